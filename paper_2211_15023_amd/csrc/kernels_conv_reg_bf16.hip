// Convolution kernels with register-resident weights, bf16 instantiations.
#include "conv_kernel.h"

namespace accerl {

hipError_t conv_launch_reg_bf16(const ConvParams& p, int NT, int KS, int RD, int pf, dim3 grid, size_t lds, hipStream_t s) {
#define X(E, N, K, R) if (NT == N && KS == K && RD == R) return conv_go_pf<E, N, K, R>(p, pf, grid, lds, s);
    ACCERL_REG_VARIANTS_BF16(X)
#undef X
    return hipErrorInvalidValue;
}

}  // namespace accerl
