// Tuned convolution kernel variants, bf16 instantiations.
#include "conv_kernel.h"

namespace accerl {

hipError_t conv_launch_tuned_bf16(const ConvParams& p, int NT, int KS, int RD, int pf, dim3 grid, size_t lds, hipStream_t s) {
    const bool extras = p.res != nullptr || p.pool != 0;
#define X(E, N, K, R, M, P, F) if (NT == N && KS == K && RD == R && p.mode == M && pf == P && (F || !extras)) return conv_go<E, N, K, R, M, P, conv_pt(N), 4, false, F != 0>(p, grid, lds, s);
    ACCERL_TUNED_BF16(X)
#undef X
    return hipErrorNotFound;
}

}  // namespace accerl
