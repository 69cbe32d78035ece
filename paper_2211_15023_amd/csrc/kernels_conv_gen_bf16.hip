// Convolution kernels with weights in LDS (any number of MFMA steps), bf16 instantiations.
#include "conv_kernel.h"

namespace accerl {

hipError_t conv_launch_gen_bf16(const ConvParams& p, int NT, int RD, dim3 grid, size_t lds, hipStream_t s) {
    if (NT == 1) return conv_go_generic<EL_BF16, 1>(p, RD, grid, lds, s);
    if (NT == 2) return conv_go_generic<EL_BF16, 2>(p, RD, grid, lds, s);
    if (NT == 4) return conv_go_generic<EL_BF16, 4>(p, RD, grid, lds, s);
    return hipErrorInvalidValue;
}

}  // namespace accerl
