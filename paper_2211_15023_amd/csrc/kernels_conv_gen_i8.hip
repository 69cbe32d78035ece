// Convolution kernels with weights in LDS (any number of MFMA steps), i8 instantiations.
#include "conv_kernel.h"

namespace accerl {

hipError_t conv_launch_gen_i8(const ConvParams& p, int NT, int RD, dim3 grid, size_t lds, hipStream_t s) {
    if (NT == 1) return conv_go_generic<EL_I8, 1>(p, RD, grid, lds, s);
    if (NT == 2) return conv_go_generic<EL_I8, 2>(p, RD, grid, lds, s);
    if (NT == 4) return conv_go_generic<EL_I8, 4>(p, RD, grid, lds, s);
    return hipErrorInvalidValue;
}

}  // namespace accerl
