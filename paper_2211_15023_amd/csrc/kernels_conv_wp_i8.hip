// Wave-private convolution kernel variants, int8 instantiations.
#include "conv_kernel.h"

namespace accerl {

hipError_t conv_launch_wp_i8(const ConvParams& p, int NT, int RD, int PT, dim3 grid, size_t lds, hipStream_t s) {
#define X(E, N, R, P, T) if (NT == N && RD == R && PT == T) return conv_go<E, N, 0, R, CM_FLAT, P, T, CONV_WP_WAVES, true, false>(p, grid, lds, s);
    ACCERL_WP_I8(X)
#undef X
    return hipErrorNotFound;
}

}  // namespace accerl
