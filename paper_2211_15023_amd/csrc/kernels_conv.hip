// Dispatch of the convolution kernel family (template in conv_kernel.h).
#include "conv_kernel.h"

namespace accerl {

bool conv_has_reg_variant(Elem el, int NT, int KS, int RD) {
#define X(E, N, K, R) if (el == E && NT == N && KS == K && RD == R) return true;
    ACCERL_REG_VARIANTS_I8(X)
    ACCERL_REG_VARIANTS_BF16(X)
#undef X
    return false;
}

hipError_t launch_conv(const ConvParams& p, Elem el, int NT, int KS, int RD, hipStream_t s) {
    if (p.B <= 0) return hipSuccess;
    const size_t lds = (KS > 0 ? 0 : (size_t)p.w_bytes + (size_t)p.k_steps * 16) + (size_t)p.G * p.tile_stride;
    const int pf = (p.G * p.units_img + CONV_THREADS - 1) / CONV_THREADS;
    if (pf > 16 || p.groups < 1) return hipErrorInvalidValue;
    dim3 grid((unsigned)p.n_bands, (unsigned)p.groups);
    if (KS > 0) {
        if (!conv_has_reg_variant(el, NT, KS, RD)) return hipErrorInvalidValue;
        return el == EL_I8 ? conv_launch_reg_i8(p, NT, KS, RD, pf, grid, lds, s) : conv_launch_reg_bf16(p, NT, KS, RD, pf, grid, lds, s);
    }
    if (el == EL_I8) return conv_launch_gen_i8(p, NT, RD, pf, grid, lds, s);
    if (el == EL_BF16) return conv_launch_gen_bf16(p, NT, RD, pf, grid, lds, s);
    return hipErrorInvalidValue;
}

}  // namespace accerl
