// Dispatch of the convolution kernel family (template in conv_kernel.h).
#include <stdlib.h>

#include "conv_kernel.h"

namespace accerl {

// Pick the kernel variant for a layer: a tuned variant with register-resident weights (KS = k_steps)
// if one is listed, else a tuned LDS-weight variant, else the generic family.  Returns the staging
// depth (units per lane) of the chosen kernel in *PF, 0 in *KS for LDS weights; false if `pf` units
// per lane cannot be staged by any kernel.
bool conv_pick_variant(Elem el, int NT, int k_steps, int RD, int mode, int pf, bool extras, int* KS, int* PF) {
    int best_reg = 0, best_lds = 0;
#define X(E, N, K, R, M, P, F)                                                               \
    if (el == E && NT == N && RD == R && mode == M && pf <= P && (F || !extras)) {           \
        if (K == k_steps && (best_reg == 0 || P < best_reg)) best_reg = P;                   \
        if (K == 0 && (best_lds == 0 || P < best_lds)) best_lds = P;                         \
    }
    ACCERL_TUNED_I8(X)
    ACCERL_TUNED_BF16(X)
#undef X
    if (best_reg) { *KS = k_steps; *PF = best_reg; return true; }
    if (best_lds) { *KS = 0; *PF = best_lds; return true; }
    if (pf > 16) return false;
    *KS = 0; *PF = 16;
    return true;
}

int conv_num_cus() {
    static int n = 0;
    if (n <= 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v < 1) v = 256;
        n = v;
    }
    return n;
}

int conv_pixel_tiles(int NT) { return conv_pt(NT); }

// Wave-private variant for a contiguous-staging int8 layer: true if one exists for (NT, RD, PT) and a
// wavefront can stage `units` 16-byte units (one batch) by itself.
bool conv_wp_available(Elem el, int NT, int RD, int PT, int units) {
    if (el != EL_I8 || units > 64 * CONV_WP_PF) return false;
#define X(E, N, R, P, T) if (NT == N && RD == R && PT == T) return true;
    ACCERL_WP_I8(X)
#undef X
    return false;
}

hipError_t launch_conv(const ConvParams& p, Elem el, int NT, int KS, int RD, int PF, hipStream_t s) {
    if (p.B <= 0) return hipSuccess;
    static const bool no_tail = getenv("ACCERL_NO_CONV_TAIL") != nullptr;
    if (el == EL_I8 && !no_tail && conv_tail_supported(p, NT)) return launch_conv_tail(p, s);
    const size_t lds = (KS > 0 ? 0 : (size_t)p.w_bytes + (size_t)p.k_steps * 16 + CONV_LDS_CONST) + (size_t)p.lds_tiles + (size_t)(p.pool ? p.lds_otile : 0) + (size_t)p.lds_tab;
    dim3 grid((unsigned)p.n_bands, 1);
    if (p.wave_private) {
        if (KS != 0 || p.mode != CM_FLAT || p.res || p.pool || p.n_bands != 1 || p.G * p.units_img > 64 * CONV_WP_PF) return hipErrorInvalidValue;
        return conv_launch_wp_i8(p, NT, RD, p.wp_pt, grid, lds, s);
    }
    if ((p.G * p.units_img + 255) / 256 > PF) return hipErrorInvalidValue;
    hipError_t e = el == EL_I8 ? conv_launch_tuned_i8(p, NT, KS, RD, PF, grid, lds, s)
                               : conv_launch_tuned_bf16(p, NT, KS, RD, PF, grid, lds, s);
    if (e != hipErrorNotFound) return e;
    if (KS != 0 || PF != 16) return hipErrorInvalidValue;
    const int rd = RD == 16 ? 16 : 4;
    if (el == EL_I8) return conv_launch_gen_i8(p, NT, rd, grid, lds, s);
    if (el == EL_BF16) return conv_launch_gen_bf16(p, NT, rd, grid, lds, s);
    return hipErrorInvalidValue;
}

}  // namespace accerl
