// Policy heads fused with the sampler: logits and value of 16 states per wavefront on the matrix
// cores (A = head weights, B = the states' feature rows, both loaded up front into registers), then log-softmax normaliser and inverse-CDF sampling per state.
#include "accerl_internal.h"

namespace accerl {

constexpr int HD_WAVES = 1;          // one wavefront per workgroup: no workgroup barrier, 16 states each
constexpr int HD_KMAX = 16;          // most MFMA steps of K a kernel variant holds in registers per lane
constexpr int HD_PITCH = 65;         // floats per state in the logits staging area

__device__ __forceinline__ uint32_t h_relu_i8x4(uint32_t x) {
    const uint32_t neg = (x & 0x80808080u) >> 7;
    return x & ~(neg * 0xffu);
}
__device__ __forceinline__ uint32_t h_relu_bf16x2(uint32_t x) {
    const uint32_t neg = (x & 0x80008000u) >> 15;
    return x & ~(neg * 0xffffu);
}

template <int EL, int NT, int KM>
__global__ __launch_bounds__(HD_WAVES * 64) void heads_kernel(const HeadsParams p) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    float* s_l = (float*)smem;                                      // [waves][2][16][HD_PITCH]: logits, then exp terms
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = lane & 15, g = lane >> 4;
    const int64_t row0 = ((int64_t)blockIdx.x * HD_WAVES + wave) * 16;
    int64_t row = row0 + j;
    const bool live = row < p.B;
    if (!live) row = p.B - 1;

    const float u_row = p.uniforms ? p.uniforms[row] : 0.0f;      // requested first: the sampler at the end needs it
    // this lane's K chunks of its state: unconditional loads, the tail chunk rebuilt below
    v4i xb[KM];
    const char* xrow = (const char*)p.x + row * p.Kp_bytes;
#pragma unroll
    for (int st = 0; st < KM; ++st) {
        int kb = st * 64 + g * 16;
        if (kb > p.Kp_bytes - 16) kb = (p.Kp_bytes - 16) & ~3;
        xb[st] = *(const v4i*)(xrow + kb);
    }

    // weight fragments straight into registers (every wavefront needs each of them exactly once)
    v4i wa[NT][KM];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int st = 0; st < KM; ++st)
            wa[t][st] = ((const v4i*)p.wfrag)[(t * p.k_steps + min(st, p.k_steps - 1)) * 64 + lane];
    const bool whole_steps = (p.Kp_bytes & 63) == 0;   // uniform: skips the per-chunk fix-ups below
    v4i acc_i[NT];
    v4f acc_f[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        if constexpr (EL == EL_I8) acc_i[t] = *(const v4i*)((const int*)p.bias + 16 * t + 4 * g);
        else acc_f[t] = *(const v4f*)((const float*)p.bias + 16 * t + 4 * g);
    }
#pragma unroll
    for (int st = 0; st < KM; ++st) {
        if (st < p.k_steps) {
            const int kb = st * 64 + g * 16;
            v4i v = xb[st];
            if (whole_steps) {
                // rows are whole MFMA steps: no chunk reaches past the end
            } else if (kb >= p.Kp_bytes) {
                v = (v4i){0, 0, 0, 0};
            } else if (kb > p.Kp_bytes - 16) {
                const int sh = (16 - (p.Kp_bytes - kb)) >> 2;
                v4i w = {0, 0, 0, 0};
#pragma unroll
                for (int e = 0; e < 4; ++e) if (e + sh < 4) w[e] = v[(e + sh) & 3];
                v = w;
            }
            if (p.relu_in) {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    v[e] = (int)((EL == EL_I8) ? h_relu_i8x4((uint32_t)v[e]) : h_relu_bf16x2((uint32_t)v[e]));
            }
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const v4i a = wa[t][st];
                if constexpr (EL == EL_I8) acc_i[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, v, acc_i[t], 0, 0, 0);
                else acc_f[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, v), acc_f[t], 0, 0, 0);
            }
        }
    }

    const int A = p.A;
    if constexpr (NT <= 2) {
        // At most 31 actions: a state's logits and value are the 4 NT accumulators of each of its four lanes (lane
        // group g holds outputs 16t + 4g .. 16t + 4g + 3), so the normaliser, the cumulative sums and the sampled action
        // come from in-lane arithmetic plus row-pair / half-wave swaps: no staging area and no serial scan.  Sums are
        // formed block-wise instead of in index order: they differ from an index-order evaluation by rounding (1e-7
        // relative), far inside the 1e-5 band around a CDF boundary in which a sampled action may differ; the
        // exponential is the hardware's 2^x (about 1e-7 relative per unit of |logit - max|).
        auto pair16 = [](unsigned v) { return __builtin_amdgcn_permlane16_swap(v, v, false, false); };   // {even row, odd row} of the lane's row pair
        auto pair32 = [](unsigned v) { return __builtin_amdgcn_permlane32_swap(v, v, false, false); };   // {lower half, upper half}
        float o[NT][4];
        bool is_logit[NT][4];
        float m = -3.0e38f;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            v4f ml = {1.f, 1.f, 1.f, 1.f};
            if constexpr (EL == EL_I8) ml = *(const v4f*)(p.mult + 16 * t + 4 * g);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int n = 16 * t + 4 * g + r;
                if constexpr (EL == EL_I8) {
                    o[t][r] = (float)acc_i[t][r] * ml[r];
                    if (p.tap_acc && live && n <= A) p.tap_acc[row * (A + 1) + n] = acc_i[t][r];
                } else {
                    o[t][r] = acc_f[t][r];
                }
                is_logit[t][r] = n < A;
                m = fmaxf(m, is_logit[t][r] ? o[t][r] : -3.0e38f);
            }
        }
        {
            const auto a = pair16(__float_as_uint(m));
            m = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
            const auto b = pair32(__float_as_uint(m));
            m = fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
        }
        float cum[NT][4], before[NT], Z = 0.0f;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            float run = 0.0f;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                run += is_logit[t][r] ? __builtin_amdgcn_exp2f((o[t][r] - m) * 1.44269504088896341f) : 0.0f;
                cum[t][r] = run;
            }
            const auto t16 = pair16(__float_as_uint(run));
            const float s_even = __uint_as_float(t16[0]), s_pair = s_even + __uint_as_float(t16[1]);
            const auto t32 = pair32(__float_as_uint(s_pair));
            const float s_low = __uint_as_float(t32[0]);
            // exp terms in front of this lane's: all of the blocks before t, and block t's lane groups below g
            before[t] = Z + ((g & 1) ? s_even : 0.0f) + ((g & 2) ? s_low : 0.0f);
            Z += s_low + __uint_as_float(t32[1]);
        }
        if (p.logits && live) {
            // rows of A floats: 16- or 8-byte stores where the row pitch allows (neighbouring states fill the lines)
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                float* dst = p.logits + row * A + 16 * t + 4 * g;
                if ((A & 3) == 0) {
                    if (is_logit[t][3]) *(v4f*)dst = (v4f){o[t][0], o[t][1], o[t][2], o[t][3]};
                } else if ((A & 1) == 0) {
                    typedef float v2f __attribute__((ext_vector_type(2)));
                    if (is_logit[t][1]) *(v2f*)dst = (v2f){o[t][0], o[t][1]};
                    if (is_logit[t][3]) *(v2f*)(dst + 2) = (v2f){o[t][2], o[t][3]};
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (is_logit[t][r]) dst[r] = o[t][r];
                }
            }
        }
        if (p.action) {
            const float thr = u_row * Z;
            int cnt = 0;                                   // actions whose cumulative sum does not exceed the threshold
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int r = 0; r < 4; ++r) cnt += (is_logit[t][r] && !(before[t] + cum[t][r] > thr)) ? 1 : 0;
            const auto c16 = pair16((unsigned)cnt);
            cnt = (int)(c16[0] + c16[1]);
            const auto c32 = pair32((unsigned)cnt);
            cnt = (int)(c32[0] + c32[1]);
            if (live) {
                if (g == 0) p.action[row] = min(cnt, A - 1);
#pragma unroll
                for (int t = 0; t < NT; ++t)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (16 * t + 4 * g + r == A) p.value[row] = o[t][r];
            }
        }
        return;
    }
    // heads -> staging area (outputs 16t + 4g + r of state j)
    float* stage = s_l + wave * 2 * 16 * HD_PITCH;
    float* stage_e = stage + 16 * HD_PITCH;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        v4f ml = {1.f, 1.f, 1.f, 1.f};
        if constexpr (EL == EL_I8) ml = *(const v4f*)(p.mult + 16 * t + 4 * g);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int n = 16 * t + 4 * g + r;
            if (n > A) continue;
            float o;
            if constexpr (EL == EL_I8) {
                o = (float)acc_i[t][r] * ml[r];
                if (p.tap_acc && live) p.tap_acc[row * (A + 1) + n] = acc_i[t][r];
            } else {
                o = acc_f[t][r];
            }
            stage[j * HD_PITCH + n] = o;
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    if (p.logits) {
        const int rows = (int)((p.B - row0 < 16) ? (p.B - row0) : 16);
        const float inv_A = 1.0f / (float)A;
        float* dst = p.logits + row0 * A;
        for (int i = lane; i < rows * A; i += 64) {
            const int rr = (int)(((float)i + 0.5f) * inv_A), a = i - rr * A;   // i < 1024: the float quotient is exact
            dst[i] = stage[rr * HD_PITCH + a];
        }
    }
    if (p.action) {
        // every lane of a state's 4 lane groups takes the actions a = g, g+4, ... : e_a = exp(l_a - max)
        const float* lg = stage + j * HD_PITCH;
        float m = lg[0];
        for (int a = 1; a < A; ++a) m = fmaxf(m, lg[a]);
        for (int a = g; a < A; a += 4) stage_e[j * HD_PITCH + a] = expf(lg[a] - m);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        if (g == 0 && live) {   // one lane per state: normaliser and scan in index order
            const float* ex = stage_e + j * HD_PITCH;
            p.value[row] = lg[A];
            float Z = 0.0f;
            for (int a = 0; a < A; ++a) Z += ex[a];
            const float thr = p.uniforms[row] * Z;
            float cum = 0.0f;
            int act = A - 1;
            for (int a = 0; a < A; ++a) {
                cum += ex[a];
                if (cum > thr) { act = a; break; }
            }
            p.action[row] = act;
        }
    }
}

template <int EL>
static hipError_t heads_nt(const HeadsParams& p, int nt, dim3 grid, size_t lds, hipStream_t s) {
#define GO(N, K)                                                                                       \
    do {                                                                                               \
        heads_kernel<EL, N, K><<<grid, dim3(HD_WAVES * 64), lds, s>>>(p);                              \
        return hipGetLastError();                                                                      \
    } while (0)
    const int km = p.k_steps <= 4 ? 4 : p.k_steps <= 8 ? 8 : 16;
    if (km == 4) { switch (nt) { case 1: GO(1, 4); case 2: GO(2, 4); case 3: GO(3, 4); default: GO(4, 4); } }
    if (km == 8) { switch (nt) { case 1: GO(1, 8); case 2: GO(2, 8); case 3: GO(3, 8); default: GO(4, 8); } }
    switch (nt) { case 1: GO(1, 16); default: GO(2, 16); }
#undef GO
}

// a lane holds its state's K chunks and the weight fragments of nt channel tiles: at most 32 fragments
bool heads_supported(int k_steps, int Kp_bytes, int A) {
    const int nt = (A + 1 + 15) / 16;
    const int km = k_steps <= 4 ? 4 : k_steps <= 8 ? 8 : 16;
    return k_steps <= HD_KMAX && Kp_bytes >= 16 && nt <= 4 && nt * km <= 32;
}

hipError_t launch_heads(const HeadsParams& p, Elem el, hipStream_t s) {
    if (p.B <= 0) return hipSuccess;
    const int nt = (p.A + 1 + 15) / 16;
    if (!heads_supported(p.k_steps, p.Kp_bytes, p.A)) return hipErrorInvalidValue;
    const size_t lds = (size_t)HD_WAVES * 2 * 16 * HD_PITCH * 4;
    dim3 grid((unsigned)((p.B + HD_WAVES * 16 - 1) / (HD_WAVES * 16)));
    return el == EL_I8 ? heads_nt<EL_I8>(p, nt, grid, lds, s) : heads_nt<EL_BF16>(p, nt, grid, lds, s);
}

}  // namespace accerl
