// Dense layers on the matrix cores: out[b, n] = sum_k W[n, k] x[b, k], int8 (int32 accumulate) or
// bf16 (fp32 accumulate).  Output features are the MFMA rows and states the columns, so one lane ends
// up with 4 consecutive features of one state.  A workgroup owns 64 features x 64 states and walks K
// in stages of 256 bytes per row: weights through LDS, every wavefront's 16 states straight from memory
// into its B fragments; the epilogue is chosen at compile time:
// requantize to int8, bias+ReLU to bf16, policy heads (logits / value in fp32), or the LSTM cell
// (weight rows are interleaved on the host so that the 4 accumulators of a lane are the i,f,g,o
// pre-activations of one hidden unit).
#include <stdlib.h>

#include "accerl_internal.h"

namespace accerl {

constexpr int GM_THREADS = 256;
constexpr int GM_NT = 4;          // feature tiles (of 16) per workgroup
constexpr int GM_RT = 1;          // row tiles (of 16 states) per wave
constexpr int GM_WAVES = GM_THREADS / 64;
constexpr int GM_ROWS = 16 * GM_WAVES * GM_RT;   // states per workgroup
constexpr int GM_KS = 4;          // MFMA steps per LDS stage (64 bytes of K each); a multiple of 4

__device__ __forceinline__ uint32_t g_relu_i8x4(uint32_t x) {
    const uint32_t neg = (x & 0x80808080u) >> 7;
    return x & ~(neg * 0xffu);
}
__device__ __forceinline__ uint32_t g_relu_bf16x2(uint32_t x) {
    const uint32_t neg = (x & 0x80008000u) >> 15;
    return x & ~(neg * 0xffffu);
}
__device__ __forceinline__ uint32_t g_f2bf(float x) {
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return u >> 16;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ __forceinline__ float g_sigmoid(float x) { return 1.0f / (1.0f + expf(-x)); }

template <int EL, int EPI>
__global__ __launch_bounds__(GM_THREADS, GM_THREADS == 256 ? 2 : 1) void gemm_kernel(const GemmParams p) {
    extern __shared__ __attribute__((aligned(16))) char gm_smem[];
    char* s_w = gm_smem;                              // [GM_NT][GM_KS][64 lanes][16 B]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: what depends on it stays scalar
    const int j = lane & 15, g = lane >> 4;
    const int64_t b0 = (int64_t)blockIdx.x * GM_ROWS;
    const int nt0 = blockIdx.y * GM_NT;
    const int nts = (p.n_tiles - nt0 < GM_NT) ? (p.n_tiles - nt0) : GM_NT;

    // accumulators start from the bias (features n = 16*(nt0+t) + 4g + r)
    v4i acc_i[GM_RT][GM_NT];
    v4f acc_f[GM_RT][GM_NT];
#pragma unroll
    for (int t = 0; t < GM_NT; ++t) {
        const int n0 = (nt0 + (t < nts ? t : 0)) * 16 + 4 * g;
#pragma unroll
        for (int u = 0; u < GM_RT; ++u) {
            if constexpr (EL == EL_I8) acc_i[u][t] = *(const v4i*)((const int*)p.bias + n0);
            else acc_f[u][t] = *(const v4f*)((const float*)p.bias + n0);
        }
    }

    // Stage s0 of K: the weight fragments [GM_NT tiles][GM_KS steps] go through LDS (all four wavefronts
    // read them); a wavefront's own 16 states need no sharing: lane (j, g) loads state j's 16 bytes of K
    // block g straight from memory, which is exactly its MFMA B fragment.  The loads of the next stage are
    // issued into registers before the MFMA work of the current one.  They are unconditional (clamped
    // addresses, fixed up afterwards) so that nothing serialises them.
    constexpr int WPRE = GM_NT * GM_KS * 64 / GM_THREADS;       // weight units per lane
    v4i wpre[WPRE], xpre[GM_RT][GM_KS], xcur[GM_RT][GM_KS];
    const char* xptr[GM_RT];
#pragma unroll
    for (int u = 0; u < GM_RT; ++u) {
        int64_t xrow = b0 + (wave * GM_RT + u) * 16 + j;
        if (xrow >= p.B) xrow = p.B - 1;        // a state past the batch re-reads the last one; its results are not stored
        xptr[u] = (const char*)p.x + xrow * p.Kp_bytes;
        if (p.x_frag)                           // fragment order: the tile of 16 states of this wavefront, one KiB per step
            xptr[u] = (const char*)p.x + (xrow >> 4) * ((int64_t)p.k_steps << 10) + lane * 16;
    }
    auto prefetch = [&](int s0) {
        const int ns = (p.k_steps - s0 < GM_KS) ? (p.k_steps - s0) : GM_KS;
#pragma unroll
        for (int r = 0; r < WPRE; ++r) {                         // unit r of a lane: (tile, step) pair number wave + GM_WAVES * r
            const int tr = (wave + GM_WAVES * r) % GM_NT, sr = (wave + GM_WAVES * r) / GM_NT;
            const int t = (tr < nts) ? tr : 0, st = (sr < ns) ? sr : 0;
            wpre[r] = ((const v4i*)p.wfrag)[((int64_t)(nt0 + t) * p.k_steps + s0 + st) * 64 + lane];
        }
#pragma unroll
        for (int st = 0; st < GM_KS; ++st) {
            int kb = (s0 + st) * 64 + g * 16;
            if (kb > p.Kp_bytes - 16) kb = (p.Kp_bytes - 16) & ~3;
            if (p.x_frag) kb = min(s0 + st, p.k_steps - 1) << 10;
#pragma unroll
            for (int u = 0; u < GM_RT; ++u) xpre[u][st] = *(const v4i*)(xptr[u] + kb);
        }
    };
    auto commit = [&](int s0) {
        const int ns = (p.k_steps - s0 < GM_KS) ? (p.k_steps - s0) : GM_KS;
#pragma unroll
        for (int r = 0; r < WPRE; ++r) {
            const int tr = (wave + GM_WAVES * r) % GM_NT, sr = (wave + GM_WAVES * r) / GM_NT;
            v4i v = wpre[r];
            if (!(tr < nts && sr < ns)) v = (v4i){0, 0, 0, 0};
            ((v4i*)s_w)[(tr * GM_KS + sr) * 64 + lane] = v;
        }
        // only the stage that reaches the end of the rows needs the chunk fix-ups (states past the batch
        // need none: their results are never stored)
        if ((s0 + GM_KS) * 64 <= p.Kp_bytes && !p.relu_in) {
#pragma unroll
            for (int st = 0; st < GM_KS; ++st)
#pragma unroll
                for (int u = 0; u < GM_RT; ++u) xcur[u][st] = xpre[u][st];
            return;
        }
#pragma unroll
        for (int st = 0; st < GM_KS; ++st)
#pragma unroll
        for (int u = 0; u < GM_RT; ++u) {
            const int kb = (s0 + st) * 64 + g * 16;
            v4i v = xpre[u][st];
            // a chunk that starts inside the row but runs past it re-read the row's last 16 bytes: rebuild
            // it from the bytes that belong to it (rows are padded with zero weights, not zero data)
            if (kb >= p.Kp_bytes) {
                v = (v4i){0, 0, 0, 0};
            } else if (kb > p.Kp_bytes - 16) {
                const int have = p.Kp_bytes - kb;              // 4, 8 or 12 valid bytes, at the end of v
                const int sh = (16 - have) >> 2;
                v4i w = {0, 0, 0, 0};
#pragma unroll
                for (int e = 0; e < 4; ++e) if (e + sh < 4) w[e] = v[(e + sh) & 3];
                v = w;
            }
            if (p.relu_in) {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    v[e] = (int)((EL == EL_I8) ? g_relu_i8x4((uint32_t)v[e]) : g_relu_bf16x2((uint32_t)v[e]));
            }
            xcur[u][st] = v;
        }
    };

    prefetch(0);
    for (int s0 = 0; s0 < p.k_steps; s0 += GM_KS) {
        const int ns = (p.k_steps - s0 < GM_KS) ? (p.k_steps - s0) : GM_KS;
        commit(s0);
        __syncthreads();
        if (s0 + GM_KS < p.k_steps) prefetch(s0 + GM_KS);
        // the weight fragments of step st+1 are requested from LDS before the MFMAs of step st are issued
        auto load_a = [&](v4i (&a)[GM_NT], int st) {
#pragma unroll
            for (int t = 0; t < GM_NT; ++t) a[t] = *(const v4i*)(s_w + ((t * GM_KS + st) * 64 + lane) * 16);
        };
        auto mfma = [&](const v4i (&a)[GM_NT], int st) {
#pragma unroll
            for (int t = 0; t < GM_NT; ++t)
#pragma unroll
                for (int u = 0; u < GM_RT; ++u) {
                    if constexpr (EL == EL_I8) {
                        acc_i[u][t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[t], xcur[u][st], acc_i[u][t], 0, 0, 0);
                    } else {
                        acc_f[u][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            __builtin_bit_cast(v8bf, a[t]), __builtin_bit_cast(v8bf, xcur[u][st]), acc_f[u][t], 0, 0, 0);
                    }
                }
        };
        {
            v4i fa[2][GM_NT];
            load_a(fa[0], 0);
#pragma unroll
            for (int st = 0; st < GM_KS; ++st) {
                if (st < ns) {
                    if (st + 1 < ns) load_a(fa[(st + 1) & 1], st + 1);
                    mfma(fa[st & 1], st);
                }
            }
        }
        __syncthreads();
    }

    // ---- epilogue: lane holds features n0 .. n0+3 of state b
#pragma unroll
    for (int u = 0; u < GM_RT; ++u) {
        const int64_t b = b0 + (wave * GM_RT + u) * 16 + j;
        if (b >= p.B) continue;
#pragma unroll
        for (int t = 0; t < GM_NT; ++t) {
            if (t >= nts) continue;
            const int n0 = (nt0 + t) * 16 + 4 * g;
            // stored activations: rows past N up to the row pitch are written too (zero weights and bias give zeros)
            if (n0 >= ((EPI == EPI_REQUANT || EPI == EPI_BF16) ? p.Np : p.N)) continue;
            if constexpr (EPI == EPI_REQUANT) {
                const v4f ml = *(const v4f*)(p.mult + n0);
                uint32_t pk = 0;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int v = acc_i[u][t][r];
                    if (p.tap_acc && n0 + r < p.N) p.tap_acc[b * p.N + n0 + r] = v;
                    if (p.relu) {   // clamp(rint(y), 0, 127): the pack instruction rounds to nearest even, saturates at 0
                        pk = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_amdgcn_fmed3f((float)v * ml[r], 0.0f, 127.0f), r, pk);
                    } else {
                        const float y = __builtin_amdgcn_fmed3f(rintf((float)v * ml[r]), -127.0f, 127.0f);
                        pk |= ((uint32_t)(int)y & 0xffu) << (8 * r);
                    }
                }
                *(uint32_t*)((int8_t*)p.out + b * p.Np + n0) = pk;
            } else if constexpr (EPI == EPI_HEADS_I8) {
                const v4f ml = *(const v4f*)(p.mult + n0);
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int n = n0 + r;
                    if (n > p.A) continue;
                    const int v = acc_i[u][t][r];
                    if (p.tap_acc) p.tap_acc[b * (p.A + 1) + n] = v;
                    const float o = (float)v * ml[r];
                    if (p.logits) { if (n < p.A) p.logits[b * p.A + n] = o; else p.value[b] = o; }
                }
            } else if constexpr (EPI == EPI_BF16) {
                float v[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    v[r] = acc_f[u][t][r];
                    if (p.relu) v[r] = fmaxf(v[r], 0.0f);
                }
                uint32_t* d = (uint32_t*)((uint16_t*)p.out + b * p.Np + n0);
                d[0] = g_f2bf(v[0]) | (g_f2bf(v[1]) << 16);
                d[1] = g_f2bf(v[2]) | (g_f2bf(v[3]) << 16);
            } else if constexpr (EPI == EPI_HEADS_F32ACC) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int n = n0 + r;
                    if (n > p.A) continue;
                    const float o = acc_f[u][t][r];
                    if (p.logits) { if (n < p.A) p.logits[b * p.A + n] = o; else p.value[b] = o; }
                }
            } else {   // EPI_LSTM: rows 4*unit + {i,f,g,o}
                const int unit = n0 >> 2;
                const float pi = acc_f[u][t][0], pf = acc_f[u][t][1];
                const float pg = acc_f[u][t][2], po = acc_f[u][t][3];
                const float si = g_sigmoid(pi), sf = g_sigmoid(pf), tg = tanhf(pg), so = g_sigmoid(po);
                const float c_old = p.c[b * p.Hd + unit];
                const float t1 = sf * c_old;
                const float t2 = si * tg;
                const float cn = t1 + t2;
                const float hn = so * tanhf(cn);
                p.c[b * p.Hd + unit] = cn;
                p.h[b * p.Hd + unit] = hn;
                ((uint16_t*)p.out)[b * p.Np + unit] = (uint16_t)g_f2bf(hn);   // bf16 copy for the heads
            }
        }
    }
}

// ---- small batches (int8, requantizing epilogue): too few 64-state workgroups to fill the chip, and each
// would walk all of K alone.  Here a workgroup owns 16 states x 64 features and its four wavefronts split
// K: wavefront w takes the MFMA steps w, w+4, ...; weights and states both come straight from memory
// (nothing is shared between the wavefronts), two steps are kept in flight, and the four partial
// accumulators meet in LDS, where wavefront t finishes feature tile t.  Integer sums: the result does
// not depend on the split.
constexpr int GS_NT = 4;
__global__ __launch_bounds__(256) void gemm_small_i8_kernel(const GemmParams p) {
    __shared__ __attribute__((aligned(16))) int s_part[4][GS_NT][64][4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = lane & 15, g = lane >> 4;
    const int64_t b0 = (int64_t)blockIdx.x * 16;
    const int nt0 = blockIdx.y * GS_NT;
    const int nts = (p.n_tiles - nt0 < GS_NT) ? (p.n_tiles - nt0) : GS_NT;
    int64_t xrow = b0 + j;
    const bool row_live = xrow < p.B;
    if (!row_live) xrow = p.B - 1;
    const char* xptr = (const char*)p.x + xrow * p.Kp_bytes;
    if (p.x_frag) xptr = (const char*)p.x + (xrow >> 4) * ((int64_t)p.k_steps << 10) + lane * 16;

    v4i acc[GS_NT];
#pragma unroll
    for (int t = 0; t < GS_NT; ++t) acc[t] = (v4i){0, 0, 0, 0};
    auto load = [&](int st, v4i (&a)[GS_NT], v4i& x) {
        const int sc = st < p.k_steps ? st : p.k_steps - 1;          // past the end: a valid step, not used
#pragma unroll
        for (int t = 0; t < GS_NT; ++t)
            a[t] = ((const v4i*)p.wfrag)[((int64_t)(nt0 + (t < nts ? t : 0)) * p.k_steps + sc) * 64 + lane];
        int kb = sc * 64 + g * 16;
        if (kb > p.Kp_bytes - 16) kb = (p.Kp_bytes - 16) & ~3;
        if (p.x_frag) kb = sc << 10;
        x = *(const v4i*)(xptr + kb);
    };
    auto fix_x = [&](int st, v4i v) -> v4i {
        const int kb = st * 64 + g * 16;
        if (!row_live || kb >= p.Kp_bytes) {
            v = (v4i){0, 0, 0, 0};
        } else if (kb > p.Kp_bytes - 16) {                           // the row's last, partial chunk (see gemm_kernel)
            const int sh = (16 - (p.Kp_bytes - kb)) >> 2;
            v4i w = {0, 0, 0, 0};
#pragma unroll
            for (int e = 0; e < 4; ++e) if (e + sh < 4) w[e] = v[(e + sh) & 3];
            v = w;
        }
        if (p.relu_in) {
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = (int)g_relu_i8x4((uint32_t)v[e]);
        }
        return v;
    };
    v4i a0[GS_NT], a1[GS_NT], x0, x1;
    load(wave, a0, x0);
    for (int st = wave; st < p.k_steps; st += 8) {
        load(st + 4, a1, x1);
        {
            const v4i x = fix_x(st, x0);
#pragma unroll
            for (int t = 0; t < GS_NT; ++t) acc[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a0[t], x, acc[t], 0, 0, 0);
        }
        load(st + 8, a0, x0);
        if (st + 4 < p.k_steps) {
            const v4i x = fix_x(st + 4, x1);
#pragma unroll
            for (int t = 0; t < GS_NT; ++t) acc[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a1[t], x, acc[t], 0, 0, 0);
        }
    }
#pragma unroll
    for (int t = 0; t < GS_NT; ++t) *(v4i*)s_part[wave][t][lane] = acc[t];
    __syncthreads();
    // wavefront t finishes feature tile t: features n0 .. n0+3 of state b in lane (j, g)
    const int t = wave;
    const int64_t b = b0 + j;
    const int n0 = (nt0 + t) * 16 + 4 * g;
    if (t >= nts || b >= p.B || n0 >= p.Np) return;
    v4i sum = *(const v4i*)((const int*)p.bias + n0);
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const v4i v = *(const v4i*)s_part[w][t][lane];
#pragma unroll
        for (int r = 0; r < 4; ++r) sum[r] += v[r];
    }
    const v4f ml = *(const v4f*)(p.mult + n0);
    uint32_t pk = 0;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        if (p.tap_acc && n0 + r < p.N) p.tap_acc[b * p.N + n0 + r] = sum[r];
        if (p.relu) {
            pk = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_amdgcn_fmed3f((float)sum[r] * ml[r], 0.0f, 127.0f), r, pk);
        } else {
            const float y = __builtin_amdgcn_fmed3f(rintf((float)sum[r] * ml[r]), -127.0f, 127.0f);
            pk |= ((uint32_t)(int)y & 0xffu) << (8 * r);
        }
    }
    *(uint32_t*)((int8_t*)p.out + b * p.Np + n0) = pk;
}

template <int EL, int EPI>
static hipError_t gemm_go(const GemmParams& p, dim3 grid, hipStream_t s) {
    constexpr size_t lds = GM_NT * GM_KS * 1024;
    auto kfn = gemm_kernel<EL, EPI>;
    static bool set = false;   // per instantiation: the stage buffers exceed the default dynamic LDS limit
    if (!set) {
        hipError_t e = hipFuncSetAttribute((const void*)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        set = true;
    }
    kfn<<<grid, dim3(GM_THREADS), lds, s>>>(p);
    return hipGetLastError();
}

hipError_t launch_gemm(const GemmParams& p, Elem el, GemmEpi epi, hipStream_t s) {
    if (p.B <= 0) return hipSuccess;
    dim3 grid((unsigned)((p.B + GM_ROWS - 1) / GM_ROWS), (unsigned)((p.n_tiles + GM_NT - 1) / GM_NT));
    if (el == EL_I8 && epi == EPI_REQUANT && (int64_t)grid.x * grid.y < 128 && p.k_steps >= 8) {
        // fewer than 128 workgroups of the large kernel: split K over the wavefronts instead
        dim3 gs((unsigned)((p.B + 15) / 16), (unsigned)((p.n_tiles + GS_NT - 1) / GS_NT));
        gemm_small_i8_kernel<<<gs, dim3(256), 0, s>>>(p);
        return hipGetLastError();
    }
    if (el == EL_I8 && epi == EPI_REQUANT) {
        static const bool no_stream = getenv("ACCERL_NO_GEMM_STREAM") != nullptr;
        if (!no_stream && gemm_stream_supported(p)) return launch_gemm_stream(p, s);
        return gemm_go<EL_I8, EPI_REQUANT>(p, grid, s);
    }
    if (el == EL_I8 && epi == EPI_HEADS_I8) return gemm_go<EL_I8, EPI_HEADS_I8>(p, grid, s);
    if (el == EL_BF16 && epi == EPI_BF16) return gemm_go<EL_BF16, EPI_BF16>(p, grid, s);
    if (el == EL_BF16 && epi == EPI_HEADS_F32ACC) return gemm_go<EL_BF16, EPI_HEADS_F32ACC>(p, grid, s);
    if (el == EL_BF16 && epi == EPI_LSTM) return gemm_go<EL_BF16, EPI_LSTM>(p, grid, s);
    return hipErrorInvalidValue;
}

}  // namespace accerl
