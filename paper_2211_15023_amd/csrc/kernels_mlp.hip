// Fused int8 MLP actor: observation quantizer, every dense layer, the heads, log-softmax and the
// inverse-CDF sampler in one kernel.  One wavefront owns 16 states at a time: the states are the 16
// columns of 16x16x64 int8 MFMA tiles, the weights (at most 64 units per layer) live in registers for
// the whole kernel, and the requantized output of one layer is already laid out as the B operand of
// the next (the K order of the next layer's weights is permuted on the host to match the accumulator
// layout), so activations never leave registers.  HBM traffic is the observations in and the
// logits / value / action out.
#include "accerl_internal.h"

namespace accerl {

// clamp(rint(y), -127, 127) as the bits of y + 1.5 * 2^23 (the addition rounds to the nearest integer, ties
// to even, into the low mantissa bits; float bit patterns order like the values, so an integer clamp also
// catches every |y| too large for the trick); the caller keeps the low byte.
__device__ __forceinline__ int m_rne_clamp127(float y) {
    const int b = (int)__float_as_uint(y + 12582912.0f);
    return min(max(b, 0x4B400000 - 127), 0x4B400000 + 127);
}
__device__ __forceinline__ uint32_t m_pack_low_bytes(const int (&q)[4]) {
    return __builtin_amdgcn_perm((uint32_t)q[1], (uint32_t)q[0], 0x0c0c0400u) | __builtin_amdgcn_perm((uint32_t)q[3], (uint32_t)q[2], 0x04000c0cu);
}
// four requantized values -> four int8 in a dword: lower clamp 0 (fused ReLU: the pack instruction rounds to
// nearest even and saturates at 0, the median caps at 127) or -127
__device__ __forceinline__ uint32_t requant4(const float (&y)[4], bool relu) {
    if (relu) {
        uint32_t w = 0;
#pragma unroll
        for (int r = 0; r < 4; ++r) w = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_amdgcn_fmed3f(y[r], 0.0f, 127.0f), r, w);
        return w;
    }
    int q[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) q[r] = m_rne_clamp127(y[r]);
    return m_pack_low_bytes(q);
}

__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

constexpr int MLP_WAVES = 4;          // waves per workgroup
constexpr int MLP_LOGIT_PITCH = 65;   // floats per row in the per-wave logits staging area

// TAPS: the debug taps are compiled in (forward calls run the kernel without them).
// The loop over the tiles of 16 states is written without divergent branches: observation loads are
// unconditional (clamped addresses, zeroed afterwards), the next tile's observations are requested before the
// current tile is multiplied, and the exp terms of the sampler are spread over the four lane groups of a state.
// RELU: every hidden layer has the fused ReLU (lower clamp 0), known at compile time.
// P23 (with RELU): every hidden accumulator stays below 2^23, so the accumulators start at bias + 0x4B000000, read as
// floats they are 2^23 + acc exactly, and one fused multiply-add with c = -2^23 m gives acc * m rounded once (the
// same float the convert-and-multiply form gives; a negative acc gives a negative product and the clamp's 0).
// KM: layout of the first layer -- 0: K = 64 MFMA (16 features per lane), 1: K = 32 MFMA (8 features per lane, for
// observations of at most 32 features), 2: decided at run time from the plan (debug and non-ReLU variants).
template <int NH, int HT, bool TAPS, bool RELU, bool P23, int KM>
__global__ __launch_bounds__(MLP_WAVES * 64, NH <= 2 ? 3 : 2) void mlp_i8_kernel(MlpParams p) {
    __shared__ float s_logits[MLP_WAVES][2 * 16 * MLP_LOGIT_PITCH];   // per wavefront: logits, then exp terms
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int j = lane & 15;   // state within the tile (MFMA column)
    const int g = lane >> 4;   // lane group: k-block of operands, row block of results

    // the first tile's observations are requested before anything else: on the small configured batches the kernel is one
    // chain of memory latencies, and this one then runs alongside the loads of the weights
    const int64_t n_tiles = (p.B + 15) / 16;
    const int64_t wave_id = (int64_t)blockIdx.x * MLP_WAVES + wave;
    const int64_t n_waves = (int64_t)gridDim.x * MLP_WAVES;
    float* stage = s_logits[wave];
    float* stage_e = stage + 16 * MLP_LOGIT_PITCH;
    const int D = p.D, A = p.A;
    const float inv_A = 1.0f / (float)A;
    const bool vec_obs = (D & 3) == 0;          // rows are whole 16-byte groups: four floats per load
    // observations of at most 32 features: the first layer runs on the K = 32 MFMA, a lane holds 8 features (8g .. 8g+7)
    // instead of 16 -- half the loads and half the quantizer instructions per tile
    const bool k32 = KM == 2 ? p.k32 != 0 : KM == 1;
    const int fpl = k32 ? 8 : 16;               // features per lane
    const int ngr = k32 ? 2 : 4;                // groups of four floats per lane

    // this lane's 16 features (16g .. 16g+15) of its state, as four groups of four floats; a group past the row
    // (or a state past the batch) re-reads a valid address and is zeroed by `keep`
    float keep[4];
    int goff[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int f0 = fpl * g + 4 * q;
        keep[q] = (f0 < D && q < ngr) ? p.inv_s0 : 0.0f;            // the quantizer's multiplier, or 0 for padding
        goff[q] = vec_obs ? min(f0, D - 4) : 0;
    }
    float u_next = 0.0f;                          // the state's uniform draw travels with its observation
    auto load_obs = [&](int64_t tile, v4f (&raw)[4]) {
        int64_t row = tile * 16 + j;
        if (row >= p.B) row = p.B - 1;
        if (HT == 1 && p.uniforms) u_next = p.uniforms[row];
        const float* src = p.obs + row * D;
        if (vec_obs) {
            raw[0] = *(const v4f*)(src + goff[0]);
            raw[1] = *(const v4f*)(src + goff[1]);
            if (!k32) {
                raw[2] = *(const v4f*)(src + goff[2]);
                raw[3] = *(const v4f*)(src + goff[3]);
            }
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int e = 0; e < 4; ++e) raw[q][e] = src[min(fpl * g + 4 * q + e, D - 1)];
        }
    };
    v4f raw[4];
    if (wave_id < n_tiles) load_obs(wave_id, raw);

    // weights into registers; the hidden layers' biases and multipliers wait in LDS (a tile reads them again:
    // broadcast reads, and 64 registers fewer double the wavefronts a SIMD can hold)
    __shared__ __attribute__((aligned(16))) int s_bs[NH][64];
    __shared__ __attribute__((aligned(16))) float s_ml[NH][64];
    __shared__ __attribute__((aligned(16))) float s_cf[P23 ? NH : 1][64];
    for (int i = threadIdx.x; i < NH * 64; i += MLP_WAVES * 64) {
        (&s_bs[0][0])[i] = p.bias[i] + (P23 ? 0x4B000000 : 0);
        (&s_ml[0][0])[i] = p.mult[i];
        if constexpr (P23) (&s_cf[0][0])[i] = p.cfma[i];
    }
    v4i wf[NH][4];
#pragma unroll
    for (int l = 0; l < NH; ++l)
#pragma unroll
        for (int t = 0; t < 4; ++t) wf[l][t] = p.wfrag[(l * 4 + t) * 64 + lane];
    __syncthreads();
    v4i hw[HT];
    v4i hb[HT];
    v4f hd[HT];
#pragma unroll
    for (int t = 0; t < HT; ++t) {
        hw[t] = p.wfrag[(NH * 4 + t) * 64 + lane];
        hb[t] = *(const v4i*)(p.bias + NH * 64 + 16 * t + 4 * g);
        hd[t] = *(const v4f*)(p.mult + NH * 64 + 16 * t + 4 * g);
    }


    for (int64_t tile = wave_id; tile < n_tiles; tile += n_waves) {
        const int64_t row = tile * 16 + j;
        const bool live = row < p.B;
        // the layer constants are read from LDS again in every tile (96 registers if kept): nothing is hoisted past here
        asm volatile("" ::: "memory");
        // ---- observation -> int8 B operand
        v4i x = {0, 0, 0, 0};
        auto quant_group = [&](int q) {
            float y[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float k = keep[q];
                if (!vec_obs) k = (fpl * g + 4 * q + e < D && q < ngr) ? p.inv_s0 : 0.0f;
                y[e] = raw[q][e] * k;
            }
            return (int)requant4(y, false);
        };
        const float u_cur = u_next;
        x[0] = quant_group(0);
        x[1] = quant_group(1);
        if (!k32) {
            x[2] = quant_group(2);
            x[3] = quant_group(3);
        }
        if (tile + n_waves < n_tiles) load_obs(tile + n_waves, raw);      // in flight while this tile is multiplied
        if constexpr (TAPS) {
            if (p.tap_act && p.tap_layer == -1 && live) {
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int f = fpl * g + 4 * q + e;
                        if (f < D && q < ngr) p.tap_act[row * D + f] = (int8_t)((uint32_t)x[q] >> (8 * e));
                    }
            }
        }
        // ---- hidden layers, chained in registers
#pragma unroll
        for (int l = 0; l < NH; ++l) {
            v4i nx;
            const bool relu = RELU || p.lo[l] == 0;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                // the bias rides in the accumulator
                const v4i bs = *(const v4i*)&s_bs[l][16 * t + 4 * g];
                v4i acc;
                if (l == 0 && k32) {
                    const long a8 = ((long)(uint32_t)wf[l][t][0]) | ((long)wf[l][t][1] << 32);
                    const long b8 = ((long)(uint32_t)x[0]) | ((long)x[1] << 32);
                    acc = __builtin_amdgcn_mfma_i32_16x16x32_i8(a8, b8, bs, 0, 0, 0);
                } else {
                    acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(wf[l][t], x, bs, 0, 0, 0);
                }
                const v4f mq = *(const v4f*)&s_ml[l][16 * t + 4 * g];
                float y[4];
                if constexpr (P23) {
                    const v4f cq = *(const v4f*)&s_cf[l][16 * t + 4 * g];
#pragma unroll
                    for (int r = 0; r < 4; ++r) y[r] = __builtin_fmaf(__int_as_float(acc[r]), mq[r], cq[r]);
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r) y[r] = (float)acc[r] * mq[r];
                }
                const uint32_t pk = requant4(y, relu);
                if constexpr (TAPS) {
                    if (p.tap_layer == l && live) {
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const int n = 16 * t + 4 * g + r;
                            if (n < p.tap_n) {
                                if (p.tap_acc) p.tap_acc[row * p.tap_n + n] = acc[r];
                                if (p.tap_act) p.tap_act[row * p.tap_n + n] = (int8_t)(pk >> (8 * r));
                            }
                        }
                    }
                }
                nx[t] = (int)pk;   // result tile t, rows 4g..4g+3 -> k slots 4t..4t+3 of lane group g
            }
            x = nx;
        }
        // ---- heads: logits and value from the accumulators
        if constexpr (HT == 1) {
            // At most 15 actions: a state's logits and value are the 16 accumulators of its four lanes (lane group g
            // holds outputs 4g .. 4g+3), so normaliser, cumulative sums and the sampled action come from in-lane
            // arithmetic plus row-pair / half-wave swaps -- no staging, no loops over the actions.  The sums are
            // formed pairwise instead of in index order: they differ from an index-order evaluation by rounding
            // (1e-7 relative), far inside the 1e-5 band around a CDF boundary in which a sampled action may differ.
            const v4i acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(hw[0], x, hb[0], 0, 0, 0);
            float o[4], e[4];
            bool is_logit[4];
            float m = -3.0e38f;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int n = 4 * g + r;
                o[r] = (float)acc[r] * hd[0][r];
                is_logit[r] = n < A;
                m = fmaxf(m, is_logit[r] ? o[r] : -3.0e38f);
                if constexpr (TAPS) {
                    if (p.tap_layer == NH && p.tap_acc && live && n <= A) p.tap_acc[row * (A + 1) + n] = acc[r];
                }
            }
            if (A <= 4) {
                // all logits of a state sit in its first lane (group 0, outputs 0 .. 3): maximum, normaliser and scan are
                // plain in-lane arithmetic there, no exchange between the lane groups (the other groups compute along)
                float cum[4], run = 0.0f;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    run += (r < A) ? __builtin_amdgcn_exp2f((o[r] - m) * 1.44269504088896341f) : 0.0f;
                    cum[r] = run;
                }
                if (p.logits && live && g == 0) {
                    float* dst = p.logits + row * A;
                    if (A == 4) *(v4f*)dst = (v4f){o[0], o[1], o[2], o[3]};
                    else {
#pragma unroll
                        for (int r = 0; r < 3; ++r)
                            if (r < A) dst[r] = o[r];
                    }
                }
                if (p.action && live) {
                    const float thr = u_cur * run;
                    int cnt = 0;
#pragma unroll
                    for (int r = 0; r < 4; ++r) cnt += (r < A && !(cum[r] > thr)) ? 1 : 0;
                    if (g == 0) p.action[row] = min(cnt, A - 1);
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (4 * g + r == A) p.value[row] = o[r];
                }
                continue;
            }
            auto pair16 = [](unsigned v) { return __builtin_amdgcn_permlane16_swap(v, v, false, false); };   // {even row, odd row} of the lane's row pair
            auto pair32 = [](unsigned v) { return __builtin_amdgcn_permlane32_swap(v, v, false, false); };   // {lower half, upper half}
            {
                const auto a = pair16(__float_as_uint(m));
                m = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
                const auto b = pair32(__float_as_uint(m));
                m = fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
            }
            float cum[4], run = 0.0f;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                e[r] = is_logit[r] ? __builtin_amdgcn_exp2f((o[r] - m) * 1.44269504088896341f) : 0.0f;
                run += e[r];
                cum[r] = run;
            }
            const auto t16 = pair16(__float_as_uint(run));
            const float s_even = __uint_as_float(t16[0]), s_pair = s_even + __uint_as_float(t16[1]);
            const auto t32 = pair32(__float_as_uint(s_pair));
            const float s_low = __uint_as_float(t32[0]), Z = s_low + __uint_as_float(t32[1]);
            const float before = ((g & 1) ? s_even : 0.0f) + ((g & 2) ? s_low : 0.0f);   // exp terms of the lane groups below this one
            if (p.logits && live) {
                // a row of A floats: 16-byte stores where the lane's four outputs are all logits of a row that starts
                // on a 16-byte boundary (A a multiple of 4: neighbouring states then fill whole cache lines)
                float* dst = p.logits + row * A + 4 * g;
                if ((A & 3) == 0) {
                    if (is_logit[3]) *(v4f*)dst = (v4f){o[0], o[1], o[2], o[3]};
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (is_logit[r]) dst[r] = o[r];
                }
            }
            if (p.action) {
                const float thr = u_cur * Z;
                int cnt = 0;                               // actions whose cumulative sum does not exceed the threshold
#pragma unroll
                for (int r = 0; r < 4; ++r) cnt += (is_logit[r] && !(before + cum[r] > thr)) ? 1 : 0;
                const auto c16 = pair16((unsigned)cnt);
                cnt = (int)(c16[0] + c16[1]);
                const auto c32 = pair32((unsigned)cnt);
                cnt = (int)(c32[0] + c32[1]);
                if (live) {
                    if (g == 0) p.action[row] = min(cnt, A - 1);
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (4 * g + r == A) p.value[row] = o[r];
                }
            }
            continue;
        }
#pragma unroll
        for (int t = 0; t < HT; ++t) {
            const v4i acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(hw[t], x, hb[t], 0, 0, 0);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int n = 16 * t + 4 * g + r;
                const int v = acc[r];
                const float o = (float)v * hd[t][r];
                if (n <= A) stage[j * MLP_LOGIT_PITCH + n] = o;
                if constexpr (TAPS) {
                    if (p.tap_layer == NH && p.tap_acc && live && n <= A) p.tap_acc[row * (A + 1) + n] = v;
                }
            }
        }
        wave_lds_fence();
        // ---- outputs: coalesced logits, then the sampler
        if (p.logits) {
            const int64_t row0 = tile * 16;
            const int rows = (int)((p.B - row0 < 16) ? (p.B - row0) : 16);
            float* dst = p.logits + row0 * A;
            for (int i = lane; i < rows * A; i += 64) {
                const int rr = (int)(((float)i + 0.5f) * inv_A), a = i - rr * A;   // i < 1024: the float quotient is exact
                dst[i] = stage[rr * MLP_LOGIT_PITCH + a];
            }
        }
        if (p.action) {
            // every lane of a state's four lane groups takes the actions a = g, g+4, ... : e_a = exp(l_a - max)
            const float* lg = stage + j * MLP_LOGIT_PITCH;
            float m = lg[0];
            for (int a = 1; a < A; ++a) m = fmaxf(m, lg[a]);
            // e_a = 2^((l_a - max) log2 e) on the hardware's exp2: about 1e-7 relative per unit of |l_a - max|, far inside
            // the 1e-5 band around a CDF boundary in which a sampled action may differ from an exact evaluation
            for (int a = g; a < A; a += 4) stage_e[j * MLP_LOGIT_PITCH + a] = __builtin_amdgcn_exp2f((lg[a] - m) * 1.44269504088896341f);
            wave_lds_fence();
            if (g == 0 && live) {   // one lane per state: normaliser and scan in index order
                const float* ex = stage_e + j * MLP_LOGIT_PITCH;
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
        wave_lds_fence();
    }
}

template <int NH, bool TAPS, bool RELU, bool P23, int KM>
static hipError_t launch_nh(const MlpParams& p, int ht, int blocks, hipStream_t s) {
    dim3 grid(blocks), block(MLP_WAVES * 64);
    switch (ht) {
        case 1: mlp_i8_kernel<NH, 1, TAPS, RELU, P23, KM><<<grid, block, 0, s>>>(p); break;
        case 2: mlp_i8_kernel<NH, 2, TAPS, RELU, P23, KM><<<grid, block, 0, s>>>(p); break;
        case 3: mlp_i8_kernel<NH, 3, TAPS, RELU, P23, KM><<<grid, block, 0, s>>>(p); break;
        default: mlp_i8_kernel<NH, 4, TAPS, RELU, P23, KM><<<grid, block, 0, s>>>(p); break;
    }
    return hipGetLastError();
}

hipError_t launch_mlp_i8(const MlpParams& p, hipStream_t s) {
    if (p.B <= 0) return hipSuccess;
    const int ht = (p.A + 1 + 15) / 16;
    const int64_t tiles = (p.B + 15) / 16;
    int64_t blocks = (tiles + MLP_WAVES - 1) / MLP_WAVES;
    const int64_t cap = 256 * 8;   // a few workgroups per compute unit; waves loop over the rest
    if (blocks > cap) blocks = cap;
    const bool taps = p.tap_acc != nullptr || p.tap_act != nullptr;
    bool relu = true;
    for (int l = 0; l < p.n_hidden; ++l) relu = relu && p.lo[l] == 0;
    const bool p23 = relu && p.p23 != 0 && p.cfma != nullptr;
    const bool k32 = p.k32 != 0;
#define GO(N)                                                                                                 \
    case N:                                                                                                   \
        if (taps) return launch_nh<N, true, false, false, 2>(p, ht, (int)blocks, s);                          \
        if (!relu) return launch_nh<N, false, false, false, 2>(p, ht, (int)blocks, s);                        \
        if (p23) return k32 ? launch_nh<N, false, true, true, 1>(p, ht, (int)blocks, s)                       \
                            : launch_nh<N, false, true, true, 0>(p, ht, (int)blocks, s);                      \
        return k32 ? launch_nh<N, false, true, false, 1>(p, ht, (int)blocks, s)                               \
                   : launch_nh<N, false, true, false, 0>(p, ht, (int)blocks, s);
    switch (p.n_hidden) {
        GO(1) GO(2) GO(3) GO(4)
        default: return hipErrorInvalidValue;
    }
#undef GO
}

}  // namespace accerl
