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
template <int NH, int HT, bool TAPS, bool RELU>
__global__ __launch_bounds__(MLP_WAVES * 64, NH <= 2 ? 3 : 2) void mlp_i8_kernel(MlpParams p) {
    __shared__ float s_logits[MLP_WAVES][2 * 16 * MLP_LOGIT_PITCH];   // per wavefront: logits, then exp terms
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int j = lane & 15;   // state within the tile (MFMA column)
    const int g = lane >> 4;   // lane group: k-block of operands, row block of results

    // weights into registers; the hidden layers' biases and multipliers wait in LDS (a tile reads them again:
    // broadcast reads, and 64 registers fewer double the wavefronts a SIMD can hold)
    __shared__ __attribute__((aligned(16))) int s_bs[NH][64];
    __shared__ __attribute__((aligned(16))) float s_ml[NH][64];
    for (int i = threadIdx.x; i < NH * 64; i += MLP_WAVES * 64) {
        (&s_bs[0][0])[i] = p.bias[i];
        (&s_ml[0][0])[i] = p.mult[i];
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

    const int64_t n_tiles = (p.B + 15) / 16;
    const int64_t wave_id = (int64_t)blockIdx.x * MLP_WAVES + wave;
    const int64_t n_waves = (int64_t)gridDim.x * MLP_WAVES;
    float* stage = s_logits[wave];
    float* stage_e = stage + 16 * MLP_LOGIT_PITCH;
    const int D = p.D, A = p.A;
    const float inv_A = 1.0f / (float)A;
    const bool vec_obs = (D & 3) == 0;          // rows are whole 16-byte groups: four floats per load

    // this lane's 16 features (16g .. 16g+15) of its state, as four groups of four floats; a group past the row
    // (or a state past the batch) re-reads a valid address and is zeroed by `keep`
    float keep[4];
    int goff[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int f0 = 16 * g + 4 * q;
        keep[q] = (f0 < D) ? p.inv_s0 : 0.0f;                       // the quantizer's multiplier, or 0 for padding
        goff[q] = vec_obs ? min(f0, D - 4) : 0;
    }
    auto load_obs = [&](int64_t tile, v4f (&raw)[4]) {
        int64_t row = tile * 16 + j;
        if (row >= p.B) row = p.B - 1;
        const float* src = p.obs + row * D;
        if (vec_obs) {
#pragma unroll
            for (int q = 0; q < 4; ++q) raw[q] = *(const v4f*)(src + goff[q]);
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int e = 0; e < 4; ++e) raw[q][e] = src[min(16 * g + 4 * q + e, D - 1)];
        }
    };
    v4f raw[4];
    if (wave_id < n_tiles) load_obs(wave_id, raw);

    for (int64_t tile = wave_id; tile < n_tiles; tile += n_waves) {
        const int64_t row = tile * 16 + j;
        const bool live = row < p.B;
        // ---- observation -> int8 B operand
        v4i x;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            float y[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float k = keep[q];
                if (!vec_obs) k = (16 * g + 4 * q + e < D) ? p.inv_s0 : 0.0f;
                y[e] = raw[q][e] * k;
            }
            x[q] = (int)requant4(y, false);
        }
        if (tile + n_waves < n_tiles) load_obs(tile + n_waves, raw);      // in flight while this tile is multiplied
        if constexpr (TAPS) {
            if (p.tap_act && p.tap_layer == -1 && live) {
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int f = 16 * g + 4 * q + e;
                        if (f < D) p.tap_act[row * D + f] = (int8_t)((uint32_t)x[q] >> (8 * e));
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
                const v4i acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(wf[l][t], x, *(const v4i*)&s_bs[l][16 * t + 4 * g], 0, 0, 0);
                const v4f mq = *(const v4f*)&s_ml[l][16 * t + 4 * g];
                float y[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) y[r] = (float)acc[r] * mq[r];
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
            for (int a = g; a < A; a += 4) stage_e[j * MLP_LOGIT_PITCH + a] = expf(lg[a] - m);
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

template <int NH, bool TAPS, bool RELU>
static hipError_t launch_nh(const MlpParams& p, int ht, int blocks, hipStream_t s) {
    dim3 grid(blocks), block(MLP_WAVES * 64);
    switch (ht) {
        case 1: mlp_i8_kernel<NH, 1, TAPS, RELU><<<grid, block, 0, s>>>(p); break;
        case 2: mlp_i8_kernel<NH, 2, TAPS, RELU><<<grid, block, 0, s>>>(p); break;
        case 3: mlp_i8_kernel<NH, 3, TAPS, RELU><<<grid, block, 0, s>>>(p); break;
        default: mlp_i8_kernel<NH, 4, TAPS, RELU><<<grid, block, 0, s>>>(p); break;
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
#define GO(N)                                                                                                 \
    case N:                                                                                                   \
        return taps ? launch_nh<N, true, false>(p, ht, (int)blocks, s)                                        \
                    : relu ? launch_nh<N, false, true>(p, ht, (int)blocks, s) : launch_nh<N, false, false>(p, ht, (int)blocks, s);
    switch (p.n_hidden) {
        GO(1) GO(2) GO(3) GO(4)
        default: return hipErrorInvalidValue;
    }
#undef GO
}

}  // namespace accerl
