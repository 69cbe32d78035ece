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

template <int NH, int HT>
__global__ __launch_bounds__(MLP_WAVES * 64) void mlp_i8_kernel(MlpParams p) {
    __shared__ float s_logits[MLP_WAVES][16 * MLP_LOGIT_PITCH];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int j = lane & 15;   // state within the tile (MFMA column)
    const int g = lane >> 4;   // lane group: k-block of operands, row block of results

    // weights, biases and multipliers into registers
    v4i wf[NH][4];
    v4i bs[NH][4];
    v4f ml[NH][4];
#pragma unroll
    for (int l = 0; l < NH; ++l)
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            wf[l][t] = p.wfrag[(l * 4 + t) * 64 + lane];
            bs[l][t] = *(const v4i*)(p.bias + l * 64 + 16 * t + 4 * g);
            ml[l][t] = *(const v4f*)(p.mult + l * 64 + 16 * t + 4 * g);
        }
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
    const int D = p.D, A = p.A;
    const float inv_A = 1.0f / (float)A;

    for (int64_t tile = wave_id; tile < n_tiles; tile += n_waves) {
        const int64_t row = tile * 16 + j;
        const bool live = row < p.B;
        // ---- observation -> int8 B operand: this lane holds features 16g .. 16g+15 of its state
        v4i x = {0, 0, 0, 0};
        if (live) {
            const float* src = p.obs + row * D;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int f0 = 16 * g + 4 * q;
                float v[4] = {0.f, 0.f, 0.f, 0.f};
                if ((D & 3) == 0) {
                    if (f0 < D) { v4f t = *(const v4f*)(src + f0); v[0] = t[0]; v[1] = t[1]; v[2] = t[2]; v[3] = t[3]; }
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) if (f0 + e < D) v[e] = src[f0 + e];
                }
                float y[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) y[e] = v[e] * p.inv_s0;         // features past D are zeros: quantize to 0
                x[q] = (int)requant4(y, false);
            }
        }
        if (p.tap_act && p.tap_layer == -1 && live) {
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int f = 16 * g + 4 * q + e;
                    if (f < D) p.tap_act[row * D + f] = (int8_t)((uint32_t)x[q] >> (8 * e));
                }
        }
        // ---- hidden layers, chained in registers
#pragma unroll
        for (int l = 0; l < NH; ++l) {
            v4i nx;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                // the bias rides in the accumulator
                const v4i acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(wf[l][t], x, bs[l][t], 0, 0, 0);
                float y[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) y[r] = (float)acc[r] * ml[l][t][r];
                const uint32_t pk = requant4(y, p.lo[l] == 0);
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
                if (p.tap_layer == NH && p.tap_acc && live && n <= A) p.tap_acc[row * (A + 1) + n] = v;
            }
        }
        wave_lds_fence();
        // ---- outputs: coalesced logits, then one lane per state scans its row for the sampler
        if (p.logits) {
            const int64_t row0 = tile * 16;
            const int rows = (int)((p.B - row0 < 16) ? (p.B - row0) : 16);
            float* dst = p.logits + row0 * A;
            for (int i = lane; i < rows * A; i += 64) {
                const int rr = (int)(((float)i + 0.5f) * inv_A), a = i - rr * A;   // i < 1024: the float quotient is exact
                dst[i] = stage[rr * MLP_LOGIT_PITCH + a];
            }
        }
        if (g == 0 && live && p.action) {
            const float* lg = stage + j * MLP_LOGIT_PITCH;
            p.value[row] = lg[A];
            float m = lg[0];
            for (int a = 1; a < A; ++a) m = fmaxf(m, lg[a]);
            float Z = 0.0f;
            for (int a = 0; a < A; ++a) Z += expf(lg[a] - m);
            const float thr = p.uniforms[row] * Z;
            float cum = 0.0f;
            int act = A - 1;
            for (int a = 0; a < A; ++a) {
                cum += expf(lg[a] - m);
                if (cum > thr) { act = a; break; }
            }
            p.action[row] = act;
        }
        wave_lds_fence();
    }
}

template <int NH>
static hipError_t launch_nh(const MlpParams& p, int ht, int blocks, hipStream_t s) {
    dim3 grid(blocks), block(MLP_WAVES * 64);
    switch (ht) {
        case 1: mlp_i8_kernel<NH, 1><<<grid, block, 0, s>>>(p); break;
        case 2: mlp_i8_kernel<NH, 2><<<grid, block, 0, s>>>(p); break;
        case 3: mlp_i8_kernel<NH, 3><<<grid, block, 0, s>>>(p); break;
        default: mlp_i8_kernel<NH, 4><<<grid, block, 0, s>>>(p); break;
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
    switch (p.n_hidden) {
        case 1: return launch_nh<1>(p, ht, (int)blocks, s);
        case 2: return launch_nh<2>(p, ht, (int)blocks, s);
        case 3: return launch_nh<3>(p, ht, (int)blocks, s);
        case 4: return launch_nh<4>(p, ht, (int)blocks, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace accerl
