// Small kernels around the MFMA layers: sampler, observation quantizer, fp32 dense layer (teacher
// MLP), NHWC max pooling, LSTM operand packing, debug conversions.
#include "accerl_internal.h"

namespace accerl {

// ------------------------------------------------------------------ inverse-CDF sampler
// One lane per state: m = max logit, Z = sum exp(l - m) in index order, first a with cum > u*Z.
__global__ __launch_bounds__(256) void sample_kernel(const float* __restrict__ logits, const float* __restrict__ u,
                                                     int32_t* __restrict__ action, int64_t B, int A) {
    const int64_t b = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const float* lg = logits + b * A;
    float m = lg[0];
    for (int a = 1; a < A; ++a) m = fmaxf(m, lg[a]);
    float Z = 0.0f;
    for (int a = 0; a < A; ++a) Z += expf(lg[a] - m);
    const float thr = u[b] * Z;
    float cum = 0.0f;
    int act = A - 1;
    for (int a = 0; a < A; ++a) {
        cum += expf(lg[a] - m);
        if (cum > thr) { act = a; break; }
    }
    action[b] = act;
}

hipError_t launch_sample(const float* logits, const float* uniforms, int32_t* action, int64_t B, int A, hipStream_t s) {
    if (B <= 0) return hipSuccess;
    sample_kernel<<<dim3((unsigned)((B + 255) / 256)), dim3(256), 0, s>>>(logits, uniforms, action, B, A);
    return hipGetLastError();
}

// ------------------------------------------------------------------ fp32 observation -> int8 rows (padded)
__global__ __launch_bounds__(256) void quant_obs_kernel(const float* __restrict__ obs, int64_t B, int D, int Dpad,
                                                        float inv_s0, int8_t* __restrict__ out) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= B * Dpad) return;
    const int64_t b = i / Dpad;
    const int f = (int)(i - b * Dpad);
    int8_t q = 0;
    if (f < D) {
        float r = rintf(obs[b * D + f] * inv_s0);
        r = fminf(r, 127.0f);
        r = fmaxf(r, -127.0f);
        q = (int8_t)(int)r;
    }
    out[i] = q;
}

hipError_t launch_quant_obs(const float* obs, int64_t B, int D, int Dpad, float inv_s0, int8_t* out, hipStream_t s) {
    if (B <= 0) return hipSuccess;
    const int64_t n = B * Dpad;
    quant_obs_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>(obs, B, D, Dpad, inv_s0, out);
    return hipGetLastError();
}

// ------------------------------------------------------------------ fp32 dense layer
// 64 x 64 output tile per workgroup, 4 x 4 per lane, K staged through LDS 16 at a time; products are
// summed in ascending k with separate multiply and add (no contraction).
constexpr int GF_T = 64, GF_K = 16;
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmF32Params p) {
    __shared__ float sx[GF_K][GF_T + 4];
    __shared__ float sw[GF_K][GF_T + 4];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int64_t b0 = (int64_t)blockIdx.x * GF_T;
    const int n0 = blockIdx.y * GF_T;
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int jn = 0; jn < 4; ++jn) acc[i][jn] = 0.0f;
    for (int k0 = 0; k0 < p.K; k0 += GF_K) {
        for (int i = threadIdx.x; i < GF_T * GF_K; i += 256) {
            const int rr = i / GF_K, kk = i - rr * GF_K;
            const int64_t b = b0 + rr;
            const int n = n0 + rr;
            sx[kk][rr] = (b < p.B && k0 + kk < p.K) ? p.x[b * p.ldx + k0 + kk] : 0.0f;
            sw[kk][rr] = (n < p.N && k0 + kk < p.K) ? p.w[(int64_t)n * p.K + k0 + kk] : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < GF_K; ++kk) {
            float xv[4], wv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { xv[i] = sx[kk][ty * 4 + i]; wv[i] = sw[kk][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int jn = 0; jn < 4; ++jn) acc[i][jn] = fmaf(xv[i], wv[jn], acc[i][jn]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t b = b0 + ty * 4 + i;
        if (b >= p.B) continue;
#pragma unroll
        for (int jn = 0; jn < 4; ++jn) {
            const int n = n0 + tx * 4 + jn;
            if (n >= p.N) continue;
            float v = acc[i][jn] + p.bias[n];
            if (p.relu) v = fmaxf(v, 0.0f);
            if (p.heads) {
                if (n < p.A) p.logits[b * p.A + n] = v; else p.value[b] = v;
            } else {
                p.out[b * p.ldo + n] = v;
            }
        }
    }
}

hipError_t launch_gemm_f32(const GemmF32Params& p, hipStream_t s) {
    if (p.B <= 0) return hipSuccess;
    dim3 grid((unsigned)((p.B + GF_T - 1) / GF_T), (unsigned)((p.N + GF_T - 1) / GF_T));
    gemm_f32_kernel<<<grid, dim3(256), 0, s>>>(p);
    return hipGetLastError();
}

// ------------------------------------------------------------------ max pooling, NHWC, padding ignored
// One lane per output pixel and group of 4 stored channels (int8: one dword; bf16: two dwords).
__device__ __forceinline__ uint32_t max_i8x4(uint32_t a, uint32_t b) {
    uint32_t r = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int x = (int)(int8_t)(a >> (8 * e)), y = (int)(int8_t)(b >> (8 * e));
        r |= (uint32_t)(uint8_t)(int8_t)(x > y ? x : y) << (8 * e);
    }
    return r;
}

__device__ __forceinline__ float bf16_to_float(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }

__device__ __forceinline__ uint32_t max_bf16x2(uint32_t a, uint32_t b) {
    const float a0 = bf16_to_float((uint16_t)a), a1 = bf16_to_float((uint16_t)(a >> 16));
    const float b0 = bf16_to_float((uint16_t)b), b1 = bf16_to_float((uint16_t)(b >> 16));
    const uint32_t lo = (b0 > a0) ? (b & 0xffffu) : (a & 0xffffu);
    const uint32_t hi = (b1 > a1) ? (b >> 16) : (a >> 16);
    return lo | (hi << 16);
}

template <int EL>
__global__ __launch_bounds__(256) void maxpool_kernel(const uint32_t* __restrict__ in, uint32_t* __restrict__ out,
                                                      int64_t B, int H, int W, int Cg, int Ho, int Wo, int k, int s, int pad) {
    // Cg = groups of 4 channels per pixel; a group is 1 dword (int8) or 2 dwords (bf16)
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t total = B * Ho * Wo * Cg;
    if (i >= total) return;
    const int cg = (int)(i % Cg);
    int64_t t = i / Cg;
    const int ox = (int)(t % Wo); t /= Wo;
    const int oy = (int)(t % Ho);
    const int64_t b = t / Ho;
    constexpr int DW = (EL == EL_I8) ? 1 : 2;
    uint32_t m[DW];
    bool first = true;
    for (int ky = 0; ky < k; ++ky) {
        const int iy = oy * s + ky - pad;
        if (iy < 0 || iy >= H) continue;
        for (int kx = 0; kx < k; ++kx) {
            const int ix = ox * s + kx - pad;
            if (ix < 0 || ix >= W) continue;
            const uint32_t* src = in + (((b * H + iy) * W + ix) * Cg + cg) * DW;
#pragma unroll
            for (int d = 0; d < DW; ++d) {
                const uint32_t v = src[d];
                if (first) m[d] = v;
                else m[d] = (EL == EL_I8) ? max_i8x4(m[d], v) : max_bf16x2(m[d], v);
            }
            first = false;
        }
    }
#pragma unroll
    for (int d = 0; d < DW; ++d) out[i * DW + d] = m[d];
}

// 3x3 windows, pixels of 8 or 16 bytes per unit: one lane per output pixel and unit, nine unconditional
// vector loads (a tap outside the image re-reads the nearest pixel inside, which lies in the same window,
// so the maximum is unchanged), signed bytes compared as the high bytes of packed 16-bit lanes.
typedef short v2s __attribute__((ext_vector_type(2)));
template <int EL, int DW>
__global__ __launch_bounds__(256) void maxpool3_kernel(const uint32_t* __restrict__ in, uint32_t* __restrict__ out,
                                                       int H, int W, int upp, int Ho, int Wo, int s, int pad) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= Ho * Wo * upp) return;
    const int64_t b = blockIdx.y;
    const int px = i / upp, u = i - px * upp;
    const int oy = px / Wo, ox = px - oy * Wo;
    typedef uint32_t vec __attribute__((ext_vector_type(DW)));
    const vec* src = (const vec*)in + b * H * W * upp + u;
    vec tap[9];
#pragma unroll
    for (int ky = 0; ky < 3; ++ky) {
        const int iy = min(max(oy * s + ky - pad, 0), H - 1);
#pragma unroll
        for (int kx = 0; kx < 3; ++kx) {
            const int ix = min(max(ox * s + kx - pad, 0), W - 1);
            tap[ky * 3 + kx] = src[(iy * W + ix) * upp];
        }
    }
    vec r;
#pragma unroll
    for (int d = 0; d < DW; ++d) {
        if constexpr (EL == EL_I8) {
            v2s e = __builtin_bit_cast(v2s, (tap[0][d] & 0x00ff00ffu) << 8);
            v2s o = __builtin_bit_cast(v2s, tap[0][d] & 0xff00ff00u);
#pragma unroll
            for (int t = 1; t < 9; ++t) {
                e = __builtin_elementwise_max(e, __builtin_bit_cast(v2s, (tap[t][d] & 0x00ff00ffu) << 8));
                o = __builtin_elementwise_max(o, __builtin_bit_cast(v2s, tap[t][d] & 0xff00ff00u));
            }
            r[d] = ((__builtin_bit_cast(uint32_t, e) >> 8) & 0x00ff00ffu) | (__builtin_bit_cast(uint32_t, o) & 0xff00ff00u);
        } else {
            uint32_t m = tap[0][d];
#pragma unroll
            for (int t = 1; t < 9; ++t) m = max_bf16x2(m, tap[t][d]);
            r[d] = m;
        }
    }
    ((vec*)out)[(b * Ho * Wo + px) * upp + u] = r;
}

hipError_t launch_maxpool(const void* in, void* out, int64_t B, int H, int W, int Cs, int Ho, int Wo,
                          int k, int s, int pad, Elem el, hipStream_t stream) {
    if (B <= 0) return hipSuccess;
    const int pix_bytes = Cs * (el == EL_I8 ? 1 : 2);
    if (k == 3 && pad < 3 && pix_bytes % 8 == 0 && B <= 65535) {
        const int DW = (pix_bytes % 16 == 0) ? 4 : 2;
        const int upp = pix_bytes / (4 * DW);
        dim3 grid((unsigned)((Ho * Wo * upp + 255) / 256), (unsigned)B), block(256);
#define GO(E, D) maxpool3_kernel<E, D><<<grid, block, 0, stream>>>((const uint32_t*)in, (uint32_t*)out, H, W, upp, Ho, Wo, s, pad)
        if (el == EL_I8) { if (DW == 4) GO(EL_I8, 4); else GO(EL_I8, 2); }
        else { if (DW == 4) GO(EL_BF16, 4); else GO(EL_BF16, 2); }
#undef GO
        return hipGetLastError();
    }
    const int Cg = Cs / 4;
    const int64_t total = B * Ho * Wo * Cg;
    dim3 grid((unsigned)((total + 255) / 256)), block(256);
    if (el == EL_I8)
        maxpool_kernel<EL_I8><<<grid, block, 0, stream>>>((const uint32_t*)in, (uint32_t*)out, B, H, W, Cg, Ho, Wo, k, s, pad);
    else
        maxpool_kernel<EL_BF16><<<grid, block, 0, stream>>>((const uint32_t*)in, (uint32_t*)out, B, H, W, Cg, Ho, Wo, k, s, pad);
    return hipGetLastError();
}

// ------------------------------------------------------------------ LSTM operand packing
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float x) {
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)(u >> 16);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__global__ __launch_bounds__(256) void lstm_pack_kernel(LstmPackParams p) {
    const int K = p.In + p.Hd;
    const int f = blockIdx.x * 256 + threadIdx.x;      // one grid row per state: no division
    if (f >= K) return;
    const int64_t b = blockIdx.y;
    const int64_t i = b * K + f;
    const bool dn = p.done && p.done[b] != 0;
    float v;
    if (f < p.In) {
        const char* row = (const char*)p.x + b * p.x_pitch_bytes;
        if (p.x_elem == EL_I8) {
            int q = ((const int8_t*)row)[f];
            if (p.x_relu && q < 0) q = 0;
            v = (float)q * p.x_scale;
        } else if (p.x_elem == EL_BF16) {
            v = bf16_to_float(((const uint16_t*)row)[f]);
            if (p.x_relu) v = fmaxf(v, 0.0f);
        } else {
            v = ((const float*)row)[f];
            if (p.x_relu) v = fmaxf(v, 0.0f);
        }
    } else {
        const int jh = f - p.In;
        float hv = p.h[b * p.Hd + jh];
        if (dn) {
            hv = 0.0f;
            p.h[b * p.Hd + jh] = 0.0f;
            p.c[b * p.Hd + jh] = 0.0f;
        }
        v = hv;
    }
    p.xh[i] = f32_to_bf16_rne(v);
}

hipError_t launch_lstm_pack(const LstmPackParams& p, hipStream_t s) {
    if (p.B <= 0) return hipSuccess;
    if (p.B > 65535) return hipErrorInvalidValue;
    lstm_pack_kernel<<<dim3((unsigned)((p.In + p.Hd + 255) / 256), (unsigned)p.B), dim3(256), 0, s>>>(p);
    return hipGetLastError();
}

// ------------------------------------------------------------------ row gather / scatter (policy mixture)
// out row i = in row idx[i]; rows are row_bytes long (a multiple of 16), one workgroup per row
__global__ __launch_bounds__(256) void gather_rows_kernel(const char* __restrict__ in, const int32_t* __restrict__ idx,
                                                          int row_units, char* __restrict__ out) {
    const int64_t i = blockIdx.x;
    const v4i* src = (const v4i*)(in + (int64_t)idx[i] * row_units * 16);
    v4i* dst = (v4i*)(out + i * row_units * 16);
    for (int u = threadIdx.x; u < row_units; u += 256) dst[u] = src[u];
}

// uniforms of the chosen rows (in: [B], out: [n])
__global__ __launch_bounds__(256) void gather_f32_kernel(const float* __restrict__ in, const int32_t* __restrict__ idx, int64_t n, float* __restrict__ out) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) out[i] = in[idx[i]];
}

// results of a compacted forward back to their rows
__global__ __launch_bounds__(256) void scatter_out_kernel(const float* __restrict__ logits, const float* __restrict__ value, const int32_t* __restrict__ action,
                                                          const int32_t* __restrict__ idx, int64_t n, int A,
                                                          float* __restrict__ out_logits, float* __restrict__ out_value, int32_t* __restrict__ out_action) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const int64_t r = idx[i];
    if (out_logits) for (int a = 0; a < A; ++a) out_logits[r * A + a] = logits[i * A + a];
    if (out_value) out_value[r] = value[i];
    if (out_action) out_action[r] = action[i];
}

hipError_t launch_gather_rows(const void* in, const int32_t* idx, int64_t n, int64_t row_bytes, void* out, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    if (row_bytes % 16) return hipErrorInvalidValue;
    gather_rows_kernel<<<dim3((unsigned)n), dim3(256), 0, s>>>((const char*)in, idx, (int)(row_bytes / 16), (char*)out);
    return hipGetLastError();
}
hipError_t launch_gather_f32(const float* in, const int32_t* idx, int64_t n, float* out, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    gather_f32_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>(in, idx, n, out);
    return hipGetLastError();
}
hipError_t launch_scatter_out(const float* logits, const float* value, const int32_t* action, const int32_t* idx, int64_t n, int A,
                              float* out_logits, float* out_value, int32_t* out_action, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    scatter_out_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>(logits, value, action, idx, n, A, out_logits, out_value, out_action);
    return hipGetLastError();
}

// ------------------------------------------------------------------ debug conversion
__global__ __launch_bounds__(256) void bf16_to_f32_kernel(const uint16_t* __restrict__ in, float* __restrict__ out, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = bf16_to_float(in[i]);
}

hipError_t launch_bf16_to_f32(const uint16_t* in, float* out, int64_t n, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    bf16_to_f32_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>(in, out, n);
    return hipGetLastError();
}

}  // namespace accerl
