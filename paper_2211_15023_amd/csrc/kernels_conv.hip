// Convolution as an implicit GEMM on the matrix cores, one kernel for the int8 student and the bf16
// teacher.  A workgroup keeps the layer's weights (already in MFMA fragment order) in LDS and walks
// through images; for each image (or band of output rows) it stages the channels-last input patch in
// LDS once -- converting uint8 NCHW observations on the way for the first layer -- and every
// wavefront then takes tiles of 16 output pixels as the columns of 16x16 MFMA tiles whose rows are
// output channels.  K runs over (ky, kx, c): for a fixed ky the taps of a pixel are one contiguous
// run of the patch, read as 16-byte chunks (64 int8 or 32 bf16 per MFMA step).  The epilogue
// (integer bias, requantization multiplier, ReLU clamp, residual join / bias, ReLU, bf16 rounding)
// runs on the accumulators, and each lane stores 4 consecutive channels of one pixel.
#include "accerl_internal.h"

namespace accerl {

constexpr int CONV_THREADS = 256;
constexpr int CONV_PT = 2;   // pixel tiles per wave iteration (share each weight fragment read)

__device__ __forceinline__ uint32_t relu_i8x4(uint32_t x) {
    const uint32_t neg = (x & 0x80808080u) >> 7;
    return x & ~(neg * 0xffu);
}
__device__ __forceinline__ uint32_t relu_bf16x2(uint32_t x) {
    const uint32_t neg = (x & 0x80008000u) >> 15;
    return x & ~(neg * 0xffffu);
}
__device__ __forceinline__ float bf2f(uint32_t v) { return __uint_as_float(v << 16); }
__device__ __forceinline__ uint32_t f2bf(float x) {
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return u >> 16;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

template <int ALIGN>
__device__ __forceinline__ v4i lds_chunk(const char* p) {
    if constexpr (ALIGN >= 16) {
        return *(const v4i*)p;
    } else if constexpr (ALIGN == 8) {
        typedef int v2i __attribute__((ext_vector_type(2)));
        const v2i a = *(const v2i*)p, b = *(const v2i*)(p + 8);
        v4i r = {a[0], a[1], b[0], b[1]};
        return r;
    } else {
        const int* q = (const int*)p;
        v4i r = {q[0], q[1], q[2], q[3]};
        return r;
    }
}

template <int EL, int NT, int ALIGN>
__global__ __launch_bounds__(CONV_THREADS) void conv_kernel(ConvParams p) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int ESZ = (EL == EL_I8) ? 1 : 2;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = lane & 15, g = lane >> 4;
    const int pix = p.Cs_in * ESZ;                     // bytes per stored input pixel
    char* wl = smem;                                   // weight fragments
    int* koff = (int*)(smem + p.w_bytes);              // byte offset of each chunk inside the patch
    char* tile = smem + p.w_bytes + p.k_steps * 16;    // input patch

    // ---- once per workgroup: weights, chunk offsets, zeroed read slack behind the patch
    for (int i = tid; i < p.w_bytes / 16; i += CONV_THREADS) ((v4i*)wl)[i] = ((const v4i*)p.wfrag)[i];
    for (int i = tid; i < p.k_steps * 4; i += CONV_THREADS) {
        const int ky = i / p.cpr, cx = i - ky * p.cpr;
        koff[i] = (ky < p.k) ? ky * p.pitch + cx * 16 : 0;
    }
    for (int i = p.in_rows * p.pitch / 4 + tid; i < p.tile_bytes / 4; i += CONV_THREADS) ((int*)tile)[i] = 0;

    // per-lane epilogue constants: channels 16t + 4g + r
    v4i bi[NT];
    v4f bf[NT];
    v4f ml[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        if constexpr (EL == EL_I8) {
            bi[t] = *(const v4i*)((const int*)p.bias + 16 * t + 4 * g);
            ml[t] = *(const v4f*)(p.mult + 16 * t + 4 * g);
        } else {
            bf[t] = *(const v4f*)((const float*)p.bias + 16 * t + 4 * g);
        }
    }

    const int band = blockIdx.x;
    const int oy0 = band * p.TH;
    const int th = (p.Ho - oy0 < p.TH) ? (p.Ho - oy0) : p.TH;
    const int iy0 = oy0 * p.s - p.pad;
    const int n_pix = th * p.Wo;
    const int row_bytes_img = p.W * pix;               // bytes of one image row in the patch
    const int lead = p.pad * pix;                      // bytes of left padding
    const uint32_t padv = (EL == EL_I8 && p.src_nchw_u8) ? 0x80808080u : 0u;

    for (int64_t b = blockIdx.y; b < p.B; b += gridDim.y) {
        __syncthreads();
        // ---- stage the patch: every dword of in_rows x pitch is written (data or padding value)
        if (!p.src_nchw_u8) {
            const char* src = (const char*)p.in + b * (int64_t)p.H * row_bytes_img;
            const bool v16 = ((row_bytes_img | lead | p.pitch | (p.H * row_bytes_img)) & 15) == 0;
            for (int rr = wave; rr < p.in_rows; rr += CONV_THREADS / 64) {
                const int iy = iy0 + rr;
                const bool rin = iy >= 0 && iy < p.H;
                const char* srow = src + (int64_t)iy * row_bytes_img - lead;
                char* drow = tile + rr * p.pitch;
                if (v16) {
                    for (int o = lane * 16; o < p.pitch; o += 64 * 16) {
                        v4i v = {0, 0, 0, 0};
                        if (rin && o >= lead && o < lead + row_bytes_img) {
                            v = *(const v4i*)(srow + o);
                            if (p.relu_in) {
#pragma unroll
                                for (int e = 0; e < 4; ++e)
                                    v[e] = (int)((EL == EL_I8) ? relu_i8x4((uint32_t)v[e]) : relu_bf16x2((uint32_t)v[e]));
                            }
                        }
                        *(v4i*)(drow + o) = v;
                    }
                } else {
                    for (int o = lane * 4; o < p.pitch; o += 64 * 4) {
                        uint32_t v = 0;
                        if (rin && o >= lead && o < lead + row_bytes_img) {
                            v = *(const uint32_t*)(srow + o);
                            if (p.relu_in) v = (EL == EL_I8) ? relu_i8x4(v) : relu_bf16x2(v);
                        }
                        *(uint32_t*)(drow + o) = v;
                    }
                }
            }
        } else {
            // uint8 planes [C, H, W] -> channels-last pixels of 4 stored channels
            const uint8_t* src = (const uint8_t*)p.in + b * (int64_t)p.Cin_real * p.H * p.W;
            const int plane = p.H * p.W;
            const int wq = p.W >> 2;                   // groups of 4 pixels per row (W % 4 == 0)
            for (int rr = wave; rr < p.in_rows; rr += CONV_THREADS / 64) {
                const int iy = iy0 + rr;
                const bool rin = iy >= 0 && iy < p.H;
                char* drow = tile + rr * p.pitch;
                // padding columns and the tail of the row
                for (int o = lane * 4; o < p.pitch; o += 64 * 4)
                    if (!rin || o < lead || o >= lead + row_bytes_img) *(uint32_t*)(drow + o) = padv;
                if (!rin) continue;
                for (int xq = lane; xq < wq; xq += 64) {
                    uint32_t P[4];
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        P[c] = (c < p.Cin_real) ? *(const uint32_t*)(src + c * plane + iy * p.W + 4 * xq) : 0u;
                    const uint32_t lo01 = __builtin_amdgcn_perm(P[1], P[0], 0x05010400u);
                    const uint32_t hi01 = __builtin_amdgcn_perm(P[1], P[0], 0x07030602u);
                    const uint32_t lo23 = __builtin_amdgcn_perm(P[3], P[2], 0x05010400u);
                    const uint32_t hi23 = __builtin_amdgcn_perm(P[3], P[2], 0x07030602u);
                    uint32_t px[4];
                    px[0] = __builtin_amdgcn_perm(lo23, lo01, 0x05040100u);
                    px[1] = __builtin_amdgcn_perm(lo23, lo01, 0x07060302u);
                    px[2] = __builtin_amdgcn_perm(hi23, hi01, 0x05040100u);
                    px[3] = __builtin_amdgcn_perm(hi23, hi01, 0x07060302u);
                    if constexpr (EL == EL_I8) {
                        uint32_t* d = (uint32_t*)(drow + lead + 16 * xq);
                        const uint32_t live = (p.Cin_real >= 4) ? 0xffffffffu : ((1u << (8 * p.Cin_real)) - 1u);
#pragma unroll
                        for (int e = 0; e < 4; ++e) d[e] = ((px[e] ^ 0x80808080u) & live) | (0x80808080u & ~live);
                    } else {
                        uint32_t* d = (uint32_t*)(drow + lead + 32 * xq);
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            uint32_t c0 = p.lut[px[e] & 0xff], c1 = p.lut[(px[e] >> 8) & 0xff];
                            uint32_t c2 = p.lut[(px[e] >> 16) & 0xff], c3 = p.lut[px[e] >> 24];
                            if (p.Cin_real < 2) c1 = 0;
                            if (p.Cin_real < 3) c2 = 0;
                            if (p.Cin_real < 4) c3 = 0;
                            d[2 * e] = c0 | (c1 << 16);
                            d[2 * e + 1] = c2 | (c3 << 16);
                        }
                    }
                }
            }
        }
        __syncthreads();

        // ---- MFMA over pairs of pixel tiles
        const int n_tiles = (n_pix + 15) >> 4;
        for (int t0 = wave * CONV_PT; t0 < n_tiles; t0 += (CONV_THREADS / 64) * CONV_PT) {
            int pb[CONV_PT], ppix[CONV_PT];
#pragma unroll
            for (int u = 0; u < CONV_PT; ++u) {
                int pp = (t0 + u) * 16 + j;
                ppix[u] = pp;
                if (pp >= n_pix) pp = n_pix - 1;       // clamp to a valid pixel; result not stored
                const int ty = pp / p.Wo, ox = pp - ty * p.Wo;
                pb[u] = ty * p.s * p.pitch + ox * p.s * pix;
            }
            v4i acc_i[CONV_PT][NT];
            v4f acc_f[CONV_PT][NT];
#pragma unroll
            for (int u = 0; u < CONV_PT; ++u)
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    acc_i[u][t] = (v4i){0, 0, 0, 0};
                    acc_f[u][t] = (v4f){0.f, 0.f, 0.f, 0.f};
                }
            for (int st = 0; st < p.k_steps; ++st) {
                const int off = koff[st * 4 + g];
                v4i bq[CONV_PT];
#pragma unroll
                for (int u = 0; u < CONV_PT; ++u) bq[u] = lds_chunk<ALIGN>(tile + pb[u] + off);
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const v4i a = *(const v4i*)(wl + ((st * NT + t) * 64 + lane) * 16);
#pragma unroll
                    for (int u = 0; u < CONV_PT; ++u) {
                        if constexpr (EL == EL_I8) {
                            acc_i[u][t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, bq[u], acc_i[u][t], 0, 0, 0);
                        } else {
                            acc_f[u][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                __builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, bq[u]), acc_f[u][t], 0, 0, 0);
                        }
                    }
                }
            }
            // ---- epilogue
#pragma unroll
            for (int u = 0; u < CONV_PT; ++u) {
                if (ppix[u] >= n_pix) continue;
                const int ty = ppix[u] / p.Wo, ox = ppix[u] - ty * p.Wo;
                const int64_t opix = (b * p.Ho + (oy0 + ty)) * p.Wo + ox;
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const int c0 = 16 * t + 4 * g;
                    if (c0 >= p.Cs_out) continue;
                    const int64_t o = opix * p.Cs_out + c0;
                    if constexpr (EL == EL_I8) {
                        v4i v;
#pragma unroll
                        for (int r = 0; r < 4; ++r) v[r] = acc_i[u][t][r] + bi[t][r];
                        if (p.tap_acc) *(v4i*)(p.tap_acc + o) = v;
                        uint32_t pk = 0;
                        if (p.res) {
                            const uint32_t xr = *(const uint32_t*)((const int8_t*)p.res + o);
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                const float tr = (float)(int)(int8_t)(xr >> (8 * r)) * p.r;
                                float y = rintf(fmaf((float)v[r], ml[t][r], tr));
                                y = fmaxf(fminf(y, 127.0f), -127.0f);
                                pk |= (uint32_t)(uint8_t)(int8_t)(int)y << (8 * r);
                            }
                        } else {
                            const float lo = p.relu ? 0.0f : -127.0f;
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                float y = rintf((float)v[r] * ml[t][r]);
                                y = fmaxf(fminf(y, 127.0f), lo);
                                pk |= (uint32_t)(uint8_t)(int8_t)(int)y << (8 * r);
                            }
                        }
                        *(uint32_t*)((int8_t*)p.out + o) = pk;
                    } else {
                        float v[4];
#pragma unroll
                        for (int r = 0; r < 4; ++r) v[r] = acc_f[u][t][r] + bf[t][r];
                        if (p.res) {
                            const uint32_t* xr = (const uint32_t*)((const uint16_t*)p.res + o);
                            const uint32_t x0 = xr[0], x1 = xr[1];
                            v[0] = bf2f(x0 & 0xffffu) + v[0];
                            v[1] = bf2f(x0 >> 16) + v[1];
                            v[2] = bf2f(x1 & 0xffffu) + v[2];
                            v[3] = bf2f(x1 >> 16) + v[3];
                        }
                        if (p.relu) {
#pragma unroll
                            for (int r = 0; r < 4; ++r) v[r] = fmaxf(v[r], 0.0f);
                        }
                        uint32_t* d = (uint32_t*)((uint16_t*)p.out + o);
                        d[0] = f2bf(v[0]) | (f2bf(v[1]) << 16);
                        d[1] = f2bf(v[2]) | (f2bf(v[3]) << 16);
                    }
                }
            }
        }
    }
}

template <int EL, int NT>
static hipError_t launch_al(const ConvParams& p, int align, dim3 grid, size_t lds, hipStream_t s) {
#define ACCERL_CONV_GO(AL)                                                                              \
    do {                                                                                                \
        auto kfn = conv_kernel<EL, NT, AL>;                                                             \
        hipError_t e = hipFuncSetAttribute((const void*)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); \
        if (e != hipSuccess) return e;                                                                  \
        kfn<<<grid, dim3(CONV_THREADS), lds, s>>>(p);                                                   \
    } while (0)
    if (align >= 16) ACCERL_CONV_GO(16);
    else if (align == 8) ACCERL_CONV_GO(8);
    else ACCERL_CONV_GO(4);
#undef ACCERL_CONV_GO
    return hipGetLastError();
}

template <int EL>
static hipError_t launch_nt(const ConvParams& p, int NT, int align, dim3 grid, size_t lds, hipStream_t s) {
    switch (NT) {
        case 1: return launch_al<EL, 1>(p, align, grid, lds, s);
        case 2: return launch_al<EL, 2>(p, align, grid, lds, s);
        case 4: return launch_al<EL, 4>(p, align, grid, lds, s);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_conv(const ConvParams& p, Elem el, int NT, int align, hipStream_t s) {
    if (p.B <= 0) return hipSuccess;
    const size_t lds = (size_t)p.w_bytes + (size_t)p.k_steps * 16 + (size_t)p.tile_bytes;
    int64_t groups = (p.B + p.imgs_per_block - 1) / p.imgs_per_block;
    if (groups > 65535) groups = 65535;
    dim3 grid((unsigned)p.n_bands, (unsigned)groups);
    if (el == EL_I8) return launch_nt<EL_I8>(p, NT, align, grid, lds, s);
    if (el == EL_BF16) return launch_nt<EL_BF16>(p, NT, align, grid, lds, s);
    return hipErrorInvalidValue;
}

}  // namespace accerl
