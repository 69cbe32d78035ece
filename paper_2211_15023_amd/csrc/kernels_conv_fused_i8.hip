// First two convolutions of an image policy in one kernel (int8 student).
//
// The output of the first conv layer is the largest tensor the network ever writes (12.8 KB per state
// in the paper's original network, against 28 KB of observation read); written to memory and read back
// it is a third of the forward pass's traffic.  Here a workgroup takes one observation at a time:
//   phase A  uint8 planes -> channels-last tile in LDS (byte permutes), conv A on the matrix cores with
//            its weights in registers, requantized (ReLU) output written to a second LDS tile, which is
//            exactly the channels-last image conv B reads;
//   phase B  conv B from that tile with its weights in LDS; work items are (three 16-pixel tiles, half of
//            the 64 output channels), dealt round-robin to the four wavefronts: the six tiles of a 9x9
//            output are exactly one item each; requantized output goes to memory.
// Both phases use the arithmetic of conv_kernel.h (same fragments, same epilogue), so accumulators and
// activations are bit-identical to the unfused path; debug taps run the unfused kernels.
#include <stdlib.h>

#include "conv_kernel.h"

namespace accerl {

constexpr int FUSED_PF = 8;     // staging units per lane (256 lanes): observations up to 2048 units
constexpr int FUSED_ITA = 4;    // phase A rounds per observation: first-layer outputs up to 4 * 8 * 16 = 512 pixels
constexpr int FUSED_ITB = 2;    // phase B items per wavefront: second-layer outputs up to 2 * 2 * 48 = 192 pixels

template <int NTA, int KSA>
__global__ __launch_bounds__(256, 2) void conv_fused_kernel(const ConvParams a, const ConvParams b) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: what depends on it stays scalar
    const int j = lane & 15, g = lane >> 4;
    char* wl = smem;                                             // conv B weight fragments
    int* koffB = (int*)(smem + b.w_bytes);                       // conv B chunk offsets
    char* cstB = smem + b.w_bytes + b.k_steps * 16;              // conv B bias and multipliers, [2][64] words
    char* tileA = cstB + CONV_LDS_CONST;                         // observation, channels-last
    char* tileB = tileA + a.tile_stride + 32;                    // conv A output = conv B input
    const int tileB_bytes = a.Ho * a.Wo * a.Cs_out;
    const int pixA = a.Cs_in;                                    // bytes per staged observation pixel (4)

    // ---- once per workgroup
    v4i wregA[KSA][NTA];
    int koffA[KSA];
#pragma unroll
    for (int st = 0; st < KSA; ++st) {
        const int q = 4 * st + g, ky = q / a.cpr, cx = q - ky * a.cpr;
        koffA[st] = (ky < a.k) ? ky * a.pitch + cx * 16 : 0;
#pragma unroll
        for (int t = 0; t < NTA; ++t) wregA[st][t] = ((const v4i*)a.wfrag)[(st * NTA + t) * 64 + lane];
    }
    // LDS set-up, run after the first observation's loads have been issued (their latencies overlap)
    auto setup_lds = [&]() {
        lds_copy16(wl, b.wfrag, b.w_bytes / 16, tid, 256);
        for (int i = tid; i < b.k_steps * 4; i += 256) {
            const int ky = i / b.cpr, cx = i - ky * b.cpr;
            koffB[i] = (ky < b.k) ? ky * b.pitch + cx * 16 : 0;
        }
        for (int i = tid; i < 64; i += 256) {
            ((int*)cstB)[i] = ((const int*)b.bias)[i];
            ((float*)cstB)[64 + i] = b.mult[i];
        }
        for (int i = tid; i < (a.tile_stride + 32) / 4; i += 256) ((int*)tileA)[i] = (int)0x80808080u;   // obs - 128 of a zero
        for (int i = tid; i < 8; i += 256) ((int*)(tileB + tileB_bytes))[i] = 0;                          // read slack
    };
    v4i biA[NTA];
    v4f mlA[NTA];
#pragma unroll
    for (int t = 0; t < NTA; ++t) {
        biA[t] = *(const v4i*)((const int*)a.bias + 4 * NTA * g + 4 * t);
        mlA[t] = *(const v4f*)(a.mult + 4 * NTA * g + 4 * t);
    }
    const v4i* biasB = (const v4i*)(cstB + (16 * g) * 4);              // [t] -> bias of channels 16g + 4t ..
    const v4f* multB = (const v4f*)(cstB + (64 + 16 * g) * 4);

    // ---- staging of one observation: a dword (4 pixels) from each channel plane per unit, all loads
    // unconditional (a unit past the end re-reads the last one and is dropped at commit time)
    v4i pre[FUSED_PF];
    uint32_t soff[FUSED_PF];
    int doff[FUSED_PF];
    const int lead = a.pad * pixA;
#pragma unroll
    for (int i = 0; i < FUSED_PF; ++i) {
        const int u = min(tid + i * 256, a.units_img - 1);
        const int rr = (int)fdiv((uint32_t)u, a.magic_rowunits);
        const int cu = u - rr * a.row_units;
        const int iy = rr - a.pad;
        const bool rin = iy >= 0 && iy < a.H;
        soff[i] = (uint32_t)(min(max(iy, 0), a.H - 1) * a.W + 4 * cu);
        doff[i] = rin ? rr * a.pitch + lead + 4 * cu * pixA : -1;
    }
    const int plane = a.H * a.W;
    auto prefetch = [&](int64_t img) {
        const uint8_t* src = (const uint8_t*)a.in + img * (int64_t)a.Cin_real * plane;
#pragma unroll
        for (int i = 0; i < FUSED_PF; ++i) {
            v4i v;
#pragma unroll
            for (int c = 0; c < 4; ++c) v[c] = *(const int*)(src + (uint32_t)(min(c, a.Cin_real - 1) * plane) + soff[i]);
            pre[i] = v;
        }
    };
    auto commit = [&]() {
#pragma unroll
        for (int i = 0; i < FUSED_PF; ++i) {
            if (tid + i * 256 >= a.units_img) break;
            if (doff[i] < 0) continue;
            const uint32_t P0 = (uint32_t)pre[i][0], P1 = (uint32_t)pre[i][1], P2 = (uint32_t)pre[i][2], P3 = (uint32_t)pre[i][3];
            const uint32_t lo01 = __builtin_amdgcn_perm(P1, P0, 0x05010400u), hi01 = __builtin_amdgcn_perm(P1, P0, 0x07030602u);
            const uint32_t lo23 = __builtin_amdgcn_perm(P3, P2, 0x05010400u), hi23 = __builtin_amdgcn_perm(P3, P2, 0x07030602u);
            uint32_t px[4];
            px[0] = __builtin_amdgcn_perm(lo23, lo01, 0x05040100u) ^ 0x80808080u;
            px[1] = __builtin_amdgcn_perm(lo23, lo01, 0x07060302u) ^ 0x80808080u;
            px[2] = __builtin_amdgcn_perm(hi23, hi01, 0x05040100u) ^ 0x80808080u;
            px[3] = __builtin_amdgcn_perm(hi23, hi01, 0x07060302u) ^ 0x80808080u;
            if ((lead & 15) == 0) {
                *(v4i*)(tileA + doff[i]) = (v4i){(int)px[0], (int)px[1], (int)px[2], (int)px[3]};
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) *(uint32_t*)(tileA + doff[i] + 4 * e) = px[e];
            }
        }
    };

    const int npixA = a.Ho * a.Wo, tilesA = (npixA + 15) >> 4;
    const int npixB = b.Ho * b.Wo, tilesB = (npixB + 15) >> 4;
    const int rowA = a.s * a.pitch, colA = a.sx * pixA;
    const int rowB = b.s * b.pitch, colB = b.sx * b.Cs_in;

    // Which pixels a lane works on, and where they sit in the LDS tiles, is the same for every observation:
    // worked out once (phase A: up to FUSED_ITA rounds of two tiles per wavefront; phase B: up to FUSED_ITB
    // items of three tiles).
    int pbA[FUSED_ITA][2];
#pragma unroll
    for (int r = 0; r < FUSED_ITA; ++r)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int pc = min((wave * 2 + 8 * r + u) * 16 + j, npixA - 1);
            const int ty = qdiv(pc, a.inv_wo, a.hinv_wo), ox = pc - __mul24(ty, a.Wo);
            pbA[r][u] = __mul24(ty, rowA) + __mul24(ox, colA);
        }
    int pbB[FUSED_ITB][3];
#pragma unroll
    for (int r = 0; r < FUSED_ITB; ++r)
#pragma unroll
        for (int u = 0; u < 3; ++u) {
            const int pc = min((((wave + 4 * r) >> 1) * 3 + u) * 16 + j, npixB - 1);
            const int ty = qdiv(pc, b.inv_wo, b.hinv_wo), ox = pc - __mul24(ty, b.Wo);
            pbB[r][u] = __mul24(ty, rowB) + __mul24(ox, colB);
        }

    int64_t img = blockIdx.x;
    if (img < a.B) prefetch(img);
    setup_lds();
    __syncthreads();
    for (; img < a.B; img += gridDim.x) {
        commit();
        __syncthreads();     // tile A complete; every wavefront has also left phase B of the image before
        if (img + gridDim.x < a.B) prefetch(img + gridDim.x);

        // ---- phase A: conv A -> tile B (two pixel tiles per wavefront and step)
#pragma unroll
        for (int r = 0; r < FUSED_ITA; ++r) {
            const int t0 = wave * 2 + 8 * r;
            if (t0 >= tilesA) break;
            int pb[2], pp[2];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                pp[u] = (t0 + u) * 16 + j;
                pb[u] = pbA[r][u];
            }
            v4i acc[2][NTA];
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int t = 0; t < NTA; ++t) acc[u][t] = biA[t];
#pragma unroll
            for (int st = 0; st < KSA; ++st) {
                v4i bq[2];
#pragma unroll
                for (int u = 0; u < 2; ++u) bq[u] = *(const v4i*)(tileA + pb[u] + koffA[st]);
#pragma unroll
                for (int t = 0; t < NTA; ++t)
#pragma unroll
                    for (int u = 0; u < 2; ++u) acc[u][t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wregA[st][t], bq[u], acc[u][t], 0, 0, 0);
            }
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                if (pp[u] >= npixA) continue;
                char* dst = tileB + __mul24(pp[u], a.Cs_out) + 4 * NTA * g;
                uint32_t wq[NTA];
#pragma unroll
                for (int t = 0; t < NTA; ++t) {
                    uint32_t w = 0;
                    if (a.relu) {
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            w = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_amdgcn_fmed3f((float)acc[u][t][r] * mlA[t][r], 0.0f, 127.0f), r, w);
                    } else {
                        int q[4];
#pragma unroll
                        for (int r = 0; r < 4; ++r) q[r] = rne_clamp127((float)acc[u][t][r] * mlA[t][r]);
                        w = pack_low_bytes(q);
                    }
                    wq[t] = w;
                }
                if (NTA == 2 && 8 * g + 8 <= a.Cs_out) {
                    typedef int v2i __attribute__((ext_vector_type(2)));
                    *(v2i*)dst = (v2i){(int)wq[0], (int)wq[NTA - 1]};
                } else {
#pragma unroll
                    for (int t = 0; t < NTA; ++t)
                        if (4 * NTA * g + 4 * t < a.Cs_out) *(uint32_t*)(dst + 4 * t) = wq[t];
                }
            }
        }
        __syncthreads();     // tile B complete

        // ---- phase B: conv B from tile B; item = (three pixel tiles, channel half): five fragment reads feed
        // six MFMAs per step, and a 9x9 output (six tiles) is exactly one item per wavefront
        char* outB = (char*)b.out + img * (int64_t)npixB * b.Cs_out;
        const int itemsB = 2 * ((tilesB + 2) / 3);
#pragma unroll
        for (int r = 0; r < FUSED_ITB; ++r) {
            const int it = wave + 4 * r;
            if (it >= itemsB) break;
            const int h = it & 1, tile0 = (it >> 1) * 3;
            int pp[3];
            const char* base[3];
#pragma unroll
            for (int u = 0; u < 3; ++u) {
                pp[u] = (tile0 + u) * 16 + j;
                base[u] = tileB + pbB[r][u];
            }
            v4i acc[3][2];
#pragma unroll
            for (int u = 0; u < 3; ++u) { acc[u][0] = biasB[2 * h]; acc[u][1] = biasB[2 * h + 1]; }
            for (int st = 0; st < b.k_steps; ++st) {
                const v4i a0 = *(const v4i*)(wl + ((st * 4 + 2 * h) * 64 + lane) * 16);
                const v4i a1 = *(const v4i*)(wl + ((st * 4 + 2 * h + 1) * 64 + lane) * 16);
                const int ko = koffB[st * 4 + g];
                v4i bq[3];
#pragma unroll
                for (int u = 0; u < 3; ++u) bq[u] = *(const v4i*)(base[u] + ko);
#pragma unroll
                for (int u = 0; u < 3; ++u) {
                    acc[u][0] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a0, bq[u], acc[u][0], 0, 0, 0);
                    acc[u][1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a1, bq[u], acc[u][1], 0, 0, 0);
                }
            }
            const v4f m0 = multB[2 * h], m1 = multB[2 * h + 1];
#pragma unroll
            for (int u = 0; u < 3; ++u) {
                if (pp[u] >= npixB) continue;
                uint32_t w0 = 0, w1 = 0;
                if (b.relu) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        w0 = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_amdgcn_fmed3f((float)acc[u][0][r] * m0[r], 0.0f, 127.0f), r, w0);
                        w1 = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_amdgcn_fmed3f((float)acc[u][1][r] * m1[r], 0.0f, 127.0f), r, w1);
                    }
                } else {
                    int q0[4], q1[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) { q0[r] = rne_clamp127((float)acc[u][0][r] * m0[r]); q1[r] = rne_clamp127((float)acc[u][1][r] * m1[r]); }
                    w0 = pack_low_bytes(q0);
                    w1 = pack_low_bytes(q1);
                }
                typedef int v2i __attribute__((ext_vector_type(2)));
                *(v2i*)(outB + __mul24(pp[u], b.Cs_out) + 16 * g + 8 * h) = (v2i){(int)w0, (int)w1};
            }
        }
    }
}

size_t conv_fused_lds(const ConvParams& a, const ConvParams& b) {
    return (size_t)b.w_bytes + (size_t)b.k_steps * 16 + CONV_LDS_CONST + (size_t)a.tile_stride + 32 + (size_t)a.Ho * a.Wo * a.Cs_out + 32;
}

// The pair of layers this kernel covers (everything else runs layer by layer).
bool conv_fused_supported(const ConvParams& a, int NTA, int KSA, int RDA, const ConvParams& b, int NTB, int KSB, int RDB) {
    if (!a.src_u8 || a.mode != CM_U8T || a.n_bands != 1 || a.pool || a.wave_private || KSA != 4 || a.k_steps != 4 || RDA != 16) return false;
    if (NTA != 1 && NTA != 2) return false;
    if (a.units_img > 256 * FUSED_PF || (a.Cs_out & 3)) return false;
    if (a.Ho * a.Wo > FUSED_ITA * 8 * 16 || b.Ho * b.Wo > FUSED_ITB * 2 * 48) return false;
    if (b.mode != CM_FLAT || b.n_bands != 1 || b.pool || b.relu_in || b.src_u8 || NTB != 4 || KSB != 0 || RDB != 16) return false;
    if (b.Cs_out != 64 || b.Cs_in != a.Cs_out || b.H != a.Ho || b.W * b.Cs_in != a.Wo * a.Cs_out) return false;
    if (a.Ho * a.Wo * a.Cs_out >= (1 << 23) || b.Ho * b.Wo * b.Cs_out >= (1 << 23)) return false;
    return conv_fused_lds(a, b) <= 78 * 1024;            // two workgroups per compute unit
}

hipError_t launch_conv_fused(const ConvParams& a, int NTA, const ConvParams& b, hipStream_t s) {
    if (a.B <= 0) return hipSuccess;
    if (a.res || b.res) return hipErrorInvalidValue;
    static const bool no_front = getenv("ACCERL_NO_CONV_FRONT") != nullptr;
    if (!no_front && conv_front_supported(a, NTA, b)) return launch_conv_front(a, b, s);
    const size_t lds = conv_fused_lds(a, b);
    const void* fn = NTA == 1 ? (const void*)conv_fused_kernel<1, 4> : (const void*)conv_fused_kernel<2, 4>;
    static size_t set_lds[2] = {0, 0};
    static int occ[2] = {0, 0};
    const int v = NTA == 1 ? 0 : 1;
    if (lds > set_lds[v]) {
        hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        set_lds[v] = lds;
        int o = 0;
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&o, fn, 256, lds);
        if (e != hipSuccess) return e;
        occ[v] = o < 1 ? 1 : o;
    }
    // resident workgroups striding over the images, in even rounds
    const int64_t cap = (int64_t)occ[v] * conv_num_cus();
    const int64_t rounds = (a.B + cap - 1) / cap;
    dim3 grid((unsigned)((a.B + rounds - 1) / rounds));
    if (NTA == 1) conv_fused_kernel<1, 4><<<grid, dim3(256), lds, s>>>(a, b);
    else conv_fused_kernel<2, 4><<<grid, dim3(256), lds, s>>>(a, b);
    return hipGetLastError();
}

}  // namespace accerl
