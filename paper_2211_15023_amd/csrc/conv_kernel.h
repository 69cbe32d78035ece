// Convolution as an implicit GEMM on the matrix cores, one kernel family for the int8 student and
// the bf16 teacher.
//
// Work split.  A workgroup (4 wavefronts) walks over batches of G images.  For a batch it stages the
// input tiles in LDS once and every wavefront then takes tiles of 16 output pixels -- numbered across
// the G images, so ragged image sizes (81 or 49 pixels) do not waste MFMA columns -- as the columns of
// 16x16 MFMA tiles whose rows are output channels.  K runs over (ky, kx, c) of the channels-last tile:
// for a fixed ky the taps of a pixel are one contiguous run, read as 16-byte chunks (64 int8 or 32 bf16
// per MFMA step).  uint8 observations arrive as channel planes; staging reads one dword (4 pixels)
// from each plane and interleaves them with byte permutes into 4-byte channels-last pixels, so that
// under the 8x8/4 first layer of the paper's networks consecutive output pixels sit 16 bytes apart.
//
// Weights are the A operand.  When they fit (KS steps x NT tiles x 4 VGPRs) they live in registers for
// the whole kernel, so LDS only feeds the pixel operand: one 16-byte read per lane serves NT MFMAs.
// Otherwise they sit in LDS in fragment order.
//
// Wave-private variant (WP).  For layers whose tiles are plain copies, every wavefront of a workgroup
// (8 of them) owns its own batch of images and its own LDS region, shares only the weights, and never
// meets the others at a barrier after start-up: while one wavefront requantizes or stages, the other
// one on its SIMD keeps the matrix core busy.
//
// Latency.  The global loads of batch i+1 are issued into registers before the MFMA work of batch i
// and written to LDS afterwards, so HBM latency hides behind compute inside one workgroup.
//
// Epilogue.  MFMA row i of tile t is output channel 4*NT*(i/4) + 4*t + i%4 (weights are laid out that
// way on the host), so a lane ends up with 4*NT consecutive channels of one pixel: bias, requantize
// (or bias/ReLU/bf16 rounding), optional residual join, one contiguous store.
#pragma once
#include "accerl_internal.h"

namespace accerl {


// max(x, 0) on four signed bytes: a negative byte's sign bit t gives t - (t >> 7) = 0x7f, and 0x7f | t = 0xff is its mask
// (full-rate instructions only: a 32-bit multiply takes four issue slots)
__device__ __forceinline__ uint32_t relu_i8x4(uint32_t x) {
    const uint32_t t = x & 0x80808080u;
    return x & ~((t - (t >> 7)) | t);
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
__device__ __forceinline__ uint32_t fdiv(uint32_t n, uint32_t magic) { return magic ? __umulhi(n, magic) : n; }
// floor(n / d) for 0 <= n < 2^20 from inv = 1/d and hinv = 0.5/d: the true value of (n + 0.5)/d is at least
// 0.5/d away from an integer, more than the rounding error of the two float operations.
__device__ __forceinline__ int qdiv(int n, float inv, float hinv) { return (int)__builtin_fmaf((float)n, inv, hinv); }
template <int RD>
__device__ __forceinline__ v4i read_chunk(const char* p) {
    if constexpr (RD == 16) {
        return *(const v4i*)p;
    } else if constexpr (RD == 8) {
        typedef int v2i __attribute__((ext_vector_type(2)));
        const v2i a = *(const v2i*)p, b = *(const v2i*)(p + 8);
        return (v4i){a[0], a[1], b[0], b[1]};
    } else {
        const int* q = (const int*)p;
        return (v4i){q[0], q[1], q[2], q[3]};
    }
}

// Per-byte signed maximum over many dwords, bytes compared as the high bytes of packed 16-bit lanes: each dword
// is split once into its even and its odd bytes (two instructions), the running maxima stay in that form (two
// packed maxima per dword), and one byte permute puts them together at the end.
struct I8x4Max {
    typedef short v2s __attribute__((ext_vector_type(2)));
    v2s e, o;
    __device__ __forceinline__ explicit I8x4Max(uint32_t x)
        : e(__builtin_bit_cast(v2s, __builtin_amdgcn_perm(x, x, 0x020c000cu))), o(__builtin_bit_cast(v2s, x & 0xff00ff00u)) {}
    __device__ __forceinline__ void take(uint32_t x) {
        const I8x4Max t(x);
        e = __builtin_elementwise_max(e, t.e);
        o = __builtin_elementwise_max(o, t.o);
    }
    __device__ __forceinline__ uint32_t get() const {
        return __builtin_amdgcn_perm(__builtin_bit_cast(uint32_t, o), __builtin_bit_cast(uint32_t, e), 0x07030501u);
    }
};
__device__ __forceinline__ uint32_t pmax_bf16x2(uint32_t a, uint32_t b) {
    const float a0 = bf2f(a & 0xffffu), a1 = bf2f(a >> 16), b0 = bf2f(b & 0xffffu), b1 = bf2f(b >> 16);
    return ((b0 > a0) ? (b & 0xffffu) : (a & 0xffffu)) | (((b1 > a1) ? (b >> 16) : (a >> 16)) << 16);
}

// clamp(rint(y), -127, 127) as the bits of y + 1.5 * 2^23: the addition rounds y to the nearest integer
// (ties to even), which then sits in the low mantissa bits; float bit patterns order like the values, so
// the clamp is an integer median and also catches every |y| too large for the trick.  The caller keeps
// only the low byte.
__device__ __forceinline__ int rne_clamp127(float y) {
    const int b = (int)__float_as_uint(y + 12582912.0f);
    return min(max(b, 0x4B400000 - 127), 0x4B400000 + 127);
}
// bytes 0 of q[0..3] -> one dword
__device__ __forceinline__ uint32_t pack_low_bytes(const int (&q)[4]) {
    const uint32_t lo = __builtin_amdgcn_perm((uint32_t)q[1], (uint32_t)q[0], 0x0c0c0400u);
    const uint32_t hi = __builtin_amdgcn_perm((uint32_t)q[3], (uint32_t)q[2], 0x04000c0cu);
    return lo | hi;
}

// Requantization with the fused ReLU, clamp(rint(float(acc) * m), 0, 127), of four accumulators into four bytes.
// P23 = false: as written (convert, multiply, clamp, pack: four instructions per value).
// P23 = true (ConvParams::pos23 layers, accumulators started at bias + 0x4B000000): the integer 0x4B000000 + acc, read
// as a float, is exactly 2^23 + acc for 0 <= acc < 2^23, so fma(that, m, -2^23 * m) is acc * m rounded once -- the very
// float the definition rounds to an integer (the conversion of acc is exact) -- in three instructions per value.  A
// negative acc gives a float below 2^23, hence a negative product, and the clamp returns the same 0.  c = -2^23 * m
// is exact (a power of two times m).
template <bool P23>
__device__ __forceinline__ uint32_t requant_relu4_p23(v4i acc, v4f m, v4f c) {
    uint32_t w = 0;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const float y = P23 ? __builtin_fmaf(__int_as_float(acc[r]), m[r], c[r]) : (float)acc[r] * m[r];
        w = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_amdgcn_fmed3f(y, 0.0f, 127.0f), r, w);
    }
    return w;
}
constexpr int P23_MAGIC = 0x4B000000;

// Copy n16 16-byte units from memory to LDS with `nthr` lanes: eight loads per lane are in flight before
// the first LDS store (a plain copy loop would wait for every load in turn).
__device__ __forceinline__ void lds_copy16(char* dst, const void* src, int n16, int tid, int nthr) {
    for (int base = 0; base < n16; base += 8 * nthr) {
        v4i r[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) r[k] = ((const v4i*)src)[min(base + k * nthr + tid, n16 - 1)];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int i = base + k * nthr + tid;
            if (i < n16) ((v4i*)dst)[i] = r[k];
        }
    }
}

__device__ __forceinline__ void conv_wave_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// NW: wavefronts per workgroup.  WP: wave-private batches (see above); else the workgroup shares one batch.
// Workgroups per compute unit the register budget is set for: four when weights, staging registers and
// accumulators are few (thin layers, which need the extra wavefronts to hide their latencies), else two.
constexpr int conv_min_blocks(int NT, int KS, int PF, int PT, int NW, int MODE) {
    if (NW != 4) return 1;
    const int regs = 4 * KS * NT + 4 * PF + (MODE == CM_FLAT ? 0 : MODE == CM_ROWS ? 4 * PF : 2 * PF) + 8 * PT * NT + 4 * PT + 8 * NT + 40;
    return regs <= 120 ? 4 : 2;
}

// EX: residual join and fused max-pooling compiled in (kernels for layers that need neither do without their registers).
template <int EL, int NT, int KS, int RD, int MODE, int PF, int PT, int NW, bool WP, bool EX>
__global__ __launch_bounds__(NW * 64, conv_min_blocks(NT, KS, PF, PT, NW, MODE)) void conv_kernel(const ConvParams p) {
    constexpr int CONV_THREADS = NW * 64;
    constexpr int SN = WP ? 64 : CONV_THREADS;      // lanes that stage one batch together
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int ESZ = (EL == EL_I8) ? 1 : 2;
    constexpr int KSR = KS > 0 ? KS : 1;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: what depends on it stays scalar
    const bool has_res = EX && p.res != nullptr, do_pool = EX && p.pool != 0;
    const int j = lane & 15, g = lane >> 4;
    const int pix = p.Cs_in * ESZ;                          // bytes per stored input pixel
    char* wl = smem;                                        // KS == 0: weight fragments + chunk offsets
    int* koff_lds = (int*)(smem + p.w_bytes);
    char* cst_lds = smem + p.w_bytes + p.k_steps * 16;        // KS == 0: bias and multipliers, [2][NT*16] words
    char* tiles_all = (KS > 0) ? smem : cst_lds + CONV_LDS_CONST;
    char* tiles = tiles_all + (WP ? wave * p.wave_tiles : 0);
    const int stid = WP ? lane : tid;               // index of this lane among those staging its batch

    auto chunk_off = [&](int q) -> int {
        const int ky = q / p.cpr, cx = q - ky * p.cpr;
        return (ky < p.k) ? ky * p.pitch + cx * 16 : 0;
    };

    // ---- once per workgroup: weights (registers or LDS), chunk offsets, tiles filled with padding
    v4i wreg[KSR][NT];
    int koffr[KSR];
    if constexpr (KS > 0) {
#pragma unroll
        for (int st = 0; st < KS; ++st) {
            koffr[st] = chunk_off(4 * st + g);
#pragma unroll
            for (int t = 0; t < NT; ++t) wreg[st][t] = ((const v4i*)p.wfrag)[(st * NT + t) * 64 + lane];
        }
    }
    // LDS set-up (weights, chunk offsets, constants, padding fill): run after the first batch's loads have
    // been issued, so that their latency and the weights' overlap
    auto setup_lds = [&]() {
        if constexpr (KS == 0) {
            lds_copy16(wl, p.wfrag, p.w_bytes / 16, tid, CONV_THREADS);
            for (int i = tid; i < p.k_steps * 4; i += CONV_THREADS) koff_lds[i] = chunk_off(i);
            for (int i = tid; i < NT * 16; i += CONV_THREADS) {
                ((int*)cst_lds)[i] = ((const int*)p.bias)[i];
                if constexpr (EL == EL_I8) ((float*)cst_lds)[NT * 16 + i] = p.mult[i];
            }
        }
        const int padv = (EL == EL_I8 && p.src_u8) ? (int)0x80808080u : 0;
        for (int i = tid; i < p.lds_tiles / 4; i += CONV_THREADS) ((int*)tiles_all)[i] = padv;
    };

    // per-lane epilogue constants: channels 4*NT*g .. 4*NT*g + 4*NT - 1.  Register-weight kernels keep
    // them in registers; LDS-weight kernels (short on registers) keep them in LDS and fetch them per tile.
    constexpr bool CREG = KS > 0;
    v4i bi[CREG ? NT : 1];
    v4f bfl[CREG ? NT : 1];
    v4f ml[CREG ? NT : 1];
    if constexpr (CREG) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            if constexpr (EL == EL_I8) {
                bi[t] = *(const v4i*)((const int*)p.bias + 4 * NT * g + 4 * t);
                ml[t] = *(const v4f*)(p.mult + 4 * NT * g + 4 * t);
            } else {
                bfl[t] = *(const v4f*)((const float*)p.bias + 4 * NT * g + 4 * t);
            }
        }
    }
    const v4i* bias_l = (const v4i*)(cst_lds + (4 * NT * g) * 4);              // [t] -> bias of channels 4NTg+4t..
    const v4f* mult_l = (const v4f*)(cst_lds + (NT * 16 + 4 * NT * g) * 4);

    // Band of output rows this workgroup computes.  With a fused 3x3 stride-2 pad-1 max-pool a band is
    // TPH pooled rows, which need the conv rows 2*py0 - 1 .. 2*(py0 + tph) - 1 inside the image.
    const int band = blockIdx.x;
    const int py0 = band * p.TPH;
    const int tph = do_pool ? ((p.PH - py0 < p.TPH) ? (p.PH - py0) : p.TPH) : 0;
    const int oy0 = do_pool ? max(2 * py0 - 1, 0) : band * p.TH;
    const int th = do_pool ? min(2 * (py0 + tph), p.Ho) - oy0 : ((p.Ho - oy0 < p.TH) ? (p.Ho - oy0) : p.TH);
    const int iy0 = oy0 * p.s - p.pad;
    const int n_pix = th * p.Wo;
    if (th <= 0) return;                                         // band past the image (a pooling plan launched without pooling)
    const float inv_npix = 1.0f / (float)n_pix, hinv_npix = 0.5f / (float)n_pix;
    char* otile = tiles_all + p.lds_tiles;                       // pooling: requantized conv rows of the batch
    const int otile_px = p.TH * p.Wo;                            // pixels per image in otile
    // A table of the batch's pixels in LDS: pixel number -> (offset of its window in the input tiles, output
    // pixel number).  It is the same for every batch, and one 8-byte read per tile replaces the reciprocal
    // arithmetic that fills it (a third of a thin layer's vector instructions).
    typedef int v2i_t __attribute__((ext_vector_type(2)));
    v2i_t* ptab = (v2i_t*)(otile + (p.pool ? p.lds_otile : 0));
    const int row_bytes_img = p.W * pix;
    const int lead = p.pad * pix;
    const int64_t n_batch = (p.B + p.G - 1) / p.G;
    const int row_step = p.s * p.pitch, col_step = p.sx * pix;   // LDS bytes per output row / column
    const int band_skip = p.Ho * p.Wo - n_pix;                   // output pixels of an image outside this band

    // ---- staging: issue the loads of a batch into registers / write them to LDS.
    // Which bytes a lane stages, and where they land in LDS, is the same for every batch, so the source
    // offset (relative to the first image of the batch) and the LDS address of each unit are worked out
    // once.  All loads are unconditional (a unit that does not exist in a short last batch, or that lies
    // in the padding, re-reads a valid address and is dropped or zeroed at commit time): loads under
    // divergent branches would be serialised by the wait-count insertion.
    v4i pre[PF];
    constexpr int NOFF = (MODE == CM_FLAT) ? 1 : PF;
    constexpr int NGAT = (MODE == CM_ROWS) ? PF : 1;
    uint32_t soff[NOFF];      // ROWS: offset of the source row; ROWSV: of the unit; U8T: of the unit in plane 0
    int doff[NOFF];           // LDS byte offset of the unit, -1 = never written (stays padding)
    int ooff[NGAT];           // ROWS: byte offset of the unit inside its image row (may lie in the padding)
    uint32_t smask[NGAT];     // ROWS: bit e set = dword e of the unit is real data
    if constexpr (MODE != CM_FLAT) {
        const int n_units = p.G * p.units_img;
#pragma unroll
        for (int i = 0; i < PF; ++i) {
            const int u = min(stid + i * SN, n_units - 1);
            const int img = (int)fdiv((uint32_t)u, p.magic_units);
            const int w = u - img * p.units_img;
            const int rr = (int)fdiv((uint32_t)w, p.magic_rowunits);
            const int cu = w - rr * p.row_units;
            const int iy = iy0 + rr;
            const bool rin = iy >= 0 && iy < p.H;
            const int iyc = min(max(iy, 0), p.H - 1);
            if constexpr (MODE == CM_ROWSV) {
                // units are the aligned 16-byte pieces of the image rows; padding is never written
                soff[i] = (uint32_t)((img * p.H + iyc) * row_bytes_img + cu * 16);
                doff[i] = rin ? img * p.tile_stride + rr * p.pitch + lead + cu * 16 : -1;
            } else if constexpr (MODE == CM_ROWS) {
                // units are the 16-byte pieces of the padded LDS rows, gathered dword by dword
                soff[i] = (uint32_t)((img * p.H + iyc) * row_bytes_img);
                const int o = cu * 16 - lead;
                uint32_t m = 0;
#pragma unroll
                for (int e = 0; e < 4; ++e) m |= (rin && o + 4 * e >= 0 && o + 4 * e < row_bytes_img) ? (1u << e) : 0u;
                smask[i] = m;
                ooff[i] = o;
                doff[i] = img * p.tile_stride + rr * p.pitch + cu * 16;
            } else {
                soff[i] = (uint32_t)(img * p.Cin_real * p.H * p.W + iyc * p.W + 4 * cu);
                doff[i] = rin ? img * p.tile_stride + rr * p.pitch + lead + 4 * cu * pix : -1;
            }
        }
    }
    auto prefetch = [&](int64_t batch) {
        const int64_t b0 = batch * p.G;
        const int gc = (int)((p.B - b0 < p.G) ? (p.B - b0) : p.G);
        const int last = gc * p.units_img - 1;
        if constexpr (MODE == CM_FLAT) {
            // a batch of images is one contiguous range, read unit by unit
            const char* src = (const char*)p.in + b0 * (int64_t)p.img_bytes;
#pragma unroll
            for (int i = 0; i < PF; ++i) {
                const int u = min(stid + i * SN, last);
                pre[i] = *(const v4i*)(src + (uint32_t)u * 16u);
            }
        } else if constexpr (MODE == CM_ROWSV) {
            const char* src = (const char*)p.in + b0 * (int64_t)p.H * row_bytes_img;
#pragma unroll
            for (int i = 0; i < PF; ++i) {
                const uint32_t so = (stid + i * SN <= last) ? soff[i] : 0u;   // a unit of a missing image reads image 0
                pre[i] = *(const v4i*)(src + so);
            }
        } else if constexpr (MODE == CM_ROWS) {
            const char* src = (const char*)p.in + b0 * (int64_t)p.H * row_bytes_img;
#pragma unroll
            for (int i = 0; i < PF; ++i) {
                const uint32_t so = (stid + i * SN <= last) ? soff[i] : 0u;
                v4i v;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    v[e] = *(const int*)(src + so + (uint32_t)min(max(ooff[i] + 4 * e, 0), row_bytes_img - 4));
                pre[i] = v;
            }
        } else {   // CM_U8T: one dword (4 pixels) from each channel plane
            const uint8_t* src = (const uint8_t*)p.in + b0 * (int64_t)p.Cin_real * p.H * p.W;
            const int plane = p.H * p.W;
#pragma unroll
            for (int i = 0; i < PF; ++i) {
                const uint32_t so = (stid + i * SN <= last) ? soff[i] : 0u;
                v4i v;
#pragma unroll
                for (int c = 0; c < 4; ++c) v[c] = *(const int*)(src + (uint32_t)(min(c, p.Cin_real - 1) * plane) + so);
                pre[i] = v;
            }
        }
    };
    auto commit = [&](int64_t batch) {
        const int64_t b0 = batch * p.G;
        const int gc = (int)((p.B - b0 < p.G) ? (p.B - b0) : p.G);
        const int total = gc * p.units_img;
#pragma unroll
        for (int i = 0; i < PF; ++i) {
            const int u = stid + i * SN;
            if (u >= total) break;
            v4i v = pre[i];
            if constexpr (MODE != CM_U8T) {
                if constexpr (MODE == CM_ROWSV) {
                    if (doff[i] < 0) continue;                // row outside the image: stays padding
                } else if constexpr (MODE == CM_ROWS) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = ((smask[i] >> e) & 1u) ? v[e] : 0;
                }
                if (p.relu_in) {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        v[e] = (int)((EL == EL_I8) ? relu_i8x4((uint32_t)v[e]) : relu_bf16x2((uint32_t)v[e]));
                }
                if constexpr (MODE == CM_FLAT) {
                    *(v4i*)(tiles + u * 16) = v;              // tiles of a batch are contiguous like the images
                } else if (MODE == CM_ROWS || (lead & 15) == 0) {
                    *(v4i*)(tiles + doff[i]) = v;
                } else if ((lead & 7) == 0) {
                    typedef int v2i __attribute__((ext_vector_type(2)));
                    *(v2i*)(tiles + doff[i]) = (v2i){v[0], v[1]};
                    *(v2i*)(tiles + doff[i] + 8) = (v2i){v[2], v[3]};
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) *(int*)(tiles + doff[i] + 4 * e) = v[e];
                }
            } else {
                if (doff[i] < 0) continue;                    // row outside the image: stays padding
                const uint32_t P0 = (uint32_t)v[0], P1 = (uint32_t)v[1], P2 = (uint32_t)v[2], P3 = (uint32_t)v[3];
                const uint32_t lo01 = __builtin_amdgcn_perm(P1, P0, 0x05010400u);
                const uint32_t hi01 = __builtin_amdgcn_perm(P1, P0, 0x07030602u);
                const uint32_t lo23 = __builtin_amdgcn_perm(P3, P2, 0x05010400u);
                const uint32_t hi23 = __builtin_amdgcn_perm(P3, P2, 0x07030602u);
                uint32_t px[4];
                px[0] = __builtin_amdgcn_perm(lo23, lo01, 0x05040100u);
                px[1] = __builtin_amdgcn_perm(lo23, lo01, 0x07060302u);
                px[2] = __builtin_amdgcn_perm(hi23, hi01, 0x05040100u);
                px[3] = __builtin_amdgcn_perm(hi23, hi01, 0x07060302u);
                if constexpr (EL == EL_I8) {
                    if ((lead & 15) == 0) {
                        *(v4i*)(tiles + doff[i]) = (v4i){(int)(px[0] ^ 0x80808080u), (int)(px[1] ^ 0x80808080u),
                                                         (int)(px[2] ^ 0x80808080u), (int)(px[3] ^ 0x80808080u)};
                    } else {
                        uint32_t* d = (uint32_t*)(tiles + doff[i]);
#pragma unroll
                        for (int e = 0; e < 4; ++e) d[e] = px[e] ^ 0x80808080u;
                    }
                } else {
                    uint32_t* d = (uint32_t*)(tiles + doff[i]);
                    if (p.lut == nullptr) {
                        // bf16(v / 255) as bf16(float(v) * (1 / 255)): the host has checked all 256 values against the table
                        typedef float v2f __attribute__((ext_vector_type(2)));
                        typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
                        const float k255 = 1.0f / 255.0f;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            v2f lo = {(float)(px[e] & 0xff) * k255, (float)((px[e] >> 8) & 0xff) * k255};
                            v2f hi = {(float)((px[e] >> 16) & 0xff) * k255, (float)(px[e] >> 24) * k255};
                            if (p.Cin_real < 2) lo[1] = 0.0f;
                            if (p.Cin_real < 3) hi[0] = 0.0f;
                            if (p.Cin_real < 4) hi[1] = 0.0f;
                            d[2 * e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, v2bf));
                            d[2 * e + 1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, v2bf));
                        }
                    } else {
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
    };

    int64_t batch = WP ? (int64_t)blockIdx.y * NW + wave : blockIdx.y;
    const int64_t bstride = WP ? (int64_t)gridDim.y * NW : gridDim.y;
    if (batch < n_batch) prefetch(batch);
    setup_lds();
    {
        for (int pp = tid; pp < p.G * n_pix; pp += CONV_THREADS) {
            const int img = qdiv(pp, inv_npix, hinv_npix);
            const int rem = pp - __mul24(img, n_pix);
            const int ty = qdiv(rem, p.inv_wo, p.hinv_wo), ox = rem - __mul24(ty, p.Wo);
            int second = do_pool ? __mul24(img, otile_px) + rem : pp + __mul24(img, band_skip);
            if (p.out_frag) {
                // fragment order of the dense layer that follows: image number in the batch, and the offset of the
                // pixel's first channel inside a tile of 16 states (K index k = rem * Cs_out: step k / 64, block k % 64 / 16)
                const int k = __mul24(rem, p.Cs_out);
                second = (img << 20) | (((k >> 6) << 10) + (((k & 63) >> 4) << 8) + (k & 15));
            }
            ptab[pp] = (v2i_t){__mul24(img, p.tile_stride) + __mul24(ty, row_step) + __mul24(ox, col_step), second};
        }
    }
    __syncthreads();   // padding fill (and LDS weights) visible before the first commit / compute
    for (; batch < n_batch; batch += bstride) {
        commit(batch);
        if constexpr (WP) conv_wave_fence(); else __syncthreads();
        if (batch + bstride < n_batch) prefetch(batch + bstride);

        const int64_t b0 = batch * p.G;
        const int gc = (int)((p.B - b0 < p.G) ? (p.B - b0) : p.G);
        const int total_pix = gc * n_pix;
        const int n_tiles = (total_pix + 15) >> 4;
        const int64_t base_el = ((b0 * p.Ho + oy0) * p.Wo) * (int64_t)p.Cs_out;   // first element this block writes
        char* out_b = (char*)p.out + base_el * ESZ;
        const char* res_b = (const char*)p.res + base_el * ESZ;
        int32_t* tap_b = p.tap_acc + base_el;
        for (int t0 = (WP ? 0 : wave * PT); t0 < n_tiles; t0 += (WP ? 1 : NW) * PT) {
            int pb[PT], ppix[PT], prel[PT];   // window offset in the tiles, pixel number, output pixel
#pragma unroll
            for (int u = 0; u < PT; ++u) {
                const int pp = (t0 + u) * 16 + j;
                ppix[u] = pp;
                const v2i_t e = ptab[min(pp, total_pix - 1)];   // past the end: a valid pixel, result not stored
                pb[u] = e[0];
                prel[u] = e[1];
            }
            v4i acc_i[PT][NT];
            v4f acc_f[PT][NT];
#pragma unroll
            for (int u = 0; u < PT; ++u)
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    // the bias rides in the accumulator
                    if constexpr (EL == EL_I8) acc_i[u][t] = CREG ? bi[CREG ? t : 0] : bias_l[t];
                    else acc_f[u][t] = CREG ? bfl[CREG ? t : 0] : __builtin_bit_cast(v4f, bias_l[t]);
                }
            // residual stream of the tile's pixels: requested before the MFMA work so that the epilogue
            // finds it there (pixels past the end were clamped to a valid one above; lanes past the last
            // channel re-read a valid group)
            uint32_t xres[PT][NT][ESZ];
            if (has_res) {
#pragma unroll
                for (int u = 0; u < PT; ++u) {
                    const int pr = prel[u];
#pragma unroll
                    for (int t = 0; t < NT; ++t) {
                        const uint32_t* xp = (const uint32_t*)(res_b + ((uint32_t)__mul24(pr, p.Cs_out) + (uint32_t)min(4 * NT * g + 4 * t, p.Cs_out - 4)) * ESZ);
#pragma unroll
                        for (int e = 0; e < ESZ; ++e) xres[u][t][e] = xp[e];
                    }
                }
            }
            auto load_b = [&](v4i (&bq)[PT], int off) {
#pragma unroll
                for (int u = 0; u < PT; ++u) bq[u] = read_chunk<RD>(tiles + pb[u] + off);
            };
            auto load_a = [&](v4i (&a)[NT], int st) {
#pragma unroll
                for (int t = 0; t < NT; ++t) a[t] = *(const v4i*)(wl + ((st * NT + t) * 64 + lane) * 16);
            };
            auto mfma = [&](const v4i (&a)[NT], const v4i (&bq)[PT]) {
#pragma unroll
                for (int t = 0; t < NT; ++t)
#pragma unroll
                    for (int u = 0; u < PT; ++u) {
                        if constexpr (EL == EL_I8) {
                            acc_i[u][t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[t], bq[u], acc_i[u][t], 0, 0, 0);
                        } else {
                            acc_f[u][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                __builtin_bit_cast(v8bf, a[t]), __builtin_bit_cast(v8bf, bq[u]), acc_f[u][t], 0, 0, 0);
                        }
                    }
            };
            if constexpr (KS > 0) {
#pragma unroll
                for (int st = 0; st < KS; ++st) {
                    v4i bq[PT];
                    load_b(bq, koffr[st]);
                    mfma(wreg[st], bq);
                }
            } else {
                for (int st = 0; st < p.k_steps; ++st) {
                    v4i a[NT], bq[PT];
                    load_a(a, st);
                    load_b(bq, koff_lds[st * 4 + g]);
                    mfma(a, bq);
                }
            }
            // ---- epilogue: this lane owns channels c0 .. c0 + 4*NT - 1 of its pixel
#pragma unroll
            for (int u = 0; u < PT; ++u) {
                if (ppix[u] >= total_pix) continue;
                const int c0 = 4 * NT * g;
                const uint32_t o_res = (uint32_t)__mul24(prel[u], p.Cs_out);
                const uint32_t o = o_res + (uint32_t)c0;
                if constexpr (EL == EL_I8) {
                    uint32_t pk[NT];
                    v4f mq[NT];
#pragma unroll
                    for (int t = 0; t < NT; ++t) mq[t] = CREG ? ml[CREG ? t : 0] : mult_l[t];
#pragma unroll
                    for (int t = 0; t < NT; ++t) {
                        const v4i v = acc_i[u][t];
                        if (p.tap_acc && c0 + 4 * t < p.Cs_out) *(v4i*)(tap_b + o + 4 * t) = v;
                        uint32_t w = 0;
                        if (has_res) {
                            int q[4];
#pragma unroll
                            for (int r = 0; r < 4; ++r) {
                                const float tr = (float)(int)(int8_t)(xres[u][t][0] >> (8 * r)) * p.r;
                                q[r] = rne_clamp127(fmaf((float)v[r], mq[t][r], tr));
                            }
                            w = pack_low_bytes(q);
                        } else if (p.relu) {
                            // clamp(rint(y), 0, 127): the pack instruction rounds to nearest even and saturates at 0
#pragma unroll
                            for (int r = 0; r < 4; ++r)
                                w = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_amdgcn_fmed3f((float)v[r] * mq[t][r], 0.0f, 127.0f), r, w);
                        } else {
                            int q[4];
#pragma unroll
                            for (int r = 0; r < 4; ++r) q[r] = rne_clamp127((float)v[r] * mq[t][r]);
                            w = pack_low_bytes(q);
                        }
                        pk[t] = w;
                    }
                    if (do_pool) {
#pragma unroll
                        for (int t = 0; t < NT; ++t)
                            if (c0 + 4 * t < p.Cs_out) *(uint32_t*)(otile + o + 4 * t) = pk[t];
                    } else {
                        int8_t* dst = (int8_t*)out_b + o;
                        if (p.out_frag) {
                            const int64_t b = b0 + (prel[u] >> 20);
                            dst = (int8_t*)p.out + (b >> 4) * ((int64_t)p.frag_ks << 10) + (prel[u] & 0xfffff) + (((int)b & 15) << 4)
                                  + ((c0 >> 4) << 8) + (c0 & 15);
                        }
                        if (NT == 4 && c0 + 16 <= p.Cs_out) {
                            *(v4i*)dst = (v4i){(int)pk[0], (int)pk[1 % NT], (int)pk[2 % NT], (int)pk[3 % NT]};
                        } else if (NT == 2 && c0 + 8 <= p.Cs_out) {
                            typedef int v2i __attribute__((ext_vector_type(2)));
                            *(v2i*)dst = (v2i){(int)pk[0], (int)pk[1 % NT]};
                        } else {
#pragma unroll
                            for (int t = 0; t < NT; ++t)
                                if (c0 + 4 * t < p.Cs_out) *(uint32_t*)(dst + 4 * t) = pk[t];
                        }
                    }
                } else {
#pragma unroll
                    for (int t = 0; t < NT; ++t) {
                        if (c0 + 4 * t >= p.Cs_out) continue;
                        float v[4];
#pragma unroll
                        for (int r = 0; r < 4; ++r) v[r] = acc_f[u][t][r];
                        if (has_res) {
                            const uint32_t x0 = xres[u][t][0], x1 = xres[u][t][ESZ - 1];
                            v[0] = bf2f(x0 & 0xffffu) + v[0];
                            v[1] = bf2f(x0 >> 16) + v[1];
                            v[2] = bf2f(x1 & 0xffffu) + v[2];
                            v[3] = bf2f(x1 >> 16) + v[3];
                        }
                        if (p.relu) {
#pragma unroll
                            for (int r = 0; r < 4; ++r) v[r] = fmaxf(v[r], 0.0f);
                        }
                        const uint32_t w0 = f2bf(v[0]) | (f2bf(v[1]) << 16), w1 = f2bf(v[2]) | (f2bf(v[3]) << 16);
                        if (do_pool) {
                            uint32_t* d = (uint32_t*)(otile + 2 * (o + 4 * t));
                            d[0] = w0; d[1] = w1;
                        } else {
                            uint32_t* d = (uint32_t*)((uint16_t*)out_b + o + 4 * t);
                            d[0] = w0; d[1] = w1;
                        }
                    }
                }
            }
        }
        if constexpr (!WP) {
            if (do_pool) {
                // max-pool the band's conv rows from LDS: one lane per pooled pixel and unit of 8 or 16 bytes.
                // A tap outside the image re-reads the nearest pixel inside, which lies in the same window.
                __syncthreads();
                const int ush = p.pool_ush, U = p.pool_unit;                  // units per real pixel = 1 << ush
                const int rowu = p.PW << ush;                                 // units per pooled row
                const int imgu = tph * rowu;
                const float inv_imgu = 1.0f / (float)imgu, hinv_imgu = 0.5f / (float)imgu;
                const int total_u = gc * imgu;
                const int Wc = p.pool_W;                                      // real (unpacked) conv pixels per row
                const int64_t out_img = (int64_t)p.PH * rowu * U;             // pooled bytes per image
                for (int idx = tid; idx < total_u; idx += CONV_THREADS) {
                    const int img = qdiv(idx, inv_imgu, hinv_imgu);
                    const int r = idx - __mul24(img, imgu);
                    const int py = qdiv(r, p.inv_prow, p.hinv_prow);
                    const int r2 = r - __mul24(py, rowu);
                    const int px = r2 >> ush, uu = r2 - (px << ush);
                    const char* src = otile + __mul24(img, otile_px) * (p.Cs_out * ESZ) + uu * U;
                    int ro[3], co[3];
#pragma unroll
                    for (int kk = 0; kk < 3; ++kk) {
                        ro[kk] = __mul24(min(max(2 * (py0 + py) - 1 + kk, 0), p.Ho - 1) - oy0, Wc);
                        co[kk] = min(max(2 * px - 1 + kk, 0), Wc - 1);
                    }
                    char* dst = (char*)p.pool_out + (b0 + img) * out_img + ((int64_t)__mul24(py0 + py, rowu) + r2) * U;
                    if (U == 16) {
                        v4i m = *(const v4i*)(src + ((ro[0] + co[0]) << ush) * 16);
                        if constexpr (EL == EL_I8) {
                            I8x4Max mx[4] = {I8x4Max((uint32_t)m[0]), I8x4Max((uint32_t)m[1]), I8x4Max((uint32_t)m[2]), I8x4Max((uint32_t)m[3])};
#pragma unroll
                            for (int t = 1; t < 9; ++t) {
                                const v4i v = *(const v4i*)(src + ((ro[t / 3] + co[t % 3]) << ush) * 16);
#pragma unroll
                                for (int e = 0; e < 4; ++e) mx[e].take((uint32_t)v[e]);
                            }
#pragma unroll
                            for (int e = 0; e < 4; ++e) m[e] = (int)mx[e].get();
                        } else {
#pragma unroll
                            for (int t = 1; t < 9; ++t) {
                                const v4i v = *(const v4i*)(src + ((ro[t / 3] + co[t % 3]) << ush) * 16);
#pragma unroll
                                for (int e = 0; e < 4; ++e) m[e] = (int)pmax_bf16x2((uint32_t)m[e], (uint32_t)v[e]);
                            }
                        }
                        *(v4i*)dst = m;
                    } else {
                        typedef int v2i __attribute__((ext_vector_type(2)));
                        v2i m = *(const v2i*)(src + ((ro[0] + co[0]) << ush) * 8);
                        if constexpr (EL == EL_I8) {
                            I8x4Max mx[2] = {I8x4Max((uint32_t)m[0]), I8x4Max((uint32_t)m[1])};
#pragma unroll
                            for (int t = 1; t < 9; ++t) {
                                const v2i v = *(const v2i*)(src + ((ro[t / 3] + co[t % 3]) << ush) * 8);
#pragma unroll
                                for (int e = 0; e < 2; ++e) mx[e].take((uint32_t)v[e]);
                            }
#pragma unroll
                            for (int e = 0; e < 2; ++e) m[e] = (int)mx[e].get();
                        } else {
#pragma unroll
                            for (int t = 1; t < 9; ++t) {
                                const v2i v = *(const v2i*)(src + ((ro[t / 3] + co[t % 3]) << ush) * 8);
#pragma unroll
                                for (int e = 0; e < 2; ++e) m[e] = (int)pmax_bf16x2((uint32_t)m[e], (uint32_t)v[e]);
                            }
                        }
                        *(v2i*)dst = m;
                    }
                }
            }
        }
        // every wave is done reading the tiles before the next commit overwrites them
        if constexpr (WP) conv_wave_fence(); else __syncthreads();
    }
}


// Launch: the grid is (bands, groups).  Every workgroup stays resident (groups is at most what the chip
// holds at this kernel's occupancy) and walks the image batches in strides of `groups`; groups is then
// lowered to the smallest count that needs the same number of rounds, so that the rounds are even.
int conv_num_cus();
template <int EL, int NT, int KS, int RD, int MODE, int PF, int PT, int NW, bool WP, bool EX>
hipError_t conv_go(const ConvParams& p, dim3 grid, size_t lds, hipStream_t s) {
    auto kfn = conv_kernel<EL, NT, KS, RD, MODE, PF, PT, NW, WP, EX>;
    static size_t set_lds = 0;   // per instantiation: raise the dynamic LDS limit when needed
    if (lds > set_lds) {
        hipError_t e = hipFuncSetAttribute((const void*)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        set_lds = lds;
    }
    // occupancy of this instantiation at this LDS size: a few sizes occur per policy, remembered in a small table
    static size_t occ_lds[4] = {~(size_t)0, ~(size_t)0, ~(size_t)0, ~(size_t)0};
    static int occ_val[4] = {1, 1, 1, 1};
    static int occ_next = 0;
    int occ = 0;
    for (int i = 0; i < 4; ++i) if (occ_lds[i] == lds) occ = occ_val[i];
    if (!occ) {
        int o = 0;
        hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&o, (const void*)kfn, NW * 64, lds);
        if (e != hipSuccess) return e;
        occ = o < 1 ? 1 : o;
        occ_val[occ_next] = occ;
        occ_lds[occ_next] = lds;
        occ_next = (occ_next + 1) & 3;
    }
    int64_t cap = (int64_t)occ * conv_num_cus() / (int64_t)grid.x;
    if (cap < 1) cap = 1;
    // a small call does not fill the chip with batches of G images: take fewer images per batch (the LDS
    // layout allows any count up to G), so that more workgroups share the work and each has a shorter chain
    ConvParams q = p;
    const int64_t slots = cap * (WP ? NW : 1);                       // batches in flight when every slot is used
    if ((q.B + q.G - 1) / q.G < slots) {
        const int64_t g = (q.B + slots - 1) / slots;
        q.G = (int)(g < 1 ? 1 : g < q.G ? g : q.G);
    }
    const int64_t n_batch = (q.B + q.G - 1) / q.G;
    const int64_t items = WP ? (n_batch + NW - 1) / NW : n_batch;     // batches a workgroup takes per round
    const int64_t rounds = (items + cap - 1) / cap;
    grid.y = (unsigned)((items + rounds - 1) / rounds);
    kfn<<<grid, dim3(NW * 64), lds, s>>>(q);
    return hipGetLastError();
}

// Pixel tiles per wave iteration of the shared-batch kernels: 4 when a layer has 4 channel tiles (each
// weight fragment read from LDS then serves 4 MFMAs), else 2.
constexpr int conv_pt(int NT) { return NT == 4 ? 4 : 2; }

// Tuned shared-batch variants: (element, NT, KS, RD, staging mode, PF).  KS > 0 keeps the weights in
// registers and unrolls that many MFMA steps; KS = 0 reads them from LDS for any number of steps.
// Last entry: 1 = residual join and fused pooling compiled in.
#define ACCERL_TUNED_I8(X)                                                                                   \
    X(EL_I8, 2, 4, 16, CM_U8T, 8, 0) X(EL_I8, 1, 4, 16, CM_U8T, 8, 0) X(EL_I8, 4, 0, 16, CM_FLAT, 8, 0)     \
    X(EL_I8, 4, 0, 16, CM_FLAT, 10, 0) X(EL_I8, 2, 4, 16, CM_FLAT, 8, 0) X(EL_I8, 1, 2, 16, CM_FLAT, 8, 0)  \
    X(EL_I8, 1, 1, 8, CM_FLAT, 8, 0) X(EL_I8, 1, 1, 4, CM_U8T, 8, 1) X(EL_I8, 1, 1, 8, CM_U8T, 8, 1)        \
    X(EL_I8, 1, 1, 8, CM_U8T, 4, 1) X(EL_I8, 1, 2, 8, CM_ROWSV, 8, 1) X(EL_I8, 1, 2, 8, CM_ROWSV, 4, 1)     \
    X(EL_I8, 1, 2, 16, CM_ROWSV, 8, 1) X(EL_I8, 1, 2, 16, CM_ROWSV, 4, 1) X(EL_I8, 1, 2, 16, CM_ROWSV, 2, 1) \
    X(EL_I8, 1, 3, 16, CM_ROWSV, 8, 1) X(EL_I8, 1, 3, 16, CM_ROWSV, 4, 1)
#define ACCERL_TUNED_BF16(X)                                                                                 \
    X(EL_BF16, 2, 8, 16, CM_U8T, 8, 0) X(EL_BF16, 1, 2, 8, CM_U8T, 8, 1) X(EL_BF16, 1, 5, 16, CM_ROWSV, 16, 1) \
    X(EL_BF16, 2, 5, 16, CM_ROWSV, 16, 1) X(EL_BF16, 2, 9, 16, CM_ROWSV, 16, 1) X(EL_BF16, 2, 9, 16, CM_ROWSV, 8, 1) \
    X(EL_BF16, 4, 0, 16, CM_FLAT, 8, 0)

// Wave-private variants (8 wavefronts, weights in LDS, contiguous staging): (element, NT, RD, PF, PT)
constexpr int CONV_WP_WAVES = 8;
constexpr int CONV_WP_PF = 14;
#define ACCERL_WP_I8(X) X(EL_I8, 4, 16, CONV_WP_PF, 3) X(EL_I8, 4, 16, CONV_WP_PF, 4)

// everything else: weights in LDS, chunk reads at 16- or 4-byte alignment, 16 staging units per lane
template <int EL, int NT>
hipError_t conv_go_generic(const ConvParams& p, int rd, dim3 grid, size_t lds, hipStream_t s) {
    const bool a16 = rd == 16;
    constexpr int PT = conv_pt(NT);
    switch (p.mode) {
        case CM_FLAT: return a16 ? conv_go<EL, NT, 0, 16, CM_FLAT, 16, PT, 4, false, true>(p, grid, lds, s) : conv_go<EL, NT, 0, 4, CM_FLAT, 16, PT, 4, false, true>(p, grid, lds, s);
        case CM_ROWS: return a16 ? conv_go<EL, NT, 0, 16, CM_ROWS, 16, PT, 4, false, true>(p, grid, lds, s) : conv_go<EL, NT, 0, 4, CM_ROWS, 16, PT, 4, false, true>(p, grid, lds, s);
        case CM_ROWSV: return a16 ? conv_go<EL, NT, 0, 16, CM_ROWSV, 16, PT, 4, false, true>(p, grid, lds, s) : conv_go<EL, NT, 0, 4, CM_ROWSV, 16, PT, 4, false, true>(p, grid, lds, s);
        case CM_U8T: return a16 ? conv_go<EL, NT, 0, 16, CM_U8T, 16, PT, 4, false, true>(p, grid, lds, s) : conv_go<EL, NT, 0, 4, CM_U8T, 16, PT, 4, false, true>(p, grid, lds, s);
        default: return hipErrorInvalidValue;
    }
}

// one translation unit per family keeps the build parallel
hipError_t conv_launch_tuned_i8(const ConvParams& p, int NT, int KS, int RD, int pf, dim3 grid, size_t lds, hipStream_t s);
hipError_t conv_launch_tuned_bf16(const ConvParams& p, int NT, int KS, int RD, int pf, dim3 grid, size_t lds, hipStream_t s);
hipError_t conv_launch_wp_i8(const ConvParams& p, int NT, int RD, int PT, dim3 grid, size_t lds, hipStream_t s);
hipError_t conv_launch_gen_i8(const ConvParams& p, int NT, int RD, dim3 grid, size_t lds, hipStream_t s);
hipError_t conv_launch_gen_bf16(const ConvParams& p, int NT, int RD, dim3 grid, size_t lds, hipStream_t s);

}  // namespace accerl
