// One residual block of the IMPALA-style student (ReLU - conv3x3 - ReLU - conv3x3 + skip, all int8, padding 1,
// the same number of channels in and out) in one kernel: the first convolution's output never leaves LDS.
// Layer by layer a block moves its stream five times through memory (conv A reads x and writes t, conv B reads t
// and x and writes x'); fused it moves it three times, and two launches become one.
//
// A workgroup (four wavefronts) takes G images at a time, G chosen so that the images' pixels fill a whole number
// of 16-column MFMA tiles per wavefront (42x42x8: one image, 21x21x16: two, 11x11x16: seven).  Per batch:
//   stage    max(x, 0) of the G images into LDS tiles with a one-pixel border of zeros (the bytes were requested
//            from memory while the batch before was multiplied);
//   conv A   columns = output pixels numbered across the G images, rows = channels (8-channel layers pack two
//            horizontally adjacent pixels into the 16 rows, as the layer-by-layer kernel does: same weight
//            fragments, same chunk order), weights in registers; requantized with the fused ReLU into a second
//            set of bordered tiles;
//   conv B   from those tiles; the epilogue reads the block's input once more (from cache) for the skip
//            connection and writes the block's output.
// Fragments, bias, multipliers and every arithmetic step are those of conv_kernel.h, so the results are
// bit-identical to the layer-by-layer path (which the debug taps still run).  Residual-block definition: network
// table of the paper's Atari experiments extended by the benchmark's IMPALA configuration.
#include <stdlib.h>

#include "conv_kernel.h"

namespace accerl {

namespace {
struct ResParams {
    const int8_t* x;         // [B, H, H, C] block input (also the skip connection)
    int8_t* out;             // [B, H, H, C]
    const v4i* wA; const int* biasA; const float* multA;
    const v4i* wB; const int* biasB; const float* multB;
    float r;                 // scale of x over scale of the output
    int64_t B;
};

constexpr int RB_THREADS = 256;
constexpr int RB_PF = 4;     // 16-byte staging units per lane

template <int C, int H>
struct RbShape {
    static constexpr int P = 16 / C;                     // output pixels per MFMA column (2 for 8 channels)
    static constexpr int WP = H / P;                     // columns per image row
    static constexpr int NPX = H * WP;                   // columns = 16-byte units per image
    static constexpr int IMG = H * H * C;                // bytes per image
    static constexpr int UPR = H * C / 16;               // 16-byte units per image row
    static constexpr int PITCH = ((H + 2) * C + 15) / 16 * 16;
    static constexpr int TILE = (H + 2) * PITCH;
    static constexpr int G = (H == 42) ? 1 : (H == 21) ? 2 : 7;
    static constexpr int COLS = G * NPX;
    static constexpr int TILES = (COLS + 15) / 16;
    static constexpr int RUN = (3 + P - 1) * C;          // bytes of one kernel row of a column
    static constexpr int CPR = (RUN + 15) / 16;          // 16-byte chunks per kernel row
    static constexpr int KS = (3 * CPR + 3) / 4;         // MFMA steps
    static constexpr int LDS = 2 * G * TILE + TILES * 16 * 4 + 64;
    static_assert(H % P == 0 && IMG == NPX * 16 && (H * C) % 16 == 0 && COLS <= RB_PF * RB_THREADS, "shape");
};

// P23: conv A's accumulators stay below 2^23 (its requantization then takes the form of requant_relu4_p23)
template <int C, int H, bool P23>
__global__ __launch_bounds__(RB_THREADS, 2) void resblock_kernel(const ResParams p) {
    typedef RbShape<C, H> S;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    char* tileX = smem;                                  // G bordered tiles of max(x, 0)
    char* tileM = smem + S::G * S::TILE;                 // G bordered tiles of conv A's output
    int* tab = (int*)(smem + 2 * S::G * S::TILE);        // column -> offset of its window in a tile set
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 15, g = lane >> 4;

    // weights, chunk offsets and epilogue constants of both convolutions (channels 4g .. 4g+3 of the lane's pixel)
    v4i wA[S::KS], wB[S::KS];
    int koff[S::KS];
#pragma unroll
    for (int st = 0; st < S::KS; ++st) {
        const int q = 4 * st + g, ky = q / S::CPR, cx = q - ky * S::CPR;
        koff[st] = (ky < 3) ? ky * S::PITCH + cx * 16 : 0;
        wA[st] = p.wA[st * 64 + lane];
        wB[st] = p.wB[st * 64 + lane];
    }
    const v4i biA = *(const v4i*)(p.biasA + 4 * g) + (P23 ? P23_MAGIC : 0), biB = *(const v4i*)(p.biasB + 4 * g);
    const v4f mlA = *(const v4f*)(p.multA + 4 * g), mlB = *(const v4f*)(p.multB + 4 * g);
    const v4f cA = mlA * -8388608.0f;

    // staging: unit u of a batch = 16 bytes of image u / NPX, row (u % NPX) / UPR; where it lands in the tiles
    v4i pre[RB_PF];
    int doff[RB_PF];
#pragma unroll
    for (int i = 0; i < RB_PF; ++i) {
        const int u = min(tid + i * RB_THREADS, S::COLS - 1);
        const int img = u / S::NPX, w = u - img * S::NPX, y = w / S::UPR, xu = w - y * S::UPR;
        doff[i] = img * S::TILE + (y + 1) * S::PITCH + C + xu * 16;
    }
    const int64_t n_batch = (p.B + S::G - 1) / S::G;
    auto prefetch = [&](int64_t batch) {
        const int64_t b0 = batch * S::G;
        const int gc = (int)((p.B - b0 < S::G) ? (p.B - b0) : S::G);
        const char* src = (const char*)p.x + b0 * (int64_t)S::IMG;
#pragma unroll
        for (int i = 0; i < RB_PF; ++i) pre[i] = *(const v4i*)(src + (uint32_t)min(tid + i * RB_THREADS, gc * S::NPX - 1) * 16u);
    };
    auto commit = [&](int64_t batch) {
        const int64_t b0 = batch * S::G;
        const int total = (int)((p.B - b0 < S::G) ? (p.B - b0) : S::G) * S::NPX;
#pragma unroll
        for (int i = 0; i < RB_PF; ++i) {
            if (tid + i * RB_THREADS >= total) break;
            v4i v = pre[i];
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = (int)relu_i8x4((uint32_t)v[e]);
            if constexpr ((C & 15) == 0) {
                *(v4i*)(tileX + doff[i]) = v;
            } else {
                typedef int v2i __attribute__((ext_vector_type(2)));
                *(v2i*)(tileX + doff[i]) = (v2i){v[0], v[1]};
                *(v2i*)(tileX + doff[i] + 8) = (v2i){v[2], v[3]};
            }
        }
    };

    int64_t batch = blockIdx.x;
    if (batch < n_batch) prefetch(batch);
    // once: borders (and everything else) zero, the column table
    for (int i = tid; i < 2 * S::G * S::TILE / 4; i += RB_THREADS) ((int*)smem)[i] = 0;
    for (int c = tid; c < S::TILES * 16; c += RB_THREADS) {
        const int cc = min(c, S::COLS - 1);              // columns past the end repeat the last one (never stored)
        const int img = cc / S::NPX, w = cc - img * S::NPX, y = w / S::WP, xp = w - y * S::WP;
        tab[c] = img * S::TILE + y * S::PITCH + xp * 16;
    }
    __syncthreads();

    for (; batch < n_batch; batch += gridDim.x) {
        commit(batch);
        __syncthreads();
        if (batch + gridDim.x < n_batch) prefetch(batch + gridDim.x);
        const int64_t b0 = batch * S::G;
        const int total = (int)((p.B - b0 < S::G) ? (p.B - b0) : S::G) * S::NPX;
        const int n_tiles = (total + 15) >> 4;

        // ---- conv A: max(x, 0) -> t, requantized with the fused ReLU into the second tile set
        for (int t = wave; t < n_tiles; t += 4) {
            const int col = t * 16 + j;
            const int base = tab[col];
            v4i acc = biA;
#pragma unroll
            for (int st = 0; st < S::KS; ++st)
                acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(wA[st], *(const v4i*)(tileX + base + koff[st]), acc, 0, 0, 0);
            const uint32_t w = requant_relu4_p23<P23>(acc, mlA, cA);
            // the column's own pixel(s) sit one row and one pixel inside its window
            if (col < total) *(uint32_t*)(tileM + base + S::PITCH + C + 4 * g) = w;
        }
        __syncthreads();

        // ---- conv B: t -> accumulator, joined with the block's input, written out
        const int8_t* xres = p.x + b0 * (int64_t)S::IMG;
        int8_t* outp = p.out + b0 * (int64_t)S::IMG;
        for (int t = wave; t < n_tiles; t += 4) {
            const int col = t * 16 + j;
            const int base = tab[col];
            const uint32_t xr = *(const uint32_t*)(xres + (uint32_t)min(col, total - 1) * 16u + 4 * g);
            v4i acc = biB;
#pragma unroll
            for (int st = 0; st < S::KS; ++st)
                acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(wB[st], *(const v4i*)(tileM + base + koff[st]), acc, 0, 0, 0);
            int q[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float tr = (float)(int)(int8_t)(xr >> (8 * r)) * p.r;
                q[r] = rne_clamp127(fmaf((float)acc[r], mlB[r], tr));
            }
            if (col < total) *(uint32_t*)(outp + (uint32_t)col * 16u + 4 * g) = pack_low_bytes(q);
        }
        __syncthreads();     // every wavefront is done with both tile sets before the next batch is staged
    }
}

template <int C, int H>
bool rb_shape_ok(const ConvParams& a, const ConvParams& b) {
    typedef RbShape<C, H> S;
    for (const ConvParams* c : {&a, &b}) {
        if (c->H != H || c->W != H || c->Cin_real != C || c->Cs_in != C || c->Ho != H || c->Wo != S::WP || c->Cs_out != 16) return false;
        if (c->k != 3 || c->s != 1 || c->pad != 1 || c->sx != S::P || c->cpr != S::CPR || c->k_steps != S::KS) return false;
        if (c->src_u8 || c->pool || c->out_frag) return false;
    }
    return true;
}

template <int C, int H, bool P23>
hipError_t rb_go(const ResParams& p, hipStream_t s) {
    typedef RbShape<C, H> S;
    static int occ = 0;
    if (!occ) {
        hipError_t e = hipFuncSetAttribute((const void*)resblock_kernel<C, H, P23>, hipFuncAttributeMaxDynamicSharedMemorySize, S::LDS);
        if (e != hipSuccess) return e;
        int o = 0;
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&o, (const void*)resblock_kernel<C, H, P23>, RB_THREADS, S::LDS);
        if (e != hipSuccess) return e;
        occ = o < 1 ? 1 : o;
    }
    // resident workgroups striding over the batches, in even rounds
    const int64_t batches = (p.B + S::G - 1) / S::G;
    const int64_t cap = (int64_t)occ * conv_num_cus();
    const int64_t rounds = (batches + cap - 1) / cap;
    dim3 grid((unsigned)((batches + rounds - 1) / rounds));
    resblock_kernel<C, H, P23><<<grid, dim3(RB_THREADS), S::LDS, s>>>(p);
    return hipGetLastError();
}
}  // namespace

// a = first convolution of the block (ReLU on its input, fused ReLU on its output, no skip), b = second
// (skip connection from a's input)
bool resblock_supported(const ConvParams& a, int NTA, const ConvParams& b, int NTB) {
    if (NTA != 1 || NTB != 1 || !a.relu_in || !a.relu || b.relu_in) return false;
    return rb_shape_ok<8, 42>(a, b) || rb_shape_ok<16, 21>(a, b) || rb_shape_ok<16, 11>(a, b);
}

hipError_t launch_resblock(const ConvParams& a, const ConvParams& b, hipStream_t s) {
    if (a.B <= 0) return hipSuccess;
    ResParams p;
    p.x = (const int8_t*)a.in; p.out = (int8_t*)b.out;
    p.wA = (const v4i*)a.wfrag; p.biasA = (const int*)a.bias; p.multA = a.mult;
    p.wB = (const v4i*)b.wfrag; p.biasB = (const int*)b.bias; p.multB = b.mult;
    p.r = b.r; p.B = a.B;
    static const bool no_p23 = getenv("ACCERL_NO_P23") != nullptr;
    const bool p23 = a.pos23 && !no_p23;
    if (rb_shape_ok<8, 42>(a, b)) return p23 ? rb_go<8, 42, true>(p, s) : rb_go<8, 42, false>(p, s);
    if (rb_shape_ok<16, 21>(a, b)) return p23 ? rb_go<16, 21, true>(p, s) : rb_go<16, 21, false>(p, s);
    if (rb_shape_ok<16, 11>(a, b)) return p23 ? rb_go<16, 11, true>(p, s) : rb_go<16, 11, false>(p, s);
    return hipErrorInvalidValue;
}

}  // namespace accerl
