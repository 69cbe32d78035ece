// The first two convolutions of the paper's original network (network table: 32 filters of 8x8 and 64
// of 4x4 on a 4x84x84 uint8 observation; strides 4 and 2, no padding) as one pipelined kernel with every
// size known at compile time.
//
// A workgroup of twelve wavefronts (one per compute unit, three per SIMD) walks over pairs of
// observations.  In one tick
//   wavefronts 4..7 and 8..11  compute the first convolution of the two observations of pair n+1 from the
//                    LDS copies of their bytes and write the requantized 20x20x32 images to LDS tiles,
//   wavefronts 0..3  compute the second convolution of the two observations of pair n from the tiles written
//                    in the tick before and store the requantized 9x9x64 images,
//   the first-layer wavefronts have the bytes of pair n+2 in flight from memory,
// then the workgroup meets, the bytes of pair n+2 go to LDS and the workgroup meets again.  Inside a
// wavefront the code is a software pipeline in straight-line form: the MFMAs of one pixel tile are
// interleaved with the requantization arithmetic of the tile before, so that matrix core and vector ALU
// work at the same time.
//
// Weights live in registers: a first-layer wavefront holds all 32 filters (32 VGPRs); a second-layer
// wavefront holds one half of the 64 filters (64 VGPRs) and computes three 16-pixel tiles with it.  The
// 81 output pixels are covered by the tiles 0..47 and 33..80: the overlap is computed twice and stored
// twice with identical bytes, which keeps the code free of per-pixel predicates.
//
// Observation tile.  Chunk u (16 bytes) of the LDS copy is dword u of each of the four channel planes,
// side by side: dword u of a plane holds 4 horizontally adjacent pixels and 84 = 21 dwords, so chunk u is
// row u / 21, pixels 4 * (u % 21) .. + 3 -- staging needs no index arithmetic and no byte shuffles, only the
// sign flip (obs - 128).  The weight fragments arrive ordered (kx, c) inside a chunk; they are
// transposed to (c, kx) once per wavefront to match.
//
// First-layer output tile.  Pixels of even and odd columns are kept in two planes, [x & 1][y][x >> 1][32
// channels]: the stride-2 second layer then reads 16 consecutive output pixels as consecutive 32-byte
// pixels (measured: 1.4 times the LDS read rate of the plain channels-last image), and the plane offset
// is an odd multiple of 16 bytes, which makes the 8-byte epilogue stores of neighbouring pixels fall into
// disjoint banks (twice the store rate).
//
// Arithmetic, fragment layouts, bias (with the zero-point correction) and multipliers are those of
// conv_kernel.h: accumulators and activations are bit-identical to the layer-by-layer path.
#include <stdlib.h>

#include "conv_kernel.h"

namespace accerl {

namespace {
constexpr int FR_THREADS = 768;
constexpr int FR_PLANE = 84 * 84;                 // bytes per channel plane
constexpr int FR_UNITS = FR_PLANE / 4;            // 16-byte chunks of the observation tile (1764)
constexpr int FR_TILE_A = FR_UNITS * 16;          // 28224
constexpr int FR_ROW_A = 21 * 16;                 // LDS bytes per observation row
constexpr int FR_ROW_B = 10 * 32;                 // one row of one column-parity plane: 10 pixels of 32 channels
constexpr int FR_PLANE_B = 20 * FR_ROW_B + 16;    // 6416: odd multiple of 16 (see above)
constexpr int FR_TILE_B = 2 * FR_PLANE_B;         // 12832
constexpr int FR_NPIX2 = 81, FR_PIX2_BYTES = 64;
constexpr int FR_LDS = 2 * FR_TILE_A + 4 * FR_TILE_B;   // two observations; per observation two output tiles
constexpr int FR_STAGERS = 256;                   // lanes that stage one observation (its four first-layer wavefronts)
constexpr int FR_PF = (FR_UNITS + FR_STAGERS - 1) / FR_STAGERS;   // staging chunks per lane (7)

struct FrontParams {
    const uint8_t* obs;      // [B, 4, 84, 84]
    int8_t* out;             // [B, 9, 9, 64]
    const v4i* wA; const int* biasA; const float* multA;
    const v4i* wB; const int* biasB; const float* multB;
    int64_t B;
};

// 4x4 byte transpose of a 16-byte chunk
__device__ __forceinline__ v4i transpose4x4(v4i v) {
    const uint32_t P0 = (uint32_t)v[0], P1 = (uint32_t)v[1], P2 = (uint32_t)v[2], P3 = (uint32_t)v[3];
    const uint32_t lo01 = __builtin_amdgcn_perm(P1, P0, 0x05010400u), hi01 = __builtin_amdgcn_perm(P1, P0, 0x07030602u);
    const uint32_t lo23 = __builtin_amdgcn_perm(P3, P2, 0x05010400u), hi23 = __builtin_amdgcn_perm(P3, P2, 0x07030602u);
    return (v4i){(int)__builtin_amdgcn_perm(lo23, lo01, 0x05040100u), (int)__builtin_amdgcn_perm(lo23, lo01, 0x07060302u),
                 (int)__builtin_amdgcn_perm(hi23, hi01, 0x05040100u), (int)__builtin_amdgcn_perm(hi23, hi01, 0x07060302u)};
}

// P23: both layers' accumulators stay below 2^23, so requantization takes the three-instruction form of requant_relu4_p23
template <bool P23>
__global__ __launch_bounds__(FR_THREADS, 3) void conv_front_kernel(const FrontParams p) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    typedef int v2i __attribute__((ext_vector_type(2)));
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 15, g = lane >> 4;
    // LDS: observation tile of slot 0, of slot 1, then the output tiles [slot][buffer]
    char* tilesB = smem + 2 * FR_TILE_A;

    // pair n of this workgroup: observations 2 * (blockIdx.x + n * gridDim.x) + {0, 1}
    const int64_t stride = 2 * (int64_t)gridDim.x;
    int64_t img = 2 * (int64_t)blockIdx.x;              // first observation of the pair whose second convolution runs this tick
    if (img >= p.B) return;

    if (wave >= 4) {
        // ================= first-layer wavefronts of slot `slot` (they also stage its observations)
        const int slot = (wave - 4) >> 2, aw = (wave - 4) & 3, stid = (tid - 256) & 255;
        char* tileA = smem + slot * FR_TILE_A;
        char* tileB = tilesB + slot * (2 * FR_TILE_B);
        img += slot;                                    // this group's observation of the current pair
        // staging: chunk u = dword u of the four planes
        uint32_t pre[FR_PF][4];
        auto stage_load_part = [&](const uint8_t* src, int k) {
            const int u = min(stid + k * FR_STAGERS, FR_UNITS - 1);
#pragma unroll
            for (int c = 0; c < 4; ++c) pre[k][c] = *(const uint32_t*)(src + c * FR_PLANE + 4 * u);
        };
        auto obs_of = [&](int64_t im) { return p.obs + min(im, p.B - 1) * (int64_t)(4 * FR_PLANE); };   // past the batch: the last observation, never used
        auto stage_load = [&](int64_t im) {
            const uint8_t* src = obs_of(im);
#pragma unroll
            for (int k = 0; k < FR_PF; ++k) stage_load_part(src, k);
        };
        auto stage_commit = [&]() {
#pragma unroll
            for (int k = 0; k < FR_PF; ++k) {
                const int u = stid + k * FR_STAGERS;
                if (u < FR_UNITS)
                    *(v4i*)(tileA + 16 * u) = (v4i){(int)(pre[k][0] ^ 0x80808080u), (int)(pre[k][1] ^ 0x80808080u),
                                                    (int)(pre[k][2] ^ 0x80808080u), (int)(pre[k][3] ^ 0x80808080u)};
            }
        };
        const bool have0 = img < p.B;
        if (have0) stage_load(img);
        v4i wA[4][2];
#pragma unroll
        for (int st = 0; st < 4; ++st)
#pragma unroll
            for (int t = 0; t < 2; ++t) wA[st][t] = transpose4x4(p.wA[(st * 2 + t) * 64 + lane]);
        v4i biA[2];
        v4f mlA[2], cA[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            biA[t] = *(const v4i*)(p.biasA + 8 * g + 4 * t);
            mlA[t] = *(const v4f*)(p.multA + 8 * g + 4 * t);
            cA[t] = mlA[t] * -8388608.0f;
            if (P23) biA[t] += P23_MAGIC;
        }
        // The 20 x 20 output pixels of the first layer are split into a block of 16 columns, whose tiles are the
        // output rows (16 pixels in a row: wavefront aw owns the five rows 5aw .. 5aw+4, a chain), and the
        // remaining 4 columns, whose five tiles are 4 x 4 pixels (wavefront aw owns tile aw, wavefront 0 also the
        // fifth).  Along a chain the windows of two vertically adjacent pixels share their lower and upper
        // halves: K steps 2 and 3 of a row (observation rows 4oy+4 .. 4oy+7) are K steps 0 and 1 of the row
        // below, so a chain tile re-reads only two of its four fragments from LDS (68 instead of 100
        // fragment reads per observation).
        // chain: window of the lane's pixel (row 5aw, column j), K step st adds two observation rows, the next
        // chain tile four; output address of that pixel, the next chain tile adds one output row
        const int rb_chain = (5 * aw) * (4 * FR_ROW_A) + j * 16 + (g >> 1) * FR_ROW_A + (g & 1) * 16;
        const int wb_chain = (j & 1) * FR_PLANE_B + (5 * aw) * FR_ROW_B + (j >> 1) * 32 + 8 * g;
        // 4 x 4 tiles: pixel (4b + j / 4, 16 + j % 4) of tile b = aw, and of tile 4 for the first wavefront
        int rb_blk[2], wb_blk[2];
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const int b = k == 0 ? aw : 4, oy = 4 * b + (j >> 2), ox = 16 + (j & 3);
            rb_blk[k] = oy * (4 * FR_ROW_A) + ox * 16 + (g >> 1) * FR_ROW_A + (g & 1) * 16;
            wb_blk[k] = (ox & 1) * FR_PLANE_B + oy * FR_ROW_B + (ox >> 1) * 32 + 8 * g;
        }

        // One tile = 8 MFMAs (4 K steps x 2 channel tiles) + 32 requantization operations.  While the matrix
        // core works on tile r, the vector ALU requantizes tile r-1 and the fragments of tile r+1 are read.
        // The group barriers pin that interleaving.  Tiles 0..4 are the chain, 5 and 6 the 4 x 4 tiles.
        auto frag_a = [&](int r, int st) {
            const int base = r < 5 ? rb_chain + r * (4 * FR_ROW_A) : rb_blk[r - 5];
            return *(const v4i*)(tileA + base + st * (2 * FR_ROW_A));
        };
        auto store_a = [&](char* dstB, int r, const v4i (&acc)[2]) {
            const uint32_t w0 = requant_relu4_p23<P23>(acc[0], mlA[0], cA[0]), w1 = requant_relu4_p23<P23>(acc[1], mlA[1], cA[1]);
            *(v2i*)(dstB + (r < 5 ? wb_chain + r * FR_ROW_B : wb_blk[r - 5])) = (v2i){(int)w0, (int)w1};
        };
        auto mfma_a = [&](const v4i (&f)[4], v4i (&acc)[2]) {
#pragma unroll
            for (int st = 0; st < 4; ++st)
#pragma unroll
                for (int t = 0; t < 2; ++t) acc[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wA[st][t], f[st], st == 0 ? biA[t] : acc[t], 0, 0, 0);
        };
        // conv_a also requests the observation `next` (the one staged after this tick), four loads per tile:
        // in one burst at the top of the tick the 28 loads cost a wavefront 14 % of the tick in issue time
        auto conv_a = [&](char* dstB, const uint8_t* next) {
            v4i f[4];
#pragma unroll
            for (int st = 0; st < 4; ++st) f[st] = frag_a(0, st);
            v4i accO[2] = {biA[0], biA[1]};
#pragma unroll
            for (int r = 0; r < 6; ++r) {
                v4i accN[2], fn[4];
                mfma_a(f, accN);
                stage_load_part(next, r);
                // fragments of tile r+1: a chain tile inherits steps 0 and 1 from steps 2 and 3 of the tile above
                if (r + 1 < 5) {
                    fn[0] = f[2]; fn[1] = f[3];
                    fn[2] = frag_a(r + 1, 2); fn[3] = frag_a(r + 1, 3);
                } else if (r + 1 == 5 || aw == 0) {     // tile 6 belongs to the first wavefront only
#pragma unroll
                    for (int st = 0; st < 4; ++st) fn[st] = frag_a(r + 1, st);
                } else {
#pragma unroll
                    for (int st = 0; st < 4; ++st) fn[st] = f[st];
                }
                if (r > 0) store_a(dstB, r - 1, accO);
                accO[0] = accN[0]; accO[1] = accN[1];
#pragma unroll
                for (int st = 0; st < 4; ++st) f[st] = fn[st];
                if (r > 0) {
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
                        if (r + 1 >= 5 || k < 2) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                        __builtin_amdgcn_sched_group_barrier(0x002, P23 ? 6 : 8, 0);
                    }
                    __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x020, 4, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            static_assert(FR_PF == 7, "six tiles carry one staging part each, the seventh follows");
            stage_load_part(next, 6);
            if (aw == 0) {                              // the fifth 4 x 4 tile
                v4i accN[2];
                mfma_a(f, accN);
                store_a(dstB, 5, accO);
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, P23 ? 6 : 8, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
                store_a(dstB, 6, accN);
            } else {
                store_a(dstB, 5, accO);
            }
        };

        if (have0) stage_commit();
        __syncthreads();                                 // observation tiles complete
        const bool more = img + stride < p.B;
        if (have0) conv_a(tileB, obs_of(img + stride));  // the second pair's observation is in flight meanwhile
        __syncthreads();                                 // first output tiles complete, observation tiles free
        if (more) stage_commit();
        __syncthreads();
        const int64_t img0 = img - slot;
        for (int n = 0;; ++n, img += stride) {
            const bool has_next = img + stride < p.B, has_next2 = img + 2 * stride < p.B;
            if (has_next) conv_a(tileB + ((n + 1) & 1) * FR_TILE_B, obs_of(img + 2 * stride));
            if (!(img0 + (n + 1) * stride < p.B)) break;          // the workgroup's pairs are done (same test in every wavefront)
            __syncthreads();
            if (has_next2) stage_commit();
            __syncthreads();
        }
    } else {
        // ================= second-layer wavefronts: both observations of the pair, one after the other
        const int h = wave & 1, p0 = (wave >> 1) ? FR_NPIX2 - 48 : 0;
        v4i wB[8][2];
#pragma unroll
        for (int st = 0; st < 8; ++st)
#pragma unroll
            for (int t = 0; t < 2; ++t) wB[st][t] = p.wB[(st * 4 + 2 * h + t) * 64 + lane];
        const v4i* biasB = (const v4i*)(p.biasB + 16 * g + 8 * h);
        const v4f* multB = (const v4f*)(p.multB + 16 * g + 8 * h);
        // window of the lane's pixel of each tile: K step st = kernel row st >> 1, column pair st & 1; the lane's
        // chunk is column parity g >> 1, channel half g & 1
        int rb[3];
#pragma unroll
        for (int u = 0; u < 3; ++u) {
            const int px = p0 + 16 * u + j;
            const int oy = (px * 7282) >> 16, ox = px - oy * 9;       // px / 9 for px < 81
            rb[u] = oy * (2 * FR_ROW_B) + ox * 32 + (g >> 1) * FR_PLANE_B + (g & 1) * 16;
        }
        const int oofs = (p0 + j) * FR_PIX2_BYTES + 16 * g + 8 * h;   // tile u adds 16 pixels

        // Three pixel tiles, one after the other: 16 MFMAs (8 K steps x 2 channel tiles) each, with the
        // requantization of the tile before interleaved.  Pixel fragments rotate through eight slots: the
        // fragment of step q + 8 is requested as soon as step q has consumed its slot.
        const v4i bi0 = biasB[0] + (P23 ? P23_MAGIC : 0), bi1 = biasB[1] + (P23 ? P23_MAGIC : 0);
        const v4f m0 = multB[0], m1 = multB[1];
        const v4f c0 = m0 * -8388608.0f, c1 = m1 * -8388608.0f;
        auto frag_b = [&](const char* srcB, int q) {
            const int u = q >> 3, st = q & 7;
            return *(const v4i*)(srcB + rb[u] + (st >> 1) * FR_ROW_B + (st & 1) * 32);
        };
        auto store_b = [&](int8_t* outp, int u, const v4i (&acc)[2]) {
            const uint32_t w0 = requant_relu4_p23<P23>(acc[0], m0, c0), w1 = requant_relu4_p23<P23>(acc[1], m1, c1);
            *(v2i*)(outp + oofs + u * (16 * FR_PIX2_BYTES)) = (v2i){(int)w0, (int)w1};
        };
        auto conv_b = [&](const char* srcB, int8_t* outp) {
            v4i gq[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) gq[q] = frag_b(srcB, q);
            v4i accO[2] = {bi0, bi1};
#pragma unroll
            for (int u = 0; u < 3; ++u) {
                v4i accN[2];
#pragma unroll
                for (int st = 0; st < 8; ++st) {
                    const int q = u * 8 + st;
                    accN[0] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wB[st][0], gq[q & 7], st == 0 ? bi0 : accN[0], 0, 0, 0);
                    accN[1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wB[st][1], gq[q & 7], st == 0 ? bi1 : accN[1], 0, 0, 0);
                    if (q + 8 < 24) gq[q & 7] = frag_b(srcB, q + 8);
                }
                if (u > 0) store_b(outp, u - 1, accO);
                accO[0] = accN[0]; accO[1] = accN[1];
                if (u > 0) {
#pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
                        if (u * 8 + k + 8 < 24) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                        __builtin_amdgcn_sched_group_barrier(0x002, P23 ? 3 : 4, 0);
                    }
                    __builtin_amdgcn_sched_group_barrier(0x040, 1, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            store_b(outp, 2, accO);
        };
        __syncthreads();
        __syncthreads();
        __syncthreads();
        for (int n = 0;; ++n, img += stride) {
            conv_b(tilesB + (n & 1) * FR_TILE_B, p.out + img * (int64_t)(FR_NPIX2 * FR_PIX2_BYTES));
            if (img + 1 < p.B)
                conv_b(tilesB + (2 + (n & 1)) * FR_TILE_B, p.out + (img + 1) * (int64_t)(FR_NPIX2 * FR_PIX2_BYTES));
            if (!(img + stride < p.B)) break;
            __syncthreads();
            __syncthreads();
        }
    }
}
}  // namespace

// Exactly the first two layers of the paper's original network as the planner describes them.
bool conv_front_supported(const ConvParams& a, int NTA, const ConvParams& b) {
    if (!a.src_u8 || a.mode != CM_U8T || a.Cin_real != 4 || a.Cs_in != 4 || a.H != 84 || a.W != 84) return false;
    if (a.k != 8 || a.s != 4 || a.sx != 4 || a.pad != 0 || a.Ho != 20 || a.Wo != 20 || a.Cs_out != 32) return false;
    if (NTA != 2 || a.k_steps != 4 || a.cpr != 2 || !a.relu || a.pool || a.res) return false;
    if (b.H != 20 || b.W != 20 || b.Cs_in != 32 || b.k != 4 || b.s != 2 || b.sx != 2 || b.pad != 0) return false;
    if (b.Ho != 9 || b.Wo != 9 || b.Cs_out != 64 || b.k_steps != 8 || b.cpr != 8 || !b.relu || b.relu_in || b.pool || b.res) return false;
    return true;
}

template <bool P23>
static hipError_t front_go(const FrontParams& p, hipStream_t s) {
    static int occ = 0;
    if (!occ) {
        hipError_t e = hipFuncSetAttribute((const void*)conv_front_kernel<P23>, hipFuncAttributeMaxDynamicSharedMemorySize, FR_LDS);
        if (e != hipSuccess) return e;
        int o = 0;
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&o, (const void*)conv_front_kernel<P23>, FR_THREADS, FR_LDS);
        if (e != hipSuccess) return e;
        occ = o < 1 ? 1 : o;
    }
    // resident workgroups striding over the pairs of observations, in even rounds
    const int64_t pairs = (p.B + 1) / 2;
    const int64_t cap = (int64_t)occ * conv_num_cus();
    const int64_t rounds = (pairs + cap - 1) / cap;
    dim3 grid((unsigned)((pairs + rounds - 1) / rounds));
    conv_front_kernel<P23><<<grid, dim3(FR_THREADS), FR_LDS, s>>>(p);
    return hipGetLastError();
}

hipError_t launch_conv_front(const ConvParams& a, const ConvParams& b, hipStream_t s) {
    if (a.B <= 0) return hipSuccess;
    FrontParams p;
    p.obs = (const uint8_t*)a.in; p.out = (int8_t*)b.out;
    p.wA = (const v4i*)a.wfrag; p.biasA = (const int*)a.bias; p.multA = a.mult;
    p.wB = (const v4i*)b.wfrag; p.biasB = (const int*)b.bias; p.multB = b.mult;
    p.B = a.B;
    static const bool no_p23 = getenv("ACCERL_NO_P23") != nullptr;
    return (a.pos23 && b.pos23 && !no_p23) ? front_go<true>(p, s) : front_go<false>(p, s);
}

}  // namespace accerl
