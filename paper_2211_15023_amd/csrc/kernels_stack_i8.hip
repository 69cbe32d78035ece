// One whole stack of the IMPALA-style student in one kernel: conv3x3 (pad 1, no ReLU) -> max-pool 3x3 / 2 (pad 1)
// -> two residual blocks (ReLU - conv3x3 - ReLU - conv3x3 + skip), all int8.  Layer by layer (even with the pool and
// each block fused) a stack moves its stream through memory nine times; here the observation (or the stack before)
// is read once and the stack's output written once, and every tensor in between lives in LDS or in registers.
//
// What bounds these layers is not the matrix cores but the vector instructions around them (requantization, pooling,
// addressing): counters of the layer-by-layer kernels show 70-80 % of all issue slots taken by vector instructions.
// The kernel is therefore organised to issue few of them:
//
//  * conv + pool without storing the convolution.  Requantization is monotone per channel, so pooling the int32
//    accumulators first and requantizing the maxima gives the same bytes with a quarter of the requantizations.  A
//    pooled pixel (py, px) needs the conv outputs of rows 2py-1..2py+1 and columns 2px-1..2px+1.  MFMA columns are
//    pooled pixels; per conv row the kernel multiplies the columns x = 2px (E) and x = 2px+1 (O): the vertical maximum
//    over the three rows is an in-lane v_max3, the horizontal one max(E, O, O of the pixel to the left), the last term
//    fetched with one DPP row shift.  Lane 0 of a tile only serves as left neighbour (tiles advance by 15 pixels), and
//    a pooled row starts with a dummy that repeats the first pixel's windows, so that a maximum never picks up a
//    value from outside its window.  Rows and columns outside the image are replaced by their nearest neighbour
//    inside, which is part of the same window, so no -infinity is needed.
//    16-channel layers: columns are "slots", the pooled pixels of the batch in raster order with the dummy in front
//    of every row; one 8-byte table entry per slot gives the window addresses.  E and O are separate MFMAs on the
//    same LDS reads: their windows together are the bordered pixels 2px .. 2px+3, whole aligned 16-byte chunks, which
//    are multiplied with the planner's weight fragments (E) and with the same fragments shifted by one pixel (O).
//    8-channel layers put E and O into the two halves of the 16 MFMA rows (the pixel packing of the layer-by-layer
//    kernel: same weight fragments): E then sits in lanes 0-31 and O in lanes 32-63.  A tile is 15 pixels of one
//    pooled row; two vertically adjacent pooled rows are processed together (they share a conv row: five MFMAs for
//    the two tiles) and one v_permlane32_swap per register brings E and O of the upper row into the lower lanes and
//    of the lower row into the upper lanes.  All addresses of a tile are a per-lane constant plus a wave-uniform row
//    offset.
//  * the pooled stream is written twice into LDS: max(x, 0) into a zero-bordered tile (the first block's conv A reads
//    it) and x itself into a plain image (the skip connection).  The blocks run as in the single-block kernel, from
//    LDS to LDS; the first block's output replaces the plain image in place, the second block's goes to memory.
//  * the next batch's input bytes are requested at the start of the current batch's last phase and land while it runs.
//
// Arithmetic, fragments and constants are those of the layer-by-layer kernels (conv_kernel.h), so results are
// bit-identical; the debug taps still run that path.  Network: the benchmark's IMPALA configuration (three such stacks).
#include <stdlib.h>

#include <type_traits>

#include "conv_kernel.h"

namespace accerl {

namespace {

struct StackParams {
    const void* in;          // uint8 planes [B, 4, HIN, HIN] or int8 [B, HIN, HIN, CI]
    int8_t* out;             // [B, H, H, C]
    const v4i* w[5];         // 0: stack convolution, 1 / 2: first block's conv A / B, 3 / 4: second block's
    const int* bias[5];
    const float* mult[5];
    float r1, r2;            // scale of a block's input over the scale of its output
    int64_t B;
};

constexpr int st_up16(int v) { return (v + 15) / 16 * 16; }

template <bool U8, int CI, int HIN, int C, int G_, int NW_>
struct StShape {
    static constexpr int G = G_;
    static constexpr int NW = NW_;                            // wavefronts per workgroup
    static constexpr int ST_THREADS = NW * 64;
    static constexpr int TU = (NW >= 8 || C == 16) ? 1 : 2;   // block column tiles per wavefront and step (two only where registers allow)
    static constexpr int P = 16 / C;                          // output pixels per MFMA column (2 for 8 channels)
    // input tile: one pixel of border on every side
    static constexpr int PITCH_IN = st_up16((HIN + 2) * CI);
    static constexpr int TILE_IN = (HIN + 2) * PITCH_IN;
    static constexpr int CPR_C = ((3 + P - 1) * CI + 15) / 16;  // 16-byte chunks per kernel row
    static constexpr int KS_C = (3 * CPR_C + 3) / 4;
    static constexpr int UPR_IN = U8 ? HIN / 4 : HIN * CI / 16; // staging units per image row
    static constexpr int UNITS_IN = HIN * UPR_IN;
    static constexpr int IMG_IN = U8 ? 4 * HIN * HIN : HIN * HIN * CI;
    static constexpr int PF = (G * UNITS_IN + ST_THREADS - 1) / ST_THREADS;
    static constexpr int RD_E = ((2 * CI) % 16 == 0) ? 16 : 8;  // alignment of the E windows (byte offset 2 px CI)
    // 16-channel layers: E (x = 2px) and O (x = 2px+1) windows together span the bordered pixels 2px .. 2px+3, which are
    // whole aligned 16-byte chunks; the kernel reads CPRK chunks per kernel row once and multiplies them with two
    // weight sets, the planner's (E) and the same shifted by one pixel (O): no second, misaligned read for O
    static constexpr int CPRK = 4 * CI / 16;                    // chunks per kernel row as read (2 or 4)
    static constexpr int KSK = (3 * CPRK + 3) / 4;              // MFMA steps over those chunks
    // pooled stream
    static constexpr int H = (HIN - 1) / 2 + 1;
    static constexpr int SLOTS = H * (H + 1);                  // per image: a dummy slot in front of every pooled row
    // residual blocks
    static constexpr int WP = H / P;                           // columns per image row
    static constexpr int NPX = H * WP;                         // columns = 16-byte units per image
    static constexpr int IMG = H * H * C;
    static constexpr int PITCH_B = st_up16((H + 2) * C);
    static constexpr int TILE_B = (H + 2) * PITCH_B;
    static constexpr int COLS = G * NPX;
    static constexpr int TILES = (COLS + 15) / 16;
    static constexpr int CPR_B = ((3 + P - 1) * C + 15) / 16;
    static constexpr int KS_B = (3 * CPR_B + 3) / 4;
    // conv + pool work items
    static constexpr int NS = (H + 14) / 15;                   // 8-channel layers: tiles (strips of 15 pixels) per pooled row
    static constexpr int NT1 = (G * SLOTS - 1 + 14) / 15;      // 16-channel layers: slot tiles per full batch
    static constexpr int T1_BYTES = (P == 2) ? NS * 64 * 16 : st_up16(G * SLOTS * 8);
    // LDS layout (bytes); 64 bytes of slack behind the input tiles: the last window of the last row reaches past it
    static constexpr int O_TX = st_up16(G * TILE_IN + 64);
    static constexpr int O_TM = O_TX + G * TILE_B;
    static constexpr int O_RAW = O_TM + G * TILE_B;
    static constexpr int O_T1 = O_RAW + G * IMG;
    static constexpr int O_TABB = O_T1 + T1_BYTES;
    static constexpr int O_CST = O_TABB + st_up16((TILES + 3 * NW * TU) * 16 * 2);   // the block loops read their table two steps ahead
    static constexpr int LDS = O_CST + 5 * 2 * 16 * 4;
    static_assert(H % P == 0 && IMG == NPX * 16 && (U8 ? (HIN % 4 == 0 && CI == 4) : (HIN * CI) % 16 == 0), "shape");
    static_assert(G * TILE_IN + 64 < 65536 && G * TILE_B < 32768 && G * SLOTS < (1 << 20) && COLS < (1 << 20), "offsets");
    static_assert(P == 1 || (G == 1 && KS_C == 1 && H % 2 == 0 && HIN % 2 == 0), "8-channel layers: one image, one MFMA step, even sizes");
    static_assert(P == 2 || (KSK == KS_C && (CI == 8 || CI == 16)), "16-channel layers: 8 or 16 stored input channels");
};

// max(v, v of the lane to its left in the same 16-lane row) for the lanes of rows `ROWS` (a 4-bit mask over the four
// rows); lane 0 of a row, and the rows not selected, keep v.  One DPP instruction: lanes without a source are not
// written and keep the destination's old value, which is v.  (The two idle cycles a DPP read needs after the vector
// instruction that wrote its source are spelled out: the compiler does not look inside the statement.)
template <int ROWS>
__device__ __forceinline__ int max_with_left(int v) {
    int d = v;
    if constexpr (ROWS == 0xC) asm("s_nop 1\n\tv_max_i32_dpp %0, %1, %1 row_shr:1 row_mask:0xc bank_mask:0xf" : "+v"(d) : "v"(v));
    else asm("s_nop 1\n\tv_max_i32_dpp %0, %1, %1 row_shr:1 row_mask:0xf bank_mask:0xf" : "+v"(d) : "v"(v));
    return d;
}

// P23: the first convolution of both blocks keeps its accumulators below 2^23 (see requant_relu4_p23)
template <bool U8, int CI, int HIN, int C, int G, int NW, int MINB, bool P23>
__global__ __launch_bounds__(NW * 64, MINB) void stack_kernel(const StackParams p) {
    typedef StShape<U8, CI, HIN, C, G, NW> S;
    constexpr int ST_THREADS = S::ST_THREADS, TU = S::TU;
    typedef int v2i __attribute__((ext_vector_type(2)));
    extern __shared__ __attribute__((aligned(16))) char smem[];
    char* tin = smem;                                    // G bordered input tiles
    char* tX = smem + S::O_TX;                           // G bordered tiles of max(stream, 0)
    char* tM = smem + S::O_TM;                           // G bordered tiles of a block's inner tensor
    char* xraw = smem + S::O_RAW;                        // G plain images of the stream (skip connection)
    char* tab1 = smem + S::O_T1;                         // conv + pool: per (strip, lane) or per slot, see below
    uint16_t* tabB = (uint16_t*)(smem + S::O_TABB);      // block column -> offset of its window in a bordered tile set
    int* cst = (int*)(smem + S::O_CST);                  // [conv][bias 16 | mult 16]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 15, g = lane >> 4;

    // ---- weights of all five convolutions and the chunk offsets of this lane
    v4i wC[S::KS_C], wO[S::P == 1 ? S::KS_C : 1], wA1[S::KS_B], wB1[S::KS_B], wA2[S::KS_B], wB2[S::KS_B];
    int koffC[S::KS_C], koffB[S::KS_B];
    if constexpr (S::P == 2) {
#pragma unroll
        for (int st = 0; st < S::KS_C; ++st) {
            const int q = 4 * st + g, ky = q / S::CPR_C, cx = q - ky * S::CPR_C;
            koffC[st] = (ky < 3) ? ky * S::PITCH_IN + cx * 16 : 0;
            wC[st] = p.w[0][st * 64 + lane];
        }
    } else {
        // chunk (ky, cx) of the planner's fragments (CPR_C chunks per kernel row), zero outside the kernel
        auto host_chunk = [&](int ky, int cx) -> v4i {
            if (ky >= 3 || cx < 0 || cx >= S::CPR_C) return (v4i){0, 0, 0, 0};
            const int qh = ky * S::CPR_C + cx;
            return p.w[0][(qh >> 2) * 64 + 16 * (qh & 3) + (lane & 15)];
        };
#pragma unroll
        for (int st = 0; st < S::KS_C; ++st) {
            const int q = 4 * st + g, ky = q / S::CPRK, cx = q - ky * S::CPRK;
            koffC[st] = (ky < 3) ? ky * S::PITCH_IN + cx * 16 : 0;
            wC[st] = host_chunk(ky, cx);
            if constexpr (CI == 16) {
                wO[st] = host_chunk(ky, cx - 1);                 // a pixel is a whole chunk
            } else {
                const v4i prev = host_chunk(ky, cx - 1), own = host_chunk(ky, cx);   // a chunk is two pixels
                wO[st] = (v4i){prev[2], prev[3], own[0], own[1]};
            }
        }
    }
#pragma unroll
    for (int st = 0; st < S::KS_B; ++st) {
        const int q = 4 * st + g, ky = q / S::CPR_B, cx = q - ky * S::CPR_B;
        koffB[st] = (ky < 3) ? ky * S::PITCH_B + cx * 16 : 0;
        wA1[st] = p.w[1][st * 64 + lane];
        wB1[st] = p.w[2][st * 64 + lane];
        wA2[st] = p.w[3][st * 64 + lane];
        wB2[st] = p.w[4][st * 64 + lane];
    }
    // the weights are in their registers before any other load is issued: the waits the compiler places in the batch
    // loop then only ever concern the loads of the next batch, not these
    __builtin_amdgcn_s_waitcnt(0x0F70);                  // vmcnt(0)

    // ---- staging: which bytes a lane requests, and where they land in the input tiles, is the same for every batch
    v4i pre[S::PF];
    uint32_t soff[S::PF];
    int doff[S::PF];
#pragma unroll
    for (int i = 0; i < S::PF; ++i) {
        const int u = min(tid + i * ST_THREADS, G * S::UNITS_IN - 1);
        const int img = u / S::UNITS_IN, w = u - img * S::UNITS_IN, row = w / S::UPR_IN, cu = w - row * S::UPR_IN;
        soff[i] = U8 ? (uint32_t)(img * S::IMG_IN + row * HIN + 4 * cu) : (uint32_t)(img * S::IMG_IN + w * 16);
        doff[i] = img * S::TILE_IN + (row + 1) * S::PITCH_IN + CI + cu * 16;
    }
    const int64_t n_batch = (p.B + G - 1) / G;
    auto prefetch = [&](int64_t batch) {
        const int64_t b0 = batch * G;
        const int gc = (int)((p.B - b0 < G) ? (p.B - b0) : G);
        const int last = gc * S::UNITS_IN - 1;
        const char* src = (const char*)p.in + b0 * (int64_t)S::IMG_IN;
#pragma unroll
        for (int i = 0; i < S::PF; ++i) {
            const uint32_t so = (tid + i * ST_THREADS <= last) ? soff[i] : 0u;     // a unit that does not exist re-reads unit 0
            if constexpr (U8) {
                v4i v;
#pragma unroll
                for (int c = 0; c < 4; ++c) v[c] = *(const int*)(src + (uint32_t)(c * HIN * HIN) + so);
                pre[i] = v;
            } else {
                pre[i] = *(const v4i*)(src + so);
            }
        }
    };
    auto commit = [&](int64_t batch) {
        const int64_t b0 = batch * G;
        const int total = (int)((p.B - b0 < G) ? (p.B - b0) : G) * S::UNITS_IN;
#pragma unroll
        for (int i = 0; i < S::PF; ++i) {
            if (tid + i * ST_THREADS >= total) break;
            const v4i v = pre[i];
            if constexpr (U8) {
                // one dword (4 pixels) of each plane -> four channels-last pixels, stored as obs - 128
                const uint32_t P0 = (uint32_t)v[0], P1 = (uint32_t)v[1], P2 = (uint32_t)v[2], P3 = (uint32_t)v[3];
                const uint32_t lo01 = __builtin_amdgcn_perm(P1, P0, 0x05010400u), hi01 = __builtin_amdgcn_perm(P1, P0, 0x07030602u);
                const uint32_t lo23 = __builtin_amdgcn_perm(P3, P2, 0x05010400u), hi23 = __builtin_amdgcn_perm(P3, P2, 0x07030602u);
                uint32_t* d = (uint32_t*)(tin + doff[i]);
                d[0] = __builtin_amdgcn_perm(lo23, lo01, 0x05040100u) ^ 0x80808080u;
                d[1] = __builtin_amdgcn_perm(lo23, lo01, 0x07060302u) ^ 0x80808080u;
                d[2] = __builtin_amdgcn_perm(hi23, hi01, 0x05040100u) ^ 0x80808080u;
                d[3] = __builtin_amdgcn_perm(hi23, hi01, 0x07060302u) ^ 0x80808080u;
            } else if constexpr ((CI & 15) == 0) {
                *(v4i*)(tin + doff[i]) = v;
            } else {
                *(v2i*)(tin + doff[i]) = (v2i){v[0], v[1]};
                *(v2i*)(tin + doff[i] + 8) = (v2i){v[2], v[3]};
            }
        }
    };

    int64_t batch = blockIdx.x;
    if (batch < n_batch) prefetch(batch);

    // ---- once per workgroup: borders, tables, constants
    {
        const int padv = U8 ? (int)0x80808080u : 0;       // a padding pixel is the observation value 0
        for (int i = tid; i < S::O_TX / 4; i += ST_THREADS) ((int*)tin)[i] = padv;
        for (int i = tid; i < (S::O_RAW - S::O_TX) / 4; i += ST_THREADS) ((int*)tX)[i] = 0;
        if constexpr (S::P == 2) {
            // per (strip, lane): window offset in an input row (chunk offset included), offsets of the lane's four
            // output bytes in the bordered tile and in the plain image (lanes 32-63 end up with the lower pooled row),
            // and whether the lane's pixel exists.  Pixel of lane j of strip s: 15 s + j - 1.
            for (int i = tid; i < S::NS * 64; i += ST_THREADS) {
                const int st = i >> 6, l = i & 63, jj = l & 15, gg = l >> 4;
                const int px = 15 * st + jj - 1, pc = min(max(px, 0), S::H - 1);
                const int ky = gg / S::CPR_C, cx = gg - ky * S::CPR_C;
                const int kf = (ky < 3) ? ky * S::PITCH_IN + cx * 16 : 0;
                ((v4i*)tab1)[i] = (v4i){2 * pc * CI + kf, (pc + 1) * C + 4 * (gg & 1) + (gg >> 1) * S::PITCH_B,
                                        pc * C + 4 * (gg & 1) + (gg >> 1) * S::H * C, (jj >= 1 && px < S::H) ? 1 : 0};
            }
        } else {
            // per slot (image, pooled row, dummy | pixel): offsets of the E window in the first and in the middle input
            // row (odd sizes: bit 0 of the first = no row below, of the second = no column to the right), offsets of the
            // pixel's output in the bordered tile and in the plain image (bit 15 = the slot is a dummy)
            for (int sidx = tid; sidx < G * S::SLOTS; sidx += ST_THREADS) {
                const int img = sidx / S::SLOTS, si = sidx - img * S::SLOTS, py = si / (S::H + 1), ps = si - py * (S::H + 1);
                const int px = max(ps - 1, 0);
                const int r0 = max(2 * py - 1, 0), r1 = 2 * py;
                const int xe = 2 * px * CI + img * S::TILE_IN;
                const int nb = (2 * py + 1 > HIN - 1) ? 1 : 0, nr = (ps > 0 && 2 * px + 1 > HIN - 1) ? 1 : 0;
                const uint32_t a0 = (uint32_t)(r0 * S::PITCH_IN + xe) | (uint32_t)nb, a1 = (uint32_t)(r1 * S::PITCH_IN + xe) | (uint32_t)nr;
                const uint32_t ox = (uint32_t)(img * S::TILE_B + (py + 1) * S::PITCH_B + (px + 1) * C) | (ps == 0 ? 0x8000u : 0u);
                const uint32_t orr = (uint32_t)(img * S::IMG + (py * S::H + px) * C);
                ((v2i*)tab1)[sidx] = (v2i){(int)(a0 | (a1 << 16)), (int)(ox | (orr << 16))};
            }
        }
        for (int c = tid; c < (S::TILES + 3 * NW * TU) * 16; c += ST_THREADS) {
            const int cc = min(c, S::COLS - 1);            // columns past the end repeat the last one (never stored)
            const int img = cc / S::NPX, w = cc - img * S::NPX, y = w / S::WP, xp = w - y * S::WP;
            tabB[c] = (uint16_t)(img * S::TILE_B + y * S::PITCH_B + xp * 16);
        }
        for (int i = tid; i < 5 * 16; i += ST_THREADS) {
            const int cv = i >> 4, n = i & 15;
            cst[cv * 32 + n] = p.bias[cv][n];
            ((float*)cst)[cv * 32 + 16 + n] = p.mult[cv][n];
        }
    }
    __syncthreads();

    for (; batch < n_batch; batch += gridDim.x) {
        commit(batch);
        __syncthreads();
        const int64_t b0 = batch * G;
        const int gc = (int)((p.B - b0 < G) ? (p.B - b0) : G);

        // ---- stack convolution + max-pool, in registers -> the bordered tile of max(x, 0) and the plain image
        {
            const v4i biC = *(const v4i*)(cst + 4 * g);
            const v4f mlC = *(const v4f*)(cst + 16 + 4 * g);
            auto finish = [&](const v4i& pooled, int ox, int orw, bool ok) {
                int q[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) q[r] = rne_clamp127((float)pooled[r] * mlC[r]);
                const uint32_t w = pack_low_bytes(q);
                if (ok) {
                    *(uint32_t*)(tX + ox) = relu_i8x4(w);
                    *(uint32_t*)(xraw + orw) = w;
                }
            };
            if constexpr (S::P == 2) {
                // work item: (pair of pooled rows rp, strip): conv rows 4rp-1 .. 4rp+3, the middle one shared.  The five
                // window reads of the next item are issued before the current item's maxima are formed and requantized.
                constexpr int N_IT = (S::H / 2) * S::NS;
                auto issue = [&](int it, v4i (&o)[5], v4i& e, int& rp) {
                    it = min(it, N_IT - 1);                  // past the end: a valid item, read and dropped
                    rp = it / S::NS;
                    e = ((const v4i*)tab1)[(it - rp * S::NS) * 64 + lane];
                    const char* a0 = tin + e[0] + max(4 * rp - 1, 0) * S::PITCH_IN;
                    const char* a1 = tin + e[0] + 4 * rp * S::PITCH_IN;
                    o[0] = read_chunk<S::RD_E>(a0);
#pragma unroll
                    for (int k = 1; k < 5; ++k) o[k] = read_chunk<S::RD_E>(a1 + (k - 1) * S::PITCH_IN);
                };
                v4i oA[5], oB[5], eA, eB;
                int rpA, rpB;
                // E in lanes 0-31, O in lanes 32-63 of each row's tile: O takes its left neighbour in, then one swap per
                // register puts E and O of the upper row into the lower lanes and of the lower row into the upper
                auto pool_store = [&](const v4i (&c)[5], const v4i& e, int rp) {
                    v4i pooled;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int x0 = max_with_left<0xC>(max(max(c[0][r], c[1][r]), c[2][r]));
                        const int x1 = max_with_left<0xC>(max(max(c[2][r], c[3][r]), c[4][r]));
                        const auto sw = __builtin_amdgcn_permlane32_swap((unsigned)x0, (unsigned)x1, false, false);
                        pooled[r] = max((int)sw[0], (int)sw[1]);
                    }
                    finish(pooled, e[1] + (2 * rp + 1) * S::PITCH_B, e[2] + 2 * rp * S::H * C, e[3] != 0);
                };
                if constexpr (NW >= 8) {
                    // four wavefronts per SIMD hide the read latency by themselves: one item at a time, fewer registers
                    for (int it = wave; it < N_IT; it += NW) {
                        issue(it, oA, eA, rpA);
                        v4i c[5];
#pragma unroll
                        for (int k = 0; k < 5; ++k) c[k] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wC[0], oA[k], biC, 0, 0, 0);
                        pool_store(c, eA, rpA);
                    }
                } else {
                issue(wave, oA, eA, rpA);
                for (int it = wave; it < N_IT; it += 2 * NW) {
                    v4i c[5];
#pragma unroll
                    for (int k = 0; k < 5; ++k) c[k] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wC[0], oA[k], biC, 0, 0, 0);
                    issue(it + NW, oB, eB, rpB);
                    pool_store(c, eA, rpA);
                    if (it + NW >= N_IT) break;
#pragma unroll
                    for (int k = 0; k < 5; ++k) c[k] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wC[0], oB[k], biC, 0, 0, 0);
                    issue(it + 2 * NW, oA, eA, rpA);
                    pool_store(c, eB, rpB);
                }
                }
            } else {
                constexpr bool ODD = (HIN & 1) != 0;
                const int n_slots = gc * S::SLOTS;
                const int n_tiles = (n_slots - 1 + 14) / 15;
                for (int t = wave; t < n_tiles; t += NW) {
                    const int s = 15 * t + j;
                    const v2i e = ((const v2i*)tab1)[min(s, n_slots - 1)];
                    const uint32_t ex = (uint32_t)e[0], ey = (uint32_t)e[1];
                    const int a0 = (int)(ex & (ODD ? 0xfffeu : 0xffffu)), a1 = (int)((ex >> 16) & (ODD ? 0xfffeu : 0xffffu));
                    const int d2 = (ODD && (ex & 1u)) ? 0 : S::PITCH_IN;            // no row below: repeat the middle one
                    const bool no_right = ODD && ((ex >> 16) & 1u);                 // no column to the right: O repeats E
                    v4i acc[2][3];
#pragma unroll
                    for (int eo = 0; eo < 2; ++eo)
#pragma unroll
                        for (int k = 0; k < 3; ++k) acc[eo][k] = biC;
#pragma unroll
                    for (int st = 0; st < S::KS_C; ++st) {
                        const char* w0 = tin + a0 + koffC[st];
                        const char* w1 = tin + a1 + koffC[st];
                        const char* wr[3] = {w0, w1, w1 + d2};
#pragma unroll
                        for (int k = 0; k < 3; ++k) {
                            const v4i b = *(const v4i*)wr[k];      // one aligned read serves the E and the O window
                            acc[0][k] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wC[st], b, acc[0][k], 0, 0, 0);
                            acc[1][k] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wO[st], b, acc[1][k], 0, 0, 0);
                        }
                    }
                    v4i pooled;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int ve = max(max(acc[0][0][r], acc[0][1][r]), acc[0][2][r]);
                        int vo = max(max(acc[1][0][r], acc[1][1][r]), acc[1][2][r]);
                        if (no_right) vo = ve;
                        pooled[r] = max(ve, max_with_left<0xF>(vo));
                    }
                    finish(pooled, (int)(ey & 0x7fffu) + 4 * g, (int)(ey >> 16) + 4 * g, s < n_slots && j >= 1 && !(ey & 0x8000u));
                }
            }
        }
        __syncthreads();

        const int total = gc * S::NPX;
        const int n_tiles = (total + 15) >> 4;
        // Block convolutions: TU column tiles per wavefront and step (tiles t, t + NW, ...); the window reads of the next
        // step are issued before the current step's epilogue, and the table entries two steps ahead of their use.
        constexpr int STEP = NW * TU;
        auto load_ops = [&](const char* src, const int (&b)[TU], v4i (&o)[TU][S::KS_B]) {
#pragma unroll
            for (int st = 0; st < S::KS_B; ++st)
#pragma unroll
                for (int u = 0; u < TU; ++u) o[u][st] = *(const v4i*)(src + b[u] + koffB[st]);
        };
        // ---- a block's first convolution: max(x, 0) -> inner tensor, requantized with the fused ReLU
        auto conv_a = [&](const v4i (&wA)[S::KS_B], int cv) {
            const v4i biA = *(const v4i*)(cst + cv * 32 + 4 * g) + (P23 ? P23_MAGIC : 0);
            const v4f mlA = *(const v4f*)(cst + cv * 32 + 16 + 4 * g);
            const v4f cA = mlA * -8388608.0f;
            int bN[TU], bNN[TU];
#pragma unroll
            for (int u = 0; u < TU; ++u) { bN[u] = tabB[(wave + NW * u) * 16 + j]; bNN[u] = tabB[(wave + STEP + NW * u) * 16 + j]; }
            v4i ops[TU][S::KS_B];
            load_ops(tX, bN, ops);
            for (int t = wave; t < n_tiles; t += STEP) {
                int base[TU];
                v4i acc[TU];
#pragma unroll
                for (int u = 0; u < TU; ++u) { base[u] = bN[u]; acc[u] = biA; }
#pragma unroll
                for (int st = 0; st < S::KS_B; ++st)
#pragma unroll
                    for (int u = 0; u < TU; ++u) acc[u] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wA[st], ops[u][st], acc[u], 0, 0, 0);
#pragma unroll
                for (int u = 0; u < TU; ++u) { bN[u] = bNN[u]; bNN[u] = tabB[(t + 2 * STEP + NW * u) * 16 + j]; }
                load_ops(tX, bN, ops);
#pragma unroll
                for (int u = 0; u < TU; ++u) {
                    const uint32_t w = requant_relu4_p23<P23>(acc[u], mlA, cA);
                    // the column's own pixel(s) sit one row and one pixel inside its window
                    if ((t + NW * u) * 16 + j < total) *(uint32_t*)(tM + base[u] + S::PITCH_B + C + 4 * g) = w;
                }
            }
        };
        // ---- a block's second convolution, joined with the block's input; LAST: to memory, else back into LDS
        auto conv_b = [&](const v4i (&wB)[S::KS_B], int cv, float rr, auto last) {
            constexpr bool LAST = decltype(last)::value;
            const v4i biB = *(const v4i*)(cst + cv * 32 + 4 * g);
            const v4f mlB = *(const v4f*)(cst + cv * 32 + 16 + 4 * g);
            int8_t* outp = p.out + b0 * (int64_t)S::IMG;
            int bN[TU], bNN[TU];
            uint32_t xn[TU];
#pragma unroll
            for (int u = 0; u < TU; ++u) {
                bN[u] = tabB[(wave + NW * u) * 16 + j];
                bNN[u] = tabB[(wave + STEP + NW * u) * 16 + j];
                xn[u] = *(const uint32_t*)(xraw + (uint32_t)min((wave + NW * u) * 16 + j, total - 1) * 16u + 4 * g);
            }
            v4i ops[TU][S::KS_B];
            load_ops(tM, bN, ops);
            for (int t = wave; t < n_tiles; t += STEP) {
                int base[TU];
                uint32_t xr[TU];
                v4i acc[TU];
#pragma unroll
                for (int u = 0; u < TU; ++u) { base[u] = bN[u]; xr[u] = xn[u]; acc[u] = biB; }
#pragma unroll
                for (int st = 0; st < S::KS_B; ++st)
#pragma unroll
                    for (int u = 0; u < TU; ++u) acc[u] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wB[st], ops[u][st], acc[u], 0, 0, 0);
#pragma unroll
                for (int u = 0; u < TU; ++u) { bN[u] = bNN[u]; bNN[u] = tabB[(t + 2 * STEP + NW * u) * 16 + j]; }
                load_ops(tM, bN, ops);
#pragma unroll
                for (int u = 0; u < TU; ++u) xn[u] = *(const uint32_t*)(xraw + (uint32_t)min((t + STEP + NW * u) * 16 + j, total - 1) * 16u + 4 * g);
#pragma unroll
                for (int u = 0; u < TU; ++u) {
                    const int col = (t + NW * u) * 16 + j;
                    int q[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const float tr = (float)(int)(int8_t)(xr[u] >> (8 * r)) * rr;
                        q[r] = rne_clamp127(fmaf((float)acc[u][r], mlB[r], tr));
                    }
                    const uint32_t w = pack_low_bytes(q);
                    if (col < total) {
                        if constexpr (LAST) {
                            *(uint32_t*)(outp + (uint32_t)col * 16u + 4 * g) = w;
                        } else {
                            *(uint32_t*)(xraw + (uint32_t)col * 16u + 4 * g) = w;
                            *(uint32_t*)(tX + base[u] + S::PITCH_B + C + 4 * g) = relu_i8x4(w);
                        }
                    }
                }
            }
        };
        conv_a(wA1, 1);
        __syncthreads();
        conv_b(wB1, 2, p.r1, std::false_type{});
        __syncthreads();
        conv_a(wA2, 3);
        __syncthreads();
        // the next batch's bytes are requested here, not earlier: their registers are then free during the phases above
        // (where the kernel needs the most), and the last phase is long enough for the loads to land
        if (batch + gridDim.x < n_batch) prefetch(batch + gridDim.x);
        conv_b(wB2, 4, p.r2, std::true_type{});
        // no barrier here: the next commit writes the input tiles only, and the barrier behind it comes before the
        // next batch writes anything that the last phase reads
    }
}

// the five convolutions of a stack as the planner laid them out: c = stack convolution (with its fused pool),
// a1 / b1 and a2 / b2 = the two blocks
template <bool U8, int CI, int HIN, int C, int G, int NW>
bool st_shape_ok(const ConvParams& c, const ConvParams& a1, const ConvParams& b1, const ConvParams& a2, const ConvParams& b2) {
    typedef StShape<U8, CI, HIN, C, G, NW> S;
    if (c.H != HIN || c.W != HIN || c.Cs_in != CI || c.Cin_real != CI || c.Ho != HIN || c.Wo != HIN / S::P || c.Cs_out != 16) return false;
    if (c.k != 3 || c.s != 1 || c.pad != 1 || c.sx != S::P || c.cpr != S::CPR_C || c.k_steps != S::KS_C) return false;
    if ((c.src_u8 != 0) != U8 || !c.pool || c.PH != S::H || c.PW != S::H || c.relu || c.relu_in || c.out_frag) return false;
    for (const ConvParams* b : {&a1, &b1, &a2, &b2}) {
        if (b->H != S::H || b->W != S::H || b->Cin_real != C || b->Cs_in != C || b->Ho != S::H || b->Wo != S::WP || b->Cs_out != 16) return false;
        if (b->k != 3 || b->s != 1 || b->pad != 1 || b->sx != S::P || b->cpr != S::CPR_B || b->k_steps != S::KS_B) return false;
        if (b->src_u8 || b->pool || b->out_frag) return false;
    }
    return a1.relu_in && a1.relu && !b1.relu_in && !b1.relu && a2.relu_in && a2.relu && !b2.relu_in && !b2.relu;
}

template <bool U8, int CI, int HIN, int C, int G, int NW, int MINB, bool P23>
hipError_t st_go(const StackParams& p, hipStream_t s) {
    typedef StShape<U8, CI, HIN, C, G, NW> S;
    auto kfn = stack_kernel<U8, CI, HIN, C, G, NW, MINB, P23>;
    static int occ = 0;
    if (!occ) {
        hipError_t e = hipFuncSetAttribute((const void*)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, S::LDS);
        if (e != hipSuccess) return e;
        int o = 0;
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&o, (const void*)kfn, S::ST_THREADS, S::LDS);
        if (e != hipSuccess) return e;
        occ = o < 1 ? 1 : o;
    }
    // resident workgroups striding over the batches, in even rounds
    const int64_t batches = (p.B + G - 1) / G;
    const int64_t cap = (int64_t)occ * conv_num_cus();
    const int64_t rounds = (batches + cap - 1) / cap;
    dim3 grid((unsigned)((batches + rounds - 1) / rounds));
    kfn<<<grid, dim3(S::ST_THREADS), S::LDS, s>>>(p);
    return hipGetLastError();
}

}  // namespace

// (uint8 source, stored input channels, input size, channels, images per batch, wavefronts per workgroup, wavefronts per
// SIMD the register budget is set for).  Stack 1 is held to two workgroups per CU by its LDS: eight wavefronts per
// workgroup at 128 registers give its SIMDs four wavefronts each (504 -> 453 us at 16384 states); stacks 2 and 3, bound by
// LDS traffic rather than by issue, gain nothing from that and keep four-wavefront workgroups, three to a CU.
#define ACCERL_STACK_SHAPES(X) X(true, 4, 84, 8, 1, 8, 4) X(false, 8, 42, 16, 1, 4, 3) X(false, 16, 21, 16, 2, 4, 3)

bool stack_supported(const ConvParams& c, int NTC, const ConvParams& a1, const ConvParams& b1, const ConvParams& a2, const ConvParams& b2) {
    if (NTC != 1) return false;
#define X(U8, CI, HIN, C, G, NW, MINB) if (st_shape_ok<U8, CI, HIN, C, G, NW>(c, a1, b1, a2, b2)) return true;
    ACCERL_STACK_SHAPES(X)
#undef X
    return false;
}

hipError_t launch_stack(const ConvParams& c, const ConvParams& a1, const ConvParams& b1, const ConvParams& a2, const ConvParams& b2, hipStream_t s) {
    if (c.B <= 0) return hipSuccess;
    StackParams p;
    p.in = c.in; p.out = (int8_t*)b2.out;
    const ConvParams* cv[5] = {&c, &a1, &b1, &a2, &b2};
    for (int i = 0; i < 5; ++i) { p.w[i] = (const v4i*)cv[i]->wfrag; p.bias[i] = (const int*)cv[i]->bias; p.mult[i] = cv[i]->mult; }
    p.r1 = b1.r; p.r2 = b2.r; p.B = c.B;
    static const bool no_p23 = getenv("ACCERL_NO_P23") != nullptr;
    const bool p23 = a1.pos23 && a2.pos23 && !no_p23;
#define X(U8, CI, HIN, C, G, NW, MINB)                                                              \
    if (st_shape_ok<U8, CI, HIN, C, G, NW>(c, a1, b1, a2, b2))                                      \
        return p23 ? st_go<U8, CI, HIN, C, G, NW, MINB, true>(p, s) : st_go<U8, CI, HIN, C, G, NW, MINB, false>(p, s);
    ACCERL_STACK_SHAPES(X)
#undef X
    return hipErrorInvalidValue;
}

}  // namespace accerl
