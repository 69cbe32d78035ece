// The first two convolutions of the paper's original network (network table: 32 filters of 8x8 and 64
// of 4x4 on a 4x84x84 uint8 observation; strides 4 and 2, no padding) as one pipelined kernel with every
// size known at compile time.
//
// A workgroup of eight wavefronts walks over observations.  In one tick
//   wavefronts 4..7  compute the first convolution of observation n+1 from the LDS copy of its bytes and
//                    write the requantized 20x20x32 image to one of two LDS tiles,
//   wavefronts 0..3  compute the second convolution of observation n from the other tile and store the
//                    requantized 9x9x64 image,
//   everyone         has the bytes of observation n+2 in flight from memory,
// then the workgroup meets, writes the bytes of observation n+2 to LDS and meets again.  The matrix-core
// work of one role overlaps the requantization arithmetic of the other inside a workgroup, and there are
// two barriers per observation.
//
// Weights live in registers: a first-layer wavefront holds all 32 filters (32 VGPRs); a second-layer
// wavefront holds one half of the 64 filters (64 VGPRs) and computes three 16-pixel tiles with it, so a
// pixel fragment read from LDS feeds two MFMAs.  The 81 output pixels are covered by the tiles
// 0..47 and 33..80: the overlap is computed twice and stored twice with identical bytes, which keeps the
// code free of per-pixel predicates.
//
// Observation tile.  Chunk u (16 bytes) of the LDS copy is dword u of each of the four channel planes,
// side by side: dword u of a plane holds 4 horizontally adjacent pixels and 84 = 21 dwords, so chunk u is
// row u / 21, pixels 4 * (u % 21) .. + 3 -- staging needs no index arithmetic and no byte shuffles, only the
// sign flip (obs - 128).  The weight fragments arrive ordered (kx, c) inside a chunk; they are
// transposed to (c, kx) once per wavefront to match.
//
// Arithmetic, fragment layouts, bias (with the zero-point correction) and multipliers are those of
// conv_kernel.h: accumulators and activations are bit-identical to the layer-by-layer path.
#include "conv_kernel.h"

namespace accerl {

namespace {
constexpr int FR_THREADS = 512;
constexpr int FR_PLANE = 84 * 84;                 // bytes per channel plane
constexpr int FR_UNITS = FR_PLANE / 4;            // 16-byte chunks of the observation tile (1764)
constexpr int FR_TILE_A = FR_UNITS * 16;          // 28224
constexpr int FR_ROW_A = 21 * 16;                 // LDS bytes per observation row
constexpr int FR_NPIX1 = 400, FR_TILES1 = 25, FR_PIX1_BYTES = 32, FR_ROW_B = 20 * 32;
constexpr int FR_TILE_B = FR_NPIX1 * FR_PIX1_BYTES;   // 12800
constexpr int FR_NPIX2 = 81, FR_PIX2_BYTES = 64;
constexpr int FR_LDS = FR_TILE_A + 2 * FR_TILE_B;
constexpr int FR_ROUNDS_A = 7;                    // tiles of the first layer per wavefront (25 over 4)
constexpr int FR_STAGERS = 256;                  // lanes of the first-layer wavefronts: they stage the observations
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

// clamp(rint(acc * m), 0, 127) of four accumulators -> four bytes
__device__ __forceinline__ uint32_t requant_relu4(v4i acc, v4f m) {
    uint32_t w = 0;
#pragma unroll
    for (int r = 0; r < 4; ++r)
        w = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_amdgcn_fmed3f((float)acc[r] * m[r], 0.0f, 127.0f), r, w);
    return w;
}

__global__ __launch_bounds__(FR_THREADS, 4) void conv_front_kernel(const FrontParams p) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    typedef int v2i __attribute__((ext_vector_type(2)));
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 15, g = lane >> 4;
    char* tileA = smem;
    char* tileB = smem + FR_TILE_A;                     // two tiles, FR_TILE_B apart
    const bool roleA = wave >= 4;

    const int64_t stride = gridDim.x;
    int64_t img = blockIdx.x;                           // observation whose second convolution runs this tick
    if (img >= p.B) return;

    if (roleA) {
        // ================= first-layer wavefronts (they also stage the observations)
        const int aw = wave - 4, stid = tid - 256;
        // staging: chunk u = dword u of the four planes
        uint32_t pre[FR_PF][4];
        auto stage_load = [&](int64_t im) {
            const uint8_t* src = p.obs + im * (int64_t)(4 * FR_PLANE);
#pragma unroll
            for (int k = 0; k < FR_PF; ++k) {
                const int u = min(stid + k * FR_STAGERS, FR_UNITS - 1);
#pragma unroll
                for (int c = 0; c < 4; ++c) pre[k][c] = *(const uint32_t*)(src + c * FR_PLANE + 4 * u);
            }
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
        stage_load(img);
        v4i wA[4][2];
#pragma unroll
        for (int st = 0; st < 4; ++st)
#pragma unroll
            for (int t = 0; t < 2; ++t) wA[st][t] = transpose4x4(p.wA[(st * 2 + t) * 64 + lane]);
        v4i biA[2];
        v4f mlA[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            biA[t] = *(const v4i*)(p.biasA + 8 * g + 4 * t);
            mlA[t] = *(const v4f*)(p.multA + 8 * g + 4 * t);
        }
        // window of this lane's pixel in each of its tiles; K step st adds two observation rows
        int rbase[FR_ROUNDS_A];
#pragma unroll
        for (int r = 0; r < FR_ROUNDS_A; ++r) {
            const int px = min((aw + 4 * r) * 16 + j, FR_NPIX1 - 1);
            const int oy = (px * 3277) >> 16, ox = px - oy * 20;       // px / 20 for px < 16384
            rbase[r] = oy * (4 * FR_ROW_A) + ox * 16 + (g >> 1) * FR_ROW_A + (g & 1) * 16;
        }
        const int wofs = (aw * 16 + j) * FR_PIX1_BYTES + 8 * g;       // tile r adds 4 * 16 pixels

        auto conv_a = [&](char* dstB) {
            v4i f[4];
#pragma unroll
            for (int st = 0; st < 4; ++st) f[st] = *(const v4i*)(tileA + rbase[0] + st * (2 * FR_ROW_A));
#pragma unroll
            for (int r = 0; r < FR_ROUNDS_A; ++r) {
                if (aw + 4 * r >= FR_TILES1) break;
                v4i acc[2];
#pragma unroll
                for (int t = 0; t < 2; ++t) acc[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wA[0][t], f[0], biA[t], 0, 0, 0);
#pragma unroll
                for (int st = 1; st < 4; ++st)
#pragma unroll
                    for (int t = 0; t < 2; ++t) acc[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wA[st][t], f[st], acc[t], 0, 0, 0);
                if (r + 1 < FR_ROUNDS_A && aw + 4 * (r + 1) < FR_TILES1) {
#pragma unroll
                    for (int st = 0; st < 4; ++st) f[st] = *(const v4i*)(tileA + rbase[r + 1 < FR_ROUNDS_A ? r + 1 : r] + st * (2 * FR_ROW_A));
                }
                const uint32_t w0 = requant_relu4(acc[0], mlA[0]), w1 = requant_relu4(acc[1], mlA[1]);
                *(v2i*)(dstB + wofs + r * (64 * FR_PIX1_BYTES)) = (v2i){(int)w0, (int)w1};
            }
        };

        stage_commit();
        __syncthreads();                                 // observation tile complete
        conv_a(tileB);
        const bool more = img + stride < p.B;
        if (more) stage_load(img + stride);
        __syncthreads();                                 // first tile B complete, observation tile free
        if (more) stage_commit();
        __syncthreads();
        for (int n = 0;; ++n, img += stride) {
            const bool has_next = img + stride < p.B, has_next2 = img + 2 * stride < p.B;
            if (has_next2) stage_load(img + 2 * stride);
            if (has_next) conv_a(tileB + ((n + 1) & 1) * FR_TILE_B);
            if (!has_next) break;
            __syncthreads();
            if (has_next2) stage_commit();
            __syncthreads();
        }
    } else {
        // ================= second-layer wavefronts
        const int h = wave & 1, p0 = (wave >> 1) ? FR_NPIX2 - 48 : 0;
        v4i wB[8][2];
#pragma unroll
        for (int st = 0; st < 8; ++st)
#pragma unroll
            for (int t = 0; t < 2; ++t) wB[st][t] = p.wB[(st * 4 + 2 * h + t) * 64 + lane];
        const v4i* biasB = (const v4i*)(p.biasB + 16 * g + 8 * h);   // fetched per observation (cache hits): no registers held
        const v4f* multB = (const v4f*)(p.multB + 16 * g + 8 * h);
        int rb[3];
#pragma unroll
        for (int u = 0; u < 3; ++u) {
            const int px = p0 + 16 * u + j;
            const int oy = (px * 7282) >> 16, ox = px - oy * 9;       // px / 9 for px < 81
            rb[u] = oy * (2 * FR_ROW_B) + ox * (2 * FR_PIX1_BYTES) + g * 16;
        }
        const int oofs = (p0 + j) * FR_PIX2_BYTES + 16 * g + 8 * h;   // tile u adds 16 pixels

        auto conv_b = [&](const char* srcB, int8_t* outp) {
            v4i acc[3][2];
            v4i cur[3], nxt[3];
            const v4i bi0 = biasB[0], bi1 = biasB[1];
#pragma unroll
            for (int u = 0; u < 3; ++u) cur[u] = *(const v4i*)(srcB + rb[u]);
#pragma unroll
            for (int st = 0; st < 8; ++st) {
                if (st + 1 < 8) {
#pragma unroll
                    for (int u = 0; u < 3; ++u) nxt[u] = *(const v4i*)(srcB + rb[u] + ((st + 1) >> 1) * FR_ROW_B + ((st + 1) & 1) * 64);
                }
#pragma unroll
                for (int u = 0; u < 3; ++u) {
                    acc[u][0] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wB[st][0], cur[u], st == 0 ? bi0 : acc[u][0], 0, 0, 0);
                    acc[u][1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wB[st][1], cur[u], st == 0 ? bi1 : acc[u][1], 0, 0, 0);
                }
#pragma unroll
                for (int u = 0; u < 3; ++u) cur[u] = nxt[u];
            }
            const v4f m0 = multB[0], m1 = multB[1];
#pragma unroll
            for (int u = 0; u < 3; ++u) {
                const uint32_t w0 = requant_relu4(acc[u][0], m0), w1 = requant_relu4(acc[u][1], m1);
                *(v2i*)(outp + oofs + u * (16 * FR_PIX2_BYTES)) = (v2i){(int)w0, (int)w1};
            }
        };

        __syncthreads();
        __syncthreads();
        __syncthreads();
        for (int n = 0;; ++n, img += stride) {
            const bool has_next = img + stride < p.B;
            conv_b(tileB + (n & 1) * FR_TILE_B, p.out + img * (int64_t)(FR_NPIX2 * FR_PIX2_BYTES));
            if (!has_next) break;
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

hipError_t launch_conv_front(const ConvParams& a, const ConvParams& b, hipStream_t s) {
    if (a.B <= 0) return hipSuccess;
    static int occ = 0;
    if (!occ) {
        hipError_t e = hipFuncSetAttribute((const void*)conv_front_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, FR_LDS);
        if (e != hipSuccess) return e;
        int o = 0;
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&o, (const void*)conv_front_kernel, FR_THREADS, FR_LDS);
        if (e != hipSuccess) return e;
        occ = o < 1 ? 1 : o;
    }
    FrontParams p;
    p.obs = (const uint8_t*)a.in; p.out = (int8_t*)b.out;
    p.wA = (const v4i*)a.wfrag; p.biasA = (const int*)a.bias; p.multA = a.mult;
    p.wB = (const v4i*)b.wfrag; p.biasB = (const int*)b.bias; p.multB = b.mult;
    p.B = a.B;
    // resident workgroups striding over the observations, in even rounds
    const int64_t cap = (int64_t)occ * conv_num_cus();
    const int64_t rounds = (a.B + cap - 1) / cap;
    dim3 grid((unsigned)((a.B + rounds - 1) / rounds));
    conv_front_kernel<<<grid, dim3(FR_THREADS), FR_LDS, s>>>(p);
    return hipGetLastError();
}

}  // namespace accerl
