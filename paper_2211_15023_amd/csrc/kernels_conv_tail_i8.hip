// The third convolution of the paper's original network (network table: 64 filters of 3x3, stride 1, no
// padding, on the 9x9x64 int8 image the second layer leaves) as a pipelined kernel with every size known
// at compile time.
//
// A workgroup of four wavefronts works on two images at a time (two workgroups share a compute unit): wavefronts
// 2s and 2s+1 own image slot s, one half of the 64 filters each, held in registers for the whole kernel (9 K
// steps -- one per filter tap, 64 input channels each -- x 2 channel tiles = 72 VGPRs).  An image's 49 output
// pixels are four tiles: three of two output rows (14 pixels) and one of the last row; the spare lanes of a tile
// repeat a pixel of the tile, so every lane reads a valid address and duplicate stores carry identical bytes.
//
// LDS holds two copies of every slot's image, each split into four planes of 16 channels,
// [channel block][pixel][16 B]: a lane's fragment (pixel j, channel block g) is then 16 bytes apart from its
// neighbour's, and the 14 pixels of a two-row tile fall into 14 different 16-byte bank groups; the planes are a
// multiple of 256 bytes apart (measured: 134 B/clock against 109 with planes of 81 * 16 bytes).  In a tick the
// bytes of image n+1 (in registers since the tick before) go to the idle copy, the bytes of image n+2 are
// requested from memory, and image n is multiplied from the other copy: one barrier per image.  Inside a
// wavefront the MFMAs of a pixel tile are interleaved with the requantization of the tile before it.
//
// Arithmetic, weight fragments, bias and multipliers are those of conv_kernel.h (bit-identical results);
// the output goes to the plain channels-last image or, when the dense layer asks for it, to its MFMA
// fragment order.
#include <stdlib.h>

#include "conv_kernel.h"

namespace accerl {

namespace {
constexpr int TL_SLOTS = 2, TL_THREADS = 128 * TL_SLOTS;
constexpr int TL_IMG = 81 * 64;                  // bytes per input image
constexpr int TL_UNITS = TL_IMG / 16;            // 324 staging chunks
constexpr int TL_PLANE = 1536;                   // one channel block of an image in LDS: 81 pixels of 16 bytes, padded to a multiple of 256
constexpr int TL_COPY = 4 * TL_PLANE;            // one LDS copy of an image
constexpr int TL_PF = (TL_UNITS + 127) / 128;    // staging chunks per lane of a slot's two wavefronts (3)
constexpr int TL_LDS = TL_SLOTS * 2 * TL_COPY;
constexpr int TL_NPIX = 49, TL_PIX_BYTES = 64;

struct TailParams {
    const int8_t* in;        // [B, 9, 9, 64]
    int8_t* out;             // [B, 7, 7, 64] or fragment order
    const v4i* w; const int* bias; const float* mult;
    int64_t B;
    int out_frag, frag_ks;
};

// P23: the layer's accumulators stay below 2^23: requantization in the three-instruction form of requant_relu4_p23
template <bool P23>
__global__ __launch_bounds__(TL_THREADS, 2) void conv_tail_kernel(const TailParams p) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    typedef int v2i __attribute__((ext_vector_type(2)));
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 15, g = lane >> 4;
    const int slot = wave >> 1, h = wave & 1;
    char* tiles = smem + slot * (2 * TL_COPY);             // two copies of this slot's image

    // image n of this slot: 4 * (blockIdx.x + n * gridDim.x) + slot
    const int64_t stride = TL_SLOTS * (int64_t)gridDim.x;
    int64_t img = TL_SLOTS * (int64_t)blockIdx.x + slot;
    const int64_t img_first = TL_SLOTS * (int64_t)blockIdx.x;     // the workgroup's first image (the same in every wavefront)
    if (img_first >= p.B) return;

    // staging: chunk u = (pixel u / 4, channel block u % 4) goes to plane u % 4
    const int stid = tid & 127;
    v4i pre[TL_PF];
    int dofs[TL_PF];
#pragma unroll
    for (int k = 0; k < TL_PF; ++k) {
        const int u = min(stid + 128 * k, TL_UNITS - 1);
        dofs[k] = (u & 3) * TL_PLANE + (u >> 2) * 16;
    }
    auto stage_load = [&](int64_t im) {
        const int8_t* src = p.in + im * (int64_t)TL_IMG;
#pragma unroll
        for (int k = 0; k < TL_PF; ++k) pre[k] = *(const v4i*)(src + 16 * min(stid + 128 * k, TL_UNITS - 1));
    };
    auto stage_commit = [&](char* dst) {
#pragma unroll
        for (int k = 0; k < TL_PF; ++k)
            if (stid + 128 * k < TL_UNITS) *(v4i*)(dst + dofs[k]) = pre[k];
    };

    if (img < p.B) stage_load(img);
    v4i w[9][2];
#pragma unroll
    for (int st = 0; st < 9; ++st)
#pragma unroll
        for (int t = 0; t < 2; ++t) w[st][t] = p.w[(st * 4 + 2 * h + t) * 64 + lane];
    const v4i bi0 = *(const v4i*)(p.bias + 16 * g + 8 * h) + (P23 ? P23_MAGIC : 0), bi1 = *(const v4i*)(p.bias + 16 * g + 8 * h + 4) + (P23 ? P23_MAGIC : 0);
    const v4f m0 = *(const v4f*)(p.mult + 16 * g + 8 * h), m1 = *(const v4f*)(p.mult + 16 * g + 8 * h + 4);
    const v4f c0 = m0 * -8388608.0f, c1 = m1 * -8388608.0f;

    // the lane's pixel in each of the four tiles: tile u = output rows 2u and 2u+1 (tile 3: row 6 and, again, row 5);
    // lanes 14 and 15 repeat lane 13's pixel
    int rb[4], oofs[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int jj = min(j, 13), r = jj >= 7 ? 1 : 0, ox = jj - 7 * r;
        const int oy = (u < 3 ? 2 * u : 5) + r;
        rb[u] = g * TL_PLANE + (oy * 9 + ox) * 16;
        const int px = oy * 7 + ox;
        oofs[u] = p.out_frag ? px * 1024 + g * 256 + 8 * h : px * TL_PIX_BYTES + 16 * g + 8 * h;
    }

    // step q = 9 * tile + tap; pixel fragments rotate through eight slots (fragment q + 8 is requested as soon
    // as step q has consumed its slot)
    auto frag = [&](const char* src, int q) {
        const int u = q / 9, st = q - 9 * u;
        return *(const v4i*)(src + rb[u] + ((st / 3) * 9 + (st % 3)) * 16);
    };
    auto store = [&](int8_t* outp, int u, const v4i (&acc)[2]) {
        const uint32_t w0 = requant_relu4_p23<P23>(acc[0], m0, c0), w1 = requant_relu4_p23<P23>(acc[1], m1, c1);
        *(v2i*)(outp + oofs[u]) = (v2i){(int)w0, (int)w1};
    };
    auto compute = [&](const char* src, int8_t* outp) {
        v4i gq[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) gq[q] = frag(src, q);
        v4i accO[2] = {bi0, bi1};
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            v4i accN[2];
#pragma unroll
            for (int st = 0; st < 9; ++st) {
                const int q = u * 9 + st;
                accN[0] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w[st][0], gq[q & 7], st == 0 ? bi0 : accN[0], 0, 0, 0);
                accN[1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w[st][1], gq[q & 7], st == 0 ? bi1 : accN[1], 0, 0, 0);
                if (q + 8 < 36) gq[q & 7] = frag(src, q + 8);
            }
            if (u > 0) store(outp, u - 1, accO);
            accO[0] = accN[0]; accO[1] = accN[1];
            if (u > 0) {
#pragma unroll
                for (int k = 0; k < 9; ++k) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
                    if (u * 9 + k + 8 < 36) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, P23 ? 3 : 4, 0);
                }
                __builtin_amdgcn_sched_group_barrier(0x040, 1, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        store(outp, 3, accO);
    };
    auto out_of = [&](int64_t im) -> int8_t* {
        return p.out_frag ? p.out + (im >> 4) * ((int64_t)p.frag_ks << 10) + (((int)im & 15) << 4)
                          : p.out + im * (int64_t)(TL_NPIX * TL_PIX_BYTES);
    };

    if (img < p.B) stage_commit(tiles);
    if (img + stride < p.B) stage_load(img + stride);
    __syncthreads();
    for (int n = 0;; ++n, img += stride) {
        // the bytes of image n+1 go to the idle copy, image n+2 is requested, image n is multiplied
        if (img + stride < p.B) stage_commit(tiles + ((n + 1) & 1) * TL_COPY);
        if (img + 2 * stride < p.B) stage_load(img + 2 * stride);
        if (img < p.B) compute(tiles + (n & 1) * TL_COPY, out_of(img));
        if (!(img_first + (n + 1) * stride < p.B)) break;
        __syncthreads();
    }
}
}  // namespace

// Exactly the third layer of the paper's original network as the planner describes it.
bool conv_tail_supported(const ConvParams& p, int NT) {
    if (p.src_u8 || p.mode != CM_FLAT || p.H != 9 || p.W != 9 || p.Cs_in != 64 || p.Cin_real != 64) return false;
    if (p.k != 3 || p.s != 1 || p.sx != 1 || p.pad != 0 || p.Ho != 7 || p.Wo != 7 || p.Cs_out != 64 || NT != 4) return false;
    if (p.k_steps != 9 || p.cpr != 12 || !p.relu || p.relu_in || p.pool || p.res || p.tap_acc) return false;
    if (p.out_frag && p.frag_ks != 49) return false;
    return true;
}

template <bool P23>
static hipError_t tail_go(const TailParams& p, hipStream_t s) {
    static int occ = 0;
    if (!occ) {
        hipError_t e = hipFuncSetAttribute((const void*)conv_tail_kernel<P23>, hipFuncAttributeMaxDynamicSharedMemorySize, TL_LDS);
        if (e != hipSuccess) return e;
        int o = 0;
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&o, (const void*)conv_tail_kernel<P23>, TL_THREADS, TL_LDS);
        if (e != hipSuccess) return e;
        occ = o < 1 ? 1 : o;
    }
    // resident workgroups striding over groups of TL_SLOTS images, in even rounds
    const int64_t groups = (p.B + TL_SLOTS - 1) / TL_SLOTS;
    const int64_t cap = (int64_t)occ * conv_num_cus();
    const int64_t rounds = (groups + cap - 1) / cap;
    dim3 grid((unsigned)((groups + rounds - 1) / rounds));
    conv_tail_kernel<P23><<<grid, dim3(TL_THREADS), TL_LDS, s>>>(p);
    return hipGetLastError();
}

hipError_t launch_conv_tail(const ConvParams& c, hipStream_t s) {
    if (c.B <= 0) return hipSuccess;
    TailParams p;
    p.in = (const int8_t*)c.in; p.out = (int8_t*)c.out;
    p.w = (const v4i*)c.wfrag; p.bias = (const int*)c.bias; p.mult = c.mult;
    p.B = c.B; p.out_frag = c.out_frag; p.frag_ks = c.frag_ks;
    static const bool no_p23 = getenv("ACCERL_NO_P23") != nullptr;
    return (c.pos23 && !no_p23) ? tail_go<true>(p, s) : tail_go<false>(p, s);
}

}  // namespace accerl
