// Large-batch int8 dense layer with requantizing epilogue, out[b, n] = requant(bias[n] + sum_k W[n, k] x[b, k]),
// as a streaming pipeline.  The tiling is gemm_kernel's (a workgroup owns 64 features and 16 states per wavefront;
// weight fragments are shared through LDS, a wavefront's state fragments come straight from memory), but
// measured per stage of four MFMA steps the generic kernel spends about as long
// issuing its burst of eight loads into a full memory pipeline and then waiting for them as it spends on
// the MFMAs.  Here
//   * every load is requested two stages before its use: the state fragments of stage s+2 go into the registers
//     that step st of stage s has just consumed, the weight fragments of stage s+3 into the registers whose
//     contents went to LDS at the top of stage s;
//   * the loads are spread between the MFMAs of the stage, two after every four MFMAs, instead of one burst;
//   * LDS holds two stages of weight fragments, so one barrier per stage suffices.
// Rows are whole MFMA steps here (Kp_bytes == 64 * k_steps, no ReLU on the input), which leaves no fix-ups in
// the loop; other shapes stay with gemm_kernel.  Integer accumulation: results are bit-identical.
#include <type_traits>

#include "accerl_internal.h"

namespace accerl {

int conv_num_cus();   // compute units of the current device

namespace {
constexpr int SG_KS = 4;                           // MFMA steps per stage
constexpr int SG_NT = 4;                           // feature tiles per workgroup (one per wavefront to fetch)
constexpr int SG_BUF = SG_NT * SG_KS * 1024;       // one stage of weight fragments: [tile][step][64 lanes][16 B]
constexpr int SG_LDS = 2 * SG_BUF;

// WAVES wavefronts of 16 states each: eight when that still gives every compute unit a workgroup (the weight
// fragments are then fetched and written to LDS once per 128 states), else four
template <int WAVES>
__global__ __launch_bounds__(64 * WAVES, 2) void gemm_stream_i8_kernel(const GemmParams p) {
    constexpr int SG_ROWS = 16 * WAVES;
    constexpr int SG_WF = SG_NT * SG_KS / WAVES;    // weight fragments a wavefront fetches per stage
    extern __shared__ __attribute__((aligned(16))) char sg_smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 15, g = lane >> 4;
    const int64_t b0 = (int64_t)blockIdx.x * SG_ROWS;
    const int nt0 = blockIdx.y * SG_NT;
    const int ks = p.k_steps;

    // a state past the batch re-reads the last one; its results are not stored
    int64_t xrow = b0 + wave * 16 + j;
    if (xrow >= p.B) xrow = p.B - 1;
    const char* xb;
    int xstep;
    if (p.x_frag) { xb = (const char*)p.x + (xrow >> 4) * ((int64_t)ks << 10) + lane * 16; xstep = 1024; }
    else { xb = (const char*)p.x + xrow * p.Kp_bytes + g * 16; xstep = 64; }
    // this wavefront fetches fragments wave * SG_WF ... of the stage's [tile][step] grid for all wavefronts
    const int wstep0 = (wave * SG_WF) % SG_KS;
    const char* wb = (const char*)p.wfrag + (int64_t)(nt0 + (wave * SG_WF) / SG_KS) * ks * 1024 + lane * 16;
    char* wdst = sg_smem + wave * SG_WF * 1024 + lane * 16;
    const char* wsrc = sg_smem + lane * 16;

    v4i acc[SG_NT];
#pragma unroll
    for (int t = 0; t < SG_NT; ++t) acc[t] = *(const v4i*)((const int*)p.bias + (nt0 + t) * 16 + 4 * g);

    // steps past the end of K load the last step again (never multiplied)
    auto load_x = [&](v4i& d, int step) { d = *(const v4i*)(xb + (int64_t)min(step, ks - 1) * xstep); };
    auto load_w = [&](v4i& d, int step) { d = *(const v4i*)(wb + (int64_t)min(step + wstep0, ks - 1) * 1024); };
    auto commit = [&](const v4i (&w)[SG_WF], int buf) {
#pragma unroll
        for (int r = 0; r < SG_WF; ++r) *(v4i*)(wdst + buf * SG_BUF + r * 1024) = w[r];
    };

    v4i xs[2][SG_KS], ws[2][SG_WF];
#pragma unroll
    for (int r = 0; r < SG_WF; ++r) load_w(ws[0][r], r);
#pragma unroll
    for (int r = 0; r < SG_KS; ++r) load_x(xs[0][r], r);
#pragma unroll
    for (int r = 0; r < SG_WF; ++r) load_w(ws[1][r], SG_KS + r);
#pragma unroll
    for (int r = 0; r < SG_KS; ++r) load_x(xs[1][r], SG_KS + r);
    commit(ws[0], 0);
#pragma unroll
    for (int r = 0; r < SG_WF; ++r) load_w(ws[0][r], 2 * SG_KS + r);
    __syncthreads();

    // stage s multiplies from LDS buffer s & 1 and the state registers xs[s & 1]; the weights of stage s+1 go
    // from ws[(s+1) & 1] to the other buffer first.  A full stage has no conditions at all (loads past the end
    // of K are clamped, the fragments they bring are never multiplied); the last, partial stage only multiplies.
    auto stage = [&](int s, auto CUR, auto FULL) {
        constexpr int cur = decltype(CUR)::value, nxt = cur ^ 1;
        constexpr bool full = decltype(FULL)::value;
        if (full) commit(ws[nxt], nxt);
        const char* src = wsrc + cur * SG_BUF;
        v4i fa[2][SG_NT];
#pragma unroll
        for (int t = 0; t < SG_NT; ++t) fa[0][t] = *(const v4i*)(src + (t * SG_KS) * 1024);
        if (full) {
            __builtin_amdgcn_sched_group_barrier(0x200, SG_WF, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, SG_NT, 0);
        }
#pragma unroll
        for (int st = 0; st < SG_KS; ++st) {
            if (st + 1 < SG_KS) {
#pragma unroll
                for (int t = 0; t < SG_NT; ++t) fa[(st + 1) & 1][t] = *(const v4i*)(src + (t * SG_KS + st + 1) * 1024);
            }
            if (full || s * SG_KS + st < ks) {
#pragma unroll
                for (int t = 0; t < SG_NT; ++t)
                    acc[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fa[st & 1][t], xs[cur][st], acc[t], 0, 0, 0);
            }
            if (full) {
                load_x(xs[cur][st], (s + 2) * SG_KS + st);
                if (st < SG_WF) load_w(ws[nxt][st], (s + 3) * SG_KS + st);
                // keep this order in the instruction stream: the LDS reads of the next step, this step's MFMAs, two loads
                if (st + 1 < SG_KS) __builtin_amdgcn_sched_group_barrier(0x100, SG_NT, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, SG_NT, 0);
                if (st < SG_WF) __builtin_amdgcn_sched_group_barrier(0x020, 2, 0);
                else __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
            }
        }
        if (full) __syncthreads();
    };
    using std::true_type; using std::false_type;
    typedef std::integral_constant<int, 0> even; typedef std::integral_constant<int, 1> odd;
    const int n_full = ks / SG_KS;
    int s = 0;
    for (; s + 2 <= n_full; s += 2) {
        stage(s, even(), true_type());
        stage(s + 1, odd(), true_type());
    }
    if (s < n_full) {
        stage(s, even(), true_type());
        if (ks % SG_KS) stage(s + 1, odd(), false_type());
    } else if (ks % SG_KS) {
        stage(s, even(), false_type());
    }

    // ---- epilogue: lane holds features n0 .. n0+3 of state b
    const int64_t b = b0 + wave * 16 + j;
    if (b >= p.B) return;
#pragma unroll
    for (int t = 0; t < SG_NT; ++t) {
        const int n0 = (nt0 + t) * 16 + 4 * g;
        if (n0 >= p.Np) continue;      // stored rows reach the row pitch (zero weights and bias give zeros)
        const v4f ml = *(const v4f*)(p.mult + n0);
        uint32_t pk = 0;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int v = acc[t][r];
            if (p.tap_acc && n0 + r < p.N) p.tap_acc[b * p.N + n0 + r] = v;
            if (p.relu) {   // clamp(rint(y), 0, 127): the pack instruction rounds to nearest even, saturates at 0
                pk = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_amdgcn_fmed3f((float)v * ml[r], 0.0f, 127.0f), r, pk);
            } else {
                const float y = __builtin_amdgcn_fmed3f(rintf((float)v * ml[r]), -127.0f, 127.0f);
                pk |= ((uint32_t)(int)y & 0xffu) << (8 * r);
            }
        }
        *(uint32_t*)((int8_t*)p.out + b * p.Np + n0) = pk;
    }
}
}  // namespace

bool gemm_stream_supported(const GemmParams& p) {
    return p.B > 0 && !p.relu_in && p.k_steps >= 2 * SG_KS && p.Kp_bytes == 64 * p.k_steps && p.n_tiles % SG_NT == 0;
}

hipError_t launch_gemm_stream(const GemmParams& p, hipStream_t s) {
    static bool set = false;
    if (!set) {
        hipError_t e = hipFuncSetAttribute((const void*)gemm_stream_i8_kernel<4>, hipFuncAttributeMaxDynamicSharedMemorySize, SG_LDS);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute((const void*)gemm_stream_i8_kernel<8>, hipFuncAttributeMaxDynamicSharedMemorySize, SG_LDS);
        if (e != hipSuccess) return e;
        set = true;
    }
    const unsigned gy = (unsigned)(p.n_tiles / SG_NT);
    const int64_t g8 = (p.B + 127) / 128, g4 = (p.B + 63) / 64;
    if (g8 * gy >= conv_num_cus()) gemm_stream_i8_kernel<8><<<dim3((unsigned)g8, gy), dim3(512), SG_LDS, s>>>(p);
    else gemm_stream_i8_kernel<4><<<dim3((unsigned)g4, gy), dim3(256), SG_LDS, s>>>(p);
    return hipGetLastError();
}

}  // namespace accerl
