// Monitor indicators and V-trace correction: the two consumers of the actor's behaviour logits.
// Both are row-wise passes over [rows, A] logit tables of the original and the smaller policy and are
// bound by HBM traffic: a wavefront copies 64 consecutive rows of both tables into LDS with coalesced
// 16-byte loads and every lane then works on its own row out of LDS.
#include <cstdio>
#include <mutex>

#include "accerl_internal.h"

namespace accerl {

constexpr int MON_AMAX = 64;        // most actions
constexpr int MON_PARTS = 2048;     // most workgroups of a reduction pass
constexpr int MON_NSTAT = 5;        // partial sums per workgroup: KL, KL^2, max KL, entropy, distillation loss

// 64 rows of `tab` starting at row r0 -> LDS (row pitch A floats).  The tile starts 256*A bytes into the
// table, so 16-byte loads are aligned whenever the table is.
__device__ __forceinline__ void stage_rows(const float* __restrict__ tab, int64_t r0, int nrows, int A, float* sm, int lane) {
    const float* src = tab + r0 * A;
    const int n = nrows * A, n4 = n >> 2;
    for (int i = lane; i < n4; i += 64) ((v4f*)sm)[i] = ((const v4f*)src)[i];
    for (int i = (n4 << 2) + lane; i < n; i += 64) sm[i] = src[i];
}

__device__ __forceinline__ void wave_sync_lds() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Row arithmetic.  With m = max_a l_a, d_a = l_a - m, e_a = exp(d_a), Z = sum_a e_a the softmax is p_a = e_a / Z and
// log p_a = d_a - log Z, so that (o = original, s = smaller policy)
//     KL(o || s) = sum_a p_o,a (log p_o,a - log p_s,a) = (sum_a e_o,a (d_o,a - d_s,a)) / Z_o - log Z_o + log Z_s
//     H(s)       = -sum_a p_s,a log p_s,a              = log Z_s - (sum_a e_s,a d_s,a) / Z_s
// two exponentials per action instead of one per probability and one per normaliser.  Identical rows give d_o = d_s and
// Z_o = Z_s bit for bit, hence KL = 0 exactly.  The exponential is the hardware's 2^x on x log2(e) (d lies in [-large, 0]:
// about 1e-6 relative error over the range the logits span), the logarithm its log2 -- well inside the 2e-4 relative
// that per-row values are held to against an fp64 evaluation.
// Lane l walks its row in LDS starting at element `rot` = l mod A, so that the lanes of a wavefront (rows A floats
// apart) do not all hit the same LDS bank when A is a multiple of 16.
__device__ __forceinline__ float fast_exp(float x) { return __builtin_amdgcn_exp2f(x * 1.44269504088896341f); }
__device__ __forceinline__ float fast_log(float x) { return __builtin_amdgcn_logf(x) * 0.693147180559945309f; }

__device__ __forceinline__ float row_max(const float* row, int A, int rot) {
    float m = row[rot];
    for (int a = 1; a < A; ++a) { int k = a + rot; k -= (k >= A) ? A : 0; m = fmaxf(m, row[k]); }
    return m;
}

// KL(o || s) and H(s) of one pair of rows
__device__ __forceinline__ void row_kl_entropy(const float* ro, const float* rs, int A, int rot, float& kl, float& h) {
    const float mo = row_max(ro, A, rot), ms = row_max(rs, A, rot);
    float zo = 0.0f, zs = 0.0f, so = 0.0f, ss = 0.0f;
    for (int a = 0; a < A; ++a) {
        int k = a + rot;
        k -= (k >= A) ? A : 0;
        const float d_o = ro[k] - mo, d_s = rs[k] - ms;
        const float eo = fast_exp(d_o), es = fast_exp(d_s);
        zo += eo; zs += es;
        so += eo * (d_o - d_s);
        ss += es * d_s;
    }
    const float lzo = fast_log(zo), lzs = fast_log(zs);
    kl = so / zo - lzo + lzs;
    h = lzs - ss / zs;
}

// log of the normaliser of one row: log p_a = (l_a - m) - lz
__device__ __forceinline__ void row_norm(const float* row, int A, int rot, float& m, float& lz) {
    m = row_max(row, A, rot);
    float Z = 0.0f;
    for (int a = 0; a < A; ++a) { int k = a + rot; k -= (k >= A) ? A : 0; Z += fast_exp(row[k] - m); }
    lz = fast_log(Z);
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
    return v;
}
__device__ __forceinline__ double wave_max(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmax(v, __shfl_down(v, o, 64));
    return v;
}

// ---- KL(original || smaller) and entropy of the smaller policy per state; per-workgroup partial sums.
// Four wavefronts per workgroup, each walking its own tiles with its own LDS region.
constexpr int MON_WAVES = 4;
__global__ __launch_bounds__(MON_WAVES * 64) void kl_rows_kernel(const float* __restrict__ lo, const float* __restrict__ ls, int64_t B, int A,
                                                                 float* __restrict__ out_kl, float* __restrict__ out_ent, double* __restrict__ parts,
                                                                 const float* __restrict__ v_o, const float* __restrict__ v_s, float beta,
                                                                 float* __restrict__ out_loss) {
    extern __shared__ __attribute__((aligned(16))) float mon_sm[];
    __shared__ double red[MON_WAVES][5];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float* so = mon_sm + wave * 128 * A;
    float* ss = so + 64 * A;
    double s_kl = 0.0, s_sq = 0.0, s_mx = -1.0, s_h = 0.0, s_loss = 0.0;
    const int64_t n_tiles = (B + 63) >> 6;
    for (int64_t tile = (int64_t)blockIdx.x * MON_WAVES + wave; tile < n_tiles; tile += (int64_t)gridDim.x * MON_WAVES) {
        const int64_t r0 = tile << 6;
        const int nrows = (int)((B - r0 < 64) ? (B - r0) : 64);
        stage_rows(lo, r0, nrows, A, so, lane);
        stage_rows(ls, r0, nrows, A, ss, lane);
        wave_sync_lds();
        if (lane < nrows) {
            const float* ro = so + lane * A;
            const float* rs = ss + lane * A;
            const int rot = lane % A;
            float kl, h;
            row_kl_entropy(ro, rs, A, rot, kl, h);
            if (out_kl) out_kl[r0 + lane] = kl;
            if (out_ent) out_ent[r0 + lane] = h;
            s_kl += (double)kl;
            s_sq += (double)kl * (double)kl;
            s_mx = fmax(s_mx, (double)kl);
            s_h += (double)h;
            if (v_o) {   // distillation loss of the state: KL + (v_original - v_smaller)^2 / 2 - beta H
                const float dv = v_o[r0 + lane] - v_s[r0 + lane];
                const float loss = kl + 0.5f * (dv * dv) - beta * h;
                if (out_loss) out_loss[r0 + lane] = loss;
                s_loss += (double)loss;
            }
        }
        wave_sync_lds();   // rows are read before the next tile overwrites them
    }
    s_kl = wave_sum(s_kl); s_sq = wave_sum(s_sq); s_h = wave_sum(s_h); s_mx = wave_max(s_mx); s_loss = wave_sum(s_loss);
    if (lane == 0) { red[wave][0] = s_kl; red[wave][1] = s_sq; red[wave][2] = s_mx; red[wave][3] = s_h; red[wave][4] = s_loss; }
    __syncthreads();
    if (threadIdx.x == 0) {
        double* p = parts + MON_NSTAT * (int64_t)blockIdx.x;
        double a0 = red[0][0], a1 = red[0][1], a2 = red[0][2], a3 = red[0][3], a4 = red[0][4];
        for (int w = 1; w < MON_WAVES; ++w) { a0 += red[w][0]; a1 += red[w][1]; a2 = fmax(a2, red[w][2]); a3 += red[w][3]; a4 += red[w][4]; }
        p[0] = a0; p[1] = a1; p[2] = a2; p[3] = a3; p[4] = a4;
    }
}

// one wavefront folds the partials in a fixed order: stats = {mean, max, population variance, entropy mean}
// (monitor) or the mean distillation loss alone (loss_only)
__global__ __launch_bounds__(64) void kl_stats_kernel(const double* __restrict__ parts, int n_parts, int64_t B, double* __restrict__ stats, int loss_only) {
    const int lane = threadIdx.x;
    double s_kl = 0.0, s_sq = 0.0, s_mx = -1.0, s_h = 0.0, s_loss = 0.0;
    for (int i = lane; i < n_parts; i += 64) {
        const double* p = parts + MON_NSTAT * i;
        s_kl += p[0]; s_sq += p[1]; s_mx = fmax(s_mx, p[2]); s_h += p[3]; s_loss += p[4];
    }
    s_kl = wave_sum(s_kl); s_sq = wave_sum(s_sq); s_h = wave_sum(s_h); s_mx = wave_max(s_mx); s_loss = wave_sum(s_loss);
    if (lane == 0) {
        const double n = (double)B, mean = s_kl / n;
        if (loss_only) {
            stats[0] = s_loss / n;
        } else {
            stats[0] = mean;
            stats[1] = s_mx;
            stats[2] = fmax(s_sq / n - mean * mean, 0.0);
            stats[3] = s_h / n;
        }
    }
}

// ---- importance ratio pi_original(a|x) / pi_smaller(a|x) of the action taken, one row per (t, b)
__global__ __launch_bounds__(MON_WAVES * 64) void is_ratio_kernel(const float* __restrict__ lo, const float* __restrict__ ls, const int32_t* __restrict__ act,
                                                                  int64_t R, int A, float* __restrict__ ratio) {
    extern __shared__ __attribute__((aligned(16))) float mon_sm[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float* so = mon_sm + wave * 128 * A;
    float* ss = so + 64 * A;
    const int64_t n_tiles = (R + 63) >> 6;
    for (int64_t tile = (int64_t)blockIdx.x * MON_WAVES + wave; tile < n_tiles; tile += (int64_t)gridDim.x * MON_WAVES) {
        const int64_t r0 = tile << 6;
        const int nrows = (int)((R - r0 < 64) ? (R - r0) : 64);
        stage_rows(lo, r0, nrows, A, so, lane);
        stage_rows(ls, r0, nrows, A, ss, lane);
        wave_sync_lds();
        if (lane < nrows) {
            const float* ro = so + lane * A;
            const float* rs = ss + lane * A;
            const int rot = lane % A;
            float mo, lzo, ms, lzs;
            row_norm(ro, A, rot, mo, lzo);
            row_norm(rs, A, rot, ms, lzs);
            int a = act[r0 + lane];
            a = min(max(a, 0), A - 1);
            ratio[r0 + lane] = fast_exp((ro[a] - mo - lzo) - (rs[a] - ms - lzs));
        }
        wave_sync_lds();
    }
}

// ---- backward scan per environment: v_s - V(x_s) = delta_s + gamma_s c_s (v_{s+1} - V(x_{s+1}))
// A scan with one lane per environment leaves the chip nearly empty (B / 64 wavefronts walking T dependent steps).  The
// recurrence a_t = delta_t + k_t a_{t+1} (k_t = gamma_t c_t) is linear, so a run of steps [t0, t1) acts on the value
// entering it as a_t0 = A + M a_t1 with A, M computed from that run alone.  A workgroup takes 64 environments; its
// wavefronts split the last (up to) NSEG * L steps into runs of L steps held in registers: each forms its (A, M) with one
// backward pass, the pairs meet in LDS, every wavefront folds the pairs of the runs behind it into the value entering
// its run and walks its registers a second time to write v_s, the clipped weights and the advantages.  Longer unrolls
// repeat this from the end of the trajectory towards its start, carrying a_t across.  delta_t needs V(x_{t+1}) only,
// which is an input.  The order of the floating-point operations is fixed by (T, L), not by the launch.
constexpr int VT_NSEG = 16;
template <int L>
__global__ __launch_bounds__(VT_NSEG * 64) void vtrace_scan_kernel(const float* __restrict__ rewards, const float* __restrict__ discounts,
                                                                   const float* __restrict__ values, const float* __restrict__ bootstrap,
                                                                   int64_t T, int64_t B, float rho_bar, float c_bar,
                                                                   float* __restrict__ rho /* in: ratio, out: clipped */,
                                                                   float* __restrict__ vs, float* __restrict__ pg_adv) {
    __shared__ float sA[VT_NSEG][64], sM[VT_NSEG][64];
    __shared__ float s_carry[64];
    const int lane = threadIdx.x & 63, seg = threadIdx.x >> 6;
    const int nseg = blockDim.x >> 6;
    const int64_t b = (int64_t)blockIdx.x * 64 + lane;
    const int64_t bc = b < B ? b : B - 1;                  // lanes past the batch repeat the last environment, store nothing
    if (seg == 0) s_carry[lane] = 0.0f;                    // a_T = v_T - V(x_T) = 0
    for (int64_t hi = T; hi > 0; hi -= (int64_t)nseg * L) {
        // this wavefront's run: steps [t0, t1) with t1 = hi - seg * L; runs past the start of the trajectory are empty
        const int64_t t1 = hi - (int64_t)seg * L;
        const int n = (int)(t1 <= 0 ? 0 : (t1 < L ? t1 : L));
        const int64_t t0 = t1 - n;
        float rh[L], kk[L], dl[L], vv[L], rw[L], gg[L];
        float v_after = 0.0f;                              // V(x_t1)
        if (n > 0) v_after = (t1 == T) ? bootstrap[bc] : values[t1 * B + bc];
#pragma unroll
        for (int i = 0; i < L; ++i) {                      // i counts back from the end of the run
            const int64_t t = t1 - 1 - i;
            const int64_t idx = (t >= 0 ? t : 0) * B + bc;
            rh[i] = rho[idx]; rw[i] = rewards[idx]; gg[i] = discounts[idx]; vv[i] = values[idx];
        }
        float A = 0.0f, M = 1.0f;
        {
            float v_next = v_after;
#pragma unroll
            for (int i = 0; i < L; ++i) {
                const float ratio = rh[i];
                const float r_c = fminf(rho_bar, ratio), c_c = fminf(c_bar, ratio);
                rh[i] = r_c;
                kk[i] = gg[i] * c_c;
                dl[i] = r_c * (rw[i] + gg[i] * v_next - vv[i]);
                if (i < n) { A = dl[i] + kk[i] * A; M = kk[i] * M; }
                v_next = vv[i];
            }
        }
        sA[seg][lane] = A;
        sM[seg][lane] = M;
        __syncthreads();
        // the value entering this run: the carry from beyond `hi`, pushed through the runs behind this one (lower seg)
        float acc = s_carry[lane];
        for (int k = 0; k < seg; ++k) acc = sA[k][lane] + sM[k][lane] * acc;
        {
            float vs_next = v_after + acc;                 // v_{t1}
#pragma unroll
            for (int i = 0; i < L; ++i) {
                if (i < n) {
                    const int64_t idx = (t1 - 1 - i) * B + b;
                    acc = dl[i] + kk[i] * acc;
                    const float vs_t = vv[i] + acc;
                    if (b < B) {
                        if (pg_adv) pg_adv[idx] = rh[i] * (rw[i] + gg[i] * vs_next - vv[i]);
                        vs[idx] = vs_t;
                        rho[idx] = rh[i];
                    }
                    vs_next = vs_t;
                }
            }
        }
        __syncthreads();                                    // every wavefront has read the pairs and the carry
        if (seg == nseg - 1) s_carry[lane] = acc;           // the run that reaches furthest back hands a_t0 on
        (void)t0;
        __syncthreads();
    }
}

static double* mon_parts(int dev) {
    static double* parts[64] = {nullptr};
    if (dev < 0 || dev >= 64) return nullptr;
    if (!parts[dev] && hipMalloc((void**)&parts[dev], (size_t)MON_PARTS * MON_NSTAT * sizeof(double)) != hipSuccess) {
        (void)hipGetLastError();
        parts[dev] = nullptr;
    }
    return parts[dev];
}

// Partial sums of the entry point that allocates nothing: a fixed array in the library's device image (every GPU the
// library runs on holds its own copy for the life of the process).  Host code never passes the array's name to a kernel
// or a copy: its device address on the current GPU is looked up once per device and kept.
constexpr int MON_STATIC_PARTS = 1024;                       // workgroups of a pass over the static array
constexpr int64_t MON_STATIC_MAX_ROWS = (int64_t)1 << 24;    // most rows per call of that entry point
static __device__ __align__(256) __attribute__((used)) double scratch[MON_STATIC_PARTS * MON_NSTAT];

static double* scratch_address(int dev, hipError_t* err) {
    static std::mutex mu;
    static double* ptr[64] = {nullptr};
    *err = hipSuccess;
    if (dev < 0 || dev >= 64) { *err = hipErrorInvalidDevice; return nullptr; }
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void* p = nullptr;
        *err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));   // the address on the device that is current now
        if (*err != hipSuccess) { (void)hipGetLastError(); return nullptr; }
        ptr[dev] = (double*)p;
    }
    return ptr[dev];
}

static int hip_fail(const char* what, hipError_t e) {
    char buf[256];
    snprintf(buf, sizeof buf, "%s: %s", what, hipGetErrorString(e));
    return set_error(ACCERL_EHIP, buf);
}

static int raise_lds(const void* fn, size_t lds) {
    if (lds <= 48 * 1024) return ACCERL_OK;
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    return e == hipSuccess ? ACCERL_OK : hip_fail("hipFuncSetAttribute", e);
}

}  // namespace accerl

using namespace accerl;

static int run_kl(const char* who, const float* logits_original, const float* logits_smaller, const float* v_o, const float* v_s,
                  float beta, int64_t B, int A, float* out_kl, float* out_entropy, float* out_loss, double* out_stats,
                  int loss_only, void* hip_stream, bool static_parts = false) {
    char msg[160];
    if (B < 0 || A < 1 || A > MON_AMAX) { snprintf(msg, sizeof msg, "%s: need B >= 0 and 1 <= A <= 64", who); return set_error(ACCERL_EINVAL, msg); }
    if (B == 0) return ACCERL_OK;
    if (!logits_original || !logits_smaller || !out_stats || (loss_only && (!v_o || !v_s))) {
        snprintf(msg, sizeof msg, "%s: NULL input or result pointer", who);
        return set_error(ACCERL_EINVAL, msg);
    }
    if (((uintptr_t)logits_original | (uintptr_t)logits_smaller) & 15) { snprintf(msg, sizeof msg, "%s: logits must be 16-byte aligned", who); return set_error(ACCERL_EINVAL, msg); }
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail("hipGetDevice", e);
    double* parts = nullptr;
    int max_parts = MON_PARTS;
    if (static_parts) {
        if (B > MON_STATIC_MAX_ROWS) {
            snprintf(msg, sizeof msg, "%s: %lld rows exceed the %lld this entry point takes per call (split the batch)", who,
                     (long long)B, (long long)MON_STATIC_MAX_ROWS);
            return set_error(ACCERL_EINVAL, msg);
        }
        parts = scratch_address(dev, &e);
        if (!parts) return hip_fail("hipGetSymbolAddress(scratch)", e);
        max_parts = MON_STATIC_PARTS;
    } else {
        parts = mon_parts(dev);
        if (!parts) return set_error(ACCERL_ENOMEM, "partial-sum buffer");
    }
    hipStream_t s = (hipStream_t)hip_stream;
    const int64_t n_tiles = (B + 63) / 64;
    const int64_t want = (n_tiles + MON_WAVES - 1) / MON_WAVES;
    const int blocks = (int)(want < max_parts ? want : max_parts);
    const size_t lds = (size_t)MON_WAVES * 2 * 64 * A * sizeof(float);
    if (int rc = raise_lds((const void*)kl_rows_kernel, lds)) return rc;
    kl_rows_kernel<<<dim3(blocks), dim3(MON_WAVES * 64), lds, s>>>(logits_original, logits_smaller, B, A, out_kl, out_entropy, parts,
                                                                  v_o, v_s, beta, out_loss);
    if ((e = hipGetLastError()) != hipSuccess) return hip_fail("kl_rows_kernel", e);
    kl_stats_kernel<<<dim3(1), dim3(64), 0, s>>>(parts, blocks, B, out_stats, loss_only);
    if ((e = hipGetLastError()) != hipSuccess) return hip_fail("kl_stats_kernel", e);
    return ACCERL_OK;
}

extern "C" int accerl_monitor_kl(const float* logits_original, const float* logits_smaller, int64_t B, int A,
                                 float* out_kl, float* out_entropy, double* out_stats, void* hip_stream) {
    return run_kl("monitor", logits_original, logits_smaller, nullptr, nullptr, 0.0f, B, A, out_kl, out_entropy, nullptr, out_stats, 0, hip_stream);
}

// Every workgroup of the row pass writes its whole record and the fold reads exactly the records of that pass, so the
// array needs no clearing between calls, whatever the call before it left there.
extern "C" int accerl_monitor_kl_noalloc(const float* logits_original, const float* logits_smaller, int64_t B, int A,
                                         float* out_kl, float* out_entropy, double* out_stats, void* hip_stream) {
    return run_kl("monitor (no allocation)", logits_original, logits_smaller, nullptr, nullptr, 0.0f, B, A, out_kl, out_entropy, nullptr,
                  out_stats, 0, hip_stream, true);
}

extern "C" int accerl_distill_loss(const float* logits_original, const float* logits_smaller, const float* value_original,
                                   const float* value_smaller, int64_t B, int A, float beta, float* out_loss, double* out_mean,
                                   void* hip_stream) {
    return run_kl("distill", logits_original, logits_smaller, value_original, value_smaller, beta, B, A, nullptr, nullptr, out_loss, out_mean, 1, hip_stream);
}

extern "C" int accerl_vtrace(const float* logits_original, const float* logits_smaller, const int32_t* actions,
                             const float* rewards, const float* discounts, const float* values, const float* bootstrap,
                             int64_t T, int64_t B, int A, float rho_bar, float c_bar,
                             float* out_vs, float* out_pg_adv, float* out_rho, void* hip_stream) {
    if (T < 0 || B < 0 || A < 1 || A > MON_AMAX) return set_error(ACCERL_EINVAL, "vtrace: need T, B >= 0 and 1 <= A <= 64");
    if (!(rho_bar >= 0.0f) || !(c_bar >= 0.0f)) return set_error(ACCERL_EINVAL, "vtrace: rho_bar and c_bar must be >= 0");
    if (T == 0 || B == 0) return ACCERL_OK;
    if (!logits_original || !logits_smaller || !actions || !rewards || !discounts || !values || !bootstrap || !out_vs || !out_rho)
        return set_error(ACCERL_EINVAL, "vtrace: NULL argument (only out_pg_adv may be NULL)");
    if (((uintptr_t)logits_original | (uintptr_t)logits_smaller) & 15) return set_error(ACCERL_EINVAL, "vtrace: logits must be 16-byte aligned");
    hipStream_t s = (hipStream_t)hip_stream;
    const int64_t R = T * B, n_tiles = (R + 63) / 64;
    const int64_t want = (n_tiles + MON_WAVES - 1) / MON_WAVES;
    const int blocks = (int)(want < 2048 ? want : 2048);
    const size_t lds = (size_t)MON_WAVES * 2 * 64 * A * sizeof(float);
    if (int rc = raise_lds((const void*)is_ratio_kernel, lds)) return rc;
    is_ratio_kernel<<<dim3(blocks), dim3(MON_WAVES * 64), lds, s>>>(logits_original, logits_smaller, actions, R, A, out_rho);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail("is_ratio_kernel", e);
    // runs of 16 steps for long unrolls, of 4 for short ones; as many wavefronts per workgroup as there are runs (at most 16)
    const dim3 vgrid((unsigned)((B + 63) / 64));
    if (T > 32) {
        const int nseg = (int)((T + 15) / 16 < VT_NSEG ? (T + 15) / 16 : VT_NSEG);
        vtrace_scan_kernel<16><<<vgrid, dim3(nseg * 64), 0, s>>>(rewards, discounts, values, bootstrap, T, B, rho_bar, c_bar, out_rho, out_vs, out_pg_adv);
    } else {
        const int nseg = (int)((T + 3) / 4);
        vtrace_scan_kernel<4><<<vgrid, dim3(nseg * 64), 0, s>>>(rewards, discounts, values, bootstrap, T, B, rho_bar, c_bar, out_rho, out_vs, out_pg_adv);
    }
    if ((e = hipGetLastError()) != hipSuccess) return hip_fail("vtrace_scan_kernel", e);
    return ACCERL_OK;
}
