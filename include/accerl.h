/*
 * accerl.h -- C ABI of the MI355X actor-forward library.
 *
 * The one operation behind this boundary is the Actor's policy inference of the AcceRL paper
 * (Section 1: the agent maps each environment state s to an action a, and this step is the
 * bottleneck of data collection; Section 2.1: the Actors run the *compressed* policy; Section
 * 2.2, Eq. 1: the network yields an action distribution pi(.|s) and a value v(s)).  The
 * compressed ("student") policy is the post-training-quantized int8 network of Section 2.2
 * "Parameter Quantization" with the Conv+ReLU / FC+ReLU fusion described there, optionally of a
 * pruned or distilled shape (Section 2.2 "Structured Pruning", "Knowledge Distillation"); the
 * original ("teacher") policy in fp32 or bf16 sits alongside because the Corrector (Section 2.3,
 * Eq. 2: rho_t = min(rho, pi_original / pi_smaller)) and the Monitor (Section 2.4, Eq. 5) need
 * both distributions on the same states.  The behaviour logits are an output for the same reason.
 *
 * General rules
 *  - Every function returns an accerl_status (0 = OK, negative = error); nothing throws or
 *    aborts across this boundary.  accerl_last_error() gives a thread-local message.
 *  - "HOST" pointers are read during the call and never kept.  "DEVICE" pointers are HIP device
 *    memory owned by the caller, 16-byte aligned, valid until the work enqueued on `stream`
 *    has finished.  The library owns only its device copy of the weights and a per-policy
 *    workspace that it grows (hipMalloc, synchronising) when a call needs more than any
 *    earlier call did.
 *  - Forward calls only enqueue work on `stream` (a hipStream_t; NULL = the default stream) and
 *    return without synchronising; the status reports argument and launch errors only.
 *    B == 0 is valid and enqueues nothing.  One policy must not be used by two streams at once
 *    (the workspace is shared).
 *  - All tensors are dense and row-major in the logical order written below.
 */
#ifndef ACCERL_H
#define ACCERL_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct accerl_policy accerl_policy; /* opaque, library-owned */

typedef enum {
    ACCERL_OK = 0,
    ACCERL_EINVAL = -1,       /* NULL / mis-shaped / misaligned argument, inconsistent arch */
    ACCERL_ENOMEM = -2,       /* host or device allocation failed */
    ACCERL_EHIP = -3,         /* a HIP runtime call or kernel launch failed */
    ACCERL_EUNSUPPORTED = -4  /* valid request outside what the kernels cover */
} accerl_status;

typedef enum { ACCERL_OBS_U8 = 0, ACCERL_OBS_F32 = 1 } accerl_obs_dtype;

typedef enum {
    ACCERL_INT8 = 0, /* student: int8 weights and activations, int32 accumulation        */
    ACCERL_FP32 = 1, /* teacher: fp32 throughout                                           */
    ACCERL_BF16 = 2  /* teacher: bf16 operands and stored activations, fp32 accumulation  */
} accerl_precision;

typedef enum {
    ACCERL_CONV = 1,     /* cin cout k stride pad relu : square kernel, zero padding        */
    ACCERL_DENSE = 2,    /* cin cout relu                                                   */
    ACCERL_MAXPOOL = 3,  /* k stride pad : taps outside the image are ignored               */
    ACCERL_RESBLOCK = 4, /* cin == cout == channels : x + convB(relu(convA(relu(x)))), 3x3 pad 1 */
    ACCERL_RELU = 5,
    ACCERL_FLATTEN = 6,  /* C,H,W order                                                     */
    ACCERL_LSTM = 7      /* cin = input width, cout = hidden units; gate order i,f,g,o      */
} accerl_layer_kind;

typedef struct {
    int32_t kind;   /* accerl_layer_kind */
    int32_t cin, cout;
    int32_t k, stride, pad;
    int32_t relu;   /* conv / dense: ReLU fused after the layer */
    int32_t reserved;
} accerl_layer;

#define ACCERL_MAX_LAYERS 48

/* A network: observation, layer list, then two implicit heads on the last layer's flat output:
 * A = n_actions logits and one value (Section 2.2, Eq. 1: pi and v). */
typedef struct {
    int32_t obs_dtype;             /* accerl_obs_dtype */
    int32_t obs_c, obs_h, obs_w;   /* image observation [C,H,W]; vector observation: obs_c = D, obs_h = obs_w = 1 */
    int32_t n_actions;             /* 1 .. 64 */
    int32_t precision;             /* accerl_precision */
    int32_t n_layers;
    accerl_layer layers[ACCERL_MAX_LAYERS];
} accerl_arch;

/*
 * Sizes of the two host blobs accerl_policy_create expects for `arch` (so a caller can check its
 * packing).  Return ACCERL_EINVAL for an inconsistent arch.
 *
 * Weight blob: the parametrised tensors in layer order -- conv: W[cout,cin,k,k], b[cout];
 * dense: W[cout,cin], b[cout]; resblock: convA W,b then convB W,b; lstm: W_ih[4H,cin], b[4H],
 * W_hh[4H,H]; finally the heads W[A+1, F], b[A+1] (row A is the value head).  Each tensor
 * starts at the next multiple of 16 bytes.  Biases are always fp32.  W is int8 (already
 * quantized, values in -127..127) for every tensor of an ACCERL_INT8 policy except the LSTM
 * matrices and the heads of a network that contains an LSTM, which are fp32; W is fp32 for
 * teacher policies (an ACCERL_BF16 policy rounds it to bf16, ties to even, on upload).
 *
 * Scale array (ACCERL_INT8 only; n_scales = 0 for teachers): first the activation scales --
 * s_0 of the observation (uint8 observations: must be 1/255, the bytes enter as integers
 * 0..255), then in layer order one scale per quantized activation: conv and dense: their
 * output; resblock: the output of conv A, then the stream after the add -- followed by the
 * per-output-channel weight scales s_w of every int8 tensor in blob order.
 */
int accerl_blob_sizes(const accerl_arch* arch, int64_t* weights_bytes, int64_t* n_scales);

/*
 * Build a policy: validates `arch`, copies and re-lays the weights for the kernels, derives the
 * integer biases and fp32 requantization multipliers, uploads everything and fixes the launch
 * plan (the library's form of the static computational graph of Section 2.2).
 *
 * Derived constants (double arithmetic, then one rounding):
 *   biasq[n] = (int32) rint(b[n] / (s_in * s_w[n]))
 *   m[n]     = (float)((s_in * s_w[n]) / s_out)         requantization multiplier
 *   r        = (float)(s_x / s_out)                     residual-stream ratio
 *   d[n]     = (float)(s_in * s_w[n])                   head dequantization
 *   inv_s0   = (float)(1 / s_0)                         fp32 observation quantizer
 *
 * weights, quant_scales: HOST, copied.  quant_scales may be NULL iff n_scales == 0.
 * *out receives the policy; destroy it with accerl_policy_destroy.  Uses the current HIP device.
 */
int accerl_policy_create(const accerl_arch* arch, const void* weights, int64_t weights_bytes,
                         const float* quant_scales, int64_t n_scales, accerl_policy** out);

void accerl_policy_destroy(accerl_policy* p);

/*
 * Student forward (Section 1 / 2.1: the Actor's inference on the compressed policy; arithmetic:
 * Section 2.2 "Parameter Quantization").  The policy must be ACCERL_INT8 and contain no LSTM.
 *
 *   states     DEVICE [B, C, H, W] uint8 or [B, D] fp32, as the arch says
 *   uniforms   DEVICE [B] fp32 in [0, 1): one draw per state for the sampler
 *   out_logits DEVICE [B, A] fp32 behaviour logits
 *   out_value  DEVICE [B] fp32
 *   out_action DEVICE [B] int32: with m = max_a logit, e_a = exp(logit_a - m), Z = sum_a e_a
 *              (index order), the first a with e_0 + .. + e_a > u * Z, else A - 1
 *
 * Per layer: acc = sum Wq * xq + biasq (exact int32); y = (float)acc * m[n];
 * q = clamp(rint(y), relu ? 0 : -127, 127); residual join y = fma((float)acc, m[n], (float)xq * r);
 * heads logit = (float)acc * d[n].
 */
int accerl_actor_forward(accerl_policy* p, const void* states, int64_t B, const float* uniforms,
                         float* out_logits, float* out_value, int32_t* out_action, void* stream);

/* Teacher forward: same arguments and outputs; the policy must be ACCERL_FP32 or ACCERL_BF16 and
 * contain no LSTM (Section 3.1: the original network runs in fp32; Section 2.2: fp16-class
 * storage is the paper's other low-bit option).  uint8 observations enter as obs / 255. */
int accerl_actor_forward_teacher(accerl_policy* p, const void* states, int64_t B, const float* uniforms,
                                 float* out_logits, float* out_value, int32_t* out_action, void* stream);

/*
 * One environment step of a recurrent policy (the arch ends in an ACCERL_LSTM layer), any
 * precision.  done: DEVICE [B] uint8; rows with done != 0 have h and c zeroed before the cell.
 * h, c: DEVICE [B, H] fp32, updated in place.  The LSTM and the heads behind it use bf16 GEMM
 * operands (fp32 for an ACCERL_FP32 policy) with fp32 accumulation and fp32 gate arithmetic:
 * c' = sig(f) * c + sig(i) * tanh(g), h' = sig(o) * tanh(c').
 */
int accerl_actor_forward_recurrent(accerl_policy* p, const void* states, int64_t B, const float* uniforms,
                                   const uint8_t* done, float* h, float* c,
                                   float* out_logits, float* out_value, int32_t* out_action, void* stream);

typedef enum {
    ACCERL_TAP_ACC = 0,   /* int32 accumulator of a conv / dense layer (resblock: of conv B); layer = n_layers: of the heads */
    ACCERL_TAP_ACT = 1,   /* stored output of the layer: int8 (student), fp32 (teachers, converted) */
    ACCERL_TAP_ACC_A = 2, /* resblock: accumulator of conv A */
    ACCERL_TAP_ACT_A = 3  /* resblock: output of conv A */
} accerl_tap;

/*
 * Debug forward for parity tests: runs the same kernels as the forward calls up to and
 * including layer `layer` and copies one intermediate tensor to `out` (DEVICE, `out_bytes`
 * must equal the tensor's size).  Image tensors are written channels-last, [B, H, W, Cs] with
 * Cs = C rounded up to a multiple of 4 (padding channels are zero); flat tensors [B, N].  Accumulator taps are student-only and include the integer bias and are
 * zero-point free (uint8 observations count as 0..255).  Recurrent policies: layers before the
 * LSTM only.  Synchronises the stream before returning.
 */
int accerl_actor_forward_debug(accerl_policy* p, const void* states, int64_t B, int32_t layer, int32_t tap,
                               void* out, int64_t out_bytes, void* stream);

/*
 * Measurement aid (not part of the method).  Between accerl_profile_begin and accerl_profile_end
 * every forward call on the policy records one HIP event after each kernel launch of its plan (and
 * one before the first), on the stream of that call; a step's time is the span between the event
 * before it and the event after it.  A step whose work was done by the step before it (a conv or a
 * max-pool fused into the preceding conv kernel) records nothing and reports zero launches.
 * accerl_profile_end waits for the events and returns, per plan step, the summed elapsed time in
 * ms, the number of launches, the arch layer the step belongs to (n_layers = heads / sampler) and the step kind (0 fused MLP, 1 observation quantizer,
 * 2 convolution, 3 MFMA dense, 4 fp32 dense, 5 max pooling, 6 LSTM packing, 7 sampler, 8 heads + sampler).  All arrays
 * are HOST, `cap` entries each; *n_steps receives the number of plan steps (also on ACCERL_EINVAL
 * when cap is too small).
 */
int accerl_profile_begin(accerl_policy* p);
int accerl_profile_end(accerl_policy* p, int32_t cap, int32_t* n_steps, float* total_ms, int64_t* launches,
                       int32_t* layer, int32_t* kind);

/*
 * Host-only aid: builds the launch plan exactly as accerl_policy_create would (same arguments, no
 * GPU needed) and writes a one-line-per-kernel description of it into `text` (HOST, `cap` bytes,
 * always NUL-terminated, truncated if too small).
 */
int accerl_plan_describe(const accerl_arch* arch, const void* weights, int64_t weights_bytes,
                         const float* quant_scales, int64_t n_scales, char* text, int64_t cap);

/*
 * Policy mixture (Section 3.2, "Knowledge Distillation Results"): the actor sends a state through the
 * smaller network with probability alpha and through the original one otherwise.  The draw is the
 * caller's (use_smaller: HOST uint8 [B], non-zero = smaller network, read during the call); the
 * library compacts the rows of each subset, runs `smaller` on the first and `original` on the second
 * (any two non-recurrent policies: int8, fp32 or bf16) and writes every row's results to its place in the
 * outputs, so each row holds exactly what the chosen network alone would have produced for it.
 * Both policies must share observation shape and number of actions and be non-recurrent.  states,
 * uniforms and the outputs are DEVICE as in accerl_actor_forward.  Asynchronous on hip_stream; the
 * compaction buffers belong to `smaller` and grow on demand (a stream synchronisation when they do),
 * so calls that share `smaller` must not overlap.  Errors as accerl_actor_forward.
 */
int accerl_actor_forward_mixture(accerl_policy* smaller, accerl_policy* original, const void* states, int64_t B,
                                 const float* uniforms, const uint8_t* use_smaller,
                                 float* out_logits, float* out_value, int32_t* out_action, void* hip_stream);

/* Host-only: the mixture probability as a function of the Monitor's KL-mean indicator (same passage):
 * 1 up to kl_lo, 0 from kl_hi on, linear in between (the paper prints no constants). */
double accerl_mixture_alpha(double kl_mean, double kl_lo, double kl_hi);

/*
 * Monitor indicators (Monitor section, KL equation): for B states on which both the original and
 * the smaller (compressed) policy were evaluated,
 *     KL_b = sum_a pi_original(a|x_b) log(pi_original(a|x_b) / pi_smaller(a|x_b)),
 *     H_b  = -sum_a pi_smaller(a|x_b) log pi_smaller(a|x_b)     (the entropy indicator; Section 2.2 Eq. 1)
 * with pi = softmax of the logits.  logits_* : DEVICE fp32 [B, A] row-major, 16-byte aligned,
 * 1 <= A <= 64.  out_kl, out_entropy: DEVICE fp32 [B] or NULL.  out_stats: DEVICE double[4] =
 * {KL mean, KL max, KL variance (population: mean of squares minus squared mean), entropy mean},
 * the indicators the Monitor's strategies read.  Per-row arithmetic is fp32, the reductions are
 * fp64 in a fixed order (results do not depend on the launch).  Asynchronous on hip_stream; the
 * library keeps one small per-device buffer of partial sums, so calls that overlap on one device
 * must use the same stream.  B == 0 is a no-op.  Errors: ACCERL_EINVAL for NULL / misaligned /
 * out-of-range arguments, ACCERL_ENOMEM, ACCERL_EHIP.
 */
int accerl_monitor_kl(const float* logits_original, const float* logits_smaller, int64_t B, int A,
                      float* out_kl, float* out_entropy, double* out_stats, void* hip_stream);

/*
 * accerl_monitor_kl for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and the same results as
 * accerl_monitor_kl; the per-workgroup partial sums go to a fixed 40 KiB array inside the library's device
 * image (1024 records of 5 doubles; each GPU the library runs on holds its own copy until the process ends)
 * instead of a buffer allocated at first use, and the call makes no hipMalloc / hipFree and no allocating
 * library call.  B is limited to 16 777 216 (2^24) rows per call; a larger B returns ACCERL_EINVAL with a
 * message and enqueues nothing (split the batch).  Every call on a GPU uses that GPU's one array: calls that
 * overlap in time on one GPU (different streams or threads) race and must be serialised by the caller; calls
 * in sequence need no clearing in between, since a pass overwrites every record that its fold reads.
 * With more than 1024 x 256 rows the row pass runs over 1024 workgroups where accerl_monitor_kl uses up to
 * 2048, so the fp64 sums may differ from it in their last bits; out_kl and out_entropy are identical.
 */
int accerl_monitor_kl_noalloc(const float* logits_original, const float* logits_smaller, int64_t B, int A,
                              float* out_kl, float* out_entropy, double* out_stats, void* hip_stream);

/*
 * Knowledge-distillation loss, forward value only (Section 2.2, Eq. 1): per state
 *     loss_b = KL(pi_original(.|s_b) || pi_smaller(.|s_b)) + (v_original(s_b) - v_smaller(s_b))^2 / 2
 *              - beta H(pi_smaller(.|s_b)),
 * the quantity the Compressor minimises when it transfers the original policy into the smaller
 * network (its gradient and the optimiser are outside this library).  logits_*: DEVICE fp32 [B, A]
 * (16-byte aligned, 1 <= A <= 64); value_*: DEVICE fp32 [B]; out_loss: DEVICE fp32 [B] or NULL;
 * out_mean: DEVICE double[1], the batch mean (fp64 reduction in a fixed order).  Same stream and
 * overlap rules as accerl_monitor_kl, whose per-device partial-sum buffer it shares.
 */
int accerl_distill_loss(const float* logits_original, const float* logits_smaller, const float* value_original,
                        const float* value_smaller, int64_t B, int A, float beta, float* out_loss, double* out_mean,
                        void* hip_stream);

/*
 * V-trace corrector (Corrector section, V-trace equation) for B trajectories of T steps collected
 * by the smaller policy and corrected towards the original one.  Time-major tensors, all DEVICE:
 *   logits_original, logits_smaller  fp32 [T, B, A], 16-byte aligned, 1 <= A <= 64
 *   actions int32 [T, B] (the a_t taken; clamped into 0..A-1), rewards, discounts, values fp32 [T, B]
 *   (discounts = gamma, or 0 where the episode ended at that step; values = V(x_t)),
 *   bootstrap fp32 [B] = V(x_T).
 *   rho_t = min(rho_bar, pi_original(a_t|x_t) / pi_smaller(a_t|x_t)),  c_t = min(c_bar, same ratio)
 *   delta_t = rho_t (r_t + gamma_t V(x_{t+1}) - V(x_t))
 *   v_s = V(x_s) + sum_{t=s}^{T-1} (prod_{i=s}^{t-1} gamma_i c_i) delta_t   (evaluated as a backward scan)
 * Outputs fp32 [T, B]: out_vs = v_s; out_rho = rho_t (also the importance weight of the Importance
 * Sampling corrector); out_pg_adv (may be NULL) = rho_t (r_t + gamma_t v_{t+1} - V(x_t)), v_T = V(x_T),
 * the advantage of the corrected actor-critic update.  out_rho is also used as scratch during the
 * call.  Asynchronous on hip_stream; allocates nothing.  T == 0 or B == 0 is a no-op.
 */
int accerl_vtrace(const float* logits_original, const float* logits_smaller, const int32_t* actions,
                  const float* rewards, const float* discounts, const float* values, const float* bootstrap,
                  int64_t T, int64_t B, int A, float rho_bar, float c_bar,
                  float* out_vs, float* out_pg_adv, float* out_rho, void* hip_stream);

/*
 * Measurement aids (not part of the method): the ceilings the kernels are compared with, as this machine
 * sustains them.  accerl_probe_mfma runs 2048 workgroups x 4 wavefronts, each issuing iters x 8 independent
 * 16x16 MFMAs on registers (int8 16x16x64, or bf16 16x16x32 if bf16 != 0): ops = 2048 * 4 * iters * 8 *
 * 2 * 16*16*K.  accerl_probe_copy streams `bytes` (a multiple of 16) from src to dst with 16-byte
 * loads and stores.  Both asynchronous on hip_stream; the caller times them.  sink: DEVICE int32[1].
 */
int accerl_probe_mfma(int32_t bf16, int32_t iters, int32_t* sink, void* hip_stream);
int accerl_probe_copy(const void* src, void* dst, int64_t bytes, void* hip_stream);
/* One launch of a kernel that does nothing (one wavefront): chains of it give the launch floor that the latency of
 * the small configured batches is quoted against. */
int accerl_probe_empty(void* hip_stream);

/* Message of the last error on this thread ("" if none). */
const char* accerl_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* ACCERL_H */
