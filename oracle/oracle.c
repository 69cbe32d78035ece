/*
 * CPU oracle for the AcceRL actor forward pass.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, direct-loop C: one function per layer type, logical NCHW / row-major
 * [B, features] tensors, no tiling, no SIMD intrinsics, no code shared with the HIP
 * library.  Only tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * What the paper fixes (Section 2.2, "Parameter Quantization"): the actor's policy is the
 * learner's network with fp32 parameters replaced by int8 (post-training quantization) and
 * adjacent layers (Conv+ReLU, FC+ReLU) fused; (Section 2.2, "Structured Pruning") pruning
 * deletes rows and columns of the weight matrices; (Section 2.2, Eq. 1) the network outputs
 * an action distribution pi(.|s) and a value v(s); (Section 3.1, network table) the
 * original CNN is conv 32(8), 64(4), 64(3) + FC on a 4x84x84 input with up to 18 actions.
 * The paper gives no arithmetic for the quantized layers; the reading implemented here
 * (symmetric per-output-channel weight scales, per-tensor activation scales, int32
 * accumulation, one fp32 multiply + round-half-even per requantization) is stated at each
 * function.  Every fp32 step below is a single IEEE-754 binary32 operation; compile with
 * -ffp-contract=off so none is fused.
 *
 * Parity status: integer accumulators, requantization, pooling, softmax and the sampler
 * are pinned by tests against brute force, library routines, closed forms and invariants.
 * End-to-end network outputs are "parity unpinned" by the paper (it prints no forward-pass
 * value); they are guarded by those per-layer pins.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void orc_set_threads(int n) {
#ifdef _OPENMP
    omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* bfloat16 = top 16 bits of binary32; round to nearest, ties to even; NaN kept. */
float orc_bf16_round_scalar(float x) {
    uint32_t u;
    memcpy(&u, &x, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return x;
    u += 0x7fffu + ((u >> 16) & 1u);
    u &= 0xffff0000u;
    memcpy(&x, &u, 4);
    return x;
}

void orc_bf16_round(const float* x, int64_t n, float* y) {
    for (int64_t i = 0; i < n; ++i) y[i] = orc_bf16_round_scalar(x[i]);
}

/* ------------------------------------------------------------------ teacher (float) */

/* y[b,co,oy,ox] = relu?( sum_{ci,ky,kx} w[co,ci,ky,kx] * x[b,ci,oy*s+ky-p,ox*s+kx-p] + bias[co] )
 * Out-of-image taps contribute 0.  Sum and bias in double, result rounded once to float.
 * bf16_operands: x and w are rounded to bfloat16 before each product (bf16 teacher). */
void orc_conv2d_f(const float* x, int64_t B, int C, int H, int W,
                  const float* w, const float* bias, int Co, int k, int s, int p,
                  int relu, int bf16_operands, float* y) {
    const int Ho = (H + 2 * p - k) / s + 1, Wo = (W + 2 * p - k) / s + 1;
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < B; ++b)
        for (int co = 0; co < Co; ++co)
            for (int oy = 0; oy < Ho; ++oy)
                for (int ox = 0; ox < Wo; ++ox) {
                    double acc = 0.0;
                    for (int ci = 0; ci < C; ++ci)
                        for (int ky = 0; ky < k; ++ky) {
                            const int iy = oy * s + ky - p;
                            if (iy < 0 || iy >= H) continue;
                            for (int kx = 0; kx < k; ++kx) {
                                const int ix = ox * s + kx - p;
                                if (ix < 0 || ix >= W) continue;
                                float xv = x[((b * C + ci) * H + iy) * W + ix];
                                float wv = w[((co * C + ci) * k + ky) * k + kx];
                                if (bf16_operands) { xv = orc_bf16_round_scalar(xv); wv = orc_bf16_round_scalar(wv); }
                                acc += (double)xv * (double)wv;
                            }
                        }
                    float r = (float)(acc + (double)bias[co]);
                    if (relu && !(r > 0.0f)) r = 0.0f;
                    y[((b * Co + co) * Ho + oy) * Wo + ox] = r;
                }
}

/* y[b,n] = relu?( sum_k w[n,k] * x[b,k] + bias[n] ); bias may be NULL (treated as 0). */
void orc_dense_f(const float* x, int64_t B, int K, const float* w, const float* bias, int N,
                 int relu, int bf16_operands, float* y) {
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < B; ++b)
        for (int n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int kk = 0; kk < K; ++kk) {
                float xv = x[b * K + kk], wv = w[(int64_t)n * K + kk];
                if (bf16_operands) { xv = orc_bf16_round_scalar(xv); wv = orc_bf16_round_scalar(wv); }
                acc += (double)xv * (double)wv;
            }
            float r = (float)(acc + (bias ? (double)bias[n] : 0.0));
            if (relu && !(r > 0.0f)) r = 0.0f;
            y[b * N + n] = r;
        }
}

/* Max over the k x k window at stride s; taps outside the image are ignored. */
void orc_maxpool_f(const float* x, int64_t B, int C, int H, int W, int k, int s, int p, float* y) {
    const int Ho = (H + 2 * p - k) / s + 1, Wo = (W + 2 * p - k) / s + 1;
#pragma omp parallel for schedule(static)
    for (int64_t bc = 0; bc < B * C; ++bc)
        for (int oy = 0; oy < Ho; ++oy)
            for (int ox = 0; ox < Wo; ++ox) {
                float m = -INFINITY;
                for (int ky = 0; ky < k; ++ky)
                    for (int kx = 0; kx < k; ++kx) {
                        const int iy = oy * s + ky - p, ix = ox * s + kx - p;
                        if (iy < 0 || iy >= H || ix < 0 || ix >= W) continue;
                        const float v = x[(bc * H + iy) * W + ix];
                        if (v > m) m = v;
                    }
                y[(bc * Ho + oy) * Wo + ox] = m;
            }
}

/* ------------------------------------------------------------------ student (int8) */

/* fp32 observation -> int8: q = clamp(rint(x * inv_s), -127, 127), one fp32 multiply. */
void orc_quantize_f32(const float* x, int64_t n, float inv_s, int8_t* q) {
    for (int64_t i = 0; i < n; ++i) {
        float r = rintf(x[i] * inv_s);
        if (r > 127.0f) r = 127.0f;
        if (r < -127.0f) r = -127.0f;
        q[i] = (int8_t)r;
    }
}

static inline int32_t load_q(const void* x, int64_t i, int is_u8, int relu_in) {
    if (is_u8) return (int32_t)((const uint8_t*)x)[i];
    int32_t v = (int32_t)((const int8_t*)x)[i];
    return (relu_in && v < 0) ? 0 : v;
}

/* acc[b,co,oy,ox] = sum wq * xq + biasq[co], exact integers.  x holds either raw uint8
 * observations (0..255, zero-point free) or int8 activations; relu_in applies max(x,0) to
 * int8 input on load (the ReLU that opens a residual branch).  Out-of-image taps add 0. */
void orc_conv2d_q_acc(const void* x, int x_is_u8, int relu_in, int64_t B, int C, int H, int W,
                      const int8_t* wq, const int32_t* biasq, int Co, int k, int s, int p,
                      int32_t* acc) {
    const int Ho = (H + 2 * p - k) / s + 1, Wo = (W + 2 * p - k) / s + 1;
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < B; ++b)
        for (int co = 0; co < Co; ++co)
            for (int oy = 0; oy < Ho; ++oy)
                for (int ox = 0; ox < Wo; ++ox) {
                    int64_t a = biasq[co];
                    for (int ci = 0; ci < C; ++ci)
                        for (int ky = 0; ky < k; ++ky) {
                            const int iy = oy * s + ky - p;
                            if (iy < 0 || iy >= H) continue;
                            for (int kx = 0; kx < k; ++kx) {
                                const int ix = ox * s + kx - p;
                                if (ix < 0 || ix >= W) continue;
                                a += (int64_t)wq[((co * C + ci) * k + ky) * k + kx] *
                                     load_q(x, ((b * C + ci) * H + iy) * W + ix, x_is_u8, relu_in);
                            }
                        }
                    acc[((b * Co + co) * Ho + oy) * Wo + ox] = (int32_t)a;
                }
}

/* acc[b,n] = sum_k wq[n,k] * xq[b,k] + biasq[n] */
void orc_dense_q_acc(const int8_t* x, int relu_in, int64_t B, int K, const int8_t* wq,
                     const int32_t* biasq, int N, int32_t* acc) {
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < B; ++b)
        for (int n = 0; n < N; ++n) {
            int64_t a = biasq[n];
            for (int kk = 0; kk < K; ++kk)
                a += (int64_t)wq[(int64_t)n * K + kk] * load_q(x, b * K + kk, 0, relu_in);
            acc[b * N + n] = (int32_t)a;
        }
}

/* Requantize a [B, Cn, HW] accumulator: y = (float)acc * m[c]; q = clamp(rint(y), lo, 127).
 * lo = 0 fuses the ReLU, lo = -127 is the plain symmetric clamp. */
void orc_requant(const int32_t* acc, int64_t B, int Cn, int HW, const float* m, int lo, int8_t* q) {
    for (int64_t b = 0; b < B; ++b)
        for (int c = 0; c < Cn; ++c)
            for (int i = 0; i < HW; ++i) {
                const int64_t o = (b * Cn + c) * HW + i;
                float y = (float)acc[o] * m[c];
                float r = rintf(y);
                if (r > 127.0f) r = 127.0f;
                if (r < (float)lo) r = (float)lo;
                q[o] = (int8_t)r;
            }
}

/* Residual join: t = (float)xq * r; y = fma((float)acc, m[c], t); q = clamp(rint(y), -127, 127). */
void orc_requant_residual(const int32_t* acc, const int8_t* xq, float r, int64_t B, int Cn, int HW,
                          const float* m, int8_t* q) {
    for (int64_t b = 0; b < B; ++b)
        for (int c = 0; c < Cn; ++c)
            for (int i = 0; i < HW; ++i) {
                const int64_t o = (b * Cn + c) * HW + i;
                float t = (float)xq[o] * r;
                float y = fmaf((float)acc[o], m[c], t);
                float v = rintf(y);
                if (v > 127.0f) v = 127.0f;
                if (v < -127.0f) v = -127.0f;
                q[o] = (int8_t)v;
            }
}

void orc_maxpool_i8(const int8_t* x, int64_t B, int C, int H, int W, int k, int s, int p, int8_t* y) {
    const int Ho = (H + 2 * p - k) / s + 1, Wo = (W + 2 * p - k) / s + 1;
#pragma omp parallel for schedule(static)
    for (int64_t bc = 0; bc < B * C; ++bc)
        for (int oy = 0; oy < Ho; ++oy)
            for (int ox = 0; ox < Wo; ++ox) {
                int m = -128;
                for (int ky = 0; ky < k; ++ky)
                    for (int kx = 0; kx < k; ++kx) {
                        const int iy = oy * s + ky - p, ix = ox * s + kx - p;
                        if (iy < 0 || iy >= H || ix < 0 || ix >= W) continue;
                        const int v = x[(bc * H + iy) * W + ix];
                        if (v > m) m = v;
                    }
                y[(bc * Ho + oy) * Wo + ox] = (int8_t)m;
            }
}

/* Head outputs from accumulators: out[b,n] = (float)acc[b,n] * d[n]. */
void orc_dequant(const int32_t* acc, int64_t B, int N, const float* d, float* out) {
    for (int64_t b = 0; b < B; ++b)
        for (int n = 0; n < N; ++n) out[b * N + n] = (float)acc[b * N + n] * d[n];
}

/* int8 activation -> float: x = (float)q * s (input of a float layer after a quantized one). */
void orc_dequant_i8(const int8_t* q, int64_t n, float s, float* x) {
    for (int64_t i = 0; i < n; ++i) x[i] = (float)q[i] * s;
}

/* ------------------------------------------------------------------ policy head */

/* Per row: m = max logit; e[a] = expf(logit[a] - m); Z = sum e in index order;
 * logp[a] = logit[a] - m - logf(Z) (optional); action = first a with cum(e) > u*Z, else A-1. */
void orc_softmax_sample(const float* logits, int64_t B, int A, const float* u,
                        int32_t* action, float* logp) {
    for (int64_t b = 0; b < B; ++b) {
        const float* l = logits + b * A;
        float m = l[0];
        for (int a = 1; a < A; ++a) if (l[a] > m) m = l[a];
        float Z = 0.0f;
        for (int a = 0; a < A; ++a) Z += expf(l[a] - m);
        if (logp) {
            const float lz = logf(Z);
            for (int a = 0; a < A; ++a) logp[b * A + a] = (l[a] - m) - lz;
        }
        if (action) {
            const float t = u[b] * Z;
            float cum = 0.0f;
            int act = A - 1;
            for (int a = 0; a < A; ++a) {
                cum += expf(l[a] - m);
                if (cum > t) { act = a; break; }
            }
            action[b] = act;
        }
    }
}

/* ------------------------------------------------------------------ LSTM core */

static inline float sigmoidf_(float x) { return 1.0f / (1.0f + expf(-x)); }

/* One step for B rows.  done[b] != 0 zeroes h[b], c[b] before the cell.  Gate order i,f,g,o:
 * pre = W_ih x + W_hh h + bias (sums in double, rounded once to float); with bf16_operands the
 * GEMM operands x, h, W_ih, W_hh are rounded to bfloat16 first.  c' = sig(f)*c + sig(i)*tanh(g),
 * h' = sig(o)*tanh(c'), each product and sum a separate fp32 operation.  h, c updated in place. */
void orc_lstm_step(const float* x, int64_t B, int In, int Hd, const uint8_t* done,
                   const float* w_ih, const float* w_hh, const float* bias, int bf16_operands,
                   float* h, float* c) {
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < B; ++b) {
        float* hb = h + b * Hd;
        float* cb = c + b * Hd;
        if (done && done[b]) for (int j = 0; j < Hd; ++j) { hb[j] = 0.0f; cb[j] = 0.0f; }
        float hn[1024], cn[1024];
        for (int j = 0; j < Hd; ++j) {
            float pre[4];
            for (int g = 0; g < 4; ++g) {
                const int row = g * Hd + j;
                double acc = 0.0;
                for (int kk = 0; kk < In; ++kk) {
                    float xv = x[b * In + kk], wv = w_ih[(int64_t)row * In + kk];
                    if (bf16_operands) { xv = orc_bf16_round_scalar(xv); wv = orc_bf16_round_scalar(wv); }
                    acc += (double)xv * (double)wv;
                }
                for (int kk = 0; kk < Hd; ++kk) {
                    float hv = hb[kk], wv = w_hh[(int64_t)row * Hd + kk];
                    if (bf16_operands) { hv = orc_bf16_round_scalar(hv); wv = orc_bf16_round_scalar(wv); }
                    acc += (double)hv * (double)wv;
                }
                pre[g] = (float)(acc + (double)bias[row]);
            }
            const float si = sigmoidf_(pre[0]), sf = sigmoidf_(pre[1]), tg = tanhf(pre[2]), so = sigmoidf_(pre[3]);
            const float t1 = sf * cb[j];
            const float t2 = si * tg;
            cn[j] = t1 + t2;
            hn[j] = so * tanhf(cn[j]);
        }
        for (int j = 0; j < Hd; ++j) { hb[j] = hn[j]; cb[j] = cn[j]; }
    }
}

/* ------------------------------------------------------------------------------------------
 * Monitor indicators and off-policy correction (paper Section 2.3 "Corrector", Section 2.4
 * "Monitor").  fp64 throughout; inputs are the fp32 logits / values the actor and the
 * learner's network produced.
 * ------------------------------------------------------------------------------------------ */

/* log-softmax of one row in double */
static void orc_logsoftmax_row(const float* l, int A, double* logp) {
    double m = (double)l[0];
    for (int a = 1; a < A; ++a) if ((double)l[a] > m) m = (double)l[a];
    double Z = 0.0;
    for (int a = 0; a < A; ++a) Z += exp((double)l[a] - m);
    const double lz = log(Z);
    for (int a = 0; a < A; ++a) logp[a] = (double)l[a] - m - lz;
}

/* Monitor section, KL equation: per state, KL(pi_original || pi_smaller) =
 * sum_a pi_original(a|x) log(pi_original(a|x) / pi_smaller(a|x)); and the policy entropy
 * H(pi_smaller) = -sum_a pi_smaller log pi_smaller (the "entropy" indicator; also the H of
 * Section 2.2 Eq. 1).  stats = {KL mean, KL max, KL variance, entropy mean} over the B states;
 * the paper names the indicators without formulas: the variance is taken as the population
 * variance mean((KL - mean)^2). */
void orc_kl_monitor(const float* logits_original, const float* logits_smaller, int64_t B, int A,
                    double* kl, double* entropy, double* stats) {
    double po[256], ps[256];
    double sum = 0.0, mx = 0.0, hsum = 0.0;
    for (int64_t b = 0; b < B; ++b) {
        orc_logsoftmax_row(logits_original + b * A, A, po);
        orc_logsoftmax_row(logits_smaller + b * A, A, ps);
        double k = 0.0, h = 0.0;
        for (int a = 0; a < A; ++a) {
            k += exp(po[a]) * (po[a] - ps[a]);
            h -= exp(ps[a]) * ps[a];
        }
        kl[b] = k;
        entropy[b] = h;
        sum += k;
        hsum += h;
        if (b == 0 || k > mx) mx = k;
    }
    const double mean = B > 0 ? sum / (double)B : 0.0;
    double var = 0.0;
    for (int64_t b = 0; b < B; ++b) var += (kl[b] - mean) * (kl[b] - mean);
    stats[0] = mean;
    stats[1] = mx;
    stats[2] = B > 0 ? var / (double)B : 0.0;
    stats[3] = B > 0 ? hsum / (double)B : 0.0;
}

/* Section 2.2 Eq. 1, knowledge-distillation loss of one state:
 * KL(pi_original || pi_smaller) + (v_original - v_smaller)^2 / 2 - beta H(pi_smaller); mean over the batch. */
void orc_distill_loss(const float* logits_original, const float* logits_smaller, const float* v_original,
                      const float* v_smaller, int64_t B, int A, double beta, double* loss, double* mean) {
    double po[256], ps[256];
    double sum = 0.0;
    for (int64_t b = 0; b < B; ++b) {
        orc_logsoftmax_row(logits_original + b * A, A, po);
        orc_logsoftmax_row(logits_smaller + b * A, A, ps);
        double k = 0.0, h = 0.0;
        for (int a = 0; a < A; ++a) {
            k += exp(po[a]) * (po[a] - ps[a]);
            h -= exp(ps[a]) * ps[a];
        }
        const double dv = (double)v_original[b] - (double)v_smaller[b];
        loss[b] = k + 0.5 * dv * dv - beta * h;
        sum += loss[b];
    }
    *mean = B > 0 ? sum / (double)B : 0.0;
}

/* Corrector section, V-trace equation, written out as printed (a sum over the remaining steps
 * of the trajectory, not a recurrence):
 *   rho_t = min(rho_bar, pi_original(a_t|x_t) / pi_smaller(a_t|x_t)),  c_i likewise with c_bar
 *   delta_t V = rho_t (r_t + gamma_t V(x_{t+1}) - V(x_t))
 *   v_s = V(x_s) + sum_{t=s}^{T-1} (prod_{i=s}^{t-1} gamma_i c_i) delta_t V
 * Tensors are time-major [T, B(, A)]; V(x_T) is the bootstrap value.  The paper's gamma^{t-s}
 * is read as the product of per-step discounts gamma_i (gamma, or 0 where an episode ended),
 * and its n as the steps left in the trajectory.  Also returned: rho_t and the importance-
 * weighted advantage rho_t (r_t + gamma_t v_{t+1} - V(x_t)) of the actor-critic update
 * (Corrector section, last equation, first line), with v_T = V(x_T). */
void orc_vtrace(const float* logits_original, const float* logits_smaller, const int32_t* actions,
                const float* rewards, const float* discounts, const float* values,
                const float* bootstrap, int64_t T, int64_t B, int A, double rho_bar, double c_bar,
                double* vs, double* pg_adv, double* rho) {
    double lo[256], ls[256];
#ifdef _OPENMP
#pragma omp parallel for schedule(static) private(lo, ls)
#endif
    for (int64_t b = 0; b < B; ++b) {
        /* rho_t, c_t are kept in rho[] and a local array */
        double cc[4096];
        for (int64_t t = 0; t < T; ++t) {
            const int64_t i = t * B + b;
            orc_logsoftmax_row(logits_original + i * A, A, lo);
            orc_logsoftmax_row(logits_smaller + i * A, A, ls);
            const double ratio = exp(lo[actions[i]] - ls[actions[i]]);
            rho[i] = ratio < rho_bar ? ratio : rho_bar;
            cc[t] = ratio < c_bar ? ratio : c_bar;
        }
        for (int64_t s = 0; s < T; ++s) {
            double acc = 0.0, prod = 1.0;
            for (int64_t t = s; t < T; ++t) {
                const int64_t i = t * B + b;
                const double vnext = (t + 1 < T) ? (double)values[(t + 1) * B + b] : (double)bootstrap[b];
                const double delta = rho[i] * ((double)rewards[i] + (double)discounts[i] * vnext - (double)values[i]);
                acc += prod * delta;
                prod *= (double)discounts[i] * cc[t];
            }
            vs[s * B + b] = (double)values[s * B + b] + acc;
        }
        for (int64_t t = 0; t < T; ++t) {
            const int64_t i = t * B + b;
            const double vnext = (t + 1 < T) ? vs[(t + 1) * B + b] : (double)bootstrap[b];
            pg_adv[i] = rho[i] * ((double)rewards[i] + (double)discounts[i] * vnext - (double)values[i]);
        }
    }
}

/* Section 3.2, "Knowledge Distillation Results": the actor uses the smaller network with probability
 * alpha and the original one with 1 - alpha, and alpha falls linearly as the KL-mean indicator
 * grows.  The paper prints no constants: alpha = 1 at kl_mean <= kl_lo, 0 at kl_mean >= kl_hi,
 * linear in between (kl_lo < kl_hi chosen by the user's strategy). */
double orc_mixture_alpha(double kl_mean, double kl_lo, double kl_hi) {
    if (kl_mean <= kl_lo) return 1.0;
    if (kl_mean >= kl_hi) return 0.0;
    return (kl_hi - kl_mean) / (kl_hi - kl_lo);
}
