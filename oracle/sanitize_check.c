/*
 * Sanitizer driver for the CPU oracle.  TEST INFRASTRUCTURE ONLY.
 *
 * Compiled together with oracle.c under -fsanitize=address,undefined (tests/test_oracle_sanitizers.py)
 * and run as a program of its own: every exported layer function is called on heap buffers of exactly
 * the size its contract states, over shapes that reach the edges of the index arithmetic (padding on
 * every side, strides that leave a remainder, kernels as large as the padded image, one-element
 * tensors, done flags, A = 1 and A = 64).  A read or write past a buffer, a signed overflow or a
 * misaligned access ends the program with a non-zero status.  No values are checked here: the pins in
 * tests/test_oracle_*.py do that.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "oracle.c"

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(void) {
    rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(rng_state >> 33);
}
static float rndf(void) { return (float)((int)(rnd() % 2001) - 1000) / 500.0f; }

static float* fbuf(int64_t n) {
    float* p = (float*)malloc((size_t)(n > 0 ? n : 1) * sizeof(float));
    for (int64_t i = 0; i < n; ++i) p[i] = rndf();
    return p;
}
static int8_t* qbuf(int64_t n, int full_range) {
    int8_t* p = (int8_t*)malloc((size_t)(n > 0 ? n : 1));
    for (int64_t i = 0; i < n; ++i) p[i] = full_range ? (int8_t)(rnd() % 255 - 127) : (int8_t)(rnd() % 15 - 7);
    return p;
}
static int32_t* ibuf(int64_t n, int32_t span) {
    int32_t* p = (int32_t*)malloc((size_t)(n > 0 ? n : 1) * sizeof(int32_t));
    for (int64_t i = 0; i < n; ++i) p[i] = (int32_t)(rnd() % (2u * (uint32_t)span + 1u)) - span;
    return p;
}
static int ohw(int h, int k, int s, int p) { return (h + 2 * p - k) / s + 1; }

static void conv_case(int B, int C, int H, int W, int Co, int k, int s, int p) {
    const int Ho = ohw(H, k, s, p), Wo = ohw(W, k, s, p);
    const int64_t nx = (int64_t)B * C * H * W, nw = (int64_t)Co * C * k * k, ny = (int64_t)B * Co * Ho * Wo;
    float *x = fbuf(nx), *w = fbuf(nw), *b = fbuf(Co), *y = fbuf(ny);
    for (int relu = 0; relu < 2; ++relu)
        for (int bf = 0; bf < 2; ++bf) orc_conv2d_f(x, B, C, H, W, w, b, Co, k, s, p, relu, bf, y);
    float* yp = fbuf((int64_t)B * C * Ho * Wo);
    if (2 * p <= k) orc_maxpool_f(x, B, C, H, W, k, s, p, yp);
    int8_t *xq = qbuf(nx, 1), *wq = qbuf(nw, 1), *q = qbuf(ny, 0), *qp = qbuf((int64_t)B * C * Ho * Wo, 0);
    uint8_t* xu = (uint8_t*)malloc((size_t)nx);
    for (int64_t i = 0; i < nx; ++i) xu[i] = (uint8_t)(rnd() & 255);
    int32_t *bq = ibuf(Co, 100000), *acc = ibuf(ny, 1);
    orc_conv2d_q_acc(xq, 0, 0, B, C, H, W, wq, bq, Co, k, s, p, acc);
    orc_conv2d_q_acc(xq, 0, 1, B, C, H, W, wq, bq, Co, k, s, p, acc);
    orc_conv2d_q_acc(xu, 1, 0, B, C, H, W, wq, bq, Co, k, s, p, acc);
    float* m = fbuf(Co);
    orc_requant(acc, B, Co, Ho * Wo, m, 0, q);
    orc_requant(acc, B, Co, Ho * Wo, m, -127, q);
    int8_t* res = qbuf(ny, 1);
    orc_requant_residual(acc, res, 0.75f, B, Co, Ho * Wo, m, q);
    if (2 * p <= k) orc_maxpool_i8(xq, B, C, H, W, k, s, p, qp);
    free(x); free(w); free(b); free(y); free(yp); free(xq); free(wq); free(q); free(qp); free(xu);
    free(bq); free(acc); free(m); free(res);
}

static void dense_case(int B, int K, int N) {
    float *x = fbuf((int64_t)B * K), *w = fbuf((int64_t)N * K), *b = fbuf(N), *y = fbuf((int64_t)B * N);
    orc_dense_f(x, B, K, w, b, N, 1, 0, y);
    orc_dense_f(x, B, K, w, NULL, N, 0, 1, y);
    orc_bf16_round(x, (int64_t)B * K, x);
    int8_t *xq = qbuf((int64_t)B * K, 1), *wq = qbuf((int64_t)N * K, 1);
    int32_t *bq = ibuf(N, 1000), *acc = ibuf((int64_t)B * N, 1);
    orc_dense_q_acc(xq, 0, B, K, wq, bq, N, acc);
    orc_dense_q_acc(xq, 1, B, K, wq, bq, N, acc);
    float* d = fbuf(N);
    orc_dequant(acc, B, N, d, y);
    orc_dequant_i8(xq, (int64_t)B * K, 0.125f, x);
    orc_quantize_f32(y, (int64_t)B * N, 3.0f, (int8_t*)acc);   /* B*N bytes of the B*N*4 available */
    free(x); free(w); free(b); free(y); free(xq); free(wq); free(bq); free(acc); free(d);
}

static void policy_case(int B, int A) {
    float *lo = fbuf((int64_t)B * A), *ls = fbuf((int64_t)B * A), *u = fbuf(B);
    for (int i = 0; i < B; ++i) u[i] = (float)(rnd() % 1000) / 1000.0f;
    int32_t* act = ibuf(B, 1);
    float* logp = fbuf((int64_t)B * A);
    orc_softmax_sample(lo, B, A, u, act, logp);
    orc_softmax_sample(lo, B, A, u, act, NULL);
    double *kl = (double*)malloc(sizeof(double) * (size_t)B), *en = (double*)malloc(sizeof(double) * (size_t)B), st[4], mean;
    orc_kl_monitor(lo, ls, B, A, kl, en, st);
    float *vo = fbuf(B), *vs_ = fbuf(B);
    orc_distill_loss(lo, ls, vo, vs_, B, A, 0.01, kl, &mean);
    free(lo); free(ls); free(u); free(act); free(logp); free(kl); free(en); free(vo); free(vs_);
}

static void vtrace_case(int T, int B, int A) {
    const int64_t n = (int64_t)T * B;
    float *lo = fbuf(n * A), *ls = fbuf(n * A), *r = fbuf(n), *g = fbuf(n), *v = fbuf(n), *boot = fbuf(B);
    int32_t* a = ibuf(n, 1);
    for (int64_t i = 0; i < n; ++i) { a[i] = (int32_t)(rnd() % (uint32_t)A); g[i] = (rnd() % 10) ? 0.99f : 0.0f; }
    double *vs = (double*)malloc(sizeof(double) * (size_t)n), *pg = (double*)malloc(sizeof(double) * (size_t)n),
           *rho = (double*)malloc(sizeof(double) * (size_t)n);
    orc_vtrace(lo, ls, a, r, g, v, boot, T, B, A, 1.0, 1.0, vs, pg, rho);
    free(lo); free(ls); free(r); free(g); free(v); free(boot); free(a); free(vs); free(pg); free(rho);
}

static void lstm_case(int B, int In, int Hd) {
    float *x = fbuf((int64_t)B * In), *h = fbuf((int64_t)B * Hd), *c = fbuf((int64_t)B * Hd);
    float *wi = fbuf((int64_t)4 * Hd * In), *wh = fbuf((int64_t)4 * Hd * Hd), *b = fbuf(4 * Hd);
    uint8_t* done = (uint8_t*)malloc((size_t)B);
    for (int i = 0; i < B; ++i) done[i] = (uint8_t)(rnd() % 3 == 0);
    orc_lstm_step(x, B, In, Hd, done, wi, wh, b, 1, h, c);
    orc_lstm_step(x, B, In, Hd, NULL, wi, wh, b, 0, h, c);
    free(x); free(h); free(c); free(wi); free(wh); free(b); free(done);
}

int main(void) {
    orc_set_threads(orc_num_threads() > 4 ? 4 : orc_num_threads());
    /* the benchmark networks' layer shapes at reduced image sizes, then edge shapes */
    conv_case(2, 4, 20, 20, 5, 8, 4, 0);
    conv_case(2, 3, 9, 9, 6, 4, 2, 0);
    conv_case(1, 6, 7, 7, 4, 3, 1, 0);
    conv_case(3, 4, 11, 11, 3, 3, 1, 1);
    conv_case(2, 2, 11, 11, 2, 3, 2, 1);     /* the 3x3 stride-2 pad-1 pooling shape, odd size */
    conv_case(2, 2, 10, 12, 2, 3, 2, 1);     /* even sizes, H != W */
    conv_case(1, 1, 1, 1, 1, 1, 1, 0);
    conv_case(1, 2, 2, 2, 3, 3, 1, 1);       /* kernel larger than the image, all taps but one in the padding */
    conv_case(1, 1, 5, 5, 1, 5, 3, 2);       /* stride leaves a remainder */
    dense_case(1, 1, 1);
    dense_case(3, 24, 64);
    dense_case(5, 67, 19);
    policy_case(1, 1);
    policy_case(7, 18);
    policy_case(3, 64);
    vtrace_case(1, 1, 2);
    vtrace_case(16, 5, 18);
    lstm_case(1, 1, 1);
    lstm_case(4, 9, 6);
    volatile float z = orc_bf16_round_scalar(1.00390625f) + (float)orc_mixture_alpha(0.5, 0.1, 1.0);
    (void)z;
    puts("sanitize_check ok");
    return 0;
}
