/*
 * Memory-safety driver for the CPU oracle.  TEST INFRASTRUCTURE ONLY.
 *
 * Built together with s4tf_oracle.c under -fsanitize=address,undefined and run as a
 * plain executable by the CPU tests: it calls every function of the oracle once per
 * shape on buffers that are malloc'ed to exactly the documented sizes, so that any
 * access outside an operand, any signed overflow or misaligned access in the oracle's
 * loop nests aborts the run.  It checks no values (those are pinned by the Python
 * tests); it prints "ok" and returns 0 when every call came back.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

void orc_round_bf16(double* a, size_t n);
void orc_round_bf16_slow(double* a, size_t n);
void orc_conv2d_fwd(const double* x, const double* w, const double* bias, double* y, int N, int H, int W, int C,
                    int K, int R, int S, int stride, int pad, int groups);
void orc_conv2d_vjp(const double* x, const double* w, const double* dy, double* dx, double* dw, double* dbias, int N,
                    int H, int W, int C, int K, int R, int S, int stride, int pad, int groups);
void orc_bias_act_fwd(const double* x, const double* bias, double* y, size_t M, int C, int act);
void orc_bias_act_vjp(const double* y, const double* dy, double* dx, double* dbias, size_t M, int C, int act);
void orc_bn_act_fwd(const double* x, const double* res, const double* gamma, const double* beta, double* y,
                    double* save_mean, double* save_invstd, size_t M, int C, double eps, int act);
void orc_bn_act_vjp(const double* x, const double* y, const double* gamma, const double* save_mean,
                    const double* save_invstd, const double* dy, double* dx, double* dres, double* dgamma,
                    double* dbeta, size_t M, int C, int act);
void orc_avgpool2_fwd(const double* x, double* y, int N, int H, int W, int C);
void orc_avgpool2_vjp(const double* dy, double* dx, int N, int H, int W, int C);
void orc_maxpool3s2_fwd(const double* x, double* y, int N, int H, int W, int C);
void orc_maxpool3s2_vjp(const double* x, const double* dy, double* dx, int N, int H, int W, int C);
void orc_head_fwd_vjp(const double* x, const double* Wt, const double* b, const int32_t* labels, double* loss,
                      double* dx, double* dW, double* db, double* logits, int N, int H, int W, int C, int classes);
void orc_sgd_momentum(size_t count, double* param, double* velocity, const double* grad, double lr, double momentum);

void orc_gather_rows_fwd(const double* x, const int32_t* index, double* y, int rows, int cols, int count);
void orc_gather_rows_vjp(const double* dy, const int32_t* index, double* dx, int rows, int cols, int count);
void orc_bn_inference_fwd(const double* x, const double* res, const double* gamma, const double* beta, const double* rm,
                          const double* rv, double* y, size_t M, int C, double eps, int act);
void orc_bn_update_running(const double* mean, const double* invstd, double* rm, double* rv, int C, size_t M,
                           double momentum, double eps);
void orc_bn_fold(const double* w, const double* bias, const double* gamma, const double* beta, const double* rm,
                 const double* rv, double* w_out, double* bias_out, size_t rows, int K, double eps);

static uint64_t state = 88172645463325252ull;
static double rnd(void) { /* xorshift64, mapped to (-1, 1) */
  state ^= state << 13;
  state ^= state >> 7;
  state ^= state << 17;
  return (double)(state >> 11) / 4503599627370496.0 - 1.0;
}
static double* buf(size_t n) { /* exactly n doubles, filled */
  double* p = (double*)malloc(sizeof(double) * (n ? n : 1));
  if (!p) abort();
  for (size_t i = 0; i < n; ++i) p[i] = rnd();
  return p;
}

static void conv_case(int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int groups) {
  int P = (H + 2 * pad - R) / stride + 1, Q = (W + 2 * pad - S) / stride + 1;
  size_t xs = (size_t)N * H * W * C, ys = (size_t)N * P * Q * K, wsz = (size_t)R * S * (C / groups) * K;
  double *x = buf(xs), *w = buf(wsz), *b = buf(K), *y = buf(ys), *dy = buf(ys), *dx = buf(xs), *dw = buf(wsz), *db = buf(K);
  orc_conv2d_fwd(x, w, b, y, N, H, W, C, K, R, S, stride, pad, groups);
  orc_conv2d_fwd(x, w, NULL, y, N, H, W, C, K, R, S, stride, pad, groups);
  orc_conv2d_vjp(x, w, dy, dx, dw, db, N, H, W, C, K, R, S, stride, pad, groups);
  orc_conv2d_vjp(x, w, dy, NULL, dw, NULL, N, H, W, C, K, R, S, stride, pad, groups);
  free(x); free(w); free(b); free(y); free(dy); free(dx); free(dw); free(db);
}

static void bn_case(size_t M, int C, int act, int with_res) {
  size_t n = M * C;
  double *x = buf(n), *res = with_res ? buf(n) : NULL, *g = buf(C), *be = buf(C), *y = buf(n), *mean = buf(C),
         *invstd = buf(C), *dy = buf(n), *dx = buf(n), *dres = with_res ? buf(n) : NULL, *dg = buf(C), *db = buf(C);
  orc_bn_act_fwd(x, res, g, be, y, mean, invstd, M, C, 1e-5, act);
  orc_bn_act_vjp(x, y, g, mean, invstd, dy, dx, dres, dg, db, M, C, act);
  orc_bias_act_fwd(x, be, y, M, C, act);
  orc_bias_act_fwd(x, NULL, y, M, C, act);
  orc_bias_act_vjp(y, dy, dx, db, M, C, act);
  orc_bias_act_vjp(y, dy, dx, NULL, M, C, act);
  free(x); free(res); free(g); free(be); free(y); free(mean); free(invstd); free(dy); free(dx); free(dres); free(dg); free(db);
}

static void pool_case(int N, int H, int W, int C) {
  size_t xs = (size_t)N * H * W * C;
  if (H >= 2 && W >= 2) {
    size_t ys = (size_t)N * (H / 2) * (W / 2) * C;
    double *x = buf(xs), *y = buf(ys), *dy = buf(ys), *dx = buf(xs);
    orc_avgpool2_fwd(x, y, N, H, W, C);
    orc_avgpool2_vjp(dy, dx, N, H, W, C);
    free(x); free(y); free(dy); free(dx);
  }
  size_t ym = (size_t)N * ((H - 1) / 2 + 1) * ((W - 1) / 2 + 1) * C;
  double *x = buf(xs), *y = buf(ym), *dy = buf(ym), *dx = buf(xs);
  for (size_t i = 0; i < xs; i += 3) x[i] = 0.0; /* ties among zeros */
  orc_maxpool3s2_fwd(x, y, N, H, W, C);
  orc_maxpool3s2_vjp(x, dy, dx, N, H, W, C);
  free(x); free(y); free(dy); free(dx);
}

static void head_case(int N, int H, int W, int C, int classes) {
  size_t xs = (size_t)N * H * W * C;
  double *x = buf(xs), *Wt = buf((size_t)C * classes), *b = buf(classes), *dx = buf(xs), *dW = buf((size_t)C * classes),
         *db = buf(classes), *logits = buf((size_t)N * classes), loss = 0.0;
  int32_t* labels = (int32_t*)malloc(sizeof(int32_t) * N);
  for (int n = 0; n < N; ++n) labels[n] = (int32_t)(n % classes);
  orc_head_fwd_vjp(x, Wt, b, labels, &loss, dx, dW, db, logits, N, H, W, C, classes);
  orc_head_fwd_vjp(x, Wt, b, labels, &loss, NULL, dW, db, NULL, N, H, W, C, classes);
  free(x); free(Wt); free(b); free(dx); free(dW); free(db); free(logits); free(labels);
}

int main(void) {
  /* N H W C K R S stride pad groups */
  conv_case(2, 5, 5, 3, 4, 3, 3, 1, 1, 1);
  conv_case(2, 6, 5, 3, 4, 3, 3, 2, 1, 1);
  conv_case(1, 7, 7, 2, 3, 5, 5, 2, 2, 1);
  conv_case(2, 5, 6, 4, 6, 3, 3, 1, 0, 2);
  conv_case(2, 6, 6, 4, 4, 3, 3, 2, 1, 4);
  conv_case(1, 4, 4, 3, 5, 1, 1, 2, 0, 1);
  conv_case(2, 5, 5, 2, 3, 3, 3, 1, 2, 1);
  conv_case(2, 6, 7, 3, 4, 1, 3, 1, 1, 1);
  conv_case(1, 9, 8, 2, 2, 5, 3, 2, 2, 1);
  conv_case(3, 1, 1, 7, 5, 1, 1, 1, 0, 1);
  conv_case(17, 3, 3, 2, 2, 3, 3, 1, 1, 1); /* more images than threads */
  for (int act = 0; act < 3; ++act) {
    bn_case(1, 1, act, 0);
    bn_case(35, 6, act, 1);
    bn_case(64, 19, act, act != 1); /* a channel count that is not a multiple of the channel block */
  }
  pool_case(2, 7, 9, 5);
  pool_case(1, 2, 2, 3);
  pool_case(1, 1, 1, 2);
  pool_case(3, 10, 10, 4);
  head_case(4, 3, 2, 6, 5);
  head_case(1, 1, 1, 3, 2);
  head_case(9, 1, 1, 8, 10);
  {
    double *p = buf(1001), *v = buf(1001), *g = buf(1001);
    orc_sgd_momentum(1001, p, v, g, 0.1, 0.9);
    orc_sgd_momentum(0, p, v, g, 0.1, 0.9);
    p[0] = 0.0; p[1] = 1e-40; p[2] = 3.3e38; p[3] = -1e39; p[4] = 1.0 / 0.0;
    orc_round_bf16(p, 1001);
    orc_round_bf16_slow(v, 1001);
    free(p); free(v); free(g);
  }
  {
    int32_t idx[6] = {3, 9, 3, 0, -1, 10};
    double *x = buf(10 * 5), *y = buf(6 * 5), *dy = buf(6 * 5), *dx = buf(10 * 5);
    orc_gather_rows_fwd(x, idx, y, 10, 5, 6);
    orc_gather_rows_vjp(dy, idx, dx, 10, 5, 6);
    orc_gather_rows_fwd(x, idx, y, 10, 5, 0);
    free(x); free(y); free(dy); free(dx);
  }
  {
    double *x = buf(35 * 6), *res = buf(35 * 6), *g = buf(6), *be = buf(6), *rm = buf(6), *rv = buf(6), *y = buf(35 * 6);
    double *w = buf(27 * 6), *b = buf(6), *wo = buf(27 * 6), *bo = buf(6), *is = buf(6);
    for (int c = 0; c < 6; ++c) { rv[c] = 0.5 + rv[c] * rv[c]; is[c] = 0.5 + is[c] * is[c]; }
    for (int act = 0; act < 3; ++act) orc_bn_inference_fwd(x, act ? res : NULL, g, be, rm, rv, y, 35, 6, 1e-5, act);
    orc_bn_update_running(rm, is, rm, rv, 6, 35, 0.1, 1e-5);
    orc_bn_update_running(rm, is, rm, rv, 6, 1, 1.0, 0.0);
    orc_bn_fold(w, b, g, be, rm, rv, wo, bo, 27, 6, 1e-5);
    orc_bn_fold(w, NULL, g, be, rm, rv, wo, bo, 27, 6, 1e-5);
    free(x); free(res); free(g); free(be); free(rm); free(rv); free(y); free(w); free(b); free(wo); free(bo); free(is);
  }
  printf("ok\n");
  return 0;
}
