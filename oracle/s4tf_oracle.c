/*
 * CPU oracle for one differentiated training step of a convolutional network.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the GPU
 * library is checked against.  It shares no code, header, table or helper with the
 * GPU path and nothing in the product path may call it.
 *
 * What a "step" is follows the paper's training loop (Section 4.2, the figure
 * "Training LeNet on a simple dataset"): take the gradient of the scalar loss
 * softmaxCrossEntropy(logits: model(x), labels: y) with respect to the model, then
 * let the optimizer update the model in place.  Each op below is one primitive with
 * a hand-written pullback, i.e. one of the "base case" derivatives of Section 2.1
 * (a VJP returns the value plus a map from the output cotangent to the input
 * cotangents).  The paper names the ops (Conv2D, AvgPool2D, Dense,
 * softmaxCrossEntropy, the LeNet figure of Section 4.1) but does not define their
 * arithmetic; the definitions used here are the textbook ones and every reading the
 * paper leaves open is listed in the design notes of this repository.
 *
 * Conventions: activations NHWC, filters (R,S,C/groups,K) as in the LeNet figure's
 * filterShape (5,5,1,6) = (H,W,Cin,Cout); convolution is cross-correlation with
 * symmetric zero padding; P = floor((H + 2 pad - R)/stride) + 1.  Everything is
 * double precision.  OpenMP is used over the outermost independent index only.
 * Pullbacks of conv are written as the adjoint scatter of the forward loop nest,
 * not as a gather.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define IDX4(n, h, w, c, H, W, C) ((((size_t)(n) * (H) + (h)) * (W) + (w)) * (C) + (c))

int orc_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ---- bf16 rounding (round to nearest, ties to even) of a double, result kept in a
 * double.  bf16 = 1 sign, 8 exponent, 7 explicit mantissa bits (8 significant). ---- */
static double round_bf16_one(double v) {
  if (v == 0.0 || isnan(v) || isinf(v)) return v;
  int e;
  double m = frexp(v, &e);          /* v = m * 2^e, 0.5 <= |m| < 1 */
  int emin = -126;                  /* smallest normal exponent of bf16 (same as fp32) */
  int ebits = e - 1;                /* v = (2m) * 2^(e-1), 1 <= |2m| < 2 */
  int shift = 7;                    /* keep 7 fractional bits of 2m */
  if (ebits < emin) shift -= (emin - ebits); /* subnormal: fewer bits */
  double scaled = ldexp(m, shift + 1);       /* (2m) * 2^shift */
  double r = nearbyint(scaled);              /* default rounding mode = ties-to-even */
  double out = ldexp(r, ebits - shift);
  if (fabs(out) > 3.3895313892515355e38) out = copysign(INFINITY, v);
  return out;
}

/* Same rounding on the bit pattern of the double, valid when the result is a normal bf16
 * number: a double has 52 explicit mantissa bits, bf16 keeps 7, so 45 bits are dropped with
 * round-half-to-even.  Anything near the subnormal or overflow range takes the slow path. */
static double round_bf16_fast(double v) {
  double av = fabs(v);
  if (!(av >= 1.1754943508222875e-38 && av < 1.0e38)) return round_bf16_one(v);
  uint64_t u;
  memcpy(&u, &v, sizeof u);
  u += 0x00000FFFFFFFFFFFull + ((u >> 45) & 1ull);
  u &= ~0x00001FFFFFFFFFFFull;
  memcpy(&v, &u, sizeof u);
  return v;
}

void orc_round_bf16(double* a, size_t n) {
#pragma omp parallel for schedule(static)
  for (size_t i = 0; i < n; ++i) a[i] = round_bf16_fast(a[i]);
}

/* slow path only, for testing the fast path against it */
void orc_round_bf16_slow(double* a, size_t n) {
  for (size_t i = 0; i < n; ++i) a[i] = round_bf16_one(a[i]);
}

static double act_apply(double z, int act) {
  if (act == 1) return z > 0.0 ? z : 0.0;
  if (act == 2) return z < 0.0 ? 0.0 : (z > 6.0 ? 6.0 : z);
  return z;
}
/* derivative mask evaluated on the stored output y: relu 0<y, relu6 0<y<6 */
static double act_mask(double y, int act) {
  if (act == 1) return y > 0.0 ? 1.0 : 0.0;
  if (act == 2) return (y > 0.0 && y < 6.0) ? 1.0 : 0.0;
  return 1.0;
}

/* ---------------------------------------------------------------------------------
 * conv2d forward:  y[n,p,q,k] = b[k] + sum_{r,s,c} x[n, p*st+r-pad, q*st+s-pad, g*Cg+c]
 *                                              * w[r,s,c,k],   g = k / (K/groups)
 * --------------------------------------------------------------------------------- */
void orc_conv2d_fwd(const double* x, const double* w, const double* bias, double* y,
                    int N, int H, int W, int C, int K, int R, int S, int stride, int pad,
                    int groups) {
  int P = (H + 2 * pad - R) / stride + 1, Q = (W + 2 * pad - S) / stride + 1;
  int Cg = C / groups, Kg = K / groups;
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int p = 0; p < P; ++p) {
      double* acc = (double*)malloc(sizeof(double) * (size_t)K);
      for (int q = 0; q < Q; ++q) {
        for (int k = 0; k < K; ++k) acc[k] = bias ? bias[k] : 0.0;
        for (int r = 0; r < R; ++r) {
          int h = p * stride + r - pad;
          if (h < 0 || h >= H) continue;
          for (int s = 0; s < S; ++s) {
            int ww = q * stride + s - pad;
            if (ww < 0 || ww >= W) continue;
            for (int g = 0; g < groups; ++g)
              for (int c = 0; c < Cg; ++c) {
                double xv = x[IDX4(n, h, ww, g * Cg + c, H, W, C)];
                const double* wp = w + (((size_t)r * S + s) * Cg + c) * K + (size_t)g * Kg;
                double* ap = acc + (size_t)g * Kg;
                for (int k = 0; k < Kg; ++k) ap[k] += xv * wp[k];
              }
          }
        }
        memcpy(y + IDX4(n, p, q, 0, P, Q, K), acc, sizeof(double) * (size_t)K);
      }
      free(acc);
    }
}

/* ---------------------------------------------------------------------------------
 * conv2d pullback.  For every forward term (n,p,q,k,r,s,c) with in-range (h,w):
 *     dx[n,h,w,c]  += dy[n,p,q,k] * w[r,s,c,k]
 *     dw[r,s,c,k]  += x[n,h,w,c]  * dy[n,p,q,k]
 *     db[k]        += dy[n,p,q,k]
 * dx may be NULL (no consumer), dbias may be NULL.  dx and dw are overwritten.
 * Images are independent for dx; dw/db are accumulated per thread over a static
 * partition of the images and the per-thread results added in thread order.
 * --------------------------------------------------------------------------------- */
void orc_conv2d_vjp(const double* x, const double* w, const double* dy, double* dx, double* dw,
                    double* dbias, int N, int H, int W, int C, int K, int R, int S, int stride,
                    int pad, int groups) {
  int P = (H + 2 * pad - R) / stride + 1, Q = (W + 2 * pad - S) / stride + 1;
  int Cg = C / groups, Kg = K / groups;
  size_t wsz = (size_t)R * S * Cg * K;
  int T = orc_num_threads();
  if (T > N) T = N;
  if (T < 1) T = 1;
  double* dw_part = (double*)calloc((size_t)T * wsz, sizeof(double));
  double* db_part = (double*)calloc((size_t)T * K, sizeof(double));
  if (dx) memset(dx, 0, sizeof(double) * (size_t)N * H * W * C);
#pragma omp parallel for schedule(static) num_threads(T)
  for (int t = 0; t < T; ++t) {
    double* dwt = dw_part + (size_t)t * wsz;
    double* dbt = db_part + (size_t)t * K;
    int n0 = (int)(((long)N * t) / T), n1 = (int)(((long)N * (t + 1)) / T);
    for (int n = n0; n < n1; ++n)
      for (int p = 0; p < P; ++p)
        for (int q = 0; q < Q; ++q) {
          const double* dyp = dy + IDX4(n, p, q, 0, P, Q, K);
          for (int k = 0; k < K; ++k) dbt[k] += dyp[k];
          for (int r = 0; r < R; ++r) {
            int h = p * stride + r - pad;
            if (h < 0 || h >= H) continue;
            for (int s = 0; s < S; ++s) {
              int ww = q * stride + s - pad;
              if (ww < 0 || ww >= W) continue;
              for (int g = 0; g < groups; ++g)
                for (int c = 0; c < Cg; ++c) {
                  size_t xi = IDX4(n, h, ww, g * Cg + c, H, W, C);
                  size_t wi = (((size_t)r * S + s) * Cg + c) * K + (size_t)g * Kg;
                  const double* wp = w + wi;
                  const double* dyg = dyp + (size_t)g * Kg;
                  double* dwp = dwt + wi;
                  double xv = x[xi];
                  double sdx = 0.0;
#pragma omp simd reduction(+ : sdx)
                  for (int k = 0; k < Kg; ++k) {
                    sdx += dyg[k] * wp[k];
                    dwp[k] += xv * dyg[k];
                  }
                  if (dx) dx[xi] += sdx;
                }
            }
          }
        }
  }
  for (size_t i = 0; i < wsz; ++i) {
    double s = 0.0;
    for (int t = 0; t < T; ++t) s += dw_part[(size_t)t * wsz + i];
    dw[i] = s;
  }
  if (dbias)
    for (int k = 0; k < K; ++k) {
      double s = 0.0;
      for (int t = 0; t < T; ++t) s += db_part[(size_t)t * K + k];
      dbias[k] = s;
    }
  free(dw_part);
  free(db_part);
}

/* ---------------------------------------------------------------------------------
 * bias + activation (LeNet's conv/dense "activation: relu"):  y = act(x + b[c]).
 * pullback: dx = dy * mask(y);  db[c] = sum dx.   M rows of C channels.
 * --------------------------------------------------------------------------------- */
void orc_bias_act_fwd(const double* x, const double* bias, double* y, size_t M, int C, int act) {
#pragma omp parallel for schedule(static)
  for (size_t m = 0; m < M; ++m)
    for (int c = 0; c < C; ++c)
      y[m * C + c] = act_apply(x[m * C + c] + (bias ? bias[c] : 0.0), act);
}
void orc_bias_act_vjp(const double* y, const double* dy, double* dx, double* dbias, size_t M, int C,
                      int act) {
  if (dbias)
    for (int c = 0; c < C; ++c) dbias[c] = 0.0;
  for (size_t m = 0; m < M; ++m)
    for (int c = 0; c < C; ++c) {
      double d = dy[m * C + c] * act_mask(y[m * C + c], act);
      dx[m * C + c] = d;
      if (dbias) dbias[c] += d;
    }
}

/* ---------------------------------------------------------------------------------
 * BatchNorm (training mode) + optional residual + activation, per channel over
 * m = N*H*W samples:  mu = mean(x), var = mean((x-mu)^2) (biased), invstd = 1/sqrt(var+eps)
 *   xhat = (x-mu)*invstd;  z = gamma*xhat + beta (+ res);  y = act(z)
 * --------------------------------------------------------------------------------- */
void orc_bn_act_fwd(const double* x, const double* res, const double* gamma, const double* beta,
                    double* y, double* save_mean, double* save_invstd, size_t M, int C, double eps,
                    int act) {
  /* channels are independent; they are walked in groups of CB adjacent channels so that each
   * pass over the NHWC tensor uses whole cache lines */
  enum { CB = 8 };
#pragma omp parallel for schedule(dynamic)
  for (int c0 = 0; c0 < C; c0 += CB) {
    int cb = C - c0 < CB ? C - c0 : CB;
    double mu[CB], is[CB], acc[CB];
    for (int j = 0; j < cb; ++j) acc[j] = 0.0;
    for (size_t m = 0; m < M; ++m)
      for (int j = 0; j < cb; ++j) acc[j] += x[m * C + c0 + j];
    for (int j = 0; j < cb; ++j) {
      mu[j] = acc[j] / (double)M;
      acc[j] = 0.0;
    }
    for (size_t m = 0; m < M; ++m)
      for (int j = 0; j < cb; ++j) {
        double d = x[m * C + c0 + j] - mu[j];
        acc[j] += d * d;
      }
    for (int j = 0; j < cb; ++j) {
      is[j] = 1.0 / sqrt(acc[j] / (double)M + eps);
      save_mean[c0 + j] = mu[j];
      save_invstd[c0 + j] = is[j];
    }
    for (size_t m = 0; m < M; ++m)
      for (int j = 0; j < cb; ++j) {
        size_t i = m * C + c0 + j;
        double z = gamma[c0 + j] * ((x[i] - mu[j]) * is[j]) + beta[c0 + j];
        if (res) z += res[i];
        y[i] = act_apply(z, act);
      }
  }
}

/* pullback:  dz = dy*mask(y);  dres = dz;  dbeta = sum dz;  dgamma = sum dz*xhat;
 *            dx = gamma*invstd*(dz - dbeta/m - xhat*dgamma/m)                      */
void orc_bn_act_vjp(const double* x, const double* y, const double* gamma, const double* save_mean,
                    const double* save_invstd, const double* dy, double* dx, double* dres,
                    double* dgamma, double* dbeta, size_t M, int C, int act) {
  enum { CB = 8 };
#pragma omp parallel for schedule(dynamic)
  for (int c0 = 0; c0 < C; c0 += CB) {
    int cb = C - c0 < CB ? C - c0 : CB;
    double sb[CB], sg[CB];
    for (int j = 0; j < cb; ++j) sb[j] = sg[j] = 0.0;
    for (size_t m = 0; m < M; ++m)
      for (int j = 0; j < cb; ++j) {
        size_t i = m * C + c0 + j;
        double dz = dy[i] * act_mask(y[i], act);
        sb[j] += dz;
        sg[j] += dz * ((x[i] - save_mean[c0 + j]) * save_invstd[c0 + j]);
      }
    for (int j = 0; j < cb; ++j) {
      dbeta[c0 + j] = sb[j];
      dgamma[c0 + j] = sg[j];
    }
    for (size_t m = 0; m < M; ++m)
      for (int j = 0; j < cb; ++j) {
        size_t i = m * C + c0 + j;
        double is = save_invstd[c0 + j];
        double dz = dy[i] * act_mask(y[i], act);
        double xh = (x[i] - save_mean[c0 + j]) * is;
        dx[i] = gamma[c0 + j] * is * (dz - sb[j] / (double)M - xh * sg[j] / (double)M);
        if (dres) dres[i] = dz;
      }
  }
}

/* ---------------------------------------------------------------------------------
 * 2x2 stride-2 average pool, no padding (LeNet's AvgPool2D), and its pullback.
 * --------------------------------------------------------------------------------- */
void orc_avgpool2_fwd(const double* x, double* y, int N, int H, int W, int C) {
  int P = H / 2, Q = W / 2;
#pragma omp parallel for schedule(static)
  for (int n = 0; n < N; ++n)
    for (int p = 0; p < P; ++p)
      for (int q = 0; q < Q; ++q)
        for (int c = 0; c < C; ++c) {
          double s = 0.0;
          for (int r = 0; r < 2; ++r)
            for (int t = 0; t < 2; ++t) s += x[IDX4(n, 2 * p + r, 2 * q + t, c, H, W, C)];
          y[IDX4(n, p, q, c, P, Q, C)] = s / 4.0;
        }
}
void orc_avgpool2_vjp(const double* dy, double* dx, int N, int H, int W, int C) {
  int P = H / 2, Q = W / 2;
  memset(dx, 0, sizeof(double) * (size_t)N * H * W * C);
#pragma omp parallel for schedule(static)
  for (int n = 0; n < N; ++n)
    for (int p = 0; p < P; ++p)
      for (int q = 0; q < Q; ++q)
        for (int c = 0; c < C; ++c)
          for (int r = 0; r < 2; ++r)
            for (int t = 0; t < 2; ++t)
              dx[IDX4(n, 2 * p + r, 2 * q + t, c, H, W, C)] += dy[IDX4(n, p, q, c, P, Q, C)] / 4.0;
}

/* ---------------------------------------------------------------------------------
 * 3x3 stride-2 pad-1 max pool.  Padding never wins (treated as -inf).  The pullback
 * routes the whole dy to the first maximum in row-major (r,s) window order.
 * --------------------------------------------------------------------------------- */
void orc_maxpool3s2_fwd(const double* x, double* y, int N, int H, int W, int C) {
  int P = (H + 2 - 3) / 2 + 1, Q = (W + 2 - 3) / 2 + 1;
#pragma omp parallel for schedule(static)
  for (int n = 0; n < N; ++n)
    for (int p = 0; p < P; ++p)
      for (int q = 0; q < Q; ++q)
        for (int c = 0; c < C; ++c) {
          double best = -INFINITY;
          for (int r = 0; r < 3; ++r)
            for (int s = 0; s < 3; ++s) {
              int h = 2 * p + r - 1, w = 2 * q + s - 1;
              if (h < 0 || h >= H || w < 0 || w >= W) continue;
              double v = x[IDX4(n, h, w, c, H, W, C)];
              if (v > best) best = v;
            }
          y[IDX4(n, p, q, c, P, Q, C)] = best;
        }
}
void orc_maxpool3s2_vjp(const double* x, const double* dy, double* dx, int N, int H, int W, int C) {
  int P = (H + 2 - 3) / 2 + 1, Q = (W + 2 - 3) / 2 + 1;
  memset(dx, 0, sizeof(double) * (size_t)N * H * W * C);
#pragma omp parallel for schedule(static)
  for (int n = 0; n < N; ++n)
    for (int p = 0; p < P; ++p)
      for (int q = 0; q < Q; ++q)
        for (int c = 0; c < C; ++c) {
          double best = -INFINITY;
          size_t arg = (size_t)-1;
          for (int r = 0; r < 3; ++r)
            for (int s = 0; s < 3; ++s) {
              int h = 2 * p + r - 1, w = 2 * q + s - 1;
              if (h < 0 || h >= H || w < 0 || w >= W) continue;
              size_t i = IDX4(n, h, w, c, H, W, C);
              if (x[i] > best) {
                best = x[i];
                arg = i;
              }
            }
          if (arg != (size_t)-1) dx[arg] += dy[IDX4(n, p, q, c, P, Q, C)];
        }
}

/* ---------------------------------------------------------------------------------
 * Head: global average pool + dense + mean softmax cross-entropy, value and pullback.
 *   pbar[n,c] = mean_{h,w} x[n,h,w,c];  z = pbar W + b;
 *   L = -(1/N) sum_n log softmax(z_n)[label_n];   dz = (softmax(z) - onehot)/N
 *   dW = pbar^T dz;  db = sum_n dz;  dx[n,h,w,c] = (dz W^T)[n,c] / (H*W)
 * W is [C, classes] (y = xW + b).  logits (nullable) receives z.
 * --------------------------------------------------------------------------------- */
void orc_head_fwd_vjp(const double* x, const double* Wt, const double* b, const int32_t* labels,
                      double* loss, double* dx, double* dW, double* db, double* logits, int N,
                      int H, int W, int C, int classes) {
  size_t HW = (size_t)H * W;
  double* pbar = (double*)calloc((size_t)N * C, sizeof(double));
  double* dz = (double*)calloc((size_t)N * classes, sizeof(double));
  for (int n = 0; n < N; ++n)
    for (size_t i = 0; i < HW; ++i)
      for (int c = 0; c < C; ++c) pbar[(size_t)n * C + c] += x[((size_t)n * HW + i) * C + c];
  for (size_t i = 0; i < (size_t)N * C; ++i) pbar[i] /= (double)HW;
  double L = 0.0;
  for (int n = 0; n < N; ++n) {
    double* z = dz + (size_t)n * classes; /* holds logits first, then the cotangent */
    for (int j = 0; j < classes; ++j) z[j] = b[j];
    for (int c = 0; c < C; ++c) {
      double pv = pbar[(size_t)n * C + c];
      for (int j = 0; j < classes; ++j) z[j] += pv * Wt[(size_t)c * classes + j];
    }
    if (logits) memcpy(logits + (size_t)n * classes, z, sizeof(double) * (size_t)classes);
    double zmax = z[0];
    for (int j = 1; j < classes; ++j)
      if (z[j] > zmax) zmax = z[j];
    double se = 0.0;
    for (int j = 0; j < classes; ++j) se += exp(z[j] - zmax);
    double lse = zmax + log(se);
    L += lse - z[labels[n]];
    for (int j = 0; j < classes; ++j) z[j] = exp(z[j] - lse) / (double)N;
    z[labels[n]] -= 1.0 / (double)N;
  }
  *loss = L / (double)N;
  for (size_t i = 0; i < (size_t)C * classes; ++i) dW[i] = 0.0;
  for (int j = 0; j < classes; ++j) db[j] = 0.0;
  for (int n = 0; n < N; ++n) {
    for (int j = 0; j < classes; ++j) db[j] += dz[(size_t)n * classes + j];
    for (int c = 0; c < C; ++c) {
      double pv = pbar[(size_t)n * C + c];
      double s = 0.0;
      for (int j = 0; j < classes; ++j) {
        dW[(size_t)c * classes + j] += pv * dz[(size_t)n * classes + j];
        s += dz[(size_t)n * classes + j] * Wt[(size_t)c * classes + j];
      }
      if (dx)
        for (size_t i = 0; i < HW; ++i) dx[((size_t)n * HW + i) * C + c] = s / (double)HW;
    }
  }
  free(pbar);
  free(dz);
}

/* ---------------------------------------------------------------------------------
 * SGD with momentum, in place:  v <- mu v + g;  theta <- theta - lr v.
 * --------------------------------------------------------------------------------- */
void orc_sgd_momentum(size_t count, double* param, double* velocity, const double* grad, double lr,
                      double momentum) {
  for (size_t i = 0; i < count; ++i) {
    velocity[i] = momentum * velocity[i] + grad[i];
    param[i] -= lr * velocity[i];
  }
}

/* ---------------------------------------------------------------------------------
 * Indexing and its pullback in the `inout` formulation (the paper's Section 4.3 and the
 * listing of its Appendix B use x[i] as the example: a pullback (T) -> [T] has to build
 * an array of zeros, one of type (T, inout [T]) -> Void adds the cotangent in place).
 *   fwd:  y[j,:] = x[index[j],:]
 *   vjp:  dx[index[j],:] += dy[j,:]  for j = 0, 1, ... in that order; dx is inout and only
 *         the named rows are touched.  An index outside [0, rows) is skipped (y row = 0).
 * --------------------------------------------------------------------------------- */
void orc_gather_rows_fwd(const double* x, const int32_t* index, double* y, int rows, int cols, int count) {
  for (int j = 0; j < count; ++j)
    for (int c = 0; c < cols; ++c)
      y[(size_t)j * cols + c] = (index[j] >= 0 && index[j] < rows) ? x[(size_t)index[j] * cols + c] : 0.0;
}
void orc_gather_rows_vjp(const double* dy, const int32_t* index, double* dx, int rows, int cols, int count) {
  for (int j = 0; j < count; ++j) {
    if (index[j] < 0 || index[j] >= rows) continue;
    for (int c = 0; c < cols; ++c) dx[(size_t)index[j] * cols + c] += dy[(size_t)j * cols + c];
  }
}

/* ---------------------------------------------------------------------------------
 * BatchNorm in inference mode (running statistics instead of batch statistics), the
 * update of the running statistics from a training-mode forward pass, and the folding
 * of an inference-mode BatchNorm into the convolution in front of it.  The paper only
 * mentions starting from trained checkpoints (Section 1); the arithmetic is the usual:
 *   inference:  y = act(gamma (x - rm)/sqrt(rv + eps) + beta (+ res))
 *   update:     rm <- (1-mom) rm + mom mean;  rv <- (1-mom) rv + mom var m/(m-1)
 *               with var = 1/invstd^2 - eps the biased batch variance
 *   fold:       w'[.,k] = w[.,k] s_k,  b'_k = beta_k + (b_k - rm_k) s_k,  s_k = gamma_k/sqrt(rv_k + eps)
 *               so that conv(x, w') + b' = BN_inference(conv(x, w) + b)
 * --------------------------------------------------------------------------------- */
void orc_bn_inference_fwd(const double* x, const double* res, const double* gamma, const double* beta,
                          const double* rm, const double* rv, double* y, size_t M, int C, double eps, int act) {
  for (size_t m = 0; m < M; ++m)
    for (int c = 0; c < C; ++c) {
      double z = gamma[c] * (x[m * C + c] - rm[c]) / sqrt(rv[c] + eps) + beta[c];
      if (res) z += res[m * C + c];
      y[m * C + c] = act_apply(z, act);
    }
}
void orc_bn_update_running(const double* mean, const double* invstd, double* rm, double* rv, int C, size_t M,
                           double momentum, double eps) {
  for (int c = 0; c < C; ++c) {
    double var = 1.0 / (invstd[c] * invstd[c]) - eps;
    double unbiased = M > 1 ? var * (double)M / (double)(M - 1) : var;
    rm[c] = (1.0 - momentum) * rm[c] + momentum * mean[c];
    rv[c] = (1.0 - momentum) * rv[c] + momentum * unbiased;
  }
}
void orc_bn_fold(const double* w, const double* bias, const double* gamma, const double* beta, const double* rm,
                 const double* rv, double* w_out, double* bias_out, size_t rows, int K, double eps) {
  for (int k = 0; k < K; ++k) {
    double s = gamma[k] / sqrt(rv[k] + eps);
    bias_out[k] = beta[k] + ((bias ? bias[k] : 0.0) - rm[k]) * s;
    for (size_t i = 0; i < rows; ++i) w_out[i * K + k] = w[i * K + k] * s;
  }
}
