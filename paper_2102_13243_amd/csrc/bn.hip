// BatchNorm (training mode) + residual + ReLU/ReLU6, forward and pullback, NHWC.
// Every kernel here is bound by HBM bandwidth.  All of them use the same decomposition:
// grid = (channel blocks, pixel chunks); a thread = (channel vector of V adjacent channels,
// pixel lane) keeps its per-channel constants in registers and walks its pixels with 16-byte
// accesses, so a wavefront reads whole contiguous runs of the NHWC tensor.
//   forward   stats: per-channel sum and sum of squares of (x - pivot), pivot = x at pixel 0
//             (keeps the one-pass variance free of cancellation); lanes are added in LDS in a
//             fixed order, chunks are added in double by a finalize kernel -> mean, invstd
//             apply:  y = act(gamma*(x-mean)*invstd + beta (+ residual))
//   pullback  reduce: dbeta = sum dz, dgamma = sum dz*xhat with dz = dy*act'(y)
//             apply:  dx = gamma*invstd*(dz - dbeta/m - xhat*dgamma/m),  dresidual (+)= dz
#include "s4tf_internal.h"
#include "pack.h"

namespace s4tf {
namespace {

struct Plan {
  int V, cvb, cblocks, pl, chunks;
  long long per;  // pixels per chunk
};

Plan make_plan(size_t M, int C, int dtype) {
  Plan p;
  int V = dtype == S4TF_BF16 ? 8 : 4;
  if (C % V) V = 1;
  p.V = V;
  int CV = C / V;
  int cvb = 1;
  while (cvb * 2 <= CV && cvb * 2 <= 64) cvb *= 2;
  p.cvb = cvb;
  p.cblocks = (CV + cvb - 1) / cvb;
  p.pl = 256 / cvb;
  long long want = 2048 / p.cblocks;
  if (want < 1) want = 1;
  long long per = ((long long)M + want - 1) / want;
  long long minper = (long long)p.pl * 4;
  if (per < minper) per = minper;
  p.per = per;
  p.chunks = (int)(((long long)M + per - 1) / per);
  return p;
}

// add the pixel lanes of a block in a fixed order; result valid for pl == 0
template <int NV>
__device__ inline void block_lane_sum(float (&v)[NV], float* red, int cvb, int pl_count, int cvl, int pl) {
  float* mine = red + (size_t)(pl * cvb + cvl) * NV;
#pragma unroll
  for (int e = 0; e < NV; ++e) mine[e] = v[e];
  __syncthreads();
  if (pl == 0) {
#pragma unroll
    for (int e = 0; e < NV; ++e) {
      float s = 0.f;
      for (int l = 0; l < pl_count; ++l) s += red[(size_t)(l * cvb + cvl) * NV + e];
      v[e] = s;
    }
  }
}

template <typename T, int V>
__global__ __launch_bounds__(256) void bn_stats_kernel(const T* __restrict__ x, float* __restrict__ part, long long M,
                                                       int C, int cvb, long long per) {
  extern __shared__ float red[];
  const int CV = C / V, pl_count = blockDim.x / cvb;
  const int cvl = threadIdx.x % cvb, pl = threadIdx.x / cvb;
  const int cv = blockIdx.x * cvb + cvl;
  const bool live = cv < CV;
  const int c = live ? cv * V : 0;
  float acc[2 * V];
#pragma unroll
  for (int e = 0; e < 2 * V; ++e) acc[e] = 0.f;
  Pack<T, V> pv = ldp<T, V>(x + c);
  const long long p0 = (long long)blockIdx.y * per, p1 = p0 + per < M ? p0 + per : M;
  if (live)
    for (long long m = p0 + pl; m < p1; m += pl_count) {
      Pack<T, V> xv = ldp<T, V>(x + m * C + c);
#pragma unroll
      for (int e = 0; e < V; ++e) {
        float d = xv.get(e) - pv.get(e);
        acc[e] += d;
        acc[V + e] += d * d;
      }
    }
  block_lane_sum<2 * V>(acc, red, cvb, pl_count, cvl, pl);
  if (pl == 0 && live) {
    float* dst = part + (long long)blockIdx.y * 2 * C;
#pragma unroll
    for (int e = 0; e < V; ++e) {
      dst[c + e] = acc[e];
      dst[C + c + e] = acc[V + e];
    }
  }
}

template <typename T>
__global__ void bn_stats_finalize_kernel(const T* __restrict__ x, const float* __restrict__ part, int chunks,
                                         long long M, int C, float eps, float* __restrict__ mean,
                                         float* __restrict__ invstd) {
  int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= C) return;
  double s1 = 0.0, s2 = 0.0;
  for (int z = 0; z < chunks; ++z) {
    s1 += (double)part[(long long)z * 2 * C + c];
    s2 += (double)part[(long long)z * 2 * C + C + c];
  }
  double pivot = (double)to_f32<T>(x[c]);
  double ms = s1 / (double)M;
  double var = s2 / (double)M - ms * ms;
  if (var < 0.0) var = 0.0;
  mean[c] = (float)(pivot + ms);
  invstd[c] = (float)(1.0 / sqrt(var + (double)eps));
}

template <typename T, int V>
__global__ __launch_bounds__(256) void bn_apply_kernel(const T* __restrict__ x, const T* __restrict__ res,
                                                       const float* __restrict__ gamma, const float* __restrict__ beta,
                                                       const float* __restrict__ mean, const float* __restrict__ invstd,
                                                       T* __restrict__ y, long long M, int C, int cvb, long long per,
                                                       int act) {
  const int CV = C / V, pl_count = blockDim.x / cvb;
  const int cvl = threadIdx.x % cvb, pl = threadIdx.x / cvb;
  const int cv = blockIdx.x * cvb + cvl;
  if (cv >= CV) return;
  const int c = cv * V;
  float mu[V], sc[V], be[V];
#pragma unroll
  for (int e = 0; e < V; ++e) {
    mu[e] = mean[c + e];
    sc[e] = gamma[c + e] * invstd[c + e];
    be[e] = beta[c + e];
  }
  const long long p0 = (long long)blockIdx.y * per, p1 = p0 + per < M ? p0 + per : M;
  for (long long m = p0 + pl; m < p1; m += pl_count) {
    Pack<T, V> xv = ldp<T, V>(x + m * C + c), o;
    if (res) {
      Pack<T, V> rv = ldp<T, V>(res + m * C + c);
#pragma unroll
      for (int e = 0; e < V; ++e) o.set(e, act_apply((xv.get(e) - mu[e]) * sc[e] + be[e] + rv.get(e), act));
    } else {
#pragma unroll
      for (int e = 0; e < V; ++e) o.set(e, act_apply((xv.get(e) - mu[e]) * sc[e] + be[e], act));
    }
    stp<T, V>(y + m * C + c, o);
  }
}

// dbeta and dgamma are sums of cotangents whose terms largely cancel (the cotangent reaching a
// BatchNorm from a convolution that is itself followed by BatchNorm sums to almost zero), so the
// per-thread and per-block partial sums are kept in double; the kernel stays bandwidth bound.
template <typename T, int V>
__global__ __launch_bounds__(256) void bn_vjp_reduce_kernel(const T* __restrict__ x, const T* __restrict__ y,
                                                            const T* __restrict__ dy, const float* __restrict__ mean,
                                                            const float* __restrict__ invstd, double* __restrict__ part,
                                                            long long M, int C, int cvb, long long per, int act) {
  extern __shared__ double redd[];
  const int CV = C / V, pl_count = blockDim.x / cvb;
  const int cvl = threadIdx.x % cvb, pl = threadIdx.x / cvb;
  const int cv = blockIdx.x * cvb + cvl;
  const bool live = cv < CV;
  const int c = live ? cv * V : 0;
  double acc[2 * V], mu[V], is[V];
#pragma unroll
  for (int e = 0; e < V; ++e) {
    acc[e] = acc[V + e] = 0.0;
    mu[e] = (double)mean[c + e];
    is[e] = (double)invstd[c + e];
  }
  const long long p0 = (long long)blockIdx.y * per, p1 = p0 + per < M ? p0 + per : M;
  if (live)
    for (long long m = p0 + pl; m < p1; m += pl_count) {
      Pack<T, V> xv = ldp<T, V>(x + m * C + c), dv = ldp<T, V>(dy + m * C + c);
      float dz[V];
      if (act != S4TF_ACT_NONE) {
        Pack<T, V> yv = ldp<T, V>(y + m * C + c);
#pragma unroll
        for (int e = 0; e < V; ++e) dz[e] = dv.get(e) * act_mask(yv.get(e), act);
      } else {
#pragma unroll
        for (int e = 0; e < V; ++e) dz[e] = dv.get(e);
      }
#pragma unroll
      for (int e = 0; e < V; ++e) {
        acc[e] += (double)dz[e];
        acc[V + e] += (double)dz[e] * (((double)xv.get(e) - mu[e]) * is[e]);
      }
    }
  double* mine = redd + (size_t)(pl * cvb + cvl) * 2 * V;
#pragma unroll
  for (int e = 0; e < 2 * V; ++e) mine[e] = acc[e];
  __syncthreads();
  if (pl == 0 && live) {
    double* dst = part + (long long)blockIdx.y * 2 * C;
#pragma unroll
    for (int e = 0; e < 2 * V; ++e) {
      double sum = 0.0;
      for (int l = 0; l < pl_count; ++l) sum += redd[(size_t)(l * cvb + cvl) * 2 * V + e];
      if (e < V) dst[c + e] = sum; else dst[C + c + (e - V)] = sum;
    }
  }
}

__global__ void bn_vjp_finalize_kernel(const double* __restrict__ part, int chunks, int C, float* __restrict__ dgamma,
                                       float* __restrict__ dbeta) {
  int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= C) return;
  double s1 = 0.0, s2 = 0.0;
  for (int z = 0; z < chunks; ++z) {
    s1 += part[(long long)z * 2 * C + c];
    s2 += part[(long long)z * 2 * C + C + c];
  }
  dbeta[c] = (float)s1;
  dgamma[c] = (float)s2;
}

template <typename T, int V>
__global__ __launch_bounds__(256) void bn_vjp_apply_kernel(const T* __restrict__ x, const T* __restrict__ y,
                                                           const T* __restrict__ dy, const float* __restrict__ gamma,
                                                           const float* __restrict__ mean, const float* __restrict__ invstd,
                                                           const float* __restrict__ dgamma, const float* __restrict__ dbeta,
                                                           T* __restrict__ dx, T* __restrict__ dres, int acc_dres,
                                                           long long M, int C, int cvb, long long per, int act) {
  const int CV = C / V, pl_count = blockDim.x / cvb;
  const int cvl = threadIdx.x % cvb, pl = threadIdx.x / cvb;
  const int cv = blockIdx.x * cvb + cvl;
  if (cv >= CV) return;
  const int c = cv * V;
  const float invM = 1.0f / (float)M;
  float mu[V], is[V], gs[V], mb[V], mg[V];
#pragma unroll
  for (int e = 0; e < V; ++e) {
    mu[e] = mean[c + e];
    is[e] = invstd[c + e];
    gs[e] = gamma[c + e] * is[e];
    mb[e] = dbeta[c + e] * invM;
    mg[e] = dgamma[c + e] * invM;
  }
  const long long p0 = (long long)blockIdx.y * per, p1 = p0 + per < M ? p0 + per : M;
  for (long long m = p0 + pl; m < p1; m += pl_count) {
    Pack<T, V> xv = ldp<T, V>(x + m * C + c), dv = ldp<T, V>(dy + m * C + c), o, r;
    float dz[V];
    if (act != S4TF_ACT_NONE) {
      Pack<T, V> yv = ldp<T, V>(y + m * C + c);
#pragma unroll
      for (int e = 0; e < V; ++e) dz[e] = dv.get(e) * act_mask(yv.get(e), act);
    } else {
#pragma unroll
      for (int e = 0; e < V; ++e) dz[e] = dv.get(e);
    }
#pragma unroll
    for (int e = 0; e < V; ++e) o.set(e, gs[e] * (dz[e] - mb[e] - (xv.get(e) - mu[e]) * is[e] * mg[e]));
    stp<T, V>(dx + m * C + c, o);
    if (dres) {
      if (acc_dres) {
        Pack<T, V> old = ldp<T, V>(dres + m * C + c);
#pragma unroll
        for (int e = 0; e < V; ++e) r.set(e, old.get(e) + dz[e]);
      } else {
#pragma unroll
        for (int e = 0; e < V; ++e) r.set(e, dz[e]);
      }
      stp<T, V>(dres + m * C + c, r);
    }
  }
}

constexpr int MAX_CHUNKS = 2048;

}  // namespace

size_t bn_workspace(size_t M, int C) {
  (void)M;
  return (size_t)MAX_CHUNKS * 2 * C * sizeof(double);
}

int bn_fwd(const s4tf_bn_desc& d, const void* x, const void* res, const float* gamma, const float* beta,
           void* y, float* mean, float* invstd, void* ws, hipStream_t st) {
  const long long M = (long long)d.n * d.h * d.w;
  const int C = d.c;
  Plan p = make_plan((size_t)M, C, d.dtype);
  float* part = static_cast<float*>(ws);
  dim3 grid(p.cblocks, p.chunks), block(256);
  {
    ProfScope ps(PC_BN_STATS, st);
    size_t shm = (size_t)256 * 2 * p.V * sizeof(float);
#define XT(T) (const T*)x
    if (d.dtype == S4TF_BF16) {
      if (p.V == 8) hipLaunchKernelGGL((bn_stats_kernel<bf16_t, 8>), grid, block, shm, st, XT(bf16_t), part, M, C, p.cvb, p.per);
      else hipLaunchKernelGGL((bn_stats_kernel<bf16_t, 1>), grid, block, shm, st, XT(bf16_t), part, M, C, p.cvb, p.per);
    } else {
      if (p.V == 4) hipLaunchKernelGGL((bn_stats_kernel<float, 4>), grid, block, shm, st, XT(float), part, M, C, p.cvb, p.per);
      else hipLaunchKernelGGL((bn_stats_kernel<float, 1>), grid, block, shm, st, XT(float), part, M, C, p.cvb, p.per);
    }
    int rc = launch_status("bn_stats");
    if (rc != S4TF_OK) return rc;
    if (d.dtype == S4TF_BF16)
      hipLaunchKernelGGL((bn_stats_finalize_kernel<bf16_t>), dim3((C + 63) / 64), dim3(64), 0, st, XT(bf16_t), part, p.chunks, M, C, d.eps, mean, invstd);
    else
      hipLaunchKernelGGL((bn_stats_finalize_kernel<float>), dim3((C + 63) / 64), dim3(64), 0, st, XT(float), part, p.chunks, M, C, d.eps, mean, invstd);
    rc = launch_status("bn_stats_finalize");
    if (rc != S4TF_OK) return rc;
  }
  ProfScope ps(PC_BN_APPLY, st);
  size_t shm = 0;
  if (d.dtype == S4TF_BF16) {
    typedef bf16_t T;
    if (p.V == 8) hipLaunchKernelGGL((bn_apply_kernel<T, 8>), grid, block, shm, st, (const T*)x, (const T*)res, gamma, beta, mean, invstd, (T*)y, M, C, p.cvb, p.per, d.act);
    else hipLaunchKernelGGL((bn_apply_kernel<T, 1>), grid, block, shm, st, (const T*)x, (const T*)res, gamma, beta, mean, invstd, (T*)y, M, C, p.cvb, p.per, d.act);
  } else {
    typedef float T;
    if (p.V == 4) hipLaunchKernelGGL((bn_apply_kernel<T, 4>), grid, block, shm, st, (const T*)x, (const T*)res, gamma, beta, mean, invstd, (T*)y, M, C, p.cvb, p.per, d.act);
    else hipLaunchKernelGGL((bn_apply_kernel<T, 1>), grid, block, shm, st, (const T*)x, (const T*)res, gamma, beta, mean, invstd, (T*)y, M, C, p.cvb, p.per, d.act);
  }
  return launch_status("bn_apply");
}

int bn_vjp(const s4tf_bn_desc& d, const void* x, const void* y, const float* gamma, const float* mean,
           const float* invstd, const void* dy, void* dx, void* dres, float* dgamma, float* dbeta,
           void* ws, hipStream_t st) {
  const long long M = (long long)d.n * d.h * d.w;
  const int C = d.c;
  Plan p = make_plan((size_t)M, C, d.dtype);
  double* part = static_cast<double*>(ws);
  dim3 grid(p.cblocks, p.chunks), block(256);
  {
    ProfScope ps(PC_BN_VJP_REDUCE, st);
    size_t shm = (size_t)256 * 2 * p.V * sizeof(double);
    if (d.dtype == S4TF_BF16) {
      typedef bf16_t T;
      if (p.V == 8) hipLaunchKernelGGL((bn_vjp_reduce_kernel<T, 8>), grid, block, shm, st, (const T*)x, (const T*)y, (const T*)dy, mean, invstd, part, M, C, p.cvb, p.per, d.act);
      else hipLaunchKernelGGL((bn_vjp_reduce_kernel<T, 1>), grid, block, shm, st, (const T*)x, (const T*)y, (const T*)dy, mean, invstd, part, M, C, p.cvb, p.per, d.act);
    } else {
      typedef float T;
      if (p.V == 4) hipLaunchKernelGGL((bn_vjp_reduce_kernel<T, 4>), grid, block, shm, st, (const T*)x, (const T*)y, (const T*)dy, mean, invstd, part, M, C, p.cvb, p.per, d.act);
      else hipLaunchKernelGGL((bn_vjp_reduce_kernel<T, 1>), grid, block, shm, st, (const T*)x, (const T*)y, (const T*)dy, mean, invstd, part, M, C, p.cvb, p.per, d.act);
    }
    int rc = launch_status("bn_vjp_reduce");
    if (rc != S4TF_OK) return rc;
    hipLaunchKernelGGL(bn_vjp_finalize_kernel, dim3((C + 63) / 64), dim3(64), 0, st, part, p.chunks, C, dgamma, dbeta);
    rc = launch_status("bn_vjp_finalize");
    if (rc != S4TF_OK) return rc;
  }
  ProfScope ps(PC_BN_VJP_APPLY, st);
  size_t shm = 0;
  if (d.dtype == S4TF_BF16) {
    typedef bf16_t T;
    if (p.V == 8) hipLaunchKernelGGL((bn_vjp_apply_kernel<T, 8>), grid, block, shm, st, (const T*)x, (const T*)y, (const T*)dy, gamma, mean, invstd, dgamma, dbeta, (T*)dx, (T*)dres, d.accumulate_dres, M, C, p.cvb, p.per, d.act);
    else hipLaunchKernelGGL((bn_vjp_apply_kernel<T, 1>), grid, block, shm, st, (const T*)x, (const T*)y, (const T*)dy, gamma, mean, invstd, dgamma, dbeta, (T*)dx, (T*)dres, d.accumulate_dres, M, C, p.cvb, p.per, d.act);
  } else {
    typedef float T;
    if (p.V == 4) hipLaunchKernelGGL((bn_vjp_apply_kernel<T, 4>), grid, block, shm, st, (const T*)x, (const T*)y, (const T*)dy, gamma, mean, invstd, dgamma, dbeta, (T*)dx, (T*)dres, d.accumulate_dres, M, C, p.cvb, p.per, d.act);
    else hipLaunchKernelGGL((bn_vjp_apply_kernel<T, 1>), grid, block, shm, st, (const T*)x, (const T*)y, (const T*)dy, gamma, mean, invstd, dgamma, dbeta, (T*)dx, (T*)dres, d.accumulate_dres, M, C, p.cvb, p.per, d.act);
  }
  return launch_status("bn_vjp_apply");
}

}  // namespace s4tf
