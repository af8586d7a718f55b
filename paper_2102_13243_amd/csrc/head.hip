// Head of the network: global average pool + dense + mean softmax cross-entropy, value and
// pullback in one call (`softmaxCrossEntropy(logits:labels:)` of the paper's training loop).
// Small and latency bound.  The dense part is three tiny GEMMs that reuse the implicit-GEMM
// kernels in fp32 on the pooled [n,1,1,c] tensor; the rest are reductions done in a fixed order.
//   pbar = mean_{h,w} x;  z = pbar W + b;  loss = mean_n (logsumexp(z_n) - z_n[label_n])
//   dz = (softmax(z) - onehot)/n;  dW = pbar^T dz;  db = sum_n dz;  dx = (dz W^T)/(h*w)
#include "s4tf_internal.h"

namespace s4tf {
namespace {

template <typename T>
__global__ void gap_kernel(const T* __restrict__ x, float* __restrict__ pbar, int N, int HW, int C) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;  // (n, c)
  if (i >= N * C) return;
  int c = i % C, n = i / C;
  const T* p = x + (long long)n * HW * C + c;
  float s = 0.f;
  for (int j = 0; j < HW; ++j) s += to_f32<T>(p[(long long)j * C]);
  pbar[i] = s / (float)HW;
}

// one block per sample: max, sum of exponentials, loss term, dz.  256 threads, fixed tree order.
__global__ __launch_bounds__(256) void softmax_xent_kernel(const float* __restrict__ z, const int32_t* __restrict__ labels,
                                                           float* __restrict__ dz, float* __restrict__ rowloss, int N,
                                                           int K) {
  __shared__ float red[256];
  const int n = blockIdx.x, t = threadIdx.x;
  const float* zr = z + (long long)n * K;
  float m = -INFINITY;
  for (int j = t; j < K; j += 256) m = fmaxf(m, zr[j]);
  red[t] = m;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if (t < s) red[t] = fmaxf(red[t], red[t + s]);
    __syncthreads();
  }
  m = red[0];
  __syncthreads();
  float se = 0.f;
  for (int j = t; j < K; j += 256) se += expf(zr[j] - m);
  red[t] = se;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if (t < s) red[t] += red[t + s];
    __syncthreads();
  }
  const float lse = m + logf(red[0]);
  const int lab = labels[n];
  const float invN = 1.0f / (float)N;
  for (int j = t; j < K; j += 256) {
    float p = expf(zr[j] - lse);
    dz[(long long)n * K + j] = (p - (j == lab ? 1.f : 0.f)) * invN;
  }
  if (t == 0) rowloss[n] = (lab >= 0 && lab < K) ? lse - zr[lab] : 0.f;
}

__global__ void mean_loss_kernel(const float* __restrict__ rowloss, float* __restrict__ loss, int N) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    double s = 0.0;
    for (int n = 0; n < N; ++n) s += (double)rowloss[n];
    *loss = (float)(s / (double)N);
  }
}

template <typename T>
__global__ void gap_vjp_kernel(const float* __restrict__ dpbar, T* __restrict__ dx, int N, int HW, int C) {
  const long long total = (long long)N * HW * C;
  const float inv = 1.0f / (float)HW;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
    int c = (int)(i % C);
    int n = (int)(i / ((long long)HW * C));
    dx[i] = from_f32<T>(dpbar[(long long)n * C + c] * inv);
  }
}

ConvGeom dense_geom(int N, int C, int K) {
  ConvGeom g;
  g.N = N; g.H = 1; g.W = 1; g.C = C; g.K = K; g.R = 1; g.S = 1; g.stride = 1; g.pad = 0; g.P = 1; g.Q = 1;
  return g;
}

struct Layout {
  size_t pbar, logits, dz, rowloss, dpbar, wg, total;
};
Layout layout(const s4tf_head_desc& d) {
  Layout l;
  size_t o = 0;
  l.pbar = o; o += align_up((size_t)d.n * d.c * 4, 256);
  l.logits = o; o += align_up((size_t)d.n * d.classes * 4, 256);
  l.dz = o; o += align_up((size_t)d.n * d.classes * 4, 256);
  l.rowloss = o; o += align_up((size_t)d.n * 4, 256);
  l.dpbar = o; o += align_up((size_t)d.n * d.c * 4, 256);
  l.wg = o; o += align_up(igemm_wgrad_workspace(dense_geom(d.n, d.c, d.classes), S4TF_F32), 256);
  l.total = o;
  return l;
}

}  // namespace

size_t head_workspace(const s4tf_head_desc& d) { return layout(d).total; }

int head_fwd_vjp(const s4tf_head_desc& d, const void* x, const float* W, const float* b,
                 const int32_t* labels, float* loss, void* dx, float* dW, float* db, float* logits_out,
                 void* ws, hipStream_t st) {
  Layout l = layout(d);
  char* base = static_cast<char*>(ws);
  float* pbar = reinterpret_cast<float*>(base + l.pbar);
  float* logits = logits_out ? logits_out : reinterpret_cast<float*>(base + l.logits);
  float* dz = reinterpret_cast<float*>(base + l.dz);
  float* rowloss = reinterpret_cast<float*>(base + l.rowloss);
  float* dpbar = reinterpret_cast<float*>(base + l.dpbar);
  const int HW = d.h * d.w;
  ConvGeom g = dense_geom(d.n, d.c, d.classes);
  int rc;
  {
    ProfScope ps(PC_HEAD, st);
    int total = d.n * d.c;
    if (d.dtype == S4TF_BF16)
      hipLaunchKernelGGL(gap_kernel<bf16_t>, dim3((total + 255) / 256), dim3(256), 0, st, (const bf16_t*)x, pbar, d.n, HW, d.c);
    else
      hipLaunchKernelGGL(gap_kernel<float>, dim3((total + 255) / 256), dim3(256), 0, st, (const float*)x, pbar, d.n, HW, d.c);
    if ((rc = launch_status("gap")) != S4TF_OK) return rc;
  }
  if ((rc = igemm_fwd(g, S4TF_F32, pbar, W, b, S4TF_ACT_NONE, logits, st)) != S4TF_OK) return rc;
  {
    ProfScope ps(PC_HEAD, st);
    hipLaunchKernelGGL(softmax_xent_kernel, dim3(d.n), dim3(256), 0, st, logits, labels, dz, rowloss, d.n, d.classes);
    if ((rc = launch_status("softmax_xent")) != S4TF_OK) return rc;
    hipLaunchKernelGGL(mean_loss_kernel, dim3(1), dim3(64), 0, st, rowloss, loss, d.n);
    if ((rc = launch_status("mean_loss")) != S4TF_OK) return rc;
  }
  if ((rc = igemm_wgrad(g, S4TF_F32, pbar, dz, dW, base + l.wg, l.total - l.wg, st)) != S4TF_OK) return rc;
  if ((rc = colsum(S4TF_F32, dz, (size_t)d.n, d.classes, db, st)) != S4TF_OK) return rc;
  if (dx) {
    if ((rc = igemm_dgrad(g, S4TF_F32, dz, W, dpbar, 0, st)) != S4TF_OK) return rc;
    ProfScope ps(PC_HEAD, st);
    long long total = (long long)d.n * HW * d.c;
    long long blocks = (total + 255) / 256;
    if (blocks > 16384) blocks = 16384;
    if (d.dtype == S4TF_BF16)
      hipLaunchKernelGGL(gap_vjp_kernel<bf16_t>, dim3((unsigned)blocks), dim3(256), 0, st, dpbar, (bf16_t*)dx, d.n, HW, d.c);
    else
      hipLaunchKernelGGL(gap_vjp_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, st, dpbar, (float*)dx, d.n, HW, d.c);
    if ((rc = launch_status("gap_vjp")) != S4TF_OK) return rc;
  }
  return S4TF_OK;
}

}  // namespace s4tf
