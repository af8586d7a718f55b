// Head of the network: global average pool + dense + mean softmax cross-entropy, value and
// pullback in one call (`softmaxCrossEntropy(logits:labels:)` of the paper's training loop).
// Small and latency bound.  The dense part is three tiny fp32 GEMMs on the pooled [n,c] matrix.  The two
// with few rows (logits, and the cotangent of the pooled features) would fill a handful of 128x128
// tiles, so they run as split-k register-tiled GEMMs over ~256 workgroups whose partial sums the next
// kernel in line adds up in a fixed order; dW reuses the implicit-GEMM wgrad kernel.
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

// part[s][m][j] = sum over the k of split s of A[m][k] * Bm(k, j), with Bm(k, j) = B[k][j] (B is [K][J]) or,
// BT, B[j][k] (B is [J][K]).  64x64 outputs per workgroup, 4x4 per thread, 32 k per LDS step.
constexpr int SK_T = 64, SK_KC = 32;
template <bool BT>
__global__ __launch_bounds__(256) void skinny_gemm_kernel(const float* __restrict__ A, const float* __restrict__ B,
                                                          float* __restrict__ part, int M, int J, int K, int kper) {
  __shared__ float As[SK_KC][SK_T + 4], Bs[SK_KC][SK_T + 4];
  const int t = threadIdx.x, tx = t & 15, ty = t >> 4;
  const int j0 = blockIdx.x * SK_T, m0 = blockIdx.z * SK_T;
  const int k0 = blockIdx.y * kper, k1 = min(K, k0 + kper);
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
  for (int kb = k0; kb < k1; kb += SK_KC) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {  // A[m][k]: k fastest
      const int k = t & 31, m = (t >> 5) + 8 * i;
      As[k][m] = (m0 + m < M && kb + k < k1) ? A[(long long)(m0 + m) * K + kb + k] : 0.f;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (BT) {
        const int k = t & 31, j = (t >> 5) + 8 * i;
        Bs[k][j] = (j0 + j < J && kb + k < k1) ? B[(long long)(j0 + j) * K + kb + k] : 0.f;
      } else {
        const int j = t & 63, k = (t >> 6) + 4 * i;
        Bs[k][j] = (j0 + j < J && kb + k < k1) ? B[(long long)(kb + k) * J + j0 + j] : 0.f;
      }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < SK_KC; ++k) {
      const float4 a = *reinterpret_cast<const float4*>(&As[k][ty * 4]);
      const float4 b = *reinterpret_cast<const float4*>(&Bs[k][tx * 4]);
      const float av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += av[i] * bv[j];
    }
    __syncthreads();
  }
  float* dst = part + (long long)blockIdx.y * M * J;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int col = j0 + tx * 4 + j;
      if (col < J) dst[(long long)m * J + col] = acc[i][j];
    }
  }
}

struct SkinnyPlan { int splits, kper; dim3 grid; };
SkinnyPlan skinny_plan(int M, int J, int K) {
  SkinnyPlan p;
  const int jt = (J + SK_T - 1) / SK_T, mt = (M + SK_T - 1) / SK_T;
  int want = 256 / (jt * mt);
  const int maxs = (K + SK_KC - 1) / SK_KC;
  if (want > maxs) want = maxs;
  if (want < 1) want = 1;
  p.kper = ((K + want - 1) / want + SK_KC - 1) / SK_KC * SK_KC;
  p.splits = (K + p.kper - 1) / p.kper;
  p.grid = dim3(jt, p.splits, mt);
  return p;
}

// one block per sample: logits (the split-k partial sums, added in order, plus bias), max, sum of
// exponentials, loss term, dz.  256 threads, fixed tree order; a thread meets the same classes in
// every phase, so it reads back only logits it wrote itself.
__global__ __launch_bounds__(256) void softmax_xent_kernel(const float* __restrict__ part, int splits,
                                                           const float* __restrict__ bias, float* __restrict__ z,
                                                           const int32_t* __restrict__ labels, float* __restrict__ dz,
                                                           float* __restrict__ rowloss, int N, int K) {
  __shared__ float red[256];
  const int n = blockIdx.x, t = threadIdx.x;
  float* zr = z + (long long)n * K;
  float m = -INFINITY;
  for (int j = t; j < K; j += 256) {
    float v = 0.f;
    for (int s = 0; s < splits; ++s) v += part[((long long)s * N + n) * K + j];
    v += bias[j];
    zr[j] = v;
    m = fmaxf(m, v);
  }
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
  const bool valid = lab >= 0 && lab < K;
  const float invN = 1.0f / (float)N;
  for (int j = t; j < K; j += 256) {
    float p = expf(zr[j] - lse);
    dz[(long long)n * K + j] = (p - (j == lab ? 1.f : 0.f)) * invN;
    if (j == lab) rowloss[n] = lse - zr[j];
  }
  if (!valid && t == 0) rowloss[n] = 0.f;
}

__global__ void mean_loss_kernel(const float* __restrict__ rowloss, float* __restrict__ loss, int N) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    double s = 0.0;
    for (int n = 0; n < N; ++n) s += (double)rowloss[n];
    *loss = (float)(s / (double)N);
  }
}

// dx[n][hw][c] = (sum over splits of part[s][n][c]) / HW: one thread per (n, c) walks the pixels
// (accumulate: added to what dx holds, one rounding of the sum per element)
template <typename T>
__global__ void gap_vjp_kernel(const float* __restrict__ part, int splits, T* dx, int N, int HW, int C, int accumulate) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= N * C) return;
  const int c = i % C, n = i / C;
  float v = 0.f;
  for (int s = 0; s < splits; ++s) v += part[(long long)s * N * C + i];
  v /= (float)HW;
  const T o = from_f32<T>(v);
  T* p = dx + (long long)n * HW * C + c;
  if (accumulate)
    for (int j = 0; j < HW; ++j) p[(long long)j * C] = from_f32<T>(to_f32<T>(p[(long long)j * C]) + v);
  else
    for (int j = 0; j < HW; ++j) p[(long long)j * C] = o;
}

ConvGeom dense_geom(int N, int C, int K) {
  ConvGeom g;
  g.N = N; g.H = 1; g.W = 1; g.C = C; g.K = K; g.R = 1; g.S = 1; g.stride = 1; g.pad = 0; g.P = 1; g.Q = 1;
  return g;
}

struct Layout {
  size_t pbar, logits, dz, rowloss, part, wg, total;  // part: split-k partial sums of either skinny GEMM
};
Layout layout(const s4tf_head_desc& d) {
  Layout l;
  size_t o = 0;
  l.pbar = o; o += align_up((size_t)d.n * d.c * 4, 256);
  l.logits = o; o += align_up((size_t)d.n * d.classes * 4, 256);
  l.dz = o; o += align_up((size_t)d.n * d.classes * 4, 256);
  l.rowloss = o; o += align_up((size_t)d.n * 4, 256);
  const size_t pf = (size_t)skinny_plan(d.n, d.classes, d.c).splits * d.n * d.classes;
  const size_t pb = (size_t)skinny_plan(d.n, d.c, d.classes).splits * d.n * d.c;
  l.part = o; o += align_up((pf > pb ? pf : pb) * 4, 256);
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
  float* part = reinterpret_cast<float*>(base + l.part);
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
  {
    ProfScope ps(PC_HEAD, st);
    const SkinnyPlan sp = skinny_plan(d.n, d.classes, d.c);
    hipLaunchKernelGGL(skinny_gemm_kernel<false>, sp.grid, dim3(256), 0, st, pbar, W, part, d.n, d.classes, d.c, sp.kper);
    if ((rc = launch_status("head logits")) != S4TF_OK) return rc;
    hipLaunchKernelGGL(softmax_xent_kernel, dim3(d.n), dim3(256), 0, st, part, sp.splits, b, logits, labels, dz, rowloss, d.n, d.classes);
    if ((rc = launch_status("softmax_xent")) != S4TF_OK) return rc;
    hipLaunchKernelGGL(mean_loss_kernel, dim3(1), dim3(64), 0, st, rowloss, loss, d.n);
    if ((rc = launch_status("mean_loss")) != S4TF_OK) return rc;
  }
  if ((rc = igemm_wgrad(g, S4TF_F32, pbar, dz, dW, base + l.wg, l.total - l.wg, st)) != S4TF_OK) return rc;
  if ((rc = colsum(S4TF_F32, dz, (size_t)d.n, d.classes, db, st)) != S4TF_OK) return rc;
  if (dx) {
    ProfScope ps(PC_HEAD, st);
    const SkinnyPlan sp = skinny_plan(d.n, d.c, d.classes);  // dpbar[n][c] = sum_j dz[n][j] W[c][j]
    hipLaunchKernelGGL(skinny_gemm_kernel<true>, sp.grid, dim3(256), 0, st, dz, W, part, d.n, d.c, d.classes, sp.kper);
    if ((rc = launch_status("head dpbar")) != S4TF_OK) return rc;
    const unsigned blocks = (unsigned)(((long long)d.n * d.c + 255) / 256);
    if (d.dtype == S4TF_BF16)
      hipLaunchKernelGGL(gap_vjp_kernel<bf16_t>, dim3(blocks), dim3(256), 0, st, part, sp.splits, (bf16_t*)dx, d.n, HW, d.c, d.accumulate_dx);
    else
      hipLaunchKernelGGL(gap_vjp_kernel<float>, dim3(blocks), dim3(256), 0, st, part, sp.splits, (float*)dx, d.n, HW, d.c, d.accumulate_dx);
    if ((rc = launch_status("gap_vjp")) != S4TF_OK) return rc;
  }
  return S4TF_OK;
}

}  // namespace s4tf
