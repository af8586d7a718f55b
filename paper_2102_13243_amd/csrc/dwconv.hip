// Depthwise convolution (groups == C == K), NHWC, filters (R,S,1,C).  One multiply-add per
// loaded element: bound by HBM bandwidth, so there is no MFMA here.  Threads own VEC adjacent
// channels of one pixel (16-byte accesses, channel fastest => fully coalesced); the R*S taps
// of neighbouring pixels overlap and are served by the vector L1 / L2.
//   fwd    y [n,p,q,c] = act(b[c] + sum_{r,s} x[n,p*st+r-pad,q*st+s-pad,c] w[r,s,c])
//   dgrad  dx[n,h,w,c] = sum_{r,s} dy[n,(h+pad-r)/st,(w+pad-s)/st,c] w[r,s,c]   (integer quotients)
//   wgrad  dw[r,s,c]   = sum_{n,p,q} x[n,p*st+r-pad,q*st+s-pad,c] dy[n,p,q,c]
#include "s4tf_internal.h"
#include "pack.h"

namespace s4tf {
namespace {

template <typename T, int V>
__global__ __launch_bounds__(256) void dw_fwd_kernel(ConvGeom g, const T* __restrict__ x, const T* __restrict__ w,
                                                     const float* __restrict__ bias, int act, T* __restrict__ y,
                                                     long long total) {
  const int CV = g.C / V;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (long long)gridDim.x * blockDim.x) {
    int c = (int)(i % CV) * V;
    long long pix = i / CV;
    int q = (int)(pix % g.Q);
    long long t = pix / g.Q;
    int p = (int)(t % g.P), n = (int)(t / g.P);
    float acc[V];
#pragma unroll
    for (int e = 0; e < V; ++e) acc[e] = bias ? bias[c + e] : 0.f;
    for (int r = 0; r < g.R; ++r) {
      int h = p * g.stride + r - g.pad;
      if (h < 0 || h >= g.H) continue;
      for (int s = 0; s < g.S; ++s) {
        int ww = q * g.stride + s - g.pad;
        if (ww < 0 || ww >= g.W) continue;
        Pack<T, V> xv = ldp<T, V>(x + (((long long)n * g.H + h) * g.W + ww) * g.C + c);
        Pack<T, V> wv = ldp<T, V>(w + (long long)(r * g.S + s) * g.C + c);
#pragma unroll
        for (int e = 0; e < V; ++e) acc[e] += xv.get(e) * wv.get(e);
      }
    }
    Pack<T, V> o;
#pragma unroll
    for (int e = 0; e < V; ++e) o.set(e, act_apply(acc[e], act));
    stp<T, V>(y + pix * g.C + c, o);
  }
}

template <typename T, int V>
__global__ __launch_bounds__(256) void dw_dgrad_kernel(ConvGeom g, const T* __restrict__ dy, const T* __restrict__ w,
                                                       T* __restrict__ dx, int accumulate, long long total) {
  const int CV = g.C / V;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (long long)gridDim.x * blockDim.x) {
    int c = (int)(i % CV) * V;
    long long pix = i / CV;
    int ww = (int)(pix % g.W);
    long long t = pix / g.W;
    int h = (int)(t % g.H), n = (int)(t / g.H);
    float acc[V];
#pragma unroll
    for (int e = 0; e < V; ++e) acc[e] = 0.f;
    for (int r = 0; r < g.R; ++r) {
      int hp = h + g.pad - r;
      if (hp < 0) continue;
      int p = hp / g.stride;
      if (p * g.stride != hp || p >= g.P) continue;
      for (int s = 0; s < g.S; ++s) {
        int wp = ww + g.pad - s;
        if (wp < 0) continue;
        int q = wp / g.stride;
        if (q * g.stride != wp || q >= g.Q) continue;
        Pack<T, V> dv = ldp<T, V>(dy + (((long long)n * g.P + p) * g.Q + q) * g.C + c);
        Pack<T, V> wv = ldp<T, V>(w + (long long)(r * g.S + s) * g.C + c);
#pragma unroll
        for (int e = 0; e < V; ++e) acc[e] += dv.get(e) * wv.get(e);
      }
    }
    T* dst = dx + pix * g.C + c;
    Pack<T, V> o;
    if (accumulate) {
      Pack<T, V> old = ldp<T, V>(dst);
#pragma unroll
      for (int e = 0; e < V; ++e) acc[e] += old.get(e);
    }
#pragma unroll
    for (int e = 0; e < V; ++e) o.set(e, acc[e]);
    stp<T, V>(dst, o);
  }
}

// wgrad stage 1: grid (channel blocks, pixel chunks).  Thread = (channel vector cv, pixel lane pl);
// it accumulates R*S*V sums over its pixels, the block adds the pixel lanes in LDS in a fixed
// order and writes one partial [R*S][C] slab per pixel chunk.  Stage 2 adds the slabs in order.
constexpr int DW_MAX_TAPS = 9;
template <typename T, int V>
__global__ __launch_bounds__(256) void dw_wgrad_kernel(ConvGeom g, const T* __restrict__ x, const T* __restrict__ dy,
                                                       float* __restrict__ part, int cvb, long long pix_per_chunk) {
  extern __shared__ float red[];
  const int CV = g.C / V;
  const int pl_count = blockDim.x / cvb;
  const int cvl = threadIdx.x % cvb, pl = threadIdx.x / cvb;
  const int cv = blockIdx.x * cvb + cvl;
  const int taps = g.R * g.S;
  float acc[DW_MAX_TAPS][V];
#pragma unroll
  for (int t = 0; t < DW_MAX_TAPS; ++t)
#pragma unroll
    for (int e = 0; e < V; ++e) acc[t][e] = 0.f;
  const long long total = (long long)g.N * g.P * g.Q;
  const long long p0 = (long long)blockIdx.y * pix_per_chunk;
  const long long p1 = p0 + pix_per_chunk < total ? p0 + pix_per_chunk : total;
  if (cv < CV && pl < pl_count) {
    const int c = cv * V;
    for (long long pix = p0 + pl; pix < p1; pix += pl_count) {
      int q = (int)(pix % g.Q);
      long long t = pix / g.Q;
      int p = (int)(t % g.P), n = (int)(t / g.P);
      Pack<T, V> dv = ldp<T, V>(dy + pix * g.C + c);
#pragma unroll
      for (int r = 0; r < 3; ++r) {
        if (r >= g.R) break;
        int h = p * g.stride + r - g.pad;
        if (h < 0 || h >= g.H) continue;
#pragma unroll
        for (int s = 0; s < 3; ++s) {
          if (s >= g.S) break;
          int ww = q * g.stride + s - g.pad;
          if (ww < 0 || ww >= g.W) continue;
          Pack<T, V> xv = ldp<T, V>(x + (((long long)n * g.H + h) * g.W + ww) * g.C + c);
#pragma unroll
          for (int e = 0; e < V; ++e) acc[r * 3 + s][e] += xv.get(e) * dv.get(e);
        }
      }
    }
  }
  // one tap at a time: red[pl][cvl][e], summed over pl in a fixed order by pixel lane 0
  for (int r = 0; r < g.R; ++r)
    for (int s = 0; s < g.S; ++s) {
      const int t = r * 3 + s;
      float* mine = red + (size_t)(pl * cvb + cvl) * V;
#pragma unroll
      for (int e = 0; e < V; ++e) {
        float val = 0.f;
#pragma unroll
        for (int tt = 0; tt < DW_MAX_TAPS; ++tt)
          if (tt == t) val = acc[tt][e];
        mine[e] = val;
      }
      __syncthreads();
      if (pl == 0 && cv < CV) {
        for (int e = 0; e < V; ++e) {
          float sum = 0.f;
          for (int l = 0; l < pl_count; ++l) sum += red[(size_t)(l * cvb + cvl) * V + e];
          part[((long long)blockIdx.y * taps + (r * g.S + s)) * g.C + cv * V + e] = sum;
        }
      }
      __syncthreads();
    }
}

__global__ void dw_wgrad_reduce_kernel(const float* __restrict__ part, float* __restrict__ dw, int n, int chunks) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float s = 0.f;
  for (int z = 0; z < chunks; ++z) s += part[(long long)z * n + i];
  dw[i] = s;
}

int grid_for(long long total) {
  long long b = (total + 255) / 256;
  if (b > 256 * 32) b = 256 * 32;
  if (b < 1) b = 1;
  return (int)b;
}

void wgrad_plan(const ConvGeom& g, int V, int& cvb, int& cblocks, int& chunks, long long& per) {
  int CV = g.C / V;
  cvb = CV < 64 ? CV : 64;
  // keep blockDim.x = 256 divisible: use the largest power of two <= cvb
  int p2 = 1;
  while (p2 * 2 <= cvb) p2 *= 2;
  cvb = p2;
  cblocks = (CV + cvb - 1) / cvb;
  long long total = (long long)g.N * g.P * g.Q;
  int pl = 256 / cvb;
  long long want = 2048 / cblocks;
  if (want < 1) want = 1;
  per = (total + want - 1) / want;
  long long minper = (long long)pl * 8;
  if (per < minper) per = minper;
  chunks = (int)((total + per - 1) / per);
}

int vec_of(const ConvGeom& g, int dtype) {
  int V = dtype == S4TF_BF16 ? 8 : 4;
  return g.C % V == 0 ? V : 1;
}

}  // namespace

int dwconv_fwd(const ConvGeom& g, int dtype, const void* x, const void* w, const float* bias, int act,
               void* y, hipStream_t st) {
  ProfScope ps(PC_DWCONV_FWD, st);
  int V = vec_of(g, dtype);
  long long total = (long long)g.N * g.P * g.Q * (g.C / V);
  dim3 grid(grid_for(total)), block(256);
#define DW_FWD(T, VV) hipLaunchKernelGGL((dw_fwd_kernel<T, VV>), grid, block, 0, st, g, (const T*)x, (const T*)w, bias, act, (T*)y, total)
  if (dtype == S4TF_BF16) { if (V == 8) DW_FWD(bf16_t, 8); else DW_FWD(bf16_t, 1); }
  else { if (V == 4) DW_FWD(float, 4); else DW_FWD(float, 1); }
#undef DW_FWD
  return launch_status("dwconv_fwd");
}

int dwconv_dgrad(const ConvGeom& g, int dtype, const void* dy, const void* w, void* dx, int accumulate,
                 hipStream_t st) {
  ProfScope ps(PC_DWCONV_DGRAD, st);
  int V = vec_of(g, dtype);
  long long total = (long long)g.N * g.H * g.W * (g.C / V);
  dim3 grid(grid_for(total)), block(256);
#define DW_DG(T, VV) hipLaunchKernelGGL((dw_dgrad_kernel<T, VV>), grid, block, 0, st, g, (const T*)dy, (const T*)w, (T*)dx, accumulate, total)
  if (dtype == S4TF_BF16) { if (V == 8) DW_DG(bf16_t, 8); else DW_DG(bf16_t, 1); }
  else { if (V == 4) DW_DG(float, 4); else DW_DG(float, 1); }
#undef DW_DG
  return launch_status("dwconv_dgrad");
}

size_t dwconv_wgrad_workspace(const ConvGeom& g) {
  // sized for the scalar plan, which is the larger one
  size_t worst = 0;
  for (int V = 1; V <= 8; V *= 2) {
    if (g.C % V) continue;
    int cvb, cblocks, chunks;
    long long per;
    wgrad_plan(g, V, cvb, cblocks, chunks, per);
    size_t b = (size_t)chunks * g.R * g.S * g.C * sizeof(float);
    if (b > worst) worst = b;
  }
  return worst;
}

int dwconv_wgrad(const ConvGeom& g, int dtype, const void* x, const void* dy, float* dw, void* ws,
                 hipStream_t st) {
  if (g.R > 3 || g.S > 3) return fail(S4TF_ERR_UNSUPPORTED, "depthwise wgrad supports filters up to 3x3");
  int V = vec_of(g, dtype);
  int cvb, cblocks, chunks;
  long long per;
  wgrad_plan(g, V, cvb, cblocks, chunks, per);
  dim3 grid(cblocks, chunks), block(256);
  size_t shm = (size_t)256 * V * sizeof(float);
  float* part = static_cast<float*>(ws);
  {
    ProfScope ps(PC_DWCONV_WGRAD, st);
#define DW_WG(T, VV) hipLaunchKernelGGL((dw_wgrad_kernel<T, VV>), grid, block, shm, st, g, (const T*)x, (const T*)dy, part, cvb, per)
    if (dtype == S4TF_BF16) { if (V == 8) DW_WG(bf16_t, 8); else DW_WG(bf16_t, 1); }
    else { if (V == 4) DW_WG(float, 4); else DW_WG(float, 1); }
#undef DW_WG
    int rc = launch_status("dwconv_wgrad");
    if (rc != S4TF_OK) return rc;
  }
  ProfScope ps(PC_DWCONV_WGRAD, st);
  int n = g.R * g.S * g.C;
  hipLaunchKernelGGL(dw_wgrad_reduce_kernel, dim3((n + 255) / 256), dim3(256), 0, st, part, dw, n, chunks);
  return launch_status("dwconv_wgrad_reduce");
}

}  // namespace s4tf
