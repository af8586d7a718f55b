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

// fwd, dgrad: grid (ceil(W'*CV/256), N*H') over the output rows of the pass; a thread = V channels of one
// pixel of its block's row, so the only per-thread division is by the channel-vector count.
template <typename T, int V>
__global__ __launch_bounds__(256) void dw_fwd_kernel(ConvGeom g, const T* __restrict__ x, const T* __restrict__ w,
                                                     const float* __restrict__ bias, int act, T* __restrict__ y, int row_base) {
  const int CV = g.C / V;
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= g.Q * CV) return;
  const int q = idx / CV, c = (idx - q * CV) * V;
  const int row = row_base + blockIdx.y;
  const int n = row / g.P, p = row - n * g.P;
  float acc[V];
#pragma unroll
  for (int e = 0; e < V; ++e) acc[e] = bias ? bias[c + e] : 0.f;
  const int h0 = p * g.stride - g.pad, w0 = q * g.stride - g.pad;
  const T* xn = x + (long long)n * g.H * g.W * g.C + c;
  if (g.R <= 3 && g.S <= 3) {
    // all taps loaded at once, those outside the image from pixel 0 and with a zero filter value: no
    // branch (and so no wait) between the loads
    Pack<T, V> xv[9], wv[9];
    bool on[9];
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
      for (int s = 0; s < 3; ++s) {
        const int h = h0 + r, ww = w0 + s;
        const bool ok = r < g.R && s < g.S && h >= 0 && h < g.H && ww >= 0 && ww < g.W;
        on[r * 3 + s] = ok;
        xv[r * 3 + s] = ldp<T, V>(xn + (ok ? (long long)(h * g.W + ww) * g.C : 0));
        wv[r * 3 + s] = ldp<T, V>(w + (ok ? (r * g.S + s) * g.C : 0) + c);
      }
#pragma unroll
    for (int t = 0; t < 9; ++t)
#pragma unroll
      for (int e = 0; e < V; ++e) acc[e] += (on[t] ? xv[t].get(e) : 0.f) * wv[t].get(e);
  } else {
    for (int r = 0; r < g.R; ++r) {
      const int h = h0 + r;
      if (h < 0 || h >= g.H) continue;
      for (int s = 0; s < g.S; ++s) {
        const int ww = w0 + s;
        if (ww < 0 || ww >= g.W) continue;
        const Pack<T, V> xv = ldp<T, V>(xn + (long long)(h * g.W + ww) * g.C);
        const Pack<T, V> wv = ldp<T, V>(w + (r * g.S + s) * g.C + c);
#pragma unroll
        for (int e = 0; e < V; ++e) acc[e] += xv.get(e) * wv.get(e);
      }
    }
  }
  Pack<T, V> o;
#pragma unroll
  for (int e = 0; e < V; ++e) o.set(e, act_apply(acc[e], act));
  stp<T, V>(y + ((long long)row * g.Q + q) * g.C + c, o);
}

template <typename T, int V>
__global__ __launch_bounds__(256) void dw_dgrad_kernel(ConvGeom g, const T* __restrict__ dy, const T* __restrict__ w,
                                                       T* __restrict__ dx, int accumulate, int row_base) {
  const int CV = g.C / V;
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= g.W * CV) return;
  const int ww = idx / CV, c = (idx - ww * CV) * V;
  const int row = row_base + blockIdx.y;
  const int n = row / g.H, h = row - n * g.H;
  float acc[V];
#pragma unroll
  for (int e = 0; e < V; ++e) acc[e] = 0.f;
  const T* dyn = dy + (long long)n * g.P * g.Q * g.C + c;
  if (g.R <= 3 && g.S <= 3) {
    Pack<T, V> dv[9], wv[9];
    bool on[9];
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
      for (int s = 0; s < 3; ++s) {
        const int hp = h + g.pad - r, wp = ww + g.pad - s;
        const int p = g.stride == 1 ? hp : g.stride == 2 ? (hp >> 1) : hp / g.stride;
        const int q = g.stride == 1 ? wp : g.stride == 2 ? (wp >> 1) : wp / g.stride;
        const bool ok = r < g.R && s < g.S && hp >= 0 && wp >= 0 && p * g.stride == hp && q * g.stride == wp && p < g.P && q < g.Q;
        on[r * 3 + s] = ok;
        dv[r * 3 + s] = ldp<T, V>(dyn + (ok ? (long long)(p * g.Q + q) * g.C : 0));
        wv[r * 3 + s] = ldp<T, V>(w + (ok ? (r * g.S + s) * g.C : 0) + c);
      }
#pragma unroll
    for (int t = 0; t < 9; ++t)
#pragma unroll
      for (int e = 0; e < V; ++e) acc[e] += (on[t] ? dv[t].get(e) : 0.f) * wv[t].get(e);
  } else {
    for (int r = 0; r < g.R; ++r) {
      const int hp = h + g.pad - r;
      if (hp < 0) continue;
      const int p = g.stride == 1 ? hp : g.stride == 2 ? (hp >> 1) : hp / g.stride;
      if (p * g.stride != hp || p >= g.P) continue;
      for (int s = 0; s < g.S; ++s) {
        const int wp = ww + g.pad - s;
        if (wp < 0) continue;
        const int q = g.stride == 1 ? wp : g.stride == 2 ? (wp >> 1) : wp / g.stride;
        if (q * g.stride != wp || q >= g.Q) continue;
        const Pack<T, V> dv = ldp<T, V>(dyn + (long long)(p * g.Q + q) * g.C);
        const Pack<T, V> wv = ldp<T, V>(w + (r * g.S + s) * g.C + c);
#pragma unroll
        for (int e = 0; e < V; ++e) acc[e] += dv.get(e) * wv.get(e);
      }
    }
  }
  T* dst = dx + ((long long)row * g.W + ww) * g.C + c;
  Pack<T, V> o;
  if (accumulate) {
    const Pack<T, V> old = ldp<T, V>(dst);
#pragma unroll
    for (int e = 0; e < V; ++e) acc[e] += old.get(e);
  }
#pragma unroll
  for (int e = 0; e < V; ++e) o.set(e, acc[e]);
  stp<T, V>(dst, o);
}

// wgrad stage 1: grid (channel blocks, chunks of output rows (n,p)).  Thread = (channel vector cvl, pixel lane
// pl); it walks the rows of its chunk and, inside a row, the pixels q = pl, pl + lanes, ..., accumulating
// R*S*V sums in registers (no index division in the loop).  The pixel lanes of a block are then added, first
// inside each wavefront by a shuffle butterfly (lanes that share cvl lie cvb apart), then the four
// wavefronts through LDS in a fixed order, and the block writes one partial [R*S][C] slab.  Stage 2 adds
// the slabs in order.
constexpr int DW_MAX_TAPS = 9;
template <typename T, int V>
__global__ __launch_bounds__(256) void dw_wgrad_kernel(ConvGeom g, const T* __restrict__ x, const T* __restrict__ dy,
                                                       float* __restrict__ part, int cvb, int rows_per_chunk) {
  extern __shared__ float red[];  // [4 wavefronts][min(cvb,64)][3*V]
  const int CV = g.C / V;
  const int pl_count = 256 / cvb;
  const int cvl = threadIdx.x % cvb, pl = threadIdx.x / cvb;
  const int cv = blockIdx.x * cvb + cvl;
  const int taps = g.R * g.S;
  float acc[DW_MAX_TAPS][V];
#pragma unroll
  for (int t = 0; t < DW_MAX_TAPS; ++t)
#pragma unroll
    for (int e = 0; e < V; ++e) acc[t][e] = 0.f;
  const int rows = g.N * g.P;
  const int row0 = blockIdx.y * rows_per_chunk, row1 = min(rows, row0 + rows_per_chunk);
  if (cv < CV) {
    const int c = cv * V;
    for (int row = row0; row < row1; ++row) {
      const int n = row / g.P, p = row - n * g.P;
      const int h0 = p * g.stride - g.pad;
      const T* xn = x + (long long)n * g.H * g.W * g.C + c;
      const T* dyr = dy + (long long)row * g.Q * g.C + c;
      for (int q = pl; q < g.Q; q += pl_count) {
        const Pack<T, V> dv = ldp<T, V>(dyr + (long long)q * g.C);
        const int w0 = q * g.stride - g.pad;
        // Every tap is loaded, from pixel 0 of the image when it lies outside, and a select takes it
        // out again: a branch around each load would put a wait behind each of them and the nine loads
        // of a pixel would go to memory one after the other.
        Pack<T, V> xv[DW_MAX_TAPS];
        bool on[DW_MAX_TAPS];
#pragma unroll
        for (int r = 0; r < 3; ++r)
#pragma unroll
          for (int s = 0; s < 3; ++s) {
            const int h = h0 + r, ww = w0 + s;
            const bool ok = r < g.R && s < g.S && h >= 0 && h < g.H && ww >= 0 && ww < g.W;
            on[r * 3 + s] = ok;
            xv[r * 3 + s] = ldp<T, V>(xn + (ok ? (long long)(h * g.W + ww) * g.C : 0));
          }
#pragma unroll
        for (int t = 0; t < DW_MAX_TAPS; ++t)
#pragma unroll
          for (int e = 0; e < V; ++e) acc[t][e] += (on[t] ? xv[t].get(e) : 0.f) * dv.get(e);
      }
    }
  }
  // lanes of one wavefront that share cvl: lane ids differ by multiples of cvb
  for (int off = cvb; off < 64; off <<= 1) {
#pragma unroll
    for (int t = 0; t < DW_MAX_TAPS; ++t)
#pragma unroll
      for (int e = 0; e < V; ++e) acc[t][e] += __shfl_xor(acc[t][e], off, 64);
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int cw = cvb < 64 ? cvb : 64;  // distinct cvl per wavefront (cvb <= 64 by plan): every wavefront holds them all
#pragma unroll
  for (int r = 0; r < 3; ++r) {  // one filter row at a time: red[wave][cvl][3*V]  (unrolled: acc[] stays in registers)
    if (r >= g.R) continue;  // uniform
    if (lane < cw) {
      float* mine = red + ((size_t)wave * cw + lane) * 3 * V;
#pragma unroll
      for (int s = 0; s < 3; ++s)
#pragma unroll
        for (int e = 0; e < V; ++e) mine[s * V + e] = acc[r * 3 + s][e];
    }
    __syncthreads();
    if (wave == 0 && lane < cw && cv < CV) {
      for (int s = 0; s < g.S; ++s)
#pragma unroll
        for (int e = 0; e < V; ++e) {
          float sum = 0.f;
          for (int w4 = 0; w4 < 4; ++w4) sum += red[((size_t)w4 * cw + lane) * 3 * V + s * V + e];
          part[((long long)blockIdx.y * taps + (r * g.S + s)) * g.C + cv * V + e] = sum;
        }
    }
    __syncthreads();
  }
}

// stage 2: 64 outputs per block of 1024 threads; 16 lanes per output stride over the slabs, then are added in order
__global__ __launch_bounds__(1024) void dw_wgrad_reduce_kernel(const float* __restrict__ part, float* __restrict__ dw, int n, int chunks) {
  __shared__ float red[16][64];
  const int ol = threadIdx.x & 63, zl = threadIdx.x >> 6;
  const int i = blockIdx.x * 64 + ol;
  float s = 0.f;
  if (i < n)
    for (int z = zl; z < chunks; z += 16) s += part[(long long)z * n + i];
  red[zl][ol] = s;
  __syncthreads();
  if (zl == 0 && i < n) {
    float t = 0.f;
    for (int k = 0; k < 16; ++k) t += red[k][ol];
    dw[i] = t;
  }
}

int grid_for(long long total) {
  long long b = (total + 255) / 256;
  if (b > 256 * 32) b = 256 * 32;
  if (b < 1) b = 1;
  return (int)b;
}

void wgrad_plan(const ConvGeom& g, int V, int& cvb, int& cblocks, int& chunks, int& rows_per_chunk) {
  int CV = g.C / V;
  cvb = CV < 64 ? CV : 64;
  // keep blockDim.x = 256 divisible: use the largest power of two <= cvb
  int p2 = 1;
  while (p2 * 2 <= cvb) p2 *= 2;
  cvb = p2;
  cblocks = (CV + cvb - 1) / cvb;
  const int rows = g.N * g.P;
  int want = 512 / cblocks;  // blocks in all: each pays a fixed price for adding its pixel lanes
  if (want < 1) want = 1;
  rows_per_chunk = (rows + want - 1) / want;
  // at least ~8 pixels per pixel lane and block
  const int pl = 256 / cvb;
  const int min_rows = (8 * pl + g.Q - 1) / g.Q;
  if (rows_per_chunk < min_rows) rows_per_chunk = min_rows;
  chunks = (rows + rows_per_chunk - 1) / rows_per_chunk;
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
  const int rows = g.N * g.P;
  for (int base = 0; base < rows; base += 65535) {  // grid.y is limited to 65535
    dim3 grid((unsigned)((g.Q * (g.C / V) + 255) / 256), (unsigned)(rows - base < 65535 ? rows - base : 65535)), block(256);
#define DW_FWD(T, VV) hipLaunchKernelGGL((dw_fwd_kernel<T, VV>), grid, block, 0, st, g, (const T*)x, (const T*)w, bias, act, (T*)y, base)
    if (dtype == S4TF_BF16) { if (V == 8) DW_FWD(bf16_t, 8); else DW_FWD(bf16_t, 1); }
    else { if (V == 4) DW_FWD(float, 4); else DW_FWD(float, 1); }
#undef DW_FWD
  }
  return launch_status("dwconv_fwd");
}

int dwconv_dgrad(const ConvGeom& g, int dtype, const void* dy, const void* w, void* dx, int accumulate,
                 hipStream_t st) {
  ProfScope ps(PC_DWCONV_DGRAD, st);
  int V = vec_of(g, dtype);
  const int rows = g.N * g.H;
  for (int base = 0; base < rows; base += 65535) {  // grid.y is limited to 65535
    dim3 grid((unsigned)((g.W * (g.C / V) + 255) / 256), (unsigned)(rows - base < 65535 ? rows - base : 65535)), block(256);
#define DW_DG(T, VV) hipLaunchKernelGGL((dw_dgrad_kernel<T, VV>), grid, block, 0, st, g, (const T*)dy, (const T*)w, (T*)dx, accumulate, base)
    if (dtype == S4TF_BF16) { if (V == 8) DW_DG(bf16_t, 8); else DW_DG(bf16_t, 1); }
    else { if (V == 4) DW_DG(float, 4); else DW_DG(float, 1); }
#undef DW_DG
  }
  return launch_status("dwconv_dgrad");
}

size_t dwconv_wgrad_workspace(const ConvGeom& g) {
  // sized for the scalar plan, which is the larger one
  size_t worst = 0;
  for (int V = 1; V <= 8; V *= 2) {
    if (g.C % V) continue;
    int cvb, cblocks, chunks, per;
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
  int cvb, cblocks, chunks, per;
  wgrad_plan(g, V, cvb, cblocks, chunks, per);
  dim3 grid(cblocks, chunks), block(256);
  size_t shm = (size_t)4 * (cvb < 64 ? cvb : 64) * 3 * V * sizeof(float);
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
  hipLaunchKernelGGL(dw_wgrad_reduce_kernel, dim3((n + 63) / 64), dim3(1024), 0, st, part, dw, n, chunks);
  return launch_status("dwconv_wgrad_reduce");
}

}  // namespace s4tf
