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

// stage 2: OL outputs per block of 1024 threads; 1024 / OL lanes per output stride over the slabs, then are
// added in order.  Few outputs (small C) take 64 lanes each, so that the walk over the slabs stays short.
template <int OL>
__global__ __launch_bounds__(1024) void dw_wgrad_reduce_kernel(const float* __restrict__ part, float* __restrict__ dw, int n, int chunks) {
  constexpr int ZL = 1024 / OL;
  __shared__ float red[ZL][OL];
  const int ol = threadIdx.x % OL, zl = threadIdx.x / OL;
  const int i = blockIdx.x * OL + ol;
  float s = 0.f;
  if (i < n)
    for (int z = zl; z < chunks; z += ZL) s += part[(long long)z * n + i];
  red[zl][ol] = s;
  __syncthreads();
  if (zl == 0 && i < n) {
    float t = 0.f;
    for (int k = 0; k < ZL; ++k) t += red[k][ol];
    dw[i] = t;
  }
}
void launch_wgrad_reduce(const float* part, float* dw, int n, int chunks, hipStream_t st) {
  if (n <= 64 * 64 && chunks > 64)
    hipLaunchKernelGGL(dw_wgrad_reduce_kernel<16>, dim3((n + 15) / 16), dim3(1024), 0, st, part, dw, n, chunks);
  else
    hipLaunchKernelGGL(dw_wgrad_reduce_kernel<64>, dim3((n + 63) / 64), dim3(1024), 0, st, part, dw, n, chunks);
}

// ---- 3x3, pad 1, stride 1 or 2, fp32, channel counts that are multiples of 4 -------------------------
// The kernels above issue one load per tap and output (nine for 3x3) and the address path of the CU, not
// HBM, bounds them.  Here a thread owns 4 channels of a strip of TQ adjacent output columns and walks down
// RC output rows with the input rows it needs held in registers: going down one row it loads only the
// `stride` input rows that are new, so an input pixel is loaded (TQ*stride + 3 - stride) / (TQ*stride)
// times horizontally and (RC*stride + 3 - stride) / (RC*stride) times vertically instead of 9 / stride^2.
// Work item = (image, chunk of RC output rows, strip); thread = (item, channel vector), channels fastest.
struct StripPlan {
  int RC, nstrips, nchunks;
  long long items;
};
constexpr int DW_TQ = 4;   // strip width at stride 1 (and, in column pairs, of the stride-2 input gradient)
constexpr int DW_TQ2 = 2;  // at stride 2, where a strip's window is 2*TQ + 1 columns wide

__device__ inline float4 f4sel(bool ok, const float4& v) {
  return ok ? v : make_float4(0.f, 0.f, 0.f, 0.f);
}
__device__ inline void f4fma(float4& a, const float4& x, const float4& y) {
  a.x = fmaf(x.x, y.x, a.x); a.y = fmaf(x.y, y.y, a.y); a.z = fmaf(x.z, y.z, a.z); a.w = fmaf(x.w, y.w, a.w);
}
__device__ inline float4 ld4(const float* p) { return *reinterpret_cast<const float4*>(p); }

// Input window of a strip: NC columns from column q0*ST - 1; coff[j] is the offset of column j inside a
// row (column 0 when it lies outside the image, and cok[j] false), so every load is unconditional.
template <int ST, int TQ> struct StripCols {
  static constexpr int NC = (TQ - 1) * ST + 3;
  int coff[NC];
  bool cok[NC];
  __device__ void init(int q0, int W, int C) {
#pragma unroll
    for (int j = 0; j < NC; ++j) {
      const int cin = q0 * ST - 1 + j;
      cok[j] = cin >= 0 && cin < W;
      coff[j] = (cok[j] ? cin : 0) * C;
    }
  }
  __device__ void load_row(const float* img, int hin, int H, int W, int C, float4 (&row)[NC]) const {
    const bool rok = hin >= 0 && hin < H;
    const float* xr = img + (long long)(rok ? hin : 0) * W * C;
#pragma unroll
    for (int j = 0; j < NC; ++j) row[j] = f4sel(rok && cok[j], ld4(xr + coff[j]));
  }
};

__device__ inline void strip_item(long long gid, int CV, const StripPlan& sp, int& cv, int& n, int& chunk, int& strip) {
  const int item = (int)((unsigned)gid / (unsigned)CV);  // the launcher keeps the thread count below 2^31
  cv = (int)gid - item * CV;
  strip = item % sp.nstrips;
  const int t = item / sp.nstrips;
  chunk = t % sp.nchunks;
  n = t / sp.nchunks;
}

// forward; with flip != 0 the filter is read back to front, which makes it the input gradient of a stride-1
// convolution (src = dy, dst = dx, same extents)
template <int ST, int TQ>
__global__ __launch_bounds__(256) void dw3_fwd_kernel(ConvGeom g, StripPlan sp, const float* __restrict__ src,
                                                      const float* __restrict__ w, const float* __restrict__ bias, int act,
                                                      float* __restrict__ dst, int flip, int accumulate, long long total) {
  typedef StripCols<ST, TQ> SC;
  constexpr int NC = SC::NC, CARRY = 3 - ST;
  const long long gid = (long long)blockIdx.x * 256 + threadIdx.x;
  if (gid >= total) return;
  int cv, n, chunk, strip;
  strip_item(gid, g.C / 4, sp, cv, n, chunk, strip);
  const int c = cv * 4, q0 = strip * TQ;
  const int p0 = chunk * sp.RC, p1 = min(g.P, p0 + sp.RC);
  float4 wf[9];
#pragma unroll
  for (int t = 0; t < 9; ++t) wf[t] = ld4(w + (flip ? 8 - t : t) * g.C + c);
  const float4 b4 = bias ? ld4(bias + c) : make_float4(0.f, 0.f, 0.f, 0.f);
  SC sc;
  sc.init(q0, g.W, g.C);
  const float* img = src + (long long)n * g.H * g.W * g.C + c;
  float4 win[3][NC], nxt[ST][NC];
#pragma unroll
  for (int r = 0; r < CARRY; ++r) sc.load_row(img, p0 * ST - 1 + r, g.H, g.W, g.C, win[r]);
#pragma unroll
  for (int r = 0; r < ST; ++r) sc.load_row(img, p0 * ST - 1 + CARRY + r, g.H, g.W, g.C, win[CARRY + r]);
  for (int p = p0; p < p1; ++p) {
    if (p + 1 < p1) {  // the rows that the next output row adds, requested before this one is computed
#pragma unroll
      for (int r = 0; r < ST; ++r) sc.load_row(img, (p + 1) * ST - 1 + CARRY + r, g.H, g.W, g.C, nxt[r]);
    }
    float* drow = dst + (((long long)n * g.P + p) * g.Q + q0) * g.C + c;
#pragma unroll
    for (int j = 0; j < TQ; ++j) {
      if (q0 + j >= g.Q) continue;
      float4 a = b4;
#pragma unroll
      for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int t = 0; t < 3; ++t) f4fma(a, win[r][j * ST + t], wf[r * 3 + t]);
      float4 o;
      o.x = act_apply(a.x, act); o.y = act_apply(a.y, act); o.z = act_apply(a.z, act); o.w = act_apply(a.w, act);
      float* d = drow + (long long)j * g.C;
      if (accumulate) {
        const float4 old = ld4(d);
        o.x += old.x; o.y += old.y; o.z += old.z; o.w += old.w;
      }
      *reinterpret_cast<float4*>(d) = o;
    }
    if (p + 1 < p1) {
#pragma unroll
      for (int r = 0; r < CARRY; ++r)
#pragma unroll
        for (int j = 0; j < NC; ++j) win[r][j] = win[r + ST][j];
#pragma unroll
      for (int r = 0; r < ST; ++r)
#pragma unroll
        for (int j = 0; j < NC; ++j) win[CARRY + r][j] = nxt[r][j];
    }
  }
}

// Input gradient of the stride-2 convolution.  Input rows 2a and 2a+1 receive from output rows a and a+1 only
// (row 2a through filter row 1; row 2a+1 through filter row 2 from output row a and through filter row 0 from
// output row a+1), columns likewise: a thread owns the input columns 2*b0 .. 2*b0 + 2*TQ - 1, keeps output row
// a's TQ+1 pixels in registers, loads row a+1's, and writes the two input rows.  Work item = (image, chunk of
// RC row pairs, strip of TQ column pairs).
template <int TQ>
__global__ __launch_bounds__(256) void dw3_dgrad_s2_kernel(ConvGeom g, StripPlan sp, const float* __restrict__ dy,
                                                           const float* __restrict__ w, float* __restrict__ dx,
                                                           int accumulate, long long total) {
  constexpr int NC = TQ + 1;
  const long long gid = (long long)blockIdx.x * 256 + threadIdx.x;
  if (gid >= total) return;
  int cv, n, chunk, strip;
  strip_item(gid, g.C / 4, sp, cv, n, chunk, strip);
  const int c = cv * 4, b0 = strip * TQ;
  const int HA = (g.H + 1) / 2;
  const int a0 = chunk * sp.RC, a1 = min(HA, a0 + sp.RC);
  float4 wf[9];
#pragma unroll
  for (int t = 0; t < 9; ++t) wf[t] = ld4(w + t * g.C + c);
  int coff[NC];
  bool cok[NC];
#pragma unroll
  for (int j = 0; j < NC; ++j) {
    cok[j] = b0 + j < g.Q;
    coff[j] = (cok[j] ? b0 + j : 0) * g.C;
  }
  const float* img = dy + (long long)n * g.P * g.Q * g.C + c;
  auto load_row = [&](int p, float4 (&row)[NC]) {
    const bool rok = p < g.P;
    const float* r = img + (long long)(rok ? p : 0) * g.Q * g.C;
#pragma unroll
    for (int j = 0; j < NC; ++j) row[j] = f4sel(rok && cok[j], ld4(r + coff[j]));
  };
  float4 cur[NC], nxt[NC];
  load_row(a0, cur);
  for (int a = a0; a < a1; ++a) {
    load_row(a + 1, nxt);
#pragma unroll
    for (int dh = 0; dh < 2; ++dh) {
      const int h = 2 * a + dh;
      if (h >= g.H) continue;
      float* drow = dx + (((long long)n * g.H + h) * g.W + 2 * b0) * g.C + c;
#pragma unroll
      for (int j = 0; j < TQ; ++j) {
#pragma unroll
        for (int dw = 0; dw < 2; ++dw) {
          if (2 * (b0 + j) + dw >= g.W) continue;
          float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
          // even row: filter row 1 from `cur`; odd row: filter row 2 from `cur`, filter row 0 from `nxt`
          // even column: filter column 1 from pixel j; odd: filter column 2 from pixel j, column 0 from j+1
          if (dh == 0) {
            if (dw == 0) {
              f4fma(o, cur[j], wf[1 * 3 + 1]);
            } else {
              f4fma(o, cur[j], wf[1 * 3 + 2]);
              f4fma(o, cur[j + 1], wf[1 * 3 + 0]);
            }
          } else {
            if (dw == 0) {
              f4fma(o, cur[j], wf[2 * 3 + 1]);
              f4fma(o, nxt[j], wf[0 * 3 + 1]);
            } else {
              f4fma(o, cur[j], wf[2 * 3 + 2]);
              f4fma(o, cur[j + 1], wf[2 * 3 + 0]);
              f4fma(o, nxt[j], wf[0 * 3 + 2]);
              f4fma(o, nxt[j + 1], wf[0 * 3 + 0]);
            }
          }
          float* d = drow + (long long)(2 * j + dw) * g.C;
          if (accumulate) {
            const float4 old = ld4(d);
            o.x += old.x; o.y += old.y; o.z += old.z; o.w += old.w;
          }
          *reinterpret_cast<float4*>(d) = o;
        }
      }
    }
#pragma unroll
    for (int j = 0; j < NC; ++j) cur[j] = nxt[j];
  }
}

// Filter gradient, stage 1.  grid (channel blocks, item blocks); a block has cvb channel vectors (a divisor
// of C/4, at most 64) times pl = 256 / cvb item lanes; lane il takes the items il, il + pl, ... of its
// block's range and walks each down its rows as the forward kernel does, with the strip's TQ output
// cotangents of the row beside the window: 9 x 4 sums in registers.  The item lanes are then added through
// LDS in lane order and the block writes one partial [9][C] slab; dw_wgrad_reduce_kernel adds the slabs.
template <int ST, int TQ>
__global__ __launch_bounds__(256) void dw3_wgrad_kernel(ConvGeom g, StripPlan sp, const float* __restrict__ x,
                                                        const float* __restrict__ dy, float* __restrict__ part, int cvb,
                                                        int items_per_block) {
  typedef StripCols<ST, TQ> SC;
  constexpr int NC = SC::NC, CARRY = 3 - ST;
  __shared__ float4 red[256 * 9];
  const int pl = 256 / cvb;
  const int cvl = threadIdx.x % cvb, il = threadIdx.x / cvb;
  const int cv = blockIdx.x * cvb + cvl, c = cv * 4;
  float4 acc[9];
#pragma unroll
  for (int t = 0; t < 9; ++t) acc[t] = make_float4(0.f, 0.f, 0.f, 0.f);
  const long long i0 = (long long)blockIdx.y * items_per_block;
  const long long i1 = i0 + items_per_block < sp.items ? i0 + items_per_block : sp.items;
  if (il < pl) {
    for (long long item = i0 + il; item < i1; item += pl) {
      const int strip = (int)(item % sp.nstrips);
      const int t = (int)(item / sp.nstrips);
      const int chunk = t % sp.nchunks, n = t / sp.nchunks;
      const int q0 = strip * TQ;
      const int p0 = chunk * sp.RC, p1 = min(g.P, p0 + sp.RC);
      SC sc;
      sc.init(q0, g.W, g.C);
      const float* img = x + (long long)n * g.H * g.W * g.C + c;
      // no rows are requested ahead here (the forward kernel does that): the 36 sums need the registers,
      // and three wavefronts per SIMD hide the latency instead
      float4 win[3][NC], dv[TQ];
#pragma unroll
      for (int r = 0; r < CARRY; ++r) sc.load_row(img, p0 * ST - 1 + r, g.H, g.W, g.C, win[r]);
      for (int p = p0; p < p1; ++p) {
        const float* dyr = dy + (((long long)n * g.P + p) * g.Q) * g.C + c;
#pragma unroll
        for (int j = 0; j < TQ; ++j) {
          const bool ok = q0 + j < g.Q;
          dv[j] = f4sel(ok, ld4(dyr + (long long)(ok ? q0 + j : 0) * g.C));
        }
#pragma unroll
        for (int r = 0; r < ST; ++r) sc.load_row(img, p * ST - 1 + CARRY + r, g.H, g.W, g.C, win[CARRY + r]);
#pragma unroll
        for (int j = 0; j < TQ; ++j)
#pragma unroll
          for (int r = 0; r < 3; ++r)
#pragma unroll
            for (int t2 = 0; t2 < 3; ++t2) f4fma(acc[r * 3 + t2], win[r][j * ST + t2], dv[j]);
#pragma unroll
        for (int r = 0; r < CARRY; ++r)
#pragma unroll
          for (int j = 0; j < NC; ++j) win[r][j] = win[r + ST][j];
      }
    }
#pragma unroll
    for (int t = 0; t < 9; ++t) red[(il * 9 + t) * cvb + cvl] = acc[t];
  }
  __syncthreads();
  for (int o = threadIdx.x; o < 9 * cvb; o += 256) {  // o = tap * cvb + channel vector
    float4 sum = red[o];
    for (int l = 1; l < pl; ++l) {
      const float4 v = red[l * 9 * cvb + o];
      sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
    }
    const int tap = o / cvb, cl = o - tap * cvb;
    *reinterpret_cast<float4*>(part + ((long long)blockIdx.y * 9 + tap) * g.C + (blockIdx.x * cvb + cl) * 4) = sum;
  }
}

bool strip_ok(const ConvGeom& g, int dtype) {
  if ((long long)g.N * g.H * g.W * (g.C / 4) >= (1LL << 31)) return false;  // thread ids stay 32-bit
  return dtype == S4TF_F32 && g.R == 3 && g.S == 3 && g.pad == 1 && (g.stride == 1 || g.stride == 2) && g.C % 4 == 0 &&
         g.C == g.K;
}

// rows: extent of the axis the items walk (output rows; row pairs for the stride-2 input gradient),
// cols: extent of the axis the strips cut
StripPlan strip_plan(const ConvGeom& g, int rows, int cols, bool cheap_halo, int TQ) {
  StripPlan sp;
  sp.nstrips = (cols + TQ - 1) / TQ;
  // longer walks re-load fewer halo rows, shorter ones give more threads and fewer load-then-use round
  // trips one after the other: the longest walk that still gives 2^16 threads (each keeps 6 to 18 loads of
  // 16 bytes in flight); small layers end at one row per thread
  const int cand[5] = {cheap_halo ? 7 : 14, cheap_halo ? 4 : 7, cheap_halo ? 2 : 4, cheap_halo ? 1 : 2, 1};
  sp.RC = 1;
  for (int i = 0; i < 5; ++i) {
    const long long items = (long long)g.N * ((rows + cand[i] - 1) / cand[i]) * sp.nstrips;
    if (items * (g.C / 4) >= (1 << 16)) { sp.RC = cand[i]; break; }
  }
  sp.nchunks = (rows + sp.RC - 1) / sp.RC;
  sp.items = (long long)g.N * sp.nchunks * sp.nstrips;
  return sp;
}

struct StripWgradPlan {
  StripPlan sp;
  int cvb, cblocks, yblocks, items_per_block;
};
StripWgradPlan strip_wgrad_plan(const ConvGeom& g) {
  StripWgradPlan w;
  w.sp = strip_plan(g, g.P, g.Q, g.stride == 2, g.stride == 2 ? DW_TQ2 : DW_TQ);
  const int CV = g.C / 4;
  w.cvb = 1;
  for (int d = 1; d <= 64 && d <= CV; ++d)
    if (CV % d == 0) w.cvb = d;
  w.cblocks = CV / w.cvb;
  const int pl = 256 / w.cvb;
  long long want = 1024 / w.cblocks;
  if (want < 1) want = 1;
  const long long most = (w.sp.items + pl - 1) / pl;  // at least one item per lane
  if (want > most) want = most;
  w.items_per_block = (int)((w.sp.items + want - 1) / want);
  w.yblocks = (int)((w.sp.items + w.items_per_block - 1) / w.items_per_block);
  return w;
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
  if (strip_ok(g, dtype) && aligned16(x) && aligned16(w) && aligned16(y) && (!bias || aligned16(bias))) {
    const StripPlan sp = strip_plan(g, g.P, g.Q, g.stride == 2, g.stride == 2 ? DW_TQ2 : DW_TQ);
    const long long total = sp.items * (g.C / 4);
    dim3 grid((unsigned)((total + 255) / 256)), block(256);
    if (g.stride == 1)
      hipLaunchKernelGGL((dw3_fwd_kernel<1, DW_TQ>), grid, block, 0, st, g, sp, (const float*)x, (const float*)w, bias, act, (float*)y, 0, 0, total);
    else
      hipLaunchKernelGGL((dw3_fwd_kernel<2, DW_TQ2>), grid, block, 0, st, g, sp, (const float*)x, (const float*)w, bias, act, (float*)y, 0, 0, total);
    return launch_status("dwconv_fwd");
  }
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
  if (strip_ok(g, dtype) && aligned16(dy) && aligned16(w) && aligned16(dx)) {
    if (g.stride == 1) {  // the forward kernel over dy with the filter read back to front
      const StripPlan sp = strip_plan(g, g.H, g.W, false, DW_TQ);
      const long long total = sp.items * (g.C / 4);
      hipLaunchKernelGGL((dw3_fwd_kernel<1, DW_TQ>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, g, sp, (const float*)dy,
                         (const float*)w, (const float*)nullptr, (int)S4TF_ACT_NONE, (float*)dx, 1, accumulate, total);
    } else {
      const StripPlan sp = strip_plan(g, (g.H + 1) / 2, (g.W + 1) / 2, true, DW_TQ);
      const long long total = sp.items * (g.C / 4);
      hipLaunchKernelGGL((dw3_dgrad_s2_kernel<DW_TQ>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, g, sp, (const float*)dy,
                         (const float*)w, (float*)dx, accumulate, total);
    }
    return launch_status("dwconv_dgrad");
  }
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
  if (g.R == 3 && g.S == 3 && g.pad == 1 && (g.stride == 1 || g.stride == 2) && g.C % 4 == 0) {
    const size_t b = (size_t)strip_wgrad_plan(g).yblocks * 9 * g.C * sizeof(float);
    if (b > worst) worst = b;
  }
  return worst;
}

int dwconv_wgrad(const ConvGeom& g, int dtype, const void* x, const void* dy, float* dw, void* ws,
                 hipStream_t st) {
  if (g.R > 3 || g.S > 3) return fail(S4TF_ERR_UNSUPPORTED, "depthwise wgrad supports filters up to 3x3");
  if (strip_ok(g, dtype) && aligned16(x) && aligned16(dy) && aligned16(ws)) {
    const StripWgradPlan wp = strip_wgrad_plan(g);
    float* part = static_cast<float*>(ws);
    ProfScope ps(PC_DWCONV_WGRAD, st);
    dim3 grid(wp.cblocks, wp.yblocks), block(256);
    if (g.stride == 1)
      hipLaunchKernelGGL((dw3_wgrad_kernel<1, DW_TQ>), grid, block, 0, st, g, wp.sp, (const float*)x, (const float*)dy, part, wp.cvb, wp.items_per_block);
    else
      hipLaunchKernelGGL((dw3_wgrad_kernel<2, DW_TQ2>), grid, block, 0, st, g, wp.sp, (const float*)x, (const float*)dy, part, wp.cvb, wp.items_per_block);
    int rc = launch_status("dwconv_wgrad");
    if (rc != S4TF_OK) return rc;
    const int n = 9 * g.C;
    launch_wgrad_reduce(part, dw, n, wp.yblocks, st);
    return launch_status("dwconv_wgrad_reduce");
  }
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
  launch_wgrad_reduce(part, dw, n, chunks, st);
  return launch_status("dwconv_wgrad_reduce");
}

}  // namespace s4tf
