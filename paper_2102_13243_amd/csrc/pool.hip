// Pooling forward / pullback, the activation pullback of conv/dense layers, column sums
// (bias gradients) and the SGD-momentum update.  All bound by HBM bandwidth; threads map to
// the channel-fastest NHWC index so wavefronts touch contiguous memory.
#include "s4tf_internal.h"
#include "pack.h"

namespace s4tf {
namespace {

inline int blocks_for(long long total, int per_block = 256) {
  long long b = (total + per_block - 1) / per_block;
  if (b > 256 * 64) b = 256 * 64;
  if (b < 1) b = 1;
  return (int)b;
}

// ---- 2x2 / 2 average pool (AvgPool2D of the paper's LeNet figure) -----------------------------
template <typename T>
__global__ void avgpool2_fwd_kernel(const T* __restrict__ x, T* __restrict__ y, int N, int H, int W, int C) {
  const int P = H / 2, Q = W / 2;
  const long long total = (long long)N * P * Q * C;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
    int c = (int)(i % C);
    long long t = i / C;
    int q = (int)(t % Q);
    t /= Q;
    int p = (int)(t % P), n = (int)(t / P);
    const T* b = x + (((long long)n * H + 2 * p) * W + 2 * q) * C + c;
    float s = to_f32<T>(b[0]) + to_f32<T>(b[C]) + to_f32<T>(b[(long long)W * C]) + to_f32<T>(b[(long long)W * C + C]);
    y[i] = from_f32<T>(s * 0.25f);
  }
}
template <typename T>
__global__ void avgpool2_vjp_kernel(const T* __restrict__ dy, T* __restrict__ dx, int N, int H, int W, int C, int accumulate) {
  const int P = H / 2, Q = W / 2;
  const long long total = (long long)N * H * W * C;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
    int c = (int)(i % C);
    long long t = i / C;
    int w = (int)(t % W);
    t /= W;
    int h = (int)(t % H), n = (int)(t / H);
    int p = h >> 1, q = w >> 1;
    float v = 0.f;
    if (p < P && q < Q) v = to_f32<T>(dy[(((long long)n * P + p) * Q + q) * C + c]) * 0.25f;
    if (accumulate) v += to_f32<T>(dx[i]);
    dx[i] = from_f32<T>(v);
  }
}

// ---- 3x3 / 2 pad 1 max pool --------------------------------------------------------------------
// one thread per V channels of one output pixel
// idx (optional): per output element one byte, the window position 3*r + s of the first maximum in row-major
// window order: what the pullback needs to know, so that it does not have to scan the windows again
template <typename T, int V>
__global__ void maxpool3s2_fwd_kernel(const T* __restrict__ x, T* __restrict__ y, unsigned char* __restrict__ idx, int N,
                                      int H, int W, int C) {
  const int P = (H - 1) / 2 + 1, Q = (W - 1) / 2 + 1, CV = C / V;
  const long long total = (long long)N * P * Q * CV;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
    int c = (int)(i % CV) * V;
    long long t = i / CV;
    int q = (int)(t % Q);
    t /= Q;
    int p = (int)(t % P), n = (int)(t / P);
    float best[V];
    unsigned bi[V];
#pragma unroll
    for (int v = 0; v < V; ++v) { best[v] = -INFINITY; bi[v] = 0; }
#pragma unroll
    for (int r = 0; r < 3; ++r) {
      int h = 2 * p + r - 1;
      if (h < 0 || h >= H) continue;
#pragma unroll
      for (int s = 0; s < 3; ++s) {
        int w = 2 * q + s - 1;
        if (w < 0 || w >= W) continue;
        Pack<T, V> xv = ldp<T, V>(x + (((long long)n * H + h) * W + w) * C + c);
#pragma unroll
        for (int v = 0; v < V; ++v) {
          const float e = xv.get(v);
          if (e > best[v]) { best[v] = e; bi[v] = r * 3 + s; }  // strict: the first maximum keeps the title
        }
      }
    }
    Pack<T, V> o;
#pragma unroll
    for (int v = 0; v < V; ++v) o.set(v, best[v]);
    stp<T, V>(y + i * V, o);
    if (idx) {
      if constexpr (V % 4 == 0) {  // V bytes in one store
        uint32_t w4[V / 4];
#pragma unroll
        for (int k = 0; k < V / 4; ++k) w4[k] = bi[4 * k] | (bi[4 * k + 1] << 8) | (bi[4 * k + 2] << 16) | (bi[4 * k + 3] << 24);
        if constexpr (V == 8) *reinterpret_cast<uint2*>(idx + i * V) = make_uint2(w4[0], w4[1]);
        else *reinterpret_cast<uint32_t*>(idx + i * V) = w4[0];
      } else {
#pragma unroll
        for (int v = 0; v < V; ++v) idx[i * V + v] = (unsigned char)bi[v];
      }
    }
  }
}
// gather form of the pullback: input (h,w) receives dy of every window in which it is the first
// maximum in row-major window order (so the result does not depend on thread scheduling).
// One thread per V channels of one 2x2 cell of input pixels (2a..2a+1, 2b..2b+1): the cell lies in
// the four windows (a..a+1, b..b+1) and in no other; each window is scanned once in window order with
// a strict '>' (the first maximum keeps the title) and hands its dy to the cell pixel that won, if any.
template <typename T, int V>
__global__ __launch_bounds__(256) void maxpool3s2_vjp_kernel(const T* __restrict__ x, const T* __restrict__ dy, T* __restrict__ dx,
                                                             int N, int H, int W, int C, int accumulate) {
  const int P = (H - 1) / 2 + 1, Q = (W - 1) / 2 + 1, CV = C / V;
  const int HA = (H + 1) / 2, WB = (W + 1) / 2;
  const long long total = (long long)N * HA * WB * CV;
  // Consecutive workgroup ids run on different XCDs, each with an L2 of its own.  Cells in adjacent rows
  // share two of their four input rows, so every XCD gets a contiguous run of cells (the grid is a multiple
  // of 8 workgroups) and finds the rows its previous workgroups fetched in its own L2.
  const unsigned per_xcd = gridDim.x / 8;
  const unsigned lb = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  for (long long idx = (long long)lb * blockDim.x + threadIdx.x; idx < total; idx += (long long)gridDim.x * blockDim.x) {
    const int c = (int)(idx % CV) * V;
    long long t = idx / CV;
    const int b = (int)(t % WB);
    t /= WB;
    const int a = (int)(t % HA), n = (int)(t / HA);
    // the 5x5 pixels (2a-1..2a+3, 2b-1..2b+3) that the cell's four windows cover, loaded once (36 loads
    // window by window); a pixel outside the image is loaded from the nearest one inside and counts as -inf
    Pack<T, V> nb[5][5];
    bool in[5][5];
#pragma unroll
    for (int r = 0; r < 5; ++r) {
      const int hh = 2 * a - 1 + r, hc = hh < 0 ? 0 : (hh >= H ? H - 1 : hh);
#pragma unroll
      for (int s = 0; s < 5; ++s) {
        const int ww = 2 * b - 1 + s, wc = ww < 0 ? 0 : (ww >= W ? W - 1 : ww);
        nb[r][s] = ldp<T, V>(x + (((long long)n * H + hc) * W + wc) * C + c);
        in[r][s] = hh == hc && ww == wc;
      }
    }
    float g[2][2][V];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int v = 0; v < V; ++v) g[u >> 1][u & 1][v] = 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int p = a + i;
      if (p >= P) continue;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int q = b + j;
        if (q >= Q) continue;
        float best[V];
        int bi[V];
#pragma unroll
        for (int v = 0; v < V; ++v) { best[v] = -INFINITY; bi[v] = -1; }
#pragma unroll
        for (int r = 0; r < 3; ++r)
#pragma unroll
          for (int s = 0; s < 3; ++s)
#pragma unroll
            for (int v = 0; v < V; ++v) {
              const float e = in[2 * i + r][2 * j + s] ? nb[2 * i + r][2 * j + s].get(v) : -INFINITY;
              if (e > best[v]) { best[v] = e; bi[v] = r * 3 + s; }
            }
        const Pack<T, V> dv = ldp<T, V>(dy + (((long long)n * P + p) * Q + q) * C + c);
        // cell pixel (dh, dw) sits at window position (dh + 1 - 2i, dw + 1 - 2j)
#pragma unroll
        for (int dh = 0; dh < 2; ++dh) {
          const int r = dh + 1 - 2 * i;
          if (r < 0) continue;
#pragma unroll
          for (int dw = 0; dw < 2; ++dw) {
            const int s2 = dw + 1 - 2 * j;
            if (s2 < 0) continue;
#pragma unroll
            for (int v = 0; v < V; ++v)
              if (bi[v] == r * 3 + s2) g[dh][dw][v] += dv.get(v);
          }
        }
      }
    }
#pragma unroll
    for (int dh = 0; dh < 2; ++dh) {
      const int h = 2 * a + dh;
      if (h >= H) continue;
#pragma unroll
      for (int dw = 0; dw < 2; ++dw) {
        const int w = 2 * b + dw;
        if (w >= W) continue;
        T* dst = dx + (((long long)n * H + h) * W + w) * C + c;
        Pack<T, V> o;
        if (accumulate) {
          const Pack<T, V> old = ldp<T, V>(dst);
#pragma unroll
          for (int v = 0; v < V; ++v) g[dh][dw][v] += old.get(v);
        }
#pragma unroll
        for (int v = 0; v < V; ++v) o.set(v, g[dh][dw][v]);
        stp<T, V>(dst, o);
      }
    }
  }
}

// The same pullback from the positions the forward pass saved: a 2x2 cell of input pixels reads, for each of
// its four windows, dy and the window's winner, and keeps dy where the winner is one of its own pixels.
template <typename T, int V>
__global__ __launch_bounds__(256) void maxpool3s2_vjp_idx_kernel(const unsigned char* __restrict__ idx, const T* __restrict__ dy,
                                                                 T* __restrict__ dx, int N, int H, int W, int C, int accumulate) {
  static_assert(V == 4 || V == 8, "one 4- or 8-byte load of positions per window");
  const int P = (H - 1) / 2 + 1, Q = (W - 1) / 2 + 1, CV = C / V;
  const int HA = (H + 1) / 2, WB = (W + 1) / 2;
  const long long total = (long long)N * HA * WB * CV;
  for (long long id = (long long)blockIdx.x * blockDim.x + threadIdx.x; id < total; id += (long long)gridDim.x * blockDim.x) {
    const int c = (int)(id % CV) * V;
    long long t = id / CV;
    const int b = (int)(t % WB);
    t /= WB;
    const int a = (int)(t % HA), n = (int)(t / HA);
    float g[2][2][V];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int v = 0; v < V; ++v) g[u >> 1][u & 1][v] = 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int p = a + i;
      if (p >= P) continue;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int q = b + j;
        if (q >= Q) continue;
        const long long o = (((long long)n * P + p) * Q + q) * C + c;
        const Pack<T, V> dv = ldp<T, V>(dy + o);
        uint32_t w4[2] = {0u, 0u};
        if constexpr (V == 8) {
          const uint2 u2 = *reinterpret_cast<const uint2*>(idx + o);
          w4[0] = u2.x; w4[1] = u2.y;
        } else {
          w4[0] = *reinterpret_cast<const uint32_t*>(idx + o);
        }
        // cell pixel (dh, dw) sits at window position (dh + 1 - 2i, dw + 1 - 2j)
#pragma unroll
        for (int dh = 0; dh < 2; ++dh) {
          const int r = dh + 1 - 2 * i;
          if (r < 0) continue;
#pragma unroll
          for (int dw = 0; dw < 2; ++dw) {
            const int s2 = dw + 1 - 2 * j;
            if (s2 < 0) continue;
#pragma unroll
            for (int v = 0; v < V; ++v)
              if (((w4[v >> 2] >> (8 * (v & 3))) & 0xffu) == (unsigned)(r * 3 + s2)) g[dh][dw][v] += dv.get(v);
          }
        }
      }
    }
#pragma unroll
    for (int dh = 0; dh < 2; ++dh) {
      const int h = 2 * a + dh;
      if (h >= H) continue;
#pragma unroll
      for (int dw = 0; dw < 2; ++dw) {
        const int w = 2 * b + dw;
        if (w >= W) continue;
        T* dst = dx + (((long long)n * H + h) * W + w) * C + c;
        if (accumulate) {
          const Pack<T, V> old = ldp<T, V>(dst);
#pragma unroll
          for (int v = 0; v < V; ++v) g[dh][dw][v] += old.get(v);
        }
        stp<T, V>(dst, pack_of<T, V>(g[dh][dw]));
      }
    }
  }
}

// ---- dz = dy * act'(y) ---------------------------------------------------------------------------
template <typename T>
__global__ void act_vjp_kernel(const T* __restrict__ y, const T* dy, T* dz, long long n, int act) {  // dz may be dy
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (long long)gridDim.x * blockDim.x)
    dz[i] = from_f32<T>(to_f32<T>(dy[i]) * act_mask(to_f32<T>(y[i]), act));
}

// ---- out[c] = sum over rows of a[row][c]; one block per 64 columns, fixed summation order ------
constexpr int COLSUM_CHUNKS = 512;
template <typename T>
__global__ __launch_bounds__(256) void colsum_kernel(const T* __restrict__ a, long long rows, int cols, float* __restrict__ out) {
  __shared__ double red[4][64];
  const int cl = threadIdx.x & 63, rl = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + cl;
  double s = 0.0;  // bias cotangents cancel heavily: sum in double
  if (c < cols)
    for (long long r = rl; r < rows; r += 4) s += (double)to_f32<T>(a[r * cols + c]);
  red[rl][cl] = s;
  __syncthreads();
  if (rl == 0 && c < cols) out[c] = (float)(red[0][cl] + red[1][cl] + red[2][cl] + red[3][cl]);
}

// The same in two stages for tall matrices: chunk z adds its rows (four row lanes per column, as above)
// into part[z][c], then the chunks are added in order.
template <typename T>
__global__ __launch_bounds__(256) void colsum_part_kernel(const T* __restrict__ a, long long rows, int cols, long long per,
                                                          double* __restrict__ part) {
  __shared__ double red[4][64];
  const int cl = threadIdx.x & 63, rl = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + cl;
  const long long r0 = (long long)blockIdx.y * per, r1 = r0 + per < rows ? r0 + per : rows;
  double s = 0.0;
  if (c < cols)
    for (long long r = r0 + rl; r < r1; r += 4) s += (double)to_f32<T>(a[r * cols + c]);
  red[rl][cl] = s;
  __syncthreads();
  if (rl == 0 && c < cols) part[(long long)blockIdx.y * cols + c] = red[0][cl] + red[1][cl] + red[2][cl] + red[3][cl];
}
// second stage: 64 columns x 16 chunk lanes per block; a lane adds every 16th chunk, the 16 lane sums are added in order
__global__ __launch_bounds__(1024) void colsum_final_kernel(const double* __restrict__ part, int chunks, int cols, float* __restrict__ out) {
  __shared__ double red[16][64];
  const int cl = threadIdx.x & 63, zl = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + cl;
  double s = 0.0;
  if (c < cols)
    for (int z = zl; z < chunks; z += 16) s += part[(long long)z * cols + c];
  red[zl][cl] = s;
  __syncthreads();
  if (zl == 0 && c < cols) {
    double t = 0.0;
    for (int k = 0; k < 16; ++k) t += red[k][cl];
    out[c] = (float)t;
  }
}

// ---- zero padding of one axis: dst[o][c][i] = c < C ? src[o][c][i] : 0 with Cp >= C channels -------
// (a first layer with 1 or 3 input channels is run with 8, so that it can take the 16-byte loaders)
template <typename T>
__global__ void pad_axis_kernel(const T* __restrict__ src, T* __restrict__ dst, long long outer, int C, int Cp, int inner) {
  const long long total = outer * Cp * inner;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
    const int in = (int)(i % inner);
    const long long t = i / inner;
    const int c = (int)(t % Cp);
    const long long o = t / Cp;
    dst[i] = c < C ? src[(o * C + c) * inner + in] : (T)0;
  }
}
// pixels of up to 8 bf16 channels -> 8 channels, one 16-byte store per pixel
__global__ void pad_pixels8_kernel(const bf16_t* __restrict__ src, bf16_t* __restrict__ dst, long long pixels, int C) {
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < pixels; i += (long long)gridDim.x * blockDim.x) {
    uint32_t v[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) v[c] = c < C ? (uint32_t)src[i * C + c] : 0u;
    uint4 o;
    o.x = v[0] | (v[1] << 16); o.y = v[2] | (v[3] << 16); o.z = v[4] | (v[5] << 16); o.w = v[6] | (v[7] << 16);
    reinterpret_cast<uint4*>(dst)[i] = o;
  }
}
// the reverse for gradients: dst[o][c][i] = src[o][c][i], c < C
__global__ void unpad_axis_kernel(const float* __restrict__ src, float* __restrict__ dst, long long outer, int C, int Cp, int inner) {
  const long long total = outer * C * inner;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
    const int in = (int)(i % inner);
    const long long t = i / inner;
    const int c = (int)(t % C);
    const long long o = t / C;
    dst[i] = src[(o * Cp + c) * inner + in];
  }
}

// ---- a stride-2 first layer as a stride-1 layer over 2x2 pixel blocks ---------------------------------
// A filter of odd size (R,S) with stride 2 over a batch of C <= 4 channels, padded by `pad` with H + 2 pad and
// W + 2 pad even, is the same sum as a filter of size ((R+1)/2, (S+1)/2) with stride 1 and no padding over the
// folded batch xf[n][hf][wf][(eh*2 + ew)*4 + c] = xpad[n][2 hf + eh][2 wf + ew][c] (xpad: the batch with its
// zero border; channels c >= C are zero), with wf[r'][s'][(eh*2 + ew)*4 + c][k] = w[2r' + eh][2s' + ew][c][k]
// (zero where 2r' + eh = R or 2s' + ew = S).  For a 7x7 filter on 3 channels the reduction axis is 4*4*16 = 256
// long instead of 7*7*8 = 392 (channels padded to the 16-byte loaders' 8), and every operand chunk holds two pixels.
__global__ __launch_bounds__(256) void fold2_pixels_kernel(const bf16_t* __restrict__ src, bf16_t* __restrict__ dst, int N, int H,
                                                           int W, int C, int pad, int Hf, int Wf) {
  const long long total = (long long)N * Hf * Wf * 2;  // one 16-byte chunk (eh fixed, both ew) per thread
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
    const int eh = (int)(i & 1);
    const long long pix = i >> 1;
    const int wf = (int)(pix % Wf);
    const long long t = pix / Wf;
    const int hf = (int)(t % Hf), n = (int)(t / Hf);
    const int h = 2 * hf + eh - pad;
    uint32_t v[8];
#pragma unroll
    for (int ew = 0; ew < 2; ++ew) {
      const int w = 2 * wf + ew - pad;
      const bool in = h >= 0 && h < H && w >= 0 && w < W;
      const long long base = (((long long)n * H + h) * W + w) * C;
#pragma unroll
      for (int c = 0; c < 4; ++c) v[ew * 4 + c] = (in && c < C) ? (uint32_t)src[base + c] : 0u;
    }
    uint4 o;
    o.x = v[0] | (v[1] << 16); o.y = v[2] | (v[3] << 16); o.z = v[4] | (v[5] << 16); o.w = v[6] | (v[7] << 16);
    reinterpret_cast<uint4*>(dst)[i] = o;
  }
}
__global__ void fold2_filter_kernel(const bf16_t* __restrict__ w, bf16_t* __restrict__ wf, int R, int S, int C, int K) {
  const int Sf = (S + 1) / 2, total = ((R + 1) / 2) * Sf * 16 * K;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x) {
    const int k = i % K, t = i / K, cf = t % 16, tap = t / 16;
    const int r = 2 * (tap / Sf) + (cf >> 3), s = 2 * (tap % Sf) + ((cf >> 2) & 1), c = cf & 3;
    wf[i] = (r < R && s < S && c < C) ? w[((r * S + s) * C + c) * K + k] : (bf16_t)0;
  }
}
// the filter gradient back: dw[r][s][c][k] = dwf[r/2][s/2][((r&1)*2 + (s&1))*4 + c][k]
__global__ void unfold2_filter_grad_kernel(const float* __restrict__ dwf, float* __restrict__ dw, int R, int S, int C, int K) {
  const int Sf = (S + 1) / 2, total = R * S * C * K;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x) {
    const int k = i % K, t = i / K, c = t % C, tap = t / C, r = tap / S, s = tap % S;
    dw[i] = dwf[(((r >> 1) * Sf + (s >> 1)) * 16 + ((r & 1) * 2 + (s & 1)) * 4 + c) * K + k];
  }
}

// ---- SGD with momentum ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void sgd_kernel(float* __restrict__ param, float* __restrict__ vel,
                                                  const float* __restrict__ grad, bf16_t* __restrict__ lowp,
                                                  long long n4, long long n, float lr, float mu) {
  long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const long long stride = (long long)gridDim.x * blockDim.x;
  for (; i < n4; i += stride) {
    float4 p = reinterpret_cast<float4*>(param)[i], v = reinterpret_cast<float4*>(vel)[i];
    const float4 g = reinterpret_cast<const float4*>(grad)[i];
    v.x = mu * v.x + g.x; v.y = mu * v.y + g.y; v.z = mu * v.z + g.z; v.w = mu * v.w + g.w;
    p.x -= lr * v.x; p.y -= lr * v.y; p.z -= lr * v.z; p.w -= lr * v.w;
    reinterpret_cast<float4*>(vel)[i] = v;
    reinterpret_cast<float4*>(param)[i] = p;
    if (lowp) {
      uint2 o;
      o.x = (uint32_t)f32_to_bf16(p.x) | ((uint32_t)f32_to_bf16(p.y) << 16);
      o.y = (uint32_t)f32_to_bf16(p.z) | ((uint32_t)f32_to_bf16(p.w) << 16);
      reinterpret_cast<uint2*>(lowp)[i] = o;
    }
  }
  // tail (count not a multiple of 4)
  for (long long j = n4 * 4 + (long long)blockIdx.x * blockDim.x + threadIdx.x; j < n; j += stride) {
    float v = mu * vel[j] + grad[j];
    float p = param[j] - lr * v;
    vel[j] = v;
    param[j] = p;
    if (lowp) lowp[j] = f32_to_bf16(p);
  }
}

// dst[i] = bf16(src[i]), round to nearest even
__global__ __launch_bounds__(256) void round_bf16_kernel(const float* __restrict__ src, bf16_t* __restrict__ dst,
                                                         long long n4, long long n) {
  long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const long long stride = (long long)gridDim.x * blockDim.x;
  for (; i < n4; i += stride) {
    const float4 p = reinterpret_cast<const float4*>(src)[i];
    uint2 o;
    o.x = (uint32_t)f32_to_bf16(p.x) | ((uint32_t)f32_to_bf16(p.y) << 16);
    o.y = (uint32_t)f32_to_bf16(p.z) | ((uint32_t)f32_to_bf16(p.w) << 16);
    reinterpret_cast<uint2*>(dst)[i] = o;
  }
  for (long long j = n4 * 4 + (long long)blockIdx.x * blockDim.x + threadIdx.x; j < n; j += stride) dst[j] = f32_to_bf16(src[j]);
}

// y[j, :] = x[index[j], :]; a thread copies one element, adjacent threads adjacent columns
template <typename T>
__global__ __launch_bounds__(256) void gather_rows_fwd_kernel(const T* __restrict__ x, const int32_t* __restrict__ index,
                                                              T* __restrict__ y, int rows, int cols, long long total) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const long long j = i / cols;
  const int col = (int)(i - j * cols);
  const int r = index[j];
  y[i] = (r >= 0 && r < rows) ? x[(long long)r * cols + col] : from_f32<T>(0.f);
}
// dx[index[j], :] += dy[j, :] for j = 0, 1, ... in that order: a thread owns one column and walks the gathered
// rows, so a row that is named twice receives its two contributions in a fixed order, and only the named rows of
// dx are read or written: count * cols element updates whatever the size of dx.
template <typename T>
__global__ __launch_bounds__(256) void gather_rows_vjp_kernel(const T* __restrict__ dy, const int32_t* __restrict__ index,
                                                              T* dx, int rows, int cols, int count) {
  const int col = blockIdx.x * blockDim.x + threadIdx.x;
  if (col >= cols) return;
  for (int j = 0; j < count; ++j) {
    const int r = index[j];
    if (r < 0 || r >= rows) continue;
    T* p = dx + (long long)r * cols + col;
    *p = from_f32<T>(to_f32<T>(*p) + to_f32<T>(dy[(long long)j * cols + col]));
  }
}

}  // namespace

int gather_rows_fwd(const s4tf_gather_desc& d, const void* x, const int32_t* index, void* y, hipStream_t st) {
  ProfScope ps(PC_ELEMENTWISE, st);
  const long long total = (long long)d.count * d.cols;
  const unsigned blocks = (unsigned)((total + 255) / 256);
  if (d.dtype == S4TF_BF16)
    hipLaunchKernelGGL(gather_rows_fwd_kernel<bf16_t>, dim3(blocks), dim3(256), 0, st, (const bf16_t*)x, index, (bf16_t*)y, d.rows, d.cols, total);
  else
    hipLaunchKernelGGL(gather_rows_fwd_kernel<float>, dim3(blocks), dim3(256), 0, st, (const float*)x, index, (float*)y, d.rows, d.cols, total);
  return launch_status("gather_rows_fwd");
}
int gather_rows_vjp(const s4tf_gather_desc& d, const void* dy, const int32_t* index, void* dx, hipStream_t st) {
  ProfScope ps(PC_ELEMENTWISE, st);
  const unsigned blocks = (unsigned)((d.cols + 255) / 256);
  if (d.dtype == S4TF_BF16)
    hipLaunchKernelGGL(gather_rows_vjp_kernel<bf16_t>, dim3(blocks), dim3(256), 0, st, (const bf16_t*)dy, index, (bf16_t*)dx, d.rows, d.cols, d.count);
  else
    hipLaunchKernelGGL(gather_rows_vjp_kernel<float>, dim3(blocks), dim3(256), 0, st, (const float*)dy, index, (float*)dx, d.rows, d.cols, d.count);
  return launch_status("gather_rows_vjp");
}

int round_to_bf16(size_t count, const float* src, void* dst, hipStream_t st) {
  ProfScope ps(PC_ELEMENTWISE, st);
  const long long n4 = (long long)(count / 4);
  long long blocks = (n4 + 255) / 256;
  if (blocks < 1) blocks = 1;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(round_bf16_kernel, dim3((unsigned)blocks), dim3(256), 0, st, src, (bf16_t*)dst, n4, (long long)count);
  return launch_status("round_to_bf16");
}

bool pool_saves_positions(const s4tf_pool_desc& d) {
  return d.kind == S4TF_POOL_MAX3S2 && d.c % (d.dtype == S4TF_BF16 ? 8 : 4) == 0;
}

int pool_fwd(const s4tf_pool_desc& d, const void* x, void* y, hipStream_t st, unsigned char* idx) {
  ProfScope ps(PC_POOL, st);
  const bool avg = d.kind == S4TF_POOL_AVG2;
  const int P = avg ? d.h / 2 : (d.h - 1) / 2 + 1, Q = avg ? d.w / 2 : (d.w - 1) / 2 + 1;
  dim3 grid(blocks_for((long long)d.n * P * Q * d.c)), block(256);
  const int V = d.dtype == S4TF_BF16 ? 8 : 4;
  const bool vec = d.c % V == 0 && aligned16(x) && aligned16(y);
  dim3 vgrid(blocks_for((long long)d.n * P * Q * d.c / V));
  if (d.dtype == S4TF_BF16) {
    typedef bf16_t T;
    if (avg) hipLaunchKernelGGL(avgpool2_fwd_kernel<T>, grid, block, 0, st, (const T*)x, (T*)y, d.n, d.h, d.w, d.c);
    else if (vec) hipLaunchKernelGGL((maxpool3s2_fwd_kernel<T, 8>), vgrid, block, 0, st, (const T*)x, (T*)y, idx, d.n, d.h, d.w, d.c);
    else hipLaunchKernelGGL((maxpool3s2_fwd_kernel<T, 1>), grid, block, 0, st, (const T*)x, (T*)y, (unsigned char*)nullptr, d.n, d.h, d.w, d.c);
  } else {
    typedef float T;
    if (avg) hipLaunchKernelGGL(avgpool2_fwd_kernel<T>, grid, block, 0, st, (const T*)x, (T*)y, d.n, d.h, d.w, d.c);
    else if (vec) hipLaunchKernelGGL((maxpool3s2_fwd_kernel<T, 4>), vgrid, block, 0, st, (const T*)x, (T*)y, idx, d.n, d.h, d.w, d.c);
    else hipLaunchKernelGGL((maxpool3s2_fwd_kernel<T, 1>), grid, block, 0, st, (const T*)x, (T*)y, (unsigned char*)nullptr, d.n, d.h, d.w, d.c);
  }
  return launch_status("pool_fwd");
}

int pool_vjp(const s4tf_pool_desc& d, const void* x, const void* dy, void* dx, hipStream_t st, const unsigned char* idx) {
  ProfScope ps(PC_POOL, st);
  if (idx && pool_saves_positions(d) && aligned16(x) && aligned16(dy) && aligned16(dx)) {  // the forward pass's own conditions
    const long long cells = (long long)d.n * ((d.h + 1) / 2) * ((d.w + 1) / 2);
    if (d.dtype == S4TF_BF16)
      hipLaunchKernelGGL((maxpool3s2_vjp_idx_kernel<bf16_t, 8>), dim3(blocks_for(cells * d.c / 8)), dim3(256), 0, st, idx, (const bf16_t*)dy,
                         (bf16_t*)dx, d.n, d.h, d.w, d.c, d.accumulate_dx);
    else
      hipLaunchKernelGGL((maxpool3s2_vjp_idx_kernel<float, 4>), dim3(blocks_for(cells * d.c / 4)), dim3(256), 0, st, idx, (const float*)dy,
                         (float*)dx, d.n, d.h, d.w, d.c, d.accumulate_dx);
    return launch_status("pool_vjp");
  }
  const bool avg = d.kind == S4TF_POOL_AVG2;
  dim3 grid(blocks_for((long long)d.n * d.h * d.w * d.c)), block(256);
  const int V = d.dtype == S4TF_BF16 ? 8 : 4;
  const bool vec = d.c % V == 0 && aligned16(x) && aligned16(dy) && aligned16(dx);
  dim3 vgrid(blocks_for((long long)d.n * d.h * d.w * d.c / V));
  const long long cells = (long long)d.n * ((d.h + 1) / 2) * ((d.w + 1) / 2);  // max pool: a thread per 2x2 cell
  if (!avg) {  // a multiple of 8 workgroups: the kernel hands each XCD an equal run of them
    grid = dim3((blocks_for(cells * d.c) + 7) / 8 * 8);
    vgrid = dim3((blocks_for(cells * d.c / V) + 7) / 8 * 8);
  }
  if (d.dtype == S4TF_BF16) {
    typedef bf16_t T;
    if (avg) hipLaunchKernelGGL(avgpool2_vjp_kernel<T>, grid, block, 0, st, (const T*)dy, (T*)dx, d.n, d.h, d.w, d.c, d.accumulate_dx);
    else if (vec) hipLaunchKernelGGL((maxpool3s2_vjp_kernel<T, 8>), vgrid, block, 0, st, (const T*)x, (const T*)dy, (T*)dx, d.n, d.h, d.w, d.c, d.accumulate_dx);
    else hipLaunchKernelGGL((maxpool3s2_vjp_kernel<T, 1>), grid, block, 0, st, (const T*)x, (const T*)dy, (T*)dx, d.n, d.h, d.w, d.c, d.accumulate_dx);
  } else {
    typedef float T;
    if (avg) hipLaunchKernelGGL(avgpool2_vjp_kernel<T>, grid, block, 0, st, (const T*)dy, (T*)dx, d.n, d.h, d.w, d.c, d.accumulate_dx);
    else if (vec) hipLaunchKernelGGL((maxpool3s2_vjp_kernel<T, 4>), vgrid, block, 0, st, (const T*)x, (const T*)dy, (T*)dx, d.n, d.h, d.w, d.c, d.accumulate_dx);
    else hipLaunchKernelGGL((maxpool3s2_vjp_kernel<T, 1>), grid, block, 0, st, (const T*)x, (const T*)dy, (T*)dx, d.n, d.h, d.w, d.c, d.accumulate_dx);
  }
  return launch_status("pool_vjp");
}

int act_vjp(int dtype, int act, const void* y, const void* dy, void* dz, size_t count, hipStream_t st) {
  ProfScope ps(PC_ELEMENTWISE, st);
  dim3 grid(blocks_for((long long)count)), block(256);
  if (dtype == S4TF_BF16)
    hipLaunchKernelGGL(act_vjp_kernel<bf16_t>, grid, block, 0, st, (const bf16_t*)y, (const bf16_t*)dy, (bf16_t*)dz, (long long)count, act);
  else
    hipLaunchKernelGGL(act_vjp_kernel<float>, grid, block, 0, st, (const float*)y, (const float*)dy, (float*)dz, (long long)count, act);
  return launch_status("act_vjp");
}

size_t colsum_workspace(size_t rows, int cols) {
  return rows >= 4096 ? (size_t)COLSUM_CHUNKS * cols * sizeof(double) : 0;
}

int colsum(int dtype, const void* a, size_t rows, int cols, float* out, hipStream_t st, void* ws, size_t ws_bytes) {
  ProfScope ps(PC_ELEMENTWISE, st);
  dim3 grid((cols + 63) / 64), block(256);
  const size_t need = colsum_workspace(rows, cols);
  if (need > 0 && ws && ws_bytes >= need) {  // tall: one block per 64 columns alone would walk all rows
    const long long per = ((long long)rows + COLSUM_CHUNKS - 1) / COLSUM_CHUNKS;
    const int chunks = (int)(((long long)rows + per - 1) / per);
    double* part = static_cast<double*>(ws);
    if (dtype == S4TF_BF16)
      hipLaunchKernelGGL(colsum_part_kernel<bf16_t>, dim3(grid.x, chunks), block, 0, st, (const bf16_t*)a, (long long)rows, cols, per, part);
    else
      hipLaunchKernelGGL(colsum_part_kernel<float>, dim3(grid.x, chunks), block, 0, st, (const float*)a, (long long)rows, cols, per, part);
    hipLaunchKernelGGL(colsum_final_kernel, grid, dim3(1024), 0, st, part, chunks, cols, out);
    return launch_status("colsum");
  }
  if (dtype == S4TF_BF16)
    hipLaunchKernelGGL(colsum_kernel<bf16_t>, grid, block, 0, st, (const bf16_t*)a, (long long)rows, cols, out);
  else
    hipLaunchKernelGGL(colsum_kernel<float>, grid, block, 0, st, (const float*)a, (long long)rows, cols, out);
  return launch_status("colsum");
}

int pad_channels(int dtype, const void* src, void* dst, long long outer, int C, int Cp, int inner, hipStream_t st) {
  ProfScope ps(PC_ELEMENTWISE, st);
  if (dtype == S4TF_BF16 && inner == 1 && Cp == 8) {
    hipLaunchKernelGGL(pad_pixels8_kernel, dim3(blocks_for(outer)), dim3(256), 0, st, (const bf16_t*)src, (bf16_t*)dst, outer, C);
  } else if (dtype == S4TF_BF16) {
    hipLaunchKernelGGL(pad_axis_kernel<bf16_t>, dim3(blocks_for(outer * Cp * inner)), dim3(256), 0, st, (const bf16_t*)src, (bf16_t*)dst, outer, C, Cp, inner);
  } else {
    hipLaunchKernelGGL(pad_axis_kernel<float>, dim3(blocks_for(outer * Cp * inner)), dim3(256), 0, st, (const float*)src, (float*)dst, outer, C, Cp, inner);
  }
  return launch_status("pad_channels");
}

int unpad_channels_f32(const float* src, float* dst, long long outer, int C, int Cp, int inner, hipStream_t st) {
  ProfScope ps(PC_ELEMENTWISE, st);
  hipLaunchKernelGGL(unpad_axis_kernel, dim3(blocks_for(outer * C * inner)), dim3(256), 0, st, src, dst, outer, C, Cp, inner);
  return launch_status("unpad_channels");
}

int fold2_pixels(const void* x, void* xf, int N, int H, int W, int C, int pad, hipStream_t st) {
  ProfScope ps(PC_ELEMENTWISE, st);
  const int Hf = (H + 2 * pad) / 2, Wf = (W + 2 * pad) / 2;
  hipLaunchKernelGGL(fold2_pixels_kernel, dim3(blocks_for((long long)N * Hf * Wf * 2)), dim3(256), 0, st, (const bf16_t*)x,
                     (bf16_t*)xf, N, H, W, C, pad, Hf, Wf);
  return launch_status("fold2_pixels");
}
int fold2_filter(const void* w, void* wf, int R, int S, int C, int K, hipStream_t st) {
  ProfScope ps(PC_ELEMENTWISE, st);
  hipLaunchKernelGGL(fold2_filter_kernel, dim3(blocks_for((long long)((R + 1) / 2) * ((S + 1) / 2) * 16 * K)), dim3(256), 0, st,
                     (const bf16_t*)w, (bf16_t*)wf, R, S, C, K);
  return launch_status("fold2_filter");
}
int unfold2_filter_grad(const float* dwf, float* dw, int R, int S, int C, int K, hipStream_t st) {
  ProfScope ps(PC_ELEMENTWISE, st);
  hipLaunchKernelGGL(unfold2_filter_grad_kernel, dim3(blocks_for((long long)R * S * C * K)), dim3(256), 0, st, dwf, dw, R, S, C, K);
  return launch_status("unfold2_filter_grad");
}

int sgd(size_t count, float* param, float* vel, const float* grad, void* lowp, float lr, float mu,
        hipStream_t st) {
  if (count == 0) return S4TF_OK;
  ProfScope ps(PC_SGD, st);
  long long n4 = (long long)(count / 4);
  dim3 grid(blocks_for(n4 > 0 ? n4 : 1)), block(256);
  hipLaunchKernelGGL(sgd_kernel, grid, block, 0, st, param, vel, grad, (bf16_t*)lowp, n4, (long long)count, lr, mu);
  return launch_status("sgd");
}

}  // namespace s4tf
