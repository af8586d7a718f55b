// BatchNorm (training mode) + residual + ReLU/ReLU6, forward and pullback, NHWC.
// Every kernel here is bound by HBM bandwidth.  All of them use the same decomposition:
// grid = (channel blocks, pixel chunks); a thread = (channel vector of V adjacent channels,
// pixel lane) keeps its per-channel constants in registers and walks its pixels with 16-byte
// accesses, four pixels in flight per thread, so a wavefront reads whole contiguous runs of
// the NHWC tensor and enough loads are outstanding to cover the memory latency.
//   forward   stats: per-channel sum and sum of squares of (x - pivot), pivot = x at pixel 0
//             (keeps the one-pass variance free of cancellation); the pixel lanes of a block are
//             added with wavefront shuffles and LDS in a fixed order, the blocks' partial sums
//             are added in double by a finalize kernel -> mean, invstd
//             apply:  y = act(gamma*(x-mean)*invstd + beta (+ residual))
//   pullback  reduce: dbeta = sum dz, dgamma = sum dz*xhat with dz = dy*act'(y)   (in double)
//             apply:  dx = gamma*invstd*(dz - dbeta/m - xhat*dgamma/m),  dresidual (+)= dz
#include <mutex>

#include "s4tf_internal.h"
#include "pack.h"

namespace s4tf {
namespace {

// Scratch of the forward entry point that allocates nothing (s4tf_bn_relu_fwd_static): the statistics
// kernels' per-chunk partial sums, which the plain entry point keeps in the caller's workspace.  Device
// memory that comes with the library's code object, one copy per GPU, held until the process ends.  The
// name below is a host-side stand-in, not a device address: host code only ever uses the per-device
// address that static_scratch() looks up once.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)1 << 20;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
std::mutex g_scratch_mutex;
void* g_scratch_ptr[64] = {};

int static_scratch(void** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return fail(S4TF_ERR_DEVICE, "cannot tell the current device");
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {  // once per device, with that device current: each GPU has its own copy at its own address
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return fail(S4TF_ERR_DEVICE, "cannot locate the static scratch on device %d: %s", dev, hipGetErrorString(e));
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return S4TF_OK;
}

constexpr int MAX_CHUNKS = 2048;
constexpr int UNROLL = 4;

// The finalize kernels give a block a few adjacent channels and have it walk the rows of a table of partial
// sums, a few bytes per row.  Workgroup ids are dealt round-robin to the 8 XCDs, each with an L2 of its own:
// with channel block = workgroup id, every XCD ends up fetching every line of the table.  Dealt as below, an
// XCD's blocks cover one contiguous range of channels, and a line is fetched by one L2 only (measured over a
// ResNet-50 step: the statistics finalize kernels fetch 155 MB instead of 480, the pullback's 125 instead of 241).
__device__ inline int xcd_channel_block() {
  const int n = gridDim.x, b = blockIdx.x;
  return n % 8 == 0 ? (b % 8) * (n / 8) + b / 8 : b;
}

struct Plan {
  int V, cvb, cblocks, pl, chunks;
  long long per;  // pixels per chunk
};

Plan make_plan(size_t M, int C, int dtype, int target_blocks, int min_pixels_per_lane) {
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
  long long want = target_blocks / p.cblocks;
  if (want < 1) want = 1;
  if (want > MAX_CHUNKS) want = MAX_CHUNKS;
  long long per = ((long long)M + want - 1) / want;
  long long minper = (long long)p.pl * min_pixels_per_lane;
  if (per < minper) per = minper;
  p.per = per;
  p.chunks = (int)(((long long)M + per - 1) / per);
  return p;
}

// Sum over the pixel lanes of a block; the result is valid in the threads with pl == 0.
// Thread t has cvl = t % cvb with cvb a power of two <= 64, so inside a wavefront the lanes that
// share a channel vector are the ones whose lane ids differ by multiples of cvb: a butterfly of
// lane shuffles adds them, then the four wavefronts are added through LDS.  The order of the
// additions is fixed, so the result does not depend on scheduling.
// (`first`: lane distance at which the butterfly starts; 64: the lanes of a wavefront have been added already)
template <typename A, int NV>
__device__ inline void block_lane_sum(A (&v)[NV], A* red, int first, int cvb, int cvl) {
  for (int off = first; off < 64; off <<= 1) {
#pragma unroll
    for (int e = 0; e < NV; ++e) v[e] += __shfl_xor(v[e], off, 64);
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // red[e][wavefront][cvl]: adjacent lanes touch adjacent words (no bank conflicts)
  if (lane < cvb) {
#pragma unroll
    for (int e = 0; e < NV; ++e) red[(size_t)(e * 4 + wave) * cvb + cvl] = v[e];
  }
  __syncthreads();
  if (threadIdx.x < cvb) {
#pragma unroll
    for (int e = 0; e < NV; ++e)
      v[e] = ((red[(size_t)(e * 4) * cvb + cvl] + red[(size_t)(e * 4 + 1) * cvb + cvl]) + red[(size_t)(e * 4 + 2) * cvb + cvl]) +
             red[(size_t)(e * 4 + 3) * cvb + cvl];
  }
}

template <typename A, int NV>
__device__ inline void block_lane_sum(A (&v)[NV], A* red, int cvb, int cvl) {
  block_lane_sum<A, NV>(v, red, cvb, cvb, cvl);
}

// Walk the pixels first, first+step, ... < p1 of a chunk, UNROLL at a time: `load(m, slot)` issues
// the loads of pixel m into slot, `use(m, slot)` consumes them.
template <typename Load, typename Use>
__device__ inline void walk_pixels(long long first, long long p1, long long step, Load load, Use use) {
  long long m = first;
  for (; m + (UNROLL - 1) * step < p1; m += UNROLL * step) {
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) load(m + u * step, u);
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) use(m + u * step, u);
  }
  // the last, partial round (at most UNROLL - 1 pixels) the same way: all its loads first (a slot past the end
  // re-loads pixel m and is not used), so that it costs one memory latency and not one per pixel
  if (m < p1) {
#pragma unroll
    for (int u = 0; u < UNROLL - 1; ++u) load(m + u * step < p1 ? m + u * step : m, u);
#pragma unroll
    for (int u = 0; u < UNROLL - 1; ++u)
      if (m + u * step < p1) use(m + u * step, u);
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
  const Pack<T, V> pv = ldp<T, V>(x + c);
  const long long p0 = (long long)blockIdx.y * per, p1 = p0 + per < M ? p0 + per : M;
  if (live) {
    Pack<T, V> xv[UNROLL];
    walk_pixels(p0 + pl, p1, pl_count,
                [&](long long m, int u) { xv[u] = ldp<T, V>(x + m * C + c); },
                [&](long long, int u) {
#pragma unroll
                  for (int e = 0; e < V; ++e) {
                    float d = xv[u].get(e) - pv.get(e);
                    acc[e] += d;
                    acc[V + e] += d * d;
                  }
                });
  }
  block_lane_sum<float, 2 * V>(acc, red, cvb, cvl);
  if (pl == 0 && live) {
    float* dst = part + (long long)blockIdx.y * 2 * C;
#pragma unroll
    for (int e = 0; e < V; ++e) {
      dst[c + e] = acc[e];
      dst[C + c + e] = acc[V + e];
    }
  }
}

// Adds the chunks' partial sums [chunk][2][C] of 8 channels per block of 1024 threads in double: 128
// lanes per channel stride over the chunks (several loads in flight each), a shuffle butterfly adds
// the lanes of a wavefront, thread c adds the 16 wavefront totals in order.  Result in threads 0..7.
constexpr int FIN_THREADS = 1024;
template <typename P>
__device__ inline void sum_chunks(const P* __restrict__ part, int chunks, int C, int c, double (*sh)[2][8], double& s1,
                                  double& s2) {
  const int zl = threadIdx.x >> 3, cl = threadIdx.x & 7;
  double a = 0.0, b = 0.0;
  if (c < C) {
#pragma unroll 4
    for (int z = zl; z < chunks; z += FIN_THREADS / 8) {
      a += (double)part[(long long)z * 2 * C + c];
      b += (double)part[(long long)z * 2 * C + C + c];
    }
  }
  for (int off = 8; off < 64; off <<= 1) {
    a += __shfl_xor(a, off, 64);
    b += __shfl_xor(b, off, 64);
  }
  if ((threadIdx.x & 63) < 8) {
    sh[threadIdx.x >> 6][0][cl] = a;
    sh[threadIdx.x >> 6][1][cl] = b;
  }
  __syncthreads();
  s1 = s2 = 0.0;
  if (threadIdx.x < 8)
    for (int w = 0; w < FIN_THREADS / 64; ++w) {
      s1 += sh[w][0][cl];
      s2 += sh[w][1][cl];
    }
}

template <typename T>
__global__ __launch_bounds__(FIN_THREADS) void bn_stats_finalize_kernel(const T* __restrict__ x, const float* __restrict__ part,
                                                                        int chunks, long long M, int C, float eps,
                                                                        float* __restrict__ mean, float* __restrict__ invstd) {
  __shared__ double sh[FIN_THREADS / 64][2][8];
  const int c = xcd_channel_block() * 8 + (threadIdx.x & 7);
  double s1, s2;
  sum_chunks<float>(part, chunks, C, c, sh, s1, s2);
  if (threadIdx.x >= 8 || c >= C) return;
  double pivot = (double)to_f32<T>(x[c]);
  double ms = s1 / (double)M;
  double var = s2 / (double)M - ms * ms;
  if (var < 0.0) var = 0.0;
  mean[c] = (float)(pivot + ms);
  invstd[c] = (float)(1.0 / sqrt(var + (double)eps));
}

// Statistics from the partial sums a convolution left behind: run i covers rows [i*rows, min(M, (i+1)*rows))
// and holds per channel s_i = sum x and q_i = sum (x - s_i/n_i)^2.  With S = sum s_i:
//   mean = S/M,   M*var = sum q_i + sum s_i^2/n_i - S^2/M      (all in double)
// The table is laid out channel by channel, part[(which*C + c)*runs + i]: the runs of a channel are adjacent,
// so the 1024/CPB lanes that a block gives each of its CPB channels read whole cache lines (run-major, the
// table of a 64-channel layer with thousands of runs cost every block a fetch of every line: 31 us for the
// first layer of a ResNet-50 at batch 64, 10 us for each 56x56 layer).  The lanes of a wavefront are added by
// a shuffle butterfly, the wavefronts of a channel through LDS, in a fixed order.
template <int CPB>
__global__ __launch_bounds__(1024) void bn_stats_from_runs_kernel(const float* __restrict__ part, int runs, int rows,
                                                                  long long M, int C, float eps, float* __restrict__ mean,
                                                                  float* __restrict__ invstd) {
  constexpr int ZL = 1024 / CPB, WPC = ZL / 64;  // lanes and wavefronts per channel
  static_assert(ZL % 64 == 0, "a wavefront serves one channel");
  __shared__ double sh[16][3];
  const int cl = threadIdx.x / ZL, zl = threadIdx.x % ZL, c = xcd_channel_block() * CPB + cl;
  const double inv_rows = 1.0 / (double)rows;
  const double inv_last = 1.0 / (double)(M - (long long)(runs - 1) * rows);
  double v[3] = {0.0, 0.0, 0.0};
  if (c < C) {
    const float* __restrict__ srow = part + (long long)c * runs;
    const float* __restrict__ qrow = part + ((long long)C + c) * runs;
#pragma unroll 4
    for (int i = zl; i < runs; i += ZL) {
      const double s = (double)srow[i];
      const double q = (double)qrow[i];
      v[0] += s;
      v[1] += q;
      v[2] += s * s * (i == runs - 1 ? inv_last : inv_rows);
    }
  }
  for (int off = 1; off < 64; off <<= 1) {
#pragma unroll
    for (int e = 0; e < 3; ++e) v[e] += __shfl_xor(v[e], off, 64);
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) {
#pragma unroll
    for (int e = 0; e < 3; ++e) sh[wave][e] = v[e];
  }
  __syncthreads();
  if (zl != 0 || c >= C) return;
  double S = 0.0, Q = 0.0, W = 0.0;
  for (int w = cl * WPC; w < (cl + 1) * WPC; ++w) { S += sh[w][0]; Q += sh[w][1]; W += sh[w][2]; }
  double var = (Q + W - S * S / (double)M) / (double)M;
  if (var < 0.0) var = 0.0;
  mean[c] = (float)(S / (double)M);
  invstd[c] = (float)(1.0 / sqrt(var + (double)eps));
}

// z of the forward pass.  The pullback recomputes it (and from it the activation mask) with the same
// operations in the same order, so the two agree bit for bit.
__device__ inline float bn_z(float x, float mu, float sc, float be) { return fmaf(x - mu, sc, be); }
// act'(y) read off z: y = round_T(act(z)) is positive exactly when z is (rounding keeps the sign; an fp32
// z below 2^-133 that bf16 flushes to zero is the one exception, and harmless), and below 6 exactly when z
// is below 6 (fp32) or below 6 - 2^-6, the tie that rounds up to 6 (bf16).
template <typename T> __device__ inline float remask_hi(int act) {
  return act == S4TF_ACT_RELU6 ? (sizeof(T) == 2 ? 5.984375f : 6.f) : __builtin_inff();
}

// INFER: `mean` and `invstd` are the running mean and the running VARIANCE (inference mode); a template
// parameter so that the training-mode kernel does not carry the square roots and divisions
template <typename T, int V, bool INFER>
__device__ __forceinline__ void bn_apply_body(const T* __restrict__ x, const T* __restrict__ res,
                                              const float* __restrict__ gamma, const float* __restrict__ beta,
                                              const float* __restrict__ mean, const float* __restrict__ invstd,
                                              T* __restrict__ y, unsigned char* __restrict__ bits, long long M,
                                              int C, int cvb, long long per, int act, float infer_eps) {
  const int CV = C / V, pl_count = blockDim.x / cvb;
  const int cvl = threadIdx.x % cvb, pl = threadIdx.x / cvb;
  const int cv = blockIdx.x * cvb + cvl;
  if (cv >= CV) return;
  const int c = cv * V;
  const float mhi = remask_hi<T>(act);
  float mu[V], sc[V], be[V];
#pragma unroll
  for (int e = 0; e < V; ++e) {
    mu[e] = mean[c + e];
    float is = invstd[c + e];
    if constexpr (INFER) is = 1.0f / sqrtf(is + infer_eps);
    sc[e] = gamma[c + e] * is;
    be[e] = beta[c + e];
  }
  const float act_lo = act == S4TF_ACT_NONE ? -__builtin_inff() : 0.f;
  const float act_hi = act == S4TF_ACT_RELU6 ? 6.f : __builtin_inff();
  const long long p0 = (long long)blockIdx.y * per, p1 = p0 + per < M ? p0 + per : M;
  Pack<T, V> xv[UNROLL], rv[UNROLL];
  walk_pixels(p0 + pl, p1, pl_count,
              [&](long long m, int u) {
                xv[u] = ldp<T, V>(x + m * C + c);
                if (res) rv[u] = ldp<T, V>(res + m * C + c);
              },
              [&](long long m, int u) {
                float o[V];
                unsigned b = 0;
#pragma unroll
                for (int e = 0; e < V; ++e) {
                  float z = bn_z(xv[u].get(e), mu[e], sc[e], be[e]);
                  if (res) z += rv[u].get(e);
                  o[e] = fminf(fmaxf(z, act_lo), act_hi);  // the activation as a clamp: no branch per element
                  b |= (z > 0.f && z < mhi) ? (1u << e) : 0u;
                }
                stp<T, V>(y + m * C + c, pack_of<T, V>(o));
                // act'(y) of this thread's V outputs, one bit each (see remask_hi), for the pullback
                if (bits) bits[m * CV + cv] = (unsigned char)b;
              });
}

#define BN_APPLY_ARGS                                                                                                \
  const T *__restrict__ x, const T *__restrict__ res, const float *__restrict__ gamma, const float *__restrict__ beta, \
      const float *__restrict__ mean, const float *__restrict__ invstd, T *__restrict__ y,                            \
      unsigned char *__restrict__ bits, long long M, int C, int cvb, long long per, int act, float infer_eps
template <typename T, int V> __global__ __launch_bounds__(256) void bn_apply_kernel(BN_APPLY_ARGS) {
  bn_apply_body<T, V, false>(x, res, gamma, beta, mean, invstd, y, bits, M, C, cvb, per, act, infer_eps);
}
template <typename T, int V> __global__ __launch_bounds__(256) void bn_apply_infer_kernel(BN_APPLY_ARGS) {
  bn_apply_body<T, V, true>(x, res, gamma, beta, mean, invstd, y, bits, M, C, cvb, per, act, infer_eps);
}

// dbeta and dgamma are sums of cotangents whose terms largely cancel (the cotangent reaching a
// BatchNorm from a convolution that is itself followed by BatchNorm sums to almost zero), so the
// sums across threads and blocks are kept in double.  A thread's own sum is fp32: the plan gives a
// thread a few dozen pixels (at most a few hundred for the largest tensors the library accepts), whose
// independent rounding errors stay near 1e-6 of the sum of the terms' magnitudes, and the 32 registers
// that double accumulators would hold through the loop are what lets a fourth wavefront share a SIMD
// (the kernel is bound by how many loads it keeps in flight: 898 -> 750 us over the BatchNorms of a
// ResNet-50).
template <typename T, int V, bool REMASK, bool BITS = false>
__device__ __forceinline__ void bn_vjp_reduce_body(const T* __restrict__ x, const T* __restrict__ y,
                                                   const T* __restrict__ dy, const float* __restrict__ mean,
                                                   const float* __restrict__ invstd, const float* __restrict__ gamma,
                                                   const float* __restrict__ beta, double* __restrict__ part,
                                                   long long M, int C, int cvb, long long per, int act,
                                                   const unsigned char* __restrict__ bits = nullptr) {
  extern __shared__ double redd[];
  const int CV = C / V, pl_count = blockDim.x / cvb;
  const int cvl = threadIdx.x % cvb, pl = threadIdx.x / cvb;
  const int cv = blockIdx.x * cvb + cvl;
  const bool live = cv < CV;
  const int c = live ? cv * V : 0;
  // beta given (the forward pass had no residual): the activation mask comes from z recomputed out of x,
  // and y is not read
  constexpr bool remask = REMASK;  // a template parameter: each version holds only the registers it needs
  const float mhi = remask_hi<T>(act);
  const float yhi = act == S4TF_ACT_RELU6 ? 6.f : __builtin_inff();  // act'(y) = 1 on (0, yhi); y is finite
  double acc[2 * V];
  float grp[2 * V], mu[V], is[V], sc[V], be[V];
#pragma unroll
  for (int e = 0; e < V; ++e) {
    acc[e] = acc[V + e] = 0.0;
    grp[e] = grp[V + e] = 0.f;
    mu[e] = mean[c + e];
    is[e] = invstd[c + e];
    sc[e] = remask ? gamma[c + e] * is[e] : 0.f;
    be[e] = remask ? beta[c + e] : 0.f;
  }
  const long long p0 = (long long)blockIdx.y * per, p1 = p0 + per < M ? p0 + per : M;
  if (live) {
    Pack<T, V> xv[UNROLL], dv[UNROLL], yv[UNROLL];
    unsigned char bv[UNROLL];
    walk_pixels(p0 + pl, p1, pl_count,
                [&](long long m, int u) {
                  xv[u] = ldp<T, V>(x + m * C + c);
                  dv[u] = ldp<T, V>(dy + m * C + c);
                  if (BITS) bv[u] = bits[m * CV + cv];
                  else if (act != S4TF_ACT_NONE && !remask) yv[u] = ldp<T, V>(y + m * C + c);
                },
                [&](long long, int u) {
#pragma unroll
                  for (int e = 0; e < V; ++e) {
                    float dz = dv[u].get(e);
                    if (BITS) {
                      dz = ((bv[u] >> e) & 1) ? dz : 0.f;
                    } else if (remask) {
                      const float z = bn_z(xv[u].get(e), mu[e], sc[e], be[e]);
                      dz = (z > 0.f && z < mhi) ? dz : 0.f;
                    } else if (act != S4TF_ACT_NONE) {
                      const float yy = yv[u].get(e);
                      dz = (yy > 0.f && yy < yhi) ? dz : 0.f;
                    }
                    grp[e] += dz;
                    grp[V + e] += dz * ((xv[u].get(e) - mu[e]) * is[e]);
                  }
                });
  }
  // lanes of a wavefront that share a channel vector: a butterfly in fp32 (a tree over at most 64 thread sums);
  // from there on (wavefronts of the block, blocks of the grid) the sums are double
  for (int off = cvb; off < 64; off <<= 1) {
#pragma unroll
    for (int e = 0; e < 2 * V; ++e) grp[e] += __shfl_xor(grp[e], off, 64);
  }
#pragma unroll
  for (int e = 0; e < 2 * V; ++e) acc[e] = (double)grp[e];
  block_lane_sum<double, 2 * V>(acc, redd, 64, cvb, cvl);
  if (pl == 0 && live) {
    double* dst = part + (long long)blockIdx.y * 2 * C;
#pragma unroll
    for (int e = 0; e < V; ++e) {
      dst[c + e] = acc[e];
      dst[C + c + e] = acc[V + e];
    }
  }
}

#define BN_VJP_REDUCE_ARGS                                                                                           \
  const T *__restrict__ x, const T *__restrict__ y, const T *__restrict__ dy, const float *__restrict__ mean,        \
      const float *__restrict__ invstd, const float *__restrict__ gamma, const float *__restrict__ beta,             \
      double *__restrict__ part, long long M, int C, int cvb, long long per, int act
template <typename T, int V> __global__ __launch_bounds__(256) void bn_vjp_reduce_kernel(BN_VJP_REDUCE_ARGS) {
  bn_vjp_reduce_body<T, V, false>(x, y, dy, mean, invstd, gamma, beta, part, M, C, cvb, per, act);
}
template <typename T, int V> __global__ __launch_bounds__(256) void bn_vjp_reduce_remask_kernel(BN_VJP_REDUCE_ARGS) {
  bn_vjp_reduce_body<T, V, true>(x, y, dy, mean, invstd, gamma, beta, part, M, C, cvb, per, act);
}
// act'(y) from the bits the forward pass left (here `y` points at them): one byte per thread and pixel instead of V outputs
template <typename T, int V> __global__ __launch_bounds__(256) void bn_vjp_reduce_bits_kernel(BN_VJP_REDUCE_ARGS) {
  bn_vjp_reduce_body<T, V, false, true>(x, nullptr, dy, mean, invstd, gamma, beta, part, M, C, cvb, per, act,
                                        reinterpret_cast<const unsigned char*>(y));
}

__global__ __launch_bounds__(FIN_THREADS) void bn_vjp_finalize_kernel(const double* __restrict__ part, int chunks, int C,
                                                                      float* __restrict__ dgamma, float* __restrict__ dbeta) {
  __shared__ double sh[FIN_THREADS / 64][2][8];
  const int c = xcd_channel_block() * 8 + (threadIdx.x & 7);
  double s1, s2;
  sum_chunks<double>(part, chunks, C, c, sh, s1, s2);
  if (threadIdx.x >= 8 || c >= C) return;
  dbeta[c] = (float)s1;
  dgamma[c] = (float)s2;
}

template <typename T, int V, bool REMASK, bool BITS = false, bool ACCDX = false>
__device__ __forceinline__ void bn_vjp_apply_body(const T* __restrict__ x, const T* __restrict__ y,
                                                           const T* __restrict__ dy, const float* __restrict__ gamma,
                                                           const float* __restrict__ mean, const float* __restrict__ invstd,
                                                           const float* __restrict__ beta,
                                                           const float* __restrict__ dgamma, const float* __restrict__ dbeta,
                                                           T* __restrict__ dx, T* dres, int acc_dres, long long M, int C,
                                                           int cvb, long long per, int act,
                                                           const unsigned char* __restrict__ bits = nullptr) {
  const int CV = C / V, pl_count = blockDim.x / cvb;
  const int cvl = threadIdx.x % cvb, pl = threadIdx.x / cvb;
  const int cv = blockIdx.x * cvb + cvl;
  if (cv >= CV) return;
  const int c = cv * V;
  const float invM = 1.0f / (float)M;
  constexpr bool remask = REMASK;  // as in the reduction kernel
  const float mhi = remask_hi<T>(act);
  const float yhi = act == S4TF_ACT_RELU6 ? 6.f : __builtin_inff();  // act'(y) = 1 on (0, yhi); y is finite
  // dx = gs*(dz - dbeta/M - xhat*dgamma/M) with xhat = (x - mu)*invstd, as  gs*dz - (x - mu)*a2 - a0:
  // four values per channel (five with beta) instead of five (six)
  float mu[V], gs[V], a0[V], a2[V], be[V];
#pragma unroll
  for (int e = 0; e < V; ++e) {
    const float is = invstd[c + e];
    mu[e] = mean[c + e];
    be[e] = remask ? beta[c + e] : 0.f;
    gs[e] = gamma[c + e] * is;
    a0[e] = gs[e] * (dbeta[c + e] * invM);
    a2[e] = gs[e] * (is * (dgamma[c + e] * invM));
  }
  const long long p0 = (long long)blockIdx.y * per, p1 = p0 + per < M ? p0 + per : M;
  Pack<T, V> xv[UNROLL], dv[UNROLL], yv[UNROLL], ov[UNROLL], av[UNROLL];
  unsigned char bv[UNROLL];
  walk_pixels(p0 + pl, p1, pl_count,
              [&](long long m, int u) {
                xv[u] = ldp<T, V>(x + m * C + c);
                dv[u] = ldp<T, V>(dy + m * C + c);
                if (BITS) bv[u] = bits[m * CV + cv];
                else if (act != S4TF_ACT_NONE && !remask) yv[u] = ldp<T, V>(y + m * C + c);
                if (dres && acc_dres) ov[u] = ldp<T, V>(dres + m * C + c);
                if (ACCDX) av[u] = ldp<T, V>(dx + m * C + c);  // the cotangent dx already holds
              },
              [&](long long m, int u) {
                float o[V], r[V];
#pragma unroll
                for (int e = 0; e < V; ++e) {
                  float dz = dv[u].get(e);
                  const float xc = xv[u].get(e) - mu[e];
                  if (BITS) {
                    dz = ((bv[u] >> e) & 1) ? dz : 0.f;
                  } else if (remask) {
                    const float z = fmaf(xc, gs[e], be[e]);  // bn_z, sharing the subtraction
                    dz = (z > 0.f && z < mhi) ? dz : 0.f;
                  } else if (act != S4TF_ACT_NONE) {
                    const float yy = yv[u].get(e);
                    dz = (yy > 0.f && yy < yhi) ? dz : 0.f;
                  }
                  o[e] = fmaf(gs[e], dz, -fmaf(xc, a2[e], a0[e]));
                  if (ACCDX) o[e] += av[u].get(e);
                  r[e] = (dres && acc_dres) ? ov[u].get(e) + dz : dz;
                }
                stp<T, V>(dx + m * C + c, pack_of<T, V>(o));
                if (dres) stp<T, V>(dres + m * C + c, pack_of<T, V>(r));
              });
}
#define BN_VJP_APPLY_ARGS                                                                                            \
  const T *__restrict__ x, const T *__restrict__ y, const T *__restrict__ dy, const float *__restrict__ gamma,       \
      const float *__restrict__ mean, const float *__restrict__ invstd, const float *__restrict__ beta,              \
      const float *__restrict__ dgamma, const float *__restrict__ dbeta, T *__restrict__ dx, T *dres, int acc_dres,  \
      long long M, int C, int cvb, long long per, int act
template <typename T, int V> __global__ __launch_bounds__(256) void bn_vjp_apply_kernel(BN_VJP_APPLY_ARGS) {
  bn_vjp_apply_body<T, V, false>(x, y, dy, gamma, mean, invstd, beta, dgamma, dbeta, dx, dres, acc_dres, M, C, cvb, per, act);
}
template <typename T, int V> __global__ __launch_bounds__(256) void bn_vjp_apply_remask_kernel(BN_VJP_APPLY_ARGS) {
  bn_vjp_apply_body<T, V, true>(x, y, dy, gamma, mean, invstd, beta, dgamma, dbeta, dx, dres, acc_dres, M, C, cvb, per, act);
}
template <typename T, int V> __global__ __launch_bounds__(256) void bn_vjp_apply_bits_kernel(BN_VJP_APPLY_ARGS) {
  bn_vjp_apply_body<T, V, false, true>(x, nullptr, dy, gamma, mean, invstd, beta, dgamma, dbeta, dx, dres, acc_dres, M, C,
                                       cvb, per, act, reinterpret_cast<const unsigned char*>(y));
}
// the same three, adding into the cotangent dx already holds (separate instances: the plain ones keep their registers)
template <typename T, int V> __global__ __launch_bounds__(256) void bn_vjp_apply_acc_kernel(BN_VJP_APPLY_ARGS) {
  bn_vjp_apply_body<T, V, false, false, true>(x, y, dy, gamma, mean, invstd, beta, dgamma, dbeta, dx, dres, acc_dres, M, C, cvb, per, act);
}
template <typename T, int V> __global__ __launch_bounds__(256) void bn_vjp_apply_remask_acc_kernel(BN_VJP_APPLY_ARGS) {
  bn_vjp_apply_body<T, V, true, false, true>(x, y, dy, gamma, mean, invstd, beta, dgamma, dbeta, dx, dres, acc_dres, M, C, cvb, per, act);
}
template <typename T, int V> __global__ __launch_bounds__(256) void bn_vjp_apply_bits_acc_kernel(BN_VJP_APPLY_ARGS) {
  bn_vjp_apply_body<T, V, false, true, true>(x, nullptr, dy, gamma, mean, invstd, beta, dgamma, dbeta, dx, dres, acc_dres, M, C,
                                             cvb, per, act, reinterpret_cast<const unsigned char*>(y));
}

}  // namespace

// Bytes of the activation bits of an (M, C) tensor: one byte per channel vector and pixel.  The reduction and
// the apply plans of one tensor use the same vector width, so the byte a forward thread wrote is the byte a
// pullback thread reads.
size_t bn_mask_bytes(size_t M, int C, int dtype) {
  int V = dtype == S4TF_BF16 ? 8 : 4;
  if (C % V) V = 1;
  return M * (size_t)(C / V);
}

size_t bn_workspace(size_t M, int C) {
  (void)M;
  return (size_t)MAX_CHUNKS * 2 * C * sizeof(double);
}

// KERNEL<T, V> for the descriptor's dtype and the plan's vector width
#define BN_LAUNCH(KERNEL, plan, shm, ...)                                                                       \
  do {                                                                                                          \
    dim3 grid_((plan).cblocks, (plan).chunks), block_(256);                                                     \
    if (d.dtype == S4TF_BF16) {                                                                                 \
      typedef bf16_t T;                                                                                         \
      if ((plan).V == 8) hipLaunchKernelGGL((KERNEL<T, 8>), grid_, block_, shm, st, __VA_ARGS__);               \
      else hipLaunchKernelGGL((KERNEL<T, 1>), grid_, block_, shm, st, __VA_ARGS__);                             \
    } else {                                                                                                    \
      typedef float T;                                                                                          \
      if ((plan).V == 4) hipLaunchKernelGGL((KERNEL<T, 4>), grid_, block_, shm, st, __VA_ARGS__);               \
      else hipLaunchKernelGGL((KERNEL<T, 1>), grid_, block_, shm, st, __VA_ARGS__);                             \
    }                                                                                                           \
  } while (0)

int bn_fwd(const s4tf_bn_desc& d, const void* x, const void* res, const float* gamma, const float* beta,
           void* y, float* mean, float* invstd, void* ws, hipStream_t st, const float* stats_part, int stats_rows,
           unsigned char* maskbits) {
  const long long M = (long long)d.n * d.h * d.w;
  const int C = d.c;
  const Plan pr = make_plan((size_t)M, C, d.dtype, 1024, 16);  // reduction: fewer, longer blocks
  const Plan pa = make_plan((size_t)M, C, d.dtype, 2048, UNROLL);
  float* part = static_cast<float*>(ws);
  int rc;
  if (stats_part && stats_rows > 0) {
    ProfScope ps(PC_BN_STATS, st);
    const int runs = (int)((M + stats_rows - 1) / stats_rows);
    // lanes per channel by the length of its row of the table: 128 up to 512 runs, 512 up to 2048, else 1024
    if (runs <= 512)
      hipLaunchKernelGGL(bn_stats_from_runs_kernel<8>, dim3((C + 7) / 8), dim3(1024), 0, st, stats_part, runs, stats_rows, M, C,
                         d.eps, mean, invstd);
    else if (runs <= 2048)
      hipLaunchKernelGGL(bn_stats_from_runs_kernel<2>, dim3((C + 1) / 2), dim3(1024), 0, st, stats_part, runs, stats_rows, M, C,
                         d.eps, mean, invstd);
    else
      hipLaunchKernelGGL(bn_stats_from_runs_kernel<1>, dim3(C), dim3(1024), 0, st, stats_part, runs, stats_rows, M, C,
                         d.eps, mean, invstd);
    if ((rc = launch_status("bn_stats_from_runs")) != S4TF_OK) return rc;
  } else {
    ProfScope ps(PC_BN_STATS, st);
    BN_LAUNCH(bn_stats_kernel, pr, (size_t)4 * pr.cvb * 2 * pr.V * sizeof(float), (const T*)x, part, M, C, pr.cvb, pr.per);
    if ((rc = launch_status("bn_stats")) != S4TF_OK) return rc;
    if (d.dtype == S4TF_BF16)
      hipLaunchKernelGGL((bn_stats_finalize_kernel<bf16_t>), dim3((C + 7) / 8), dim3(FIN_THREADS), 0, st, (const bf16_t*)x, part, pr.chunks, M, C, d.eps, mean, invstd);
    else
      hipLaunchKernelGGL((bn_stats_finalize_kernel<float>), dim3((C + 7) / 8), dim3(FIN_THREADS), 0, st, (const float*)x, part, pr.chunks, M, C, d.eps, mean, invstd);
    if ((rc = launch_status("bn_stats_finalize")) != S4TF_OK) return rc;
  }
  ProfScope ps(PC_BN_APPLY, st);
  BN_LAUNCH(bn_apply_kernel, pa, 0, (const T*)x, (const T*)res, gamma, beta, mean, invstd, (T*)y, maskbits, M, C, pa.cvb,
            pa.per, d.act, -1.f);
  return launch_status("bn_apply");
}

int bn_inference_fwd(const s4tf_bn_desc& d, const void* x, const void* res, const float* gamma, const float* beta,
                     const float* running_mean, const float* running_var, void* y, hipStream_t st) {
  const long long M = (long long)d.n * d.h * d.w;
  const int C = d.c;
  const Plan pa = make_plan((size_t)M, C, d.dtype, 2048, UNROLL);
  ProfScope ps(PC_BN_APPLY, st);
  BN_LAUNCH(bn_apply_infer_kernel, pa, 0, (const T*)x, (const T*)res, gamma, beta, running_mean, running_var, (T*)y,
            (unsigned char*)nullptr, M, C, pa.cvb, pa.per, d.act, d.eps);
  return launch_status("bn_inference");
}

namespace {
__global__ void bn_update_running_kernel(const float* __restrict__ mean, const float* __restrict__ invstd,
                                         float* __restrict__ rm, float* __restrict__ rv, int C, double count,
                                         float momentum, float eps) {
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= C) return;
  const double is = (double)invstd[c];
  const double var = 1.0 / (is * is) - (double)eps;                       // the biased batch variance
  const double unbiased = count > 1.0 ? var * count / (count - 1.0) : var;
  rm[c] = (float)((1.0 - (double)momentum) * (double)rm[c] + (double)momentum * (double)mean[c]);
  rv[c] = (float)((1.0 - (double)momentum) * (double)rv[c] + (double)momentum * unbiased);
}
// w'[i][k] = w[i][k] * s_k with s_k = gamma_k / sqrt(rv_k + eps); thread 0..K-1 of block 0 also writes the bias
template <typename T>
__global__ __launch_bounds__(256) void bn_fold_kernel(const T* __restrict__ w, const float* __restrict__ bias,
                                                      const float* __restrict__ gamma, const float* __restrict__ beta,
                                                      const float* __restrict__ rm, const float* __restrict__ rv,
                                                      T* __restrict__ w_out, float* __restrict__ bias_out, long long total,
                                                      int K, float eps) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < K) {
    const float s = gamma[i] / sqrtf(rv[i] + eps);
    bias_out[i] = fmaf((bias ? bias[i] : 0.f) - rm[i], s, beta[i]);
  }
  if (i >= total) return;
  const int k = (int)(i % K);
  w_out[i] = from_f32<T>(to_f32<T>(w[i]) * (gamma[k] / sqrtf(rv[k] + eps)));
}
}  // namespace

int bn_update_running(int C, size_t count, float momentum, float eps, const float* mean, const float* invstd,
                      float* rm, float* rv, hipStream_t st) {
  ProfScope ps(PC_ELEMENTWISE, st);
  hipLaunchKernelGGL(bn_update_running_kernel, dim3((C + 255) / 256), dim3(256), 0, st, mean, invstd, rm, rv, C, (double)count,
                     momentum, eps);
  return launch_status("bn_update_running");
}
int bn_fold(int dtype, long long rows, int K, const void* w, const float* bias, const float* gamma, const float* beta,
            const float* rm, const float* rv, float eps, void* w_out, float* bias_out, hipStream_t st) {
  ProfScope ps(PC_ELEMENTWISE, st);
  const long long total = rows * K;
  const long long span = total > K ? total : K;
  const unsigned blocks = (unsigned)((span + 255) / 256);
  if (dtype == S4TF_BF16)
    hipLaunchKernelGGL(bn_fold_kernel<bf16_t>, dim3(blocks), dim3(256), 0, st, (const bf16_t*)w, bias, gamma, beta, rm, rv,
                       (bf16_t*)w_out, bias_out, total, K, eps);
  else
    hipLaunchKernelGGL(bn_fold_kernel<float>, dim3(blocks), dim3(256), 0, st, (const float*)w, bias, gamma, beta, rm, rv,
                       (float*)w_out, bias_out, total, K, eps);
  return launch_status("bn_fold");
}

size_t bn_fwd_scratch_bytes(const s4tf_bn_desc& d) {
  const Plan pr = make_plan((size_t)d.n * d.h * d.w, d.c, d.dtype, 1024, 16);  // the reduction plan of bn_fwd
  return (size_t)pr.chunks * 2 * d.c * sizeof(float);
}
size_t bn_static_scratch_capacity() { return STATIC_SCRATCH_BYTES; }

int bn_fwd_static(const s4tf_bn_desc& d, const void* x, const void* res, const float* gamma, const float* beta,
                  void* y, float* mean, float* invstd, hipStream_t st) {
  const size_t want = bn_fwd_scratch_bytes(d);
  if (want > STATIC_SCRATCH_BYTES)
    return fail(S4TF_ERR_WORKSPACE, "bn: this shape needs %zu bytes of partial sums, the static scratch holds %zu", want,
                (size_t)STATIC_SCRATCH_BYTES);
  void* ptr = nullptr;
  int rc = static_scratch(&ptr);
  if (rc != S4TF_OK) return rc;
  // every partial sum the finalize kernel reads is written by the statistics kernel of the same call: nothing
  // has to start at zero, and what an earlier call left behind is never read
  return bn_fwd(d, x, res, gamma, beta, y, mean, invstd, ptr, st);
}

int bn_vjp(const s4tf_bn_desc& d, const void* x, const void* y, const float* gamma, const float* beta, const float* mean,
           const float* invstd, const void* dy, void* dx, void* dres, float* dgamma, float* dbeta,
           void* ws, hipStream_t st, const unsigned char* maskbits) {
  const long long M = (long long)d.n * d.h * d.w;
  const int C = d.c;
  if (dres || d.act == S4TF_ACT_NONE) beta = nullptr;  // with a residual z cannot be rebuilt from x alone
  if (beta || d.act == S4TF_ACT_NONE) maskbits = nullptr;
  if (maskbits) y = maskbits;  // the bits kernels take them through the y argument
  const Plan pr = make_plan((size_t)M, C, d.dtype, 512, UNROLL);  // measured over the ResNet-50 shapes: 512 blocks beat 1024 and 256
  const Plan pa = make_plan((size_t)M, C, d.dtype, 2048, UNROLL);
  double* part = static_cast<double*>(ws);
  int rc;
  {
    ProfScope ps(PC_BN_VJP_REDUCE, st);
    if (maskbits)
      BN_LAUNCH(bn_vjp_reduce_bits_kernel, pr, (size_t)4 * pr.cvb * 2 * pr.V * sizeof(double), (const T*)x, (const T*)y,
                (const T*)dy, mean, invstd, gamma, beta, part, M, C, pr.cvb, pr.per, d.act);
    else if (beta)
      BN_LAUNCH(bn_vjp_reduce_remask_kernel, pr, (size_t)4 * pr.cvb * 2 * pr.V * sizeof(double), (const T*)x, (const T*)y,
                (const T*)dy, mean, invstd, gamma, beta, part, M, C, pr.cvb, pr.per, d.act);
    else
      BN_LAUNCH(bn_vjp_reduce_kernel, pr, (size_t)4 * pr.cvb * 2 * pr.V * sizeof(double), (const T*)x, (const T*)y,
                (const T*)dy, mean, invstd, gamma, beta, part, M, C, pr.cvb, pr.per, d.act);
    if ((rc = launch_status("bn_vjp_reduce")) != S4TF_OK) return rc;
    hipLaunchKernelGGL(bn_vjp_finalize_kernel, dim3((C + 7) / 8), dim3(FIN_THREADS), 0, st, part, pr.chunks, C, dgamma, dbeta);
    if ((rc = launch_status("bn_vjp_finalize")) != S4TF_OK) return rc;
  }
  ProfScope ps(PC_BN_VJP_APPLY, st);
  if (d.accumulate_dx) {
    if (maskbits)
      BN_LAUNCH(bn_vjp_apply_bits_acc_kernel, pa, 0, (const T*)x, (const T*)y, (const T*)dy, gamma, mean, invstd, beta, dgamma, dbeta,
                (T*)dx, (T*)dres, d.accumulate_dres, M, C, pa.cvb, pa.per, d.act);
    else if (beta)
      BN_LAUNCH(bn_vjp_apply_remask_acc_kernel, pa, 0, (const T*)x, (const T*)y, (const T*)dy, gamma, mean, invstd, beta, dgamma, dbeta,
                (T*)dx, (T*)dres, d.accumulate_dres, M, C, pa.cvb, pa.per, d.act);
    else
      BN_LAUNCH(bn_vjp_apply_acc_kernel, pa, 0, (const T*)x, (const T*)y, (const T*)dy, gamma, mean, invstd, beta, dgamma, dbeta,
                (T*)dx, (T*)dres, d.accumulate_dres, M, C, pa.cvb, pa.per, d.act);
    return launch_status("bn_vjp_apply");
  }
  if (maskbits)
    BN_LAUNCH(bn_vjp_apply_bits_kernel, pa, 0, (const T*)x, (const T*)y, (const T*)dy, gamma, mean, invstd, beta, dgamma, dbeta,
              (T*)dx, (T*)dres, d.accumulate_dres, M, C, pa.cvb, pa.per, d.act);
  else if (beta)
    BN_LAUNCH(bn_vjp_apply_remask_kernel, pa, 0, (const T*)x, (const T*)y, (const T*)dy, gamma, mean, invstd, beta, dgamma, dbeta,
              (T*)dx, (T*)dres, d.accumulate_dres, M, C, pa.cvb, pa.per, d.act);
  else
    BN_LAUNCH(bn_vjp_apply_kernel, pa, 0, (const T*)x, (const T*)y, (const T*)dy, gamma, mean, invstd, beta, dgamma, dbeta,
              (T*)dx, (T*)dres, d.accumulate_dres, M, C, pa.cvb, pa.per, d.act);
  return launch_status("bn_vjp_apply");
}

}  // namespace s4tf
