// fp32 3x3 / stride 1 / padding 1 convolution for layers of few channels (16 or 32 in and out, or the 4
// padded channels of a first layer): the layers of a CIFAR ResNet.
//
// The implicit-GEMM kernel of igemm.hip gathers every k-tile of the im2col matrix from global memory, nine
// times the input in all, and pays a block barrier per 32 values of k: on a 131072 x 16 x 144 GEMM that is
// ~20 us, of which the matrix cores need 4.  Here a workgroup owns 128 consecutive output pixels (whole rows
// of one image), brings their input patch (the rows plus a one-pixel border, zeros outside the image) and the
// whole filter into LDS once, and multiplies out of LDS with no further barrier:
//   * v_mfma_f32_16x16x4_f32: 16 pixels x 16 outputs, 4 values of k = 4 adjacent channels of one tap, so a
//     16-channel layer spends nothing on padding; A: lane l = pixel l%16, channel l/16; B: lane l = channel
//     l/16, output l%16; D: register v of lane l = pixel 4*(l/16) + v, output l%16;
//   * a wavefront multiplies 32 pixels (two blocks of 16) by all outputs, so one read of a filter fragment
//     serves two MFMAs and one read of a pixel fragment serves CO/16;
//   * patch pixels are CI + 4 floats apart and filter rows CO (+16 from 32 outputs up) floats apart, which
//     spreads the 64 lanes of either fragment read over the 64 LDS banks.
// The pullback to the input (dgrad) of such a layer is the same convolution of dy with the filter turned by
// 180 degrees and its channel axes swapped: the same kernel, told to read the filter that way (FLIP).
// The forward pass can leave the partial sums of a BatchNorm that follows, per run of 32 pixels, exactly as
// igemm_fwd does.
#include "s4tf_internal.h"

namespace s4tf {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int G32 = 2;  // pixel blocks per wavefront of the 32-channel kernel

struct PatchArgs {
  const float* x;     // (N, H, W, CI)
  const float* w;     // forward: (3, 3, CI, CO); FLIP: (3, 3, CO, CI), read turned and transposed
  float* y;           // (N, H, W, CO)
  const float* bias;  // forward only, optional
  float* stats;       // forward only, optional: [sum | squared deviations][CO][runs of 32 pixels]
  int N, H, W, act, accumulate;
};

// G: blocks of 16 pixels per wavefront (2: 128 pixels per workgroup, 1: 64)
template <int CI, int CO, bool FLIP, int G>
__global__ __launch_bounds__(256) void patchconv_kernel(const PatchArgs a) {
  constexpr int TILE = 64 * G;
  constexpr int CS = CI + 4;                     // floats per patch pixel
  constexpr int WS = CO >= 32 ? CO + 16 : CO;    // floats per filter row
  constexpr int NB = CO / 16;
  constexpr int C4 = CI / 4;
  constexpr int PATCH_PIXELS = G == 2 ? 204 : 136;  // (TILE/W + 2) * (W + 2) at its largest, W = 32
  __shared__ __attribute__((aligned(16))) float wl[9 * CI * WS];
  __shared__ __attribute__((aligned(16))) float patch[PATCH_PIXELS * CS];
  const int H = a.H, W = a.W, TH = TILE / W, PW = W + 2;
  const int tiles_per_image = H / TH;
  const int n = blockIdx.x / tiles_per_image, p0 = (blockIdx.x - n * tiles_per_image) * TH;

  // Every global load of the prologue is issued before the first LDS store: one memory latency, not one per loop.
  // filter -> registers, 16 bytes at a time.  Forward: as it lies, (tap, ci) rows of CO.  FLIP: the filter lies
  // (tap, co) rows of CI; chunk i is 4 adjacent ci of row (8 - tap, co), with pairs of lanes on adjacent chunks
  // and co running over the lanes next (32-byte pieces of global memory; LDS stores two lanes to a bank)
  constexpr int WCH = 9 * CI * CO / 4;
  constexpr int WV = (WCH + 255) / 256;
  float4 wq[WV];
#pragma unroll
  for (int k = 0; k < WV; ++k) {
    const int i = threadIdx.x + k * 256;
    int src = i;
    if constexpr (FLIP) {
      const int lo = i % 2, co = (i / 2) % CO, hi = (i / (2 * CO)) % (CI / 8), tap = i / (CO * (CI / 4));
      src = ((8 - tap) * CO + co) * (CI / 4) + hi * 2 + lo;
    }
    wq[k] = i < WCH ? reinterpret_cast<const float4*>(a.w)[src] : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  // input rows p0-1 .. p0+TH, columns -1 .. W -> registers, 16 bytes (4 channels) at a time; zeros outside the image
  constexpr int PV = (PATCH_PIXELS * C4 + 255) / 256;
  const int chunks = (TH + 2) * PW * C4;
  float4 pv[PV];
#pragma unroll
  for (int k = 0; k < PV; ++k) {
    const int i = threadIdx.x + k * 256;
    const int c4 = i % C4, t = i / C4, pw = t % PW, pr = t / PW;
    const int h = p0 + pr - 1, wc = pw - 1;
    pv[k] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i < chunks && h >= 0 && h < H && wc >= 0 && wc < W)
      pv[k] = *reinterpret_cast<const float4*>(a.x + (((long long)n * H + h) * W + wc) * CI + c4 * 4);
  }
  // registers -> LDS: filter row (tap, ci), column co
#pragma unroll
  for (int k = 0; k < WV; ++k) {
    const int i = threadIdx.x + k * 256;
    if (i >= WCH) continue;
    if constexpr (FLIP) {
      const int lo = i % 2, co = (i / 2) % CO, hi = (i / (2 * CO)) % (CI / 8), tap = i / (CO * (CI / 4));
      float* dst = wl + (tap * CI + (hi * 2 + lo) * 4) * WS + co;
      dst[0] = wq[k].x; dst[WS] = wq[k].y; dst[2 * WS] = wq[k].z; dst[3 * WS] = wq[k].w;
    } else {
      const int co4 = i % (CO / 4), t = i / (CO / 4);
      *reinterpret_cast<float4*>(wl + t * WS + co4 * 4) = wq[k];
    }
  }
#pragma unroll
  for (int k = 0; k < PV; ++k) {
    const int i = threadIdx.x + k * 256;
    const int c4 = i % C4, t = i / C4;  // t = pr*PW + pw
    if (i < chunks) *reinterpret_cast<float4*>(patch + t * CS + c4 * 4) = pv[k];
  }
  __syncthreads();

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int abase[G];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    const int m = wave * 16 * G + g * 16 + (lane & 15);  // tile-local output pixel
    const int pr = m / W, pq = m - pr * W;
    abase[g] = (pr * PW + pq) * CS + (lane >> 4);
  }
  const int bbase = (lane >> 4) * WS + (lane & 15);
  f32x4 acc[G][NB];
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[g][nb] = f32x4{0.f, 0.f, 0.f, 0.f};
  // the fragments of tap t+1 are read while tap t is multiplied (the loop is unrolled: both sets are registers)
  float af[2][G][C4], bfr[2][C4][NB];
  auto read_tap = [&](int tap, int buf) {
    const int toff = ((tap / 3) * PW + (tap % 3)) * CS;
#pragma unroll
    for (int cg = 0; cg < C4; ++cg) {
#pragma unroll
      for (int g = 0; g < G; ++g) af[buf][g][cg] = patch[abase[g] + toff + cg * 4];
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) bfr[buf][cg][nb] = wl[bbase + (tap * CI + cg * 4) * WS + nb * 16];
    }
  };
  read_tap(0, 0);
#pragma unroll
  for (int tap = 0; tap < 9; ++tap) {
    if (tap + 1 < 9) read_tap(tap + 1, (tap + 1) & 1);
#pragma unroll
    for (int cg = 0; cg < C4; ++cg)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int g = 0; g < G; ++g)
          acc[g][nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(af[tap & 1][g][cg], bfr[tap & 1][cg][nb], acc[g][nb], 0, 0, 0);
  }

  const long long row0 = (long long)blockIdx.x * TILE + wave * 16 * G;  // this wavefront's first output pixel
  if (!FLIP && a.stats) {
    // per output channel over this wavefront's 16*G pixels: the sum, and the sum of squared deviations from
    // their own mean, both from deviations from a pivot (the first pixel's value) so that a channel mean of
    // many standard deviations costs no digits
    constexpr int RUN = 16 * G;
    const long long runs = (long long)a.N * H * W / RUN, run = row0 / RUN;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const float pivot = __shfl(acc[0][nb][0], lane & 15, 64);
      float s = 0.f, q = 0.f;
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const float dev = acc[g][nb][v] - pivot;
          s += dev;
          q = fmaf(dev, dev, q);
        }
      s += __shfl_xor(s, 16, 64); q += __shfl_xor(q, 16, 64);
      s += __shfl_xor(s, 32, 64); q += __shfl_xor(q, 32, 64);
      if (lane < 16) {
        const int col = nb * 16 + lane;
        a.stats[col * runs + run] = fmaf((float)RUN, pivot, s);
        a.stats[(CO + col) * runs + run] = fmaxf(q - s * s * (1.f / (float)RUN), 0.f);
      }
    }
  }
  const float act_lo = (!FLIP && a.act != S4TF_ACT_NONE) ? 0.f : -__builtin_inff();
  const float act_hi = (!FLIP && a.act == S4TF_ACT_RELU6) ? 6.f : __builtin_inff();
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const int col = nb * 16 + (lane & 15);
    const float bias = (!FLIP && a.bias) ? a.bias[col] : 0.f;
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        float* dst = a.y + (row0 + g * 16 + 4 * (lane >> 4) + v) * CO + col;
        float val = acc[g][nb][v] + bias;
        if (FLIP && a.accumulate) val += *dst;
        *dst = fminf(fmaxf(val, act_lo), act_hi);
      }
  }
}

template <int CI, int CO, bool FLIP, int G>
int launch_patch(const PatchArgs& a, hipStream_t st) {
  const unsigned tiles = (unsigned)((long long)a.N * a.H * a.W / (64 * G));
  hipLaunchKernelGGL((patchconv_kernel<CI, CO, FLIP, G>), dim3(tiles), dim3(256), 0, st, a);
  return launch_status("patchconv");
}

// pixel blocks per wavefront for a layer of C input channels
int groups_for(int C) { return C == 32 ? G32 : 2; }

bool shape_ok(const ConvGeom& g) {
  if (g.R != 3 || g.S != 3 || g.stride != 1 || g.pad != 1) return false;
  if (g.W != 16 && g.W != 32) return false;
  const int TH = 64 * groups_for(g.C) / g.W;  // rows of an image per workgroup
  return g.H % TH == 0 && (long long)g.N * g.H * g.W * (g.C > g.K ? g.C : g.K) < (1LL << 31);
}

}  // namespace

bool patchconv_fwd_ok(const ConvGeom& g, int dtype) {
  return dtype == S4TF_F32 && shape_ok(g) && ((g.C == 16 && g.K == 16) || (g.C == 32 && g.K == 32) || (g.C == 4 && g.K == 16));
}
bool patchconv_dgrad_ok(const ConvGeom& g, int dtype) {
  return dtype == S4TF_F32 && shape_ok(g) && ((g.C == 16 && g.K == 16) || (g.C == 32 && g.K == 32));
}

// y = act(conv(x, w) + bias); with `stats`, also the BatchNorm partial sums of igemm_fwd, per run of *stats_rows pixels
int patchconv_fwd(const ConvGeom& g, const void* x, const void* w, const float* bias, int act, void* y, float* stats,
                  int* stats_rows, hipStream_t st) {
  if (!aligned16(x) || !aligned16(w) || !aligned16(y)) return fail(S4TF_ERR_SHAPE, "patchconv: operands must be 16-byte aligned");
  PatchArgs a = {static_cast<const float*>(x), static_cast<const float*>(w), static_cast<float*>(y), bias, stats,
                 g.N, g.H, g.W, act, 0};
  if (stats_rows) *stats_rows = 16 * groups_for(g.C);
  if (g.C == 16) return launch_patch<16, 16, false, 2>(a, st);
  if (g.C == 32) return launch_patch<32, 32, false, G32>(a, st);
  return launch_patch<4, 16, false, 2>(a, st);
}

// dx (+)= the pullback of the same layer to its input
int patchconv_dgrad(const ConvGeom& g, const void* dy, const void* w, void* dx, int accumulate, hipStream_t st) {
  if (!aligned16(dy) || !aligned16(w) || !aligned16(dx)) return fail(S4TF_ERR_SHAPE, "patchconv: operands must be 16-byte aligned");
  PatchArgs a = {static_cast<const float*>(dy), static_cast<const float*>(w), static_cast<float*>(dx), nullptr, nullptr,
                 g.N, g.H, g.W, S4TF_ACT_NONE, accumulate};
  if (g.C == 16) return launch_patch<16, 16, true, 2>(a, st);
  return launch_patch<32, 32, true, G32>(a, st);
}

}  // namespace s4tf
