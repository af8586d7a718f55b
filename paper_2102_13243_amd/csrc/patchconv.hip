// fp32 3x3 / stride 1 / padding 1 convolution for layers of few channels (16, 32 or 64 in and out, or the 4
// padded channels of a first layer) on small images (8, 16 or 32 wide): the layers of a CIFAR ResNet.
//
// The implicit-GEMM kernel of igemm.hip gathers every k-tile of the im2col matrix from global memory, nine
// times the input in all, and pays a block barrier per 32 values of k: on a 131072 x 16 x 144 GEMM that is
// ~20 us, of which the matrix cores need 4.  Here a workgroup owns 128 consecutive output pixels (whole rows
// of one image, or two whole 8x8 images) and a block of 16 or 32 output channels, brings the pixels' input
// patch (their rows plus a one-pixel border, zeros outside the image) and its slice of the filter into LDS
// once, and multiplies out of LDS with no further barrier:
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
// 1x1 / stride 1 layers whose reduction axis is 16, 24, 32 or 64 channels (forward of an expansion layer, input
// pullback of a projection layer) take the same kernel with a single tap: 128 pixels and a block of 16, 32 or 48
// output channels per workgroup, one round of loads, a few MFMAs, the stores.  They are bound by the bytes they
// move; the implicit-GEMM kernel's fixed cost per workgroup (row decomposition, staged k-loop) was most of
// their time.
#include "s4tf_internal.h"

namespace s4tf {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int TILE = 128;          // output pixels per workgroup: 4 wavefronts x 2 blocks of 16
constexpr int PATCH_PIXELS = 204;  // the largest patch: 4 rows of a 32-wide image, (4 + 2) x (32 + 2)

struct PatchArgs {
  const float* x;     // (N, H, W, CI)
  const float* w;     // forward: (3, 3, CI, CO); FLIP: (3, 3, CO, CI), read turned and transposed
  float* y;           // (N, H, W, CO)
  const float* bias;  // forward only, optional
  float* stats;       // forward only, optional: [sum | squared deviations][KT][runs of 32 pixels]
  int N, H, W, act, accumulate;
  int KT;             // channels of y; workgroup (x, j) computes channels j*CO .. j*CO + CO-1
  int RH, IMGS;       // a tile is IMGS images x RH rows each (IMGS > 1: whole images)
};

// TAPS = 9: the 3x3 layers above.  TAPS = 1: a 1x1 / stride 1 layer with a short reduction axis (the expansion
// layers of an inverted-residual block and, with FLIP, the pullback of its projection layers): the "patch" is the
// tile's 128 pixels themselves, whatever the image shape.
template <int CI, int CO, bool FLIP, int TAPS = 9>
__global__ __launch_bounds__(256) void patchconv_kernel(const PatchArgs a) {
  constexpr int G = 2;  // blocks of 16 pixels per wavefront
  constexpr int CS = CI + 4;                                 // floats per patch pixel
  constexpr int WS = CO == 16 ? 16 : CO == 32 ? 48 : 80;     // floats per filter row: 16 or 48 modulo the 64 banks
  static_assert(CO == 16 || CO == 32 || CO == 48, "output blocks of 16, 32 or 48 channels");
  constexpr int NB = CO / 16;
  constexpr int C4 = CI / 4;
  constexpr int PPIX = TAPS == 1 ? TILE : PATCH_PIXELS;
  __shared__ __attribute__((aligned(16))) float wl[TAPS * CI * WS];
  __shared__ __attribute__((aligned(16))) float patch[PPIX * CS];
  const int H = a.H, W = a.W, PW = W + 2, RH = a.RH, PR = RH + 2, KT = a.KT, n0 = blockIdx.y * CO;
  int n = 0, p0 = 0;  // first image and first row of the tile
  if constexpr (TAPS == 1) {
  } else if (a.IMGS == 1) {
    const int tiles_per_image = H / RH;
    n = blockIdx.x / tiles_per_image;
    p0 = (blockIdx.x - n * tiles_per_image) * RH;
  } else {
    n = blockIdx.x * a.IMGS;
    p0 = 0;
  }

  // Every global load of the prologue is issued before the first LDS store: one memory latency, not one per loop.
  // filter -> registers, 16 bytes at a time.  Forward: (tap, ci) rows of KT, of which CO from n0 on.  FLIP: the filter
  // lies (tap, co) rows of CI with KT rows per tap; chunk i is 4 adjacent ci of row (TAPS-1 - tap, n0 + co), with pairs of
  // lanes on adjacent chunks and co running over the lanes next (32-byte pieces of global memory; LDS stores two
  // lanes to a bank)
  constexpr int WCH = TAPS * CI * CO / 4;
  constexpr int WV = (WCH + 255) / 256;
  float4 wq[WV];
#pragma unroll
  for (int k = 0; k < WV; ++k) {
    const int i = threadIdx.x + k * 256;
    int src;
    if constexpr (FLIP) {
      const int lo = i % 2, co = (i / 2) % CO, hi = (i / (2 * CO)) % (CI / 8), tap = i / (CO * (CI / 4));
      src = ((TAPS - 1 - tap) * KT + n0 + co) * (CI / 4) + hi * 2 + lo;
    } else {
      src = ((i / (CO / 4)) * KT + n0) / 4 + i % (CO / 4);
    }
    wq[k] = i < WCH ? reinterpret_cast<const float4*>(a.w)[src] : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  // per image of the tile, input rows p0-1 .. p0+RH, columns -1 .. W -> registers, 16 bytes (4 channels) at a
  // time; zeros outside the image
  constexpr int PV = (PPIX * C4 + 255) / 256;
  const int chunks = TAPS == 1 ? TILE * C4 : a.IMGS * PR * PW * C4;
  float4 pv[PV];
#pragma unroll
  for (int k = 0; k < PV; ++k) {
    const int i = threadIdx.x + k * 256;
    pv[k] = make_float4(0.f, 0.f, 0.f, 0.f);
    if constexpr (TAPS == 1) {
      if (i < chunks) pv[k] = reinterpret_cast<const float4*>(a.x + (long long)blockIdx.x * TILE * CI)[i];
    } else {
      const int c4 = i % C4, t = i / C4, pw = t % PW, prow = t / PW, img = prow / PR, pr = prow - img * PR;
      const int h = p0 + pr - 1, wc = pw - 1;
      if (i < chunks && h >= 0 && h < H && wc >= 0 && wc < W)
        pv[k] = *reinterpret_cast<const float4*>(a.x + (((long long)(n + img) * H + h) * W + wc) * CI + c4 * 4);
    }
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
    if constexpr (TAPS == 1) {
      abase[g] = m * CS + (lane >> 4);
    } else {
      const int row = m / W, pq = m - row * W, img = row / RH;
      abase[g] = ((row + 2 * img) * PW + pq) * CS + (lane >> 4);  // patch row img*(RH + 2) + (row - img*RH)
    }
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
    const int toff = TAPS == 1 ? 0 : ((tap / 3) * PW + (tap % 3)) * CS;
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
  for (int tap = 0; tap < TAPS; ++tap) {
    if (tap + 1 < TAPS) read_tap(tap + 1, (tap + 1) & 1);
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
        a.stats[(n0 + col) * runs + run] = fmaf((float)RUN, pivot, s);
        a.stats[(KT + n0 + col) * runs + run] = fmaxf(q - s * s * (1.f / (float)RUN), 0.f);
      }
    }
  }
  const float act_lo = (!FLIP && a.act != S4TF_ACT_NONE) ? 0.f : -__builtin_inff();
  const float act_hi = (!FLIP && a.act == S4TF_ACT_RELU6) ? 6.f : __builtin_inff();
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const int col = nb * 16 + (lane & 15);
    const float bias = (!FLIP && a.bias) ? a.bias[n0 + col] : 0.f;
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        float* dst = a.y + (row0 + g * 16 + 4 * (lane >> 4) + v) * KT + n0 + col;
        float val = acc[g][nb][v] + bias;
        if (FLIP && a.accumulate) val += *dst;
        *dst = fminf(fmaxf(val, act_lo), act_hi);
      }
  }
}

// ---- filter gradient ------------------------------------------------------------------------------------
// dw[tap][c][k] = sum over pixels m of x[m + tap][c] * dy[m][k]: per tap a (CI x pixels) x (pixels x CO) product,
// with the MFMA's k axis running over 4 adjacent pixels of an image row: A: lane l = channel l%16, pixel l/16 (read
// from the patch, 16 adjacent channels per pixel); B: lane l = pixel l/16, output l%16 (from the tile's rows of dy);
// D: register v of lane l = channel 4*(l/16) + v, output l%16.  A wavefront keeps one accumulator block per tap
// through all the tiles its workgroup walks; the workgroup then writes one partial filter gradient (its slab), and
// a reduction kernel adds the slabs in a fixed order.
// Patch pixels are 16 (48, 80) floats apart for 16 (32, 64) channels and rows of dy 16 (48) floats: 4 adjacent
// pixels x 16 adjacent channels then cover the 64 LDS banks once.
struct WgradArgs {
  const float* x;   // (N, H, W, CI)
  const float* dy;  // (N, H, W, KT)
  float* out;       // gridDim.x slabs of (3, 3, CI, KT)
  int N, H, W, KT, RH, IMGS, tiles;
  long long slab;   // floats per slab
};

template <int CI, int CO>
__global__ __launch_bounds__(256) void patchconv_wgrad_kernel(const WgradArgs a) {
  constexpr int CS = CI == 16 ? 16 : CI == 32 ? 48 : 80;
  constexpr int DS = CO == 16 ? 16 : 48;
  constexpr int NCB = CI / 16, NKB = CO / 16, C4 = CI / 4, K4 = CO / 4;
  // Four blocks of 16 x 16 outputs: a wavefront owns one of them over all 128 pixels (nothing to add across
  // wavefronts).  One block: a wavefront owns 32 of the pixels, and the four are added through LDS at the end.
  constexpr bool OWN_BLOCK = NCB * NKB == 4;
  static_assert(OWN_BLOCK || NCB * NKB == 1, "one or four output blocks per workgroup");
  constexpr int STEPS = OWN_BLOCK ? TILE / 4 : TILE / 16;  // k-steps of 4 pixels per wavefront and tile
  constexpr int TILE_FLOATS = PATCH_PIXELS * CS + TILE * DS, RED_FLOATS = OWN_BLOCK ? 0 : 9 * CI * CO;
  __shared__ __attribute__((aligned(16))) float smem[TILE_FLOATS > RED_FLOATS ? TILE_FLOATS : RED_FLOATS];
  float* patch = smem;
  float* dyt = smem + PATCH_PIXELS * CS;
  const int H = a.H, W = a.W, PW = W + 2, RH = a.RH, PR = RH + 2, KT = a.KT, n0 = blockIdx.y * CO;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int cb0 = OWN_BLOCK ? wave / NKB : 0, kb0 = OWN_BLOCK ? wave % NKB : 0;
  const int m0 = (OWN_BLOCK ? 0 : wave * 32) + (lane >> 4);  // this lane's pixel of k-step 0
  const int lw = 31 - __clz(W), lrh = a.IMGS > 1 ? 31 - __clz(RH) : 30;  // W and RH (if several images) are powers of two
  // patch offset of tile pixel m at this lane's channel: patch row = row + 2*image
  auto pix_off = [&](int m) {
    const int row = m >> lw;
    return ((row + 2 * (row >> lrh)) * PW + (m & (W - 1))) * CS + cb0 * 16 + (lane & 15);
  };
  const int bbase = m0 * DS + kb0 * 16 + (lane & 15);
  f32x4 acc[9];
#pragma unroll
  for (int t = 0; t < 9; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};

  constexpr int PV = (PATCH_PIXELS * C4 + 255) / 256, DV = (TILE * K4 + 255) / 256;
  const int chunks = a.IMGS * PR * PW * C4;
  for (int tile = blockIdx.x; tile < a.tiles; tile += gridDim.x) {
    int n, p0;
    if (a.IMGS == 1) {
      const int tiles_per_image = H / RH;
      n = tile / tiles_per_image;
      p0 = (tile - n * tiles_per_image) * RH;
    } else {
      n = tile * a.IMGS;
      p0 = 0;
    }
    float4 pv[PV], dv[DV];
#pragma unroll
    for (int k = 0; k < PV; ++k) {
      const int i = threadIdx.x + k * 256;
      const int c4 = i % C4, t = i / C4, pw = t % PW, prow = t / PW, img = prow / PR, pr = prow - img * PR;
      const int h = p0 + pr - 1, wc = pw - 1;
      pv[k] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (i < chunks && h >= 0 && h < H && wc >= 0 && wc < W)
        pv[k] = *reinterpret_cast<const float4*>(a.x + (((long long)(n + img) * H + h) * W + wc) * CI + c4 * 4);
    }
#pragma unroll
    for (int k = 0; k < DV; ++k) {
      const int i = threadIdx.x + k * 256;
      const int k4 = i % K4, m = i / K4;
      dv[k] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (i < TILE * K4) dv[k] = *reinterpret_cast<const float4*>(a.dy + ((long long)tile * TILE + m) * KT + n0 + k4 * 4);
    }
    __syncthreads();  // everyone is done with the previous tile
#pragma unroll
    for (int k = 0; k < PV; ++k) {
      const int i = threadIdx.x + k * 256;
      if (i < chunks) *reinterpret_cast<float4*>(patch + (i / C4) * CS + (i % C4) * 4) = pv[k];
    }
#pragma unroll
    for (int k = 0; k < DV; ++k) {
      const int i = threadIdx.x + k * 256;
      if (i < TILE * K4) *reinterpret_cast<float4*>(dyt + (i / K4) * DS + (i % K4) * 4) = dv[k];
    }
    __syncthreads();
    // the fragments of k-step j+1 are read while step j is multiplied
    float af[2][9], bf[2];
    auto read_step = [&](int j, int buf) {
      bf[buf] = dyt[bbase + 4 * j * DS];
      const int ab = pix_off(m0 + 4 * j);
#pragma unroll
      for (int t = 0; t < 9; ++t) af[buf][t] = patch[ab + ((t / 3) * PW + (t % 3)) * CS];
    };
    // (a rolled loop of two steps: unrolled all the way, the compiler reads every step's fragments up front and
    // the registers they fill leave one wavefront per SIMD)
    static_assert(STEPS % 2 == 0, "steps go in pairs");
    read_step(0, 0);
#pragma unroll 1
    for (int j = 0; j < STEPS; j += 2) {
      read_step(j + 1, 1);
#pragma unroll
      for (int t = 0; t < 9; ++t) acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(af[0][t], bf[0], acc[t], 0, 0, 0);
      if (j + 2 < STEPS) read_step(j + 2, 0);
#pragma unroll
      for (int t = 0; t < 9; ++t) acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(af[1][t], bf[1], acc[t], 0, 0, 0);
    }
  }
  float* slab = a.out + (long long)blockIdx.x * a.slab;
  if constexpr (OWN_BLOCK) {
#pragma unroll
    for (int t = 0; t < 9; ++t)
#pragma unroll
      for (int v = 0; v < 4; ++v)
        slab[(long long)(t * CI + cb0 * 16 + 4 * (lane >> 4) + v) * KT + n0 + kb0 * 16 + (lane & 15)] = acc[t][v];
  } else {
    // the four wavefronts' sums, added in wavefront order
    __syncthreads();
    float* red = smem;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      if (wave == w) {
#pragma unroll
        for (int t = 0; t < 9; ++t)
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            float* r = red + (t * CI + 4 * (lane >> 4) + v) * CO + (lane & 15);
            *r = w == 0 ? acc[t][v] : *r + acc[t][v];
          }
      }
      __syncthreads();
    }
    for (int i = threadIdx.x; i < 9 * CI * K4; i += 256) {
      const int row = i / K4, k4 = i - row * K4;  // row = (tap, c)
      *reinterpret_cast<float4*>(slab + (long long)row * KT + n0 + k4 * 4) = *reinterpret_cast<const float4*>(red + row * CO + k4 * 4);
    }
  }
}

template <int CI, int CO, bool FLIP, int TAPS = 9>
int launch_patch(const PatchArgs& a, hipStream_t st) {
  const unsigned tiles = (unsigned)((long long)a.N * a.H * a.W / TILE);
  hipLaunchKernelGGL((patchconv_kernel<CI, CO, FLIP, TAPS>), dim3(tiles, a.KT / CO), dim3(256), 0, st, a);
  return launch_status("patchconv");
}

// 1x1 layers: the widest block of output channels that divides their number
template <int CI, bool FLIP>
int launch_point(const PatchArgs& a, hipStream_t st) {
  if (a.KT % 48 == 0) return launch_patch<CI, 48, FLIP, 1>(a, st);
  if (a.KT % 32 == 0) return launch_patch<CI, 32, FLIP, 1>(a, st);
  return launch_patch<CI, 16, FLIP, 1>(a, st);
}
template <bool FLIP>
int launch_point(int reduce_channels, const PatchArgs& a, hipStream_t st) {
  switch (reduce_channels) {
    case 16: return launch_point<16, FLIP>(a, st);
    case 24: return launch_point<24, FLIP>(a, st);
    case 32: return launch_point<32, FLIP>(a, st);
    default: return launch_point<64, FLIP>(a, st);
  }
}
// a 1x1 / stride 1 layer whose reduction axis has `reduce` channels and whose result has `out` channels
bool point_ok(const ConvGeom& g, int reduce, int out) {
  if (g.R != 1 || g.S != 1 || g.stride != 1 || g.pad != 0) return false;
  if (reduce != 16 && reduce != 24 && reduce != 32 && reduce != 64) return false;
  const long long M = (long long)g.N * g.H * g.W;
  return out % 16 == 0 && M % TILE == 0 && M * (reduce > out ? reduce : out) < (1LL << 31);
}

// How the 128-pixel tiles lie in the images: whole rows of one image, or whole images.  False when they do not fit.
bool tiling(int N, int H, int W, int& RH, int& IMGS) {
  if (W != 8 && W != 16 && W != 32) return false;
  const int hw = H * W;
  if (hw >= TILE) {
    if (hw % TILE) return false;
    RH = TILE / W; IMGS = 1;
  } else {
    if (TILE % hw || N % (TILE / hw)) return false;
    RH = H; IMGS = TILE / hw;
  }
  return IMGS * (RH + 2) * (W + 2) <= PATCH_PIXELS;
}

bool shape_ok(const ConvGeom& g) {
  int RH, IMGS;
  if (g.R != 3 || g.S != 3 || g.stride != 1 || g.pad != 1 || !tiling(g.N, g.H, g.W, RH, IMGS)) return false;
  return (long long)g.N * g.H * g.W * (g.C > g.K ? g.C : g.K) < (1LL << 31);
}
bool channels_ok(int C, int K) { return (C == 16 && K == 16) || (C == 32 && K == 32) || (C == 64 && K == 64); }

PatchArgs make_args(const ConvGeom& g, const void* in, const void* w, void* out, int out_channels) {
  PatchArgs a = {};
  a.x = static_cast<const float*>(in); a.w = static_cast<const float*>(w); a.y = static_cast<float*>(out);
  a.N = g.N; a.H = g.H; a.W = g.W; a.KT = out_channels;
  a.RH = 1; a.IMGS = 1;  // (unused by 1x1 layers)
  if (g.R == 3) tiling(g.N, g.H, g.W, a.RH, a.IMGS);
  return a;
}

}  // namespace

bool patchconv_fwd_ok(const ConvGeom& g, int dtype) {
  if (dtype != S4TF_F32) return false;
  return point_ok(g, g.C, g.K) || (shape_ok(g) && (channels_ok(g.C, g.K) || (g.C == 4 && g.K == 16)));
}
bool patchconv_dgrad_ok(const ConvGeom& g, int dtype) {
  if (dtype != S4TF_F32) return false;
  return point_ok(g, g.K, g.C) || (shape_ok(g) && channels_ok(g.C, g.K));
}

// y = act(conv(x, w) + bias); with `stats`, also the BatchNorm partial sums of igemm_fwd, per run of *stats_rows pixels
int patchconv_fwd(const ConvGeom& g, const void* x, const void* w, const float* bias, int act, void* y, float* stats,
                  int* stats_rows, hipStream_t st) {
  if (!aligned16(x) || !aligned16(w) || !aligned16(y)) return fail(S4TF_ERR_SHAPE, "patchconv: operands must be 16-byte aligned");
  PatchArgs a = make_args(g, x, w, y, g.K);
  a.bias = bias; a.stats = stats; a.act = act;
  if (stats_rows) *stats_rows = 32;
  if (g.R == 1) return launch_point<false>(g.C, a, st);
  if (g.C == 16) return launch_patch<16, 16, false>(a, st);
  if (g.C == 32) return launch_patch<32, 32, false>(a, st);
  if (g.C == 64) return launch_patch<64, 16, false>(a, st);  // four workgroups of 16 output channels per tile
  return launch_patch<4, 16, false>(a, st);
}

// dx (+)= the pullback of the same layer to its input
int patchconv_dgrad(const ConvGeom& g, const void* dy, const void* w, void* dx, int accumulate, hipStream_t st) {
  if (!aligned16(dy) || !aligned16(w) || !aligned16(dx)) return fail(S4TF_ERR_SHAPE, "patchconv: operands must be 16-byte aligned");
  PatchArgs a = make_args(g, dy, w, dx, g.C);
  a.accumulate = accumulate;
  if (g.R == 1) return launch_point<true>(g.K, a, st);
  if (g.C == 16) return launch_patch<16, 16, true>(a, st);
  if (g.C == 32) return launch_patch<32, 32, true>(a, st);
  return launch_patch<64, 16, true>(a, st);
}

bool patchconv_wgrad_ok(const ConvGeom& g, int dtype) { return dtype == S4TF_F32 && shape_ok(g) && channels_ok(g.C, g.K); }

// Workgroups along the pixel axis = partial filter gradients (slabs) the kernel leaves: enough workgroups to fill
// the chip, each walking at most a few tiles
int patchconv_wgrad_splits(const ConvGeom& g) {
  const int tiles = (int)((long long)g.N * g.H * g.W / TILE);
  const int per_tile = g.C == 64 ? 4 : 1;  // workgroups per tile: blocks of 16 output channels for 64-channel layers
  int want = 512 / per_tile;
  if (want > tiles) want = tiles;
  const int walk = (tiles + want - 1) / want;
  return (tiles + walk - 1) / walk;
}

// `splits` slabs of (3, 3, C, K) partial sums into out (the filter gradient itself when splits == 1)
int patchconv_wgrad(const ConvGeom& g, const void* x, const void* dy, float* out, int splits, hipStream_t st) {
  if (!aligned16(x) || !aligned16(dy) || !aligned16(out)) return fail(S4TF_ERR_SHAPE, "patchconv: operands must be 16-byte aligned");
  WgradArgs a = {};
  a.x = static_cast<const float*>(x); a.dy = static_cast<const float*>(dy); a.out = out;
  a.N = g.N; a.H = g.H; a.W = g.W; a.KT = g.K;
  tiling(g.N, g.H, g.W, a.RH, a.IMGS);
  a.tiles = (int)((long long)g.N * g.H * g.W / TILE);
  a.slab = (long long)9 * g.C * g.K;
  if (g.C == 16) hipLaunchKernelGGL((patchconv_wgrad_kernel<16, 16>), dim3(splits, 1), dim3(256), 0, st, a);
  else if (g.C == 32) hipLaunchKernelGGL((patchconv_wgrad_kernel<32, 32>), dim3(splits, 1), dim3(256), 0, st, a);
  else hipLaunchKernelGGL((patchconv_wgrad_kernel<64, 16>), dim3(splits, 4), dim3(256), 0, st, a);
  return launch_status("patchconv_wgrad");
}

}  // namespace s4tf
