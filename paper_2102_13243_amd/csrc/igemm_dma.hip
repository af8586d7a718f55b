// bf16 implicit-GEMM convolution, fast path for channel counts that are multiples of 8.
//
// Same GEMM view as igemm.hip (D[i][j] = sum_k A[i][k] B[j][k] for forward / dgrad / wgrad), but
// the operand tiles go from global memory straight into LDS with 16-byte direct loads
// (global_load_lds), so no VGPRs and no LDS-store instructions are spent on staging and several
// k-tiles can be in flight: a ring of STAGES LDS buffers, one barrier per k-tile, vmcnt-based
// waits.  A direct load writes 64 lanes x 16 bytes to one contiguous KiB of LDS, lane by lane; which
// global chunk a lane fetches is free, and that freedom is the swizzle:
//   * operands whose memory is contiguous along k (im2col rows of x or dy, filters in dgrad) are
//     stored [row][k] with the 16-byte chunk index XOR-ed with (row >> 1) & 7, which makes the
//     ds_read_b128 of an MFMA fragment (32 rows, one chunk each) conflict free;
//   * operands whose memory is contiguous along the GEMM row (filters in the forward pass, x and
//     dy in wgrad) are stored as they are, [k][row], and read with ds_read_b64_tr_b16, the LDS
//     transpose load of gfx950, which hands each lane 4 consecutive k for its own row.
// The loads are buffer loads: padding (image borders, ragged tiles, stride holes in dgrad) is an
// out-of-range offset, which the hardware turns into zeros, so every lane always loads.  MFMA: v_mfma_f32_32x32x16_bf16, fp32 accumulation.
#include <utility>

#include "s4tf_internal.h"
#include "igemm_args.h"

namespace s4tf {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

constexpr int BK = 64;        // k per stage: 128 bytes per row
constexpr int ROWB = BK * 2;  // bytes per k-contiguous row

#define LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define GLB_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

typedef int i32x4 __attribute__((ext_vector_type(4)));
constexpr uint32_t OOB = 0x80000000u;  // a byte offset past every tensor on this path: such a load returns zeros

// Buffer resource over [base, base + bytes): a load whose offset is >= bytes writes zeros.
__device__ inline i32x4 make_rsrc(const void* base, uint32_t bytes) {
  const uint64_t p = (uint64_t)base;
  i32x4 r;
  r[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)p);
  r[1] = __builtin_amdgcn_readfirstlane((int)(uint32_t)(p >> 32));
  r[2] = __builtin_amdgcn_readfirstlane((int)bytes);
  r[3] = 0x00020000;
  return r;
}

// One 16-byte chunk per lane: LDS[wave_base + lane*16 .. +16) = buffer[voff .. +16), zeros if out of range.
// Issued as inline assembly on purpose: the compiler then does not count these loads, so it cannot
// turn the hand-placed partial vmcnt waits of the k-loop into full ones (every LDS read after a
// direct load it knows about gets a vmcnt(0)).  The loop orders LDS writes and reads itself: vmcnt
// wait, then barrier.  The address work per load is a handful of VALU instructions (a fixed per-lane
// offset plus a wavefront-uniform one, and a mask test): one MFMA lasts only 8 VALU issue slots.
__device__ inline void dma16(uint32_t voff, i32x4 rsrc, uint32_t lds) {  // lds: wavefront-uniform LDS byte address
  asm volatile("s_mov_b32 m0, %2\n\tbuffer_load_dwordx4 %0, %1, 0 offen lds" : : "v"(voff), "s"(rsrc), "s"(lds) : "memory");
}
// LDS byte address of a __shared__ object, as a wavefront-uniform 32-bit value
__device__ inline uint32_t lds_addr(const void* p) {
  return __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)LDS_PTR(p));
}
template <int N> __device__ inline void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0F70);  // vmcnt(N), other counters untouched
}

__device__ inline uint32_t half_of(const uint4& v, int e) {
  uint32_t d = (e >> 1) == 0 ? v.x : (e >> 1) == 1 ? v.y : (e >> 1) == 2 ? v.z : v.w;
  return (e & 1) ? (d >> 16) : (d & 0xffffu);
}
// x / d for 0 <= x < 2^31 with the host-computed (magic, shift) of Args
__device__ inline int fast_div(int x, uint32_t magic, int shift) {
  return (int)((__umulhi((uint32_t)x, magic) + (uint32_t)x) >> shift);
}
__device__ inline int log2_of(int v) { return 31 - __clz(v); }

// ---- k-contiguous operands -----------------------------------------------------------------------
// Tile-local row `row`, 16-byte chunk `kc` of its 128-byte k-run lives at byte
//   (row*8 + (kc ^ ((row >> 1) & 7))) * 16.
// Wave w fills the 1 KiB units u = w*UPW + i (8 rows each); lane l owns row 8u + l/8, slot l%8.
template <int ROWS> struct KTile {
  static constexpr int UPW = ROWS / 32;
  __device__ static int row_of(int wave, int i, int lane) { return (wave * UPW + i) * 8 + (lane >> 3); }
  __device__ static int kc_of(int wave, int i, int lane) { return (lane & 7) ^ ((row_of(wave, i, lane) >> 1) & 7); }
  __device__ static int frag_off(int row, int kc) { return (row * 8 + (kc ^ ((row >> 1) & 7))) * 16; }
};

// Gathers of an image along k = (tap, channel): forward A reads x at (p*st + r - pad, q*st + s - pad),
// dgrad A reads dy at ((h + pad - r)/st, (w + pad - s)/st).  Per row the byte offset splits into a
// fixed per-lane part and a part that depends on the tap only, and whether a tap falls inside the
// image is one bit of a per-row mask built once.  A k-tile of 64 lies inside one tap when the
// channel count is a multiple of 64 (then the tap part is wavefront-uniform); channel counts 8, 16,
// 32 put several taps in a k-tile and take the per-lane path.
template <int ROWS, bool DGRAD> struct Gather {
  typedef KTile<ROWS> TL;
  i32x4 rsrc;
  int loff[TL::UPW], kc[TL::UPW];
  uint32_t toffv[TL::UPW];  // uniform-tap path: this lane's offset for the current tap, or OOB if the tap is padding
  uint64_t mask[TL::UPW];
  int r, s, tap, cb, kt, toff;  // uniform: tap (r,s), its offset, and the channel base of the next k-tile
  int s0, tstep;                // taps visited: r = r0, r0 + tstep, ..., s likewise (all of them unless a parity class runs)
  int CH, WI, taps, S, invS, logC;
  bool uniform_tap;
  // x / stride for x >= 0
  __device__ static int sdiv(int x, int stride) { return stride == 1 ? x : stride == 2 ? (x >> 1) : x / stride; }
  // Taps (rr, ss) with rlo <= rr < rhi, slo <= ss < shi as a bit mask (bit rr*S + ss), without a loop: the column
  // bits, below 2^S, times the bits rr*S of the wanted rows (R*S <= 64, so the products do not overlap or carry)
  __device__ static uint64_t rect_mask(uint64_t rowbits, int rlo, int rhi, int slo, int shi, int S) {
    const uint64_t cols = ((1ull << shi) - 1) & ~((1ull << slo) - 1);
    const int hb = rhi * S, lb = rlo * S;
    const uint64_t rows = rowbits & (hb >= 64 ? ~0ull : ((1ull << hb) - 1)) & ~((1ull << lb) - 1);
    return cols * rows;
  }
  // tap part of the offset, in elements
  __device__ int tap_off(int rr, int ss, const ConvGeom& g) const {
    return DGRAD ? -(sdiv(rr, g.stride) * g.Q + sdiv(ss, g.stride)) * g.K : (rr * g.W + ss) * g.C;
  }
  __device__ void init(const Args& a, int row0, int wave, int lane, int kt0) {
    const ConvGeom& g = a.g;
    rsrc = make_rsrc(a.a, a.a_bytes);
    CH = DGRAD ? g.K : g.C;
    S = g.S;
    taps = g.R * g.S;
    invS = g.S == 1 ? 65536 : g.S == 3 ? 21846 : (65536 + g.S - 1) / g.S;
    uniform_tap = (CH % BK) == 0;
    logC = log2_of(CH);
    uint64_t rowbits = 0;  // bit rr*S for every filter row rr (uniform)
    for (int rr = 0; rr < g.R; ++rr) rowbits |= 1ull << (rr * g.S);
#pragma unroll
    for (int i = 0; i < TL::UPW; ++i) {
      const int row = row0 + TL::row_of(wave, i, lane);
      const bool rv = row < a.Mg;
      kc[i] = TL::kc_of(wave, i, lane);
      const int kco = uniform_tap ? kc[i] * 8 : 0;
      uint64_t m = 0;
      if (a.simple) {  // 1x1, stride 1, no padding: a plain row-major matrix
        loff[i] = (row * CH + kco) * 2;
        m = rv ? 1 : 0;
      } else if (!DGRAD) {
        const int t = fast_div(row, a.magicQ, a.shiftQ), q = row - t * g.Q;
        const int n = fast_div(t, a.magicP, a.shiftP), p = t - n * g.P;
        const int h0 = p * g.stride - g.pad, w0 = q * g.stride - g.pad;
        loff[i] = (((n * g.H + h0) * g.W + w0) * g.C + kco) * 2;
        // the taps inside the image form a rectangle: rows [rlo, rhi) x columns [slo, shi)
        const int rlo = max(0, -h0), rhi = min(g.R, g.H - h0), slo = max(0, -w0), shi = min(g.S, g.W - w0);
        if (rv && shi > slo && rhi > rlo) m = rect_mask(rowbits, rlo, rhi, slo, shi, g.S);
      } else {
        int n, h, w;
        if (a.cls) {  // rows run over the pixels (stride*hc + ph, stride*wc + pw) only
          const int t = fast_div(row, a.magicWc, a.shiftWc), wc = row - t * a.Wc;
          n = fast_div(t, a.magicHc, a.shiftHc);
          h = g.stride * (t - n * a.Hc) + a.ph;
          w = g.stride * wc + a.pw;
        } else {
          const int t = fast_div(row, a.magicW, a.shiftW);
          w = row - t * g.W;
          n = fast_div(t, a.magicH, a.shiftH);
          h = t - n * g.H;
        }
        const int hp0 = h + g.pad, wp0 = w + g.pad;
        loff[i] = (((n * g.P + sdiv(hp0, g.stride)) * g.Q + sdiv(wp0, g.stride)) * g.K + kco) * 2;
        // tap (rr, ss) reads dy at ((hp0 - rr)/stride, (wp0 - ss)/stride) when both divide exactly and
        // fall inside the output: the valid set is (valid rr) x (valid ss)
        if (g.stride == 1) {
          // every tap divides: the valid ones form a rectangle, rows [rlo, rhi) x columns [slo, shi), as in
          // the forward pass (0 <= hp0 - rr < P and 0 <= wp0 - ss < Q)
          const int rlo = max(0, hp0 - g.P + 1), rhi = min(g.R, hp0 + 1), slo = max(0, wp0 - g.Q + 1), shi = min(g.S, wp0 + 1);
          if (rv && shi > slo && rhi > rlo) m = rect_mask(rowbits, rlo, rhi, slo, shi, g.S);
        } else {
          uint64_t cols = 0;
          for (int ss = 0; ss < g.S; ++ss) {
            const int wp = wp0 - ss, wq = sdiv(wp, g.stride);
            if (wp >= 0 && wq * g.stride == wp && wq < g.Q) cols |= 1ull << ss;
          }
          if (rv)
            for (int rr = 0; rr < g.R; ++rr) {
              const int hp = hp0 - rr, hq = sdiv(hp, g.stride);
              if (hp >= 0 && hq * g.stride == hp && hq < g.P) m |= cols << (rr * g.S);
            }
        }
      }
      mask[i] = m;
    }
    kt = kt0;
    s0 = 0;
    tstep = 1;
    if (DGRAD && a.cls) {
      s0 = a.s0;
      tstep = g.stride;
      cb = 0; r = a.r0; s = a.s0; tap = r * g.S + s;
    } else if (kt0 == 0) {  // forward and dgrad launches: no division
      cb = 0; tap = 0; s = 0; r = 0;
    } else {
      const int kk = kt0 * BK;
      cb = kk % CH;
      tap = kk / CH;
      s = tap % g.S;
      r = tap / g.S;
    }
    toff = tap_off(r, s, g);
    new_tap();
  }
  __device__ void new_tap() {
    const bool in = tap < taps;
#pragma unroll
    for (int i = 0; i < TL::UPW; ++i)
      toffv[i] = (in && ((mask[i] >> tap) & 1)) ? (uint32_t)(loff[i] + toff * 2) : OOB;
  }
  __device__ void issue(const Args& a, uint32_t tile, int wave) {
    const ConvGeom& g = a.g;
    if (uniform_tap) {
      const uint32_t uni = (uint32_t)(cb * 2);  // OOB + uni stays out of range
#pragma unroll
      for (int i = 0; i < TL::UPW; ++i) dma16(toffv[i] + uni, rsrc, tile + (uint32_t)((wave * TL::UPW + i) * 1024));
      cb += BK;
      if (cb >= CH) {  // next tap: the only place that pays for its offset and its padding test
        cb = 0;
        s += tstep;
        if (s >= g.S) { s = s0; r += tstep; }
        tap = r * g.S + s;
        toff = tap_off(r, s, g);
        new_tap();
      }
    } else {
#pragma unroll
      for (int i = 0; i < TL::UPW; ++i) {
        const int kk = kt * BK + kc[i] * 8;
        const int t = kk >> logC, c = kk & (CH - 1);
        const int rr = (t * invS) >> 16, ss = t - rr * S;
        const bool ok = t < taps && ((mask[i] >> t) & 1);
        dma16(ok ? (uint32_t)(loff[i] + (tap_off(rr, ss, g) + c) * 2) : OOB, rsrc, tile + (wave * TL::UPW + i) * 1024);
      }
    }
    ++kt;
  }
};

// dgrad B: rows = input channels c, k = (r,s,ko); filters (R,S,C,K) are contiguous along ko.
// k-tiles past R*S*K run off the end of the filter tensor and read as zeros.
template <int ROWS> struct DgradB {
  typedef KTile<ROWS> TL;
  i32x4 rsrc;
  uint32_t loff[TL::UPW];
  int kc[TL::UPW], crow[TL::UPW];
  int rs, kob, kt, logK;
  int r, s, s0, tstep;  // the tap behind rs = r*S + s and how it advances (see Gather)
  bool uniform_tap;
  __device__ void init(const Args& a, int row0, int wave, int lane, int kt0) {
    const ConvGeom& g = a.g;
    rsrc = make_rsrc(a.b, a.b_bytes);
    uniform_tap = (g.K % BK) == 0;
    logK = log2_of(g.K);
#pragma unroll
    for (int i = 0; i < TL::UPW; ++i) {
      crow[i] = row0 + TL::row_of(wave, i, lane);
      kc[i] = TL::kc_of(wave, i, lane);
      loff[i] = crow[i] < a.Ng ? (uint32_t)((crow[i] * g.K + (uniform_tap ? kc[i] * 8 : 0)) * 2) : OOB;
    }
    kt = kt0;
    s0 = 0;
    tstep = 1;
    if (a.cls) {
      s0 = a.s0;
      tstep = g.stride;
      kob = 0; r = a.r0; s = a.s0;
    } else if (kt0 == 0) {
      kob = 0; r = 0; s = 0;
    } else {
      const int kk = kt0 * BK;
      kob = kk % g.K;
      const int t = kk / g.K;
      r = t / g.S;
      s = t - r * g.S;
    }
    rs = r * g.S + s;
  }
  __device__ void issue(const Args& a, uint32_t tile, int wave) {
    const ConvGeom& g = a.g;
    if (uniform_tap) {
      const uint32_t uni = (uint32_t)((rs * g.C * g.K + kob) * 2);
#pragma unroll
      for (int i = 0; i < TL::UPW; ++i) dma16(loff[i] + uni, rsrc, tile + (wave * TL::UPW + i) * 1024);
      kob += BK;
      if (kob >= g.K) {
        kob = 0;
        s += tstep;
        if (s >= g.S) { s = s0; r += tstep; }
        rs = r * g.S + s;
      }
    } else {
#pragma unroll
      for (int i = 0; i < TL::UPW; ++i) {
        const int kk = kt * BK + kc[i] * 8;
        const int t = kk >> logK, ko = kk & (g.K - 1);
        dma16(loff[i] + (uint32_t)((t * g.C * g.K + ko) * 2), rsrc, tile + (wave * TL::UPW + i) * 1024);
      }
    }
    ++kt;
  }
};

// ---- row-contiguous operands ---------------------------------------------------------------------
// Stored [k][row] as they lie in memory, a k-row being CPR 16-byte chunks of 8 adjacent rows, except for
// a swizzle of the chunk position.  LDS reads go through 64 banks of 4 bytes: a transpose read (8 bytes
// per lane) is served 32 lanes = 256 bytes at a time, and those 32 lanes fetch 64 bytes (4 chunks) from
// each of four consecutive k-rows.  k-rows lie a whole or half a 256-byte bank sweep apart, so left alone
// the four pieces would fall on the same banks; chunk c of k-row k therefore sits at position
// c ^ 4*s(k), where s(k) counts through the k-rows that share a bank window: k & 3 for 128-row tiles
// (one k-row per sweep), (k >> 1) & 1 for 64-row tiles (two per sweep).
// Wave w fills units u = w*UPW + i; a unit is KPU k-rows; lane l fills position l%CPR of k-row
// u*KPU + l/CPR (KPU is a multiple of 4, so the swizzle depends on the lane only).
template <int ROWS> struct RTile {
  static constexpr int UPW = ROWS / 32;
  static constexpr int CPR = ROWS / 8;   // chunks per k-row
  static constexpr int KPU = 64 / CPR;   // k-rows per 1 KiB unit
  static_assert(ROWS == 64 || ROWS == 128, "swizzle is written for 64- and 128-row tiles");
  __device__ static int swz(int k) { return ROWS == 128 ? ((k & 3) << 2) : (((k >> 1) & 1) << 2); }
  __device__ static int k_of(int wave, int i, int lane) { return (wave * UPW + i) * KPU + lane / CPR; }
  // the chunk of its k-row (8 adjacent rows of the tile) that a lane fetches
  __device__ static int chunk_of(int lane) { return (lane % CPR) ^ swz(lane / CPR); }
  // byte address a lane hands to ds_read_b64_tr_b16 to receive, for its own row nf + (lane & 31), the
  // 4 k-values kb .. kb+3 (kb a multiple of 4): lanes 16g..16g+15 together read k-rows kb..kb+3 x rows
  // nf+16g .. nf+16g+15
  __device__ static int tr_off(int kb, int nf, int lane) {
    const int j = lane & 15, g = (lane >> 4) & 1;
    const int k = kb + (j >> 2), n = nf + 16 * g + 4 * (j & 3);
    return k * ROWS * 2 + (((n >> 3) ^ swz(k)) << 4) + (n & 7) * 2;
  }
};

// plain [k][ld] matrix: filters in the forward pass ([(r,s,c)][ko]), dy in wgrad ([(n,p,q)][ko]).
// k-rows past the end of the tensor read as zeros.
template <int ROWS> struct PlainR {
  typedef RTile<ROWS> TL;
  i32x4 rsrc;
  uint32_t off[TL::UPW], step;
  __device__ void init(const Args& a, int col0, int wave, int lane, int kt0) {
    rsrc = make_rsrc(a.b, a.b_bytes);
    const int col = col0 + TL::chunk_of(lane) * 8;
    step = (uint32_t)(BK * a.g.K * 2);
#pragma unroll
    for (int i = 0; i < TL::UPW; ++i)
      off[i] = col < a.Ng ? (uint32_t)(((kt0 * BK + TL::k_of(wave, i, lane)) * a.g.K + col) * 2) : OOB;
  }
  __device__ void issue(const Args&, uint32_t tile, int wave) {
#pragma unroll
    for (int i = 0; i < TL::UPW; ++i) {
      dma16(off[i], rsrc, tile + (wave * TL::UPW + i) * 1024);
      off[i] += step;
    }
  }
};

// wgrad A: rows = (r,s,c) (contiguous along c), k = output pixel (n,p,q); gathers x
template <int ROWS> struct WgradA {
  typedef RTile<ROWS> TL;
  i32x4 rsrc;
  int coloff, dr, ds;  // fixed per lane: ((r-pad)*W + (s-pad))*C + c0, r - pad, s - pad
  bool cv;
  int m[TL::UPW];
  uint32_t off[TL::UPW], step;
  __device__ void init(const Args& a, int row0, int wave, int lane, int kt0) {
    const ConvGeom& g = a.g;
    rsrc = make_rsrc(a.a, a.a_bytes);
    const int i0 = row0 + TL::chunk_of(lane) * 8;
    cv = i0 < a.Mg;
    const int c0 = i0 % g.C, t2 = i0 / g.C;
    dr = t2 / g.S - g.pad;
    ds = t2 % g.S - g.pad;
    coloff = (dr * g.W + ds) * g.C + c0;
    step = (uint32_t)(BK * g.C * 2);
#pragma unroll
    for (int i = 0; i < TL::UPW; ++i) {
      m[i] = kt0 * BK + TL::k_of(wave, i, lane);
      off[i] = cv ? (uint32_t)((m[i] * g.C + c0) * 2) : OOB;  // the 1x1 / stride 1 / no padding case
    }
  }
  __device__ void issue(const Args& a, uint32_t tile, int wave) {
    const ConvGeom& g = a.g;
    if (a.simple) {
#pragma unroll
      for (int i = 0; i < TL::UPW; ++i) {
        dma16(off[i], rsrc, tile + (wave * TL::UPW + i) * 1024);
        off[i] += step;
      }
      return;
    }
#pragma unroll
    for (int i = 0; i < TL::UPW; ++i) {
      const int t = fast_div(m[i], a.magicQ, a.shiftQ), q = m[i] - t * g.Q;
      const int n = fast_div(t, a.magicP, a.shiftP), p = t - n * g.P;
      const int h = p * g.stride + dr, w = q * g.stride + ds;
      const bool ok = cv && m[i] < a.Kg && h >= 0 && h < g.H && w >= 0 && w < g.W;
      const uint32_t v = ok ? (uint32_t)((((n * g.H + p * g.stride) * g.W + q * g.stride) * g.C + coloff) * 2) : OOB;
      m[i] += BK;
      dma16(v, rsrc, tile + (wave * TL::UPW + i) * 1024);
    }
  }
};

template <int PASS, int ROWS, bool IS_A> struct Sel;
template <int ROWS> struct Sel<PASS_FWD, ROWS, true> { typedef Gather<ROWS, false> type; static constexpr bool KC = true; };
template <int ROWS> struct Sel<PASS_FWD, ROWS, false> { typedef PlainR<ROWS> type; static constexpr bool KC = false; };
template <int ROWS> struct Sel<PASS_DGRAD, ROWS, true> { typedef Gather<ROWS, true> type; static constexpr bool KC = true; };
template <int ROWS> struct Sel<PASS_DGRAD, ROWS, false> { typedef DgradB<ROWS> type; static constexpr bool KC = true; };
template <int ROWS> struct Sel<PASS_WGRAD, ROWS, true> { typedef WgradA<ROWS> type; static constexpr bool KC = false; };
template <int ROWS> struct Sel<PASS_WGRAD, ROWS, false> { typedef PlainR<ROWS> type; static constexpr bool KC = false; };

// Fragments of 32 rows x 16 k for the MFMA: 8 k-values per lane (k = 16*ks + 8*(lane>>5) + 0..7).
// Their LDS addresses are a per-lane part, computed once before the k-loop, plus a part that is known
// at compile time (ring slot, k-step): the reads in the loop need no address arithmetic at all.
template <bool KC, int ROWS> struct Frag {
  // KC: the XOR swizzle does not commute with the k-step, so one base per k-step; else one base
  static constexpr int NB = KC ? BK / 16 : 1;
  uint32_t base[NB];
  __device__ void init(uint32_t tile0, int row0, int lane) {
    if constexpr (KC) {
#pragma unroll
      for (int ks = 0; ks < NB; ++ks)
        base[ks] = tile0 + KTile<ROWS>::frag_off(row0 + (lane & 31), ks * 2 + (lane >> 5));
    } else {
      base[0] = tile0 + RTile<ROWS>::tr_off(8 * (lane >> 5), row0, lane);
    }
  }
  // slot_off: byte offset of the ring slot (and operand) inside the ring, a compile-time constant at the call
  __device__ bf16x8 load(int slot_off, int ks) const {
    if constexpr (KC) {
      return __builtin_bit_cast(bf16x8, *(const __attribute__((address_space(3))) uint4*)(uintptr_t)(base[ks] + slot_off));
    } else {
      const uint32_t a = base[0] + slot_off + ks * 16 * ROWS * 2;
      s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(uintptr_t)a);
      s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(uintptr_t)(a + 4 * ROWS * 2));
      s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      return __builtin_bit_cast(bf16x8, v);
    }
  }
};

// the value that lane ^ 32 holds
__device__ inline float other_half(float v) {
  typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
  const unsigned u = __builtin_bit_cast(unsigned, v);
  const u32x2 sw = __builtin_amdgcn_permlane32_swap(u, u, false, false);  // [lo, lo], [hi, hi]
  return __builtin_bit_cast(float, (threadIdx.x & 32) ? sw[0] : sw[1]);
}

template <typename F, int... I> __device__ inline void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F> __device__ inline void static_for(F&& f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// Staging patch of the bf16 epilogue: per wavefront 32 rows x (FN*32) columns of fp32, rows 4 banks apart
template <int FN> struct Patch {
  static constexpr int WCOLS = FN * 32, CS = WCOLS + 4, BYTES = 32 * CS * 4;
};

// STAGES >= 2: ring of LDS stages, the loads of k-tile kt+STAGES-1 fly while kt is multiplied; two
// workgroups per CU.  STAGES == 1: load, wait, multiply; half the LDS, four workgroups per CU, whose
// phases interleave: the better trade for GEMMs with only one or two k-tiles, where a ring has
// nothing to overlap and the run time is load latency plus epilogue.
template <int PASS, int STAGES, int WM, int WN, int FM, int FN>
__global__ __launch_bounds__(NT, STAGES == 1 ? 4 : STAGES >= 4 ? 1 : 2) void igemm_dma_kernel(const Args a0) {
  static_assert(WM * WN == 4, "four wavefronts");
  constexpr int BM = WM * FM * 32, BN = WN * FN * 32;
  constexpr int A_BYTES = BM * ROWB, B_BYTES = BN * ROWB, STAGE_BYTES = A_BYTES + B_BYTES;
  constexpr int LOADS = (BM + BN) / 32;  // direct loads per lane per stage
  constexpr int RING = STAGES * STAGE_BYTES;
  constexpr int SMEM = (PASS != PASS_WGRAD && 4 * Patch<FN>::BYTES > RING) ? 4 * Patch<FN>::BYTES : RING;
  typedef Sel<PASS, BM, true> SA;
  typedef Sel<PASS, BN, false> SB;
  __shared__ __attribute__((aligned(1024))) char smem[SMEM];

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t ring = lds_addr(smem);
  Args a = a0;
  int bid = blockIdx.x;
  if constexpr (PASS == PASS_DGRAD) {
    if (a.cls) {  // one launch over the four parity classes: which one this workgroup belongs to
      const int c = (bid >= a.cls_end[0]) + (bid >= a.cls_end[1]) + (bid >= a.cls_end[2]);
      bid -= c == 0 ? 0 : c == 1 ? a.cls_end[0] : c == 2 ? a.cls_end[1] : a.cls_end[2];
      a.ph = (3 - c) >> 1;  // slot c holds class 3 - c: the classes with the most taps start first
      a.pw = (3 - c) & 1;
      a.r0 = a.ph ? a.cls_r0[1] : a.cls_r0[0];
      a.s0 = a.pw ? a.cls_s0[1] : a.cls_s0[0];
      a.Hc = a.ph ? a.cls_Hc[1] : a.cls_Hc[0];
      a.Wc = a.pw ? a.cls_Wc[1] : a.cls_Wc[0];
      a.magicHc = a.ph ? a.cls_magicHc[1] : a.cls_magicHc[0];
      a.shiftHc = a.ph ? a.cls_shiftHc[1] : a.cls_shiftHc[0];
      a.magicWc = a.pw ? a.cls_magicWc[1] : a.cls_magicWc[0];
      a.shiftWc = a.pw ? a.cls_shiftWc[1] : a.cls_shiftWc[0];
      a.Mg = c == 0 ? a.cls_Mg[0] : c == 1 ? a.cls_Mg[1] : c == 2 ? a.cls_Mg[2] : a.cls_Mg[3];
      a.nk = c == 0 ? a.cls_nk[0] : c == 1 ? a.cls_nk[1] : c == 2 ? a.cls_nk[2] : a.cls_nk[3];
      a.nk_per_split = a.nk;
      a.tiles_m = c == 0 ? a.cls_tiles_m[0] : c == 1 ? a.cls_tiles_m[1] : c == 2 ? a.cls_tiles_m[2] : a.cls_tiles_m[3];
    }
  }
  int logical, split;
  if (!block_to_tile(a, bid, logical, split)) return;
  const int m0 = (logical / a.tiles_n) * BM, n0 = (logical % a.tiles_n) * BN;
  const int kt0 = split * a.nk_per_split;
  const int kt1 = min(a.nk, kt0 + a.nk_per_split);

  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  const int arow = (wave / WN) * FM * 32, brow = (wave % WN) * FN * 32;

  typename SA::type la;
  typename SB::type lb;
  la.init(a, m0, wave, lane, kt0);
  lb.init(a, n0, wave, lane, kt0);

  Frag<SA::KC, BM> fa[FM];
  Frag<SB::KC, BN> fb[FN];
#pragma unroll
  for (int i = 0; i < FM; ++i) fa[i].init(ring, arow + i * 32, lane);
#pragma unroll
  for (int j = 0; j < FN; ++j) fb[j].init(ring + A_BYTES, brow + j * 32, lane);

  // one k-tile out of ring slot `slot` (a compile-time constant): four k-steps of 16; `between(ks)` runs
  // after the MFMAs of step ks are issued, which is where the loop puts the issue of the next direct
  // loads, so that their address work overlaps the matrix pipeline instead of delaying the first LDS
  // reads after the barrier
  auto multiply = [&](auto slot, auto between) {
    constexpr int off = decltype(slot)::value * STAGE_BYTES;
    constexpr int NKS = BK / 16;
    // All fragment reads of the k-tile are issued first, in the order the MFMAs consume them: LDS
    // returns data in order, so the first MFMA waits for one LDS latency and the rest of the reads
    // stream in behind the running matrix pipeline (one exposed latency per k-tile instead of one
    // per k-step).  The scheduling barrier keeps the compiler from re-interleaving the two phases.
    // (The ring-less 128x128 variant runs four workgroups per CU on 128 registers: it reads per k-step.)
    constexpr int AHEAD = (STAGES == 1 && FM * FN == 4) ? 1 : NKS;
    bf16x8 af[NKS][FM], bf[NKS][FN];
#pragma unroll
    for (int k0 = 0; k0 < NKS; k0 += AHEAD) {
#pragma unroll
      for (int ks = k0; ks < k0 + AHEAD; ++ks) {
#pragma unroll
        for (int i = 0; i < FM; ++i) af[ks][i] = fa[i].load(off, ks);
#pragma unroll
        for (int j = 0; j < FN; ++j) bf[ks][j] = fb[j].load(off, ks);
      }
      if (AHEAD == NKS) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int ks = k0; ks < k0 + AHEAD; ++ks) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
          for (int j = 0; j < FN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks][i], bf[ks][j], acc[i][j], 0, 0, 0);
        between(ks);
      }
    }
  };

  if constexpr (STAGES == 1) {
    for (int kt = kt0; kt < kt1; ++kt) {
      if (kt > kt0) __syncthreads();  // everyone is done reading the previous k-tile
      la.issue(a, ring, wave);
      lb.issue(a, ring + A_BYTES, wave);
      wait_vmcnt<0>();
      __syncthreads();
      multiply(std::integral_constant<int, 0>{}, [](int) {});
    }
  } else {
    // prologue: k-tiles kt0 .. kt0+STAGES-2 (tiles past the end fetch zeros: the counts stay uniform)
#pragma unroll
    for (int s = 0; s < STAGES - 1; ++s) {
      la.issue(a, ring + s * STAGE_BYTES, wave);
      lb.issue(a, ring + s * STAGE_BYTES + A_BYTES, wave);
    }
    // the loop body is written out once per ring slot, so that every LDS address in it is a register
    // plus a constant
    for (int kt = kt0; kt < kt1;) {
      static_for<STAGES>([&](auto slot) {
        if (kt < kt1) {
          constexpr int nxt = (decltype(slot)::value + STAGES - 1) % STAGES;  // the slot k-tile kt-1 used
          wait_vmcnt<(STAGES - 2) * LOADS>();  // this lane's direct loads of k-tile kt have landed
          __syncthreads();                     // ... and everyone's; everyone is done reading tile kt-1
          multiply(slot, [&](int ks) {
            if (ks == 0) la.issue(a, ring + nxt * STAGE_BYTES, wave);
            if (ks == 1) lb.issue(a, ring + nxt * STAGE_BYTES + A_BYTES, wave);
          });
          ++kt;
        }
      });
    }
  }
  // Optional by-product (forward) for a BatchNorm that follows: per channel (column), over the workgroup's BM
  // output rows, the sum of the values as stored (rounded to bf16) and the sum of their squared deviations from
  // that run's own mean.  Each wavefront sums its own FM*32 rows (lanes l and l^32 hold the two halves of a
  // column); the wavefronts of the lower row block then hand their sums to the upper ones through LDS.
  // A wavefront sums deviations from a pivot, the first value of its row block (register 0 of lane l < 32):
  // sum = s + n*pivot and squared deviations = q - s^2/n, with s and q of the size of the channel's spread
  // whatever its mean, so a channel whose mean is many standard deviations loses no digits in the fp32 sums.
  float ssum[FN], sqsum[FN];
  int wcnt = 0;  // valid rows of this wavefront's row block
  if constexpr (PASS == PASS_FWD) {
    if (a.stats) {
      const int rbase = m0 + arow;
      wcnt = min(max(a.Mg - rbase, 0), FM * 32);
      const bool full = wcnt == FM * 32;  // every row of this wavefront exists
      const float inv_cnt = wcnt > 0 ? 1.f / (float)wcnt : 0.f;
#pragma unroll
      for (int j = 0; j < FN; ++j) {
        const float p0 = bf16_to_f32(f32_to_bf16(acc[0][j][0]));
        const float p1 = other_half(p0);
        const float pivot = (lane & 32) ? p1 : p0;
        // four independent chains each, then the other half of the column from lane ^ 32
        float s4[4] = {0.f, 0.f, 0.f, 0.f}, q4[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            float dev = bf16_to_f32(f32_to_bf16(acc[i][j][v])) - pivot;
            if (!full) dev = (rbase + i * 32 + 8 * (v / 4) + 4 * (lane >> 5) + (v % 4) < a.Mg) ? dev : 0.f;
            s4[v % 4] += dev;
            q4[v % 4] = fmaf(dev, dev, q4[v % 4]);
          }
        float s1 = (s4[0] + s4[1]) + (s4[2] + s4[3]);
        float q1 = (q4[0] + q4[1]) + (q4[2] + q4[3]);
        s1 += other_half(s1);
        q1 += other_half(q1);
        ssum[j] = fmaf((float)wcnt, pivot, s1);             // the row block's sum
        sqsum[j] = fmaxf(q1 - s1 * s1 * inv_cnt, 0.f);      // ... and squared deviations from its own mean
      }
    }
  }
  wait_vmcnt<0>();
  __syncthreads();  // the LDS tiles are idle: reuse them for the output tile
  if constexpr (PASS == PASS_FWD) {
    if (a.stats) {  // uniform over the workgroup: every wavefront meets the barrier below
      static_assert(WM == 2, "two row blocks of wavefronts");
      // the exchange area of a column block lies in the output patch of its upper wavefront, which reads it
      // before it overwrites it; nobody else touches that patch
      float* ex = reinterpret_cast<float*>(smem + (wave % WN) * Patch<FN>::BYTES);
      if (wave / WN == 1 && lane < 32) {
#pragma unroll
        for (int j = 0; j < FN; ++j) {
          ex[(j * 32 + lane) * 2] = ssum[j];
          ex[(j * 32 + lane) * 2 + 1] = sqsum[j];
        }
      }
      __syncthreads();
      if (wave / WN == 0 && lane < 32) {
        // two row blocks (n_a and n_b rows, sums s, squared deviations q from their own means) joined:
        // q = q_a + q_b + (s_a/n_a - s_b/n_b)^2 n_a n_b / (n_a + n_b)
        const int cnt = min(max(a.Mg - m0, 0), BM);
        const int nb = cnt - wcnt;  // valid rows of the other row block
        const float fa = (float)wcnt, fb = (float)nb;
        const float inv_a = wcnt > 0 ? 1.f / fa : 0.f, inv_b = nb > 0 ? 1.f / fb : 0.f;
        const float wgt = nb > 0 ? fa * fb / (fa + fb) : 0.f;
        // the table is channel-major: [sum | squared deviations][column][run]
        const long long runs = (a.Mg + BM - 1) / BM;
        float* part = a.stats + m0 / BM;
#pragma unroll
        for (int j = 0; j < FN; ++j) {
          const float sb = ex[(j * 32 + lane) * 2], qb = ex[(j * 32 + lane) * 2 + 1];
          const float dm = ssum[j] * inv_a - sb * inv_b;
          const int col = n0 + brow + j * 32 + lane;
          if (col < a.Ng && cnt > 0) {  // a run with no valid row has no slot
            part[col * runs] = ssum[j] + sb;
            part[(a.Ng + col) * runs] = sqsum[j] + qb + dm * dm * wgt;
          }
        }
      }
    }
  }

  // epilogue.  A 32x32 accumulator block: lane holds column (lane & 31) and, in register v,
  // row 8*(v/4) + 4*(lane >> 5) + (v % 4).
  if constexpr (PASS != PASS_WGRAD) {
    // Each wavefront turns its own sub-tile around through a private LDS patch, 32 rows x (FN*32)
    // columns of fp32 at a time, so that every lane then stores 8 adjacent bf16 outputs (16 bytes) and
    // a store instruction covers whole 128-byte runs of output rows.  No block barrier is needed.
    constexpr int WCOLS = Patch<FN>::WCOLS, CS = Patch<FN>::CS;
    float* cs = reinterpret_cast<float*>(smem + wave * Patch<FN>::BYTES);
    bf16_t* out = static_cast<bf16_t*>(a.out);
    constexpr int CPRO = WCOLS / 8;  // 16-byte output chunks per patch row
    constexpr int ITERS = 32 * CPRO / 64;
    const bool scatter = PASS == PASS_DGRAD && a.scatter2;
    // forward only: the activation as a clamp (relu: [0, inf), relu6: [0, 6], none: everything)
    const bool plain_out = PASS != PASS_FWD || (a.bias == nullptr && a.act == S4TF_ACT_NONE);
    const float act_lo = (PASS == PASS_FWD && a.act != S4TF_ACT_NONE) ? 0.f : -__builtin_inff();
    const float act_hi = (PASS == PASS_FWD && a.act == S4TF_ACT_RELU6) ? 6.f : __builtin_inff();
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      // where this lane's chunks go (-1: outside the matrix); a 1x1 / stride-2 dgrad runs over the
      // pixels of dy and scatters row (n,p,q) to pixel (n,2p,2q) of dx
      long long dsto[ITERS];
      uint4 old[ITERS];
      unsigned obits[ITERS];
#pragma unroll
      for (int it = 0; it < ITERS; ++it) {
        const int chunk = lane + it * 64;
        const int prow = chunk / CPRO, pcol = (chunk % CPRO) * 8;
        const int row = m0 + arow + i * 32 + prow, col = n0 + brow + pcol;
        dsto[it] = -1;
        if (row < a.Mg && col < a.Ng) {
          long long orow = row;
          if (PASS == PASS_DGRAD && a.cls) {
            const int t = fast_div(row, a.magicWc, a.shiftWc), wc = row - t * a.Wc;
            const int n = fast_div(t, a.magicHc, a.shiftHc), hc = t - n * a.Hc;
            orow = ((long long)n * a.g.H + a.g.stride * hc + a.ph) * a.g.W + a.g.stride * wc + a.pw;
          } else if (scatter) {
            const int t = fast_div(row, a.magicQ, a.shiftQ), q = row - t * a.g.Q;
            const int n = fast_div(t, a.magicP, a.shiftP), p = t - n * a.g.P;
            orow = ((long long)n * a.g.H + 2 * p) * a.g.W + 2 * q;
          }
          dsto[it] = orow * a.Ng + col;
          if (PASS == PASS_DGRAD && a.accumulate) {
            const bf16_t* src = a.acc_src ? static_cast<const bf16_t*>(a.acc_src) : out;
            old[it] = *reinterpret_cast<const uint4*>(src + dsto[it]);
            obits[it] = a.acc_bits ? a.acc_bits[dsto[it] >> 3] : 0xffu;
          }
        }
      }
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          cs[(8 * (v / 4) + 4 * (lane >> 5) + (v % 4)) * CS + j * 32 + (lane & 31)] = acc[i][j][v];
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int it = 0; it < ITERS; ++it) {
        const int chunk = lane + it * 64;
        const int prow = chunk / CPRO, pcol = (chunk % CPRO) * 8;
        const int col = n0 + brow + pcol;
        if (dsto[it] >= 0) {
          const float4 lo = *reinterpret_cast<const float4*>(&cs[prow * CS + pcol]);
          const float4 hi = *reinterpret_cast<const float4*>(&cs[prow * CS + pcol + 4]);
          float v8[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
          bf16_t* dst = out + dsto[it];
          if constexpr (PASS == PASS_FWD) {
            if (!plain_out) {  // bias and activation: one uniform branch per chunk, none per element
              float b8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
              if (a.bias) {
                const float4 b0 = *reinterpret_cast<const float4*>(a.bias + col);
                const float4 b1 = *reinterpret_cast<const float4*>(a.bias + col + 4);
                b8[0] = b0.x; b8[1] = b0.y; b8[2] = b0.z; b8[3] = b0.w;
                b8[4] = b1.x; b8[5] = b1.y; b8[6] = b1.z; b8[7] = b1.w;
              }
#pragma unroll
              for (int e = 0; e < 8; ++e) v8[e] = fminf(fmaxf(v8[e] + b8[e], act_lo), act_hi);
            }
          }
          if (PASS == PASS_DGRAD && a.accumulate) {
#pragma unroll
            for (int e = 0; e < 8; ++e) v8[e] += ((obits[it] >> e) & 1) ? bf16_to_f32((bf16_t)half_of(old[it], e)) : 0.f;
          }
          uint4 o;
          o.x = (uint32_t)f32_to_bf16(v8[0]) | ((uint32_t)f32_to_bf16(v8[1]) << 16);
          o.y = (uint32_t)f32_to_bf16(v8[2]) | ((uint32_t)f32_to_bf16(v8[3]) << 16);
          o.z = (uint32_t)f32_to_bf16(v8[4]) | ((uint32_t)f32_to_bf16(v8[5]) << 16);
          o.w = (uint32_t)f32_to_bf16(v8[6]) | ((uint32_t)f32_to_bf16(v8[7]) << 16);
          *reinterpret_cast<uint4*>(dst) = o;
          if (scatter && !a.accumulate) {
            // the three pixels of the 2x2 cell that no output pixel reads get a zero cotangent
            const int row = m0 + arow + i * 32 + prow;
            const int t = fast_div(row, a.magicQ, a.shiftQ), q = row - t * a.g.Q;
            const int p = t - fast_div(t, a.magicP, a.shiftP) * a.g.P;
            const uint4 z = make_uint4(0, 0, 0, 0);
            const bool wr = 2 * q + 1 < a.g.W, hd = 2 * p + 1 < a.g.H;
            if (wr) *reinterpret_cast<uint4*>(dst + a.Ng) = z;
            if (hd) *reinterpret_cast<uint4*>(dst + (long long)a.g.W * a.Ng) = z;
            if (wr && hd) *reinterpret_cast<uint4*>(dst + (long long)(a.g.W + 1) * a.Ng) = z;
          }
        }
      }
      __builtin_amdgcn_wave_barrier();
    }
  } else {
    float* dw = static_cast<float*>(a.out) + (long long)split * a.split_stride;
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j) {
        const int col = n0 + brow + j * 32 + (lane & 31);
        if (col >= a.Ng) continue;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = m0 + arow + i * 32 + 8 * (v / 4) + 4 * (lane >> 5) + (v % 4);
          if (row < a.Mg) dw[(long long)row * a.Ng + col] = acc[i][j][v];
        }
      }
  }
}

}  // namespace

bool igemm_dma_geom_ok(int pass, const ConvGeom& g) {
  auto chan_ok = [](int c) { return c % BK == 0 || c == 8 || c == 16 || c == 32; };
  const long long lim = 1LL << 30;  // elements: keeps every byte offset below 2^31
  if ((long long)g.N * g.H * g.W * g.C >= lim || (long long)g.N * g.P * g.Q * g.K >= lim ||
      (long long)g.R * g.S * g.C * g.K >= lim || g.R * g.S > 64 || g.S > 32)
    return false;
  if (pass == PASS_FWD && !chan_ok(g.C)) return false;
  if (pass == PASS_DGRAD && !chan_ok(g.K)) return false;
  return g.C % 8 == 0 && g.K % 8 == 0;
}

bool igemm_dma_ok(int pass, const ConvGeom& g, const Args& a) {
  return igemm_dma_geom_ok(pass, g) && aligned16(a.a) && aligned16(a.b) && aligned16(a.out);
}

// Tile choice.  GEMMs at most 64 columns wide take 128x64 tiles (a 128-wide tile would spend half
// its MFMAs on padding).  Otherwise 128x128 when that already gives every SIMD of the chip
// (256 CUs x 4) two wavefronts to interleave, else 64x128: twice the workgroups, which the small
// late-stage layers need more than they need the better LDS-bytes-per-MFMA ratio of the big tile.
// wgrad picks by the matrix shape alone (its workgroup count is set by the split of the reduction).
void igemm_dma_tile(int pass, int Mg, int Ng, int splits, int& BM, int& BN) {
  BM = 128;
  BN = Ng <= 64 ? 64 : 128;
  if (BN == 64) return;  // (128x64)
  if (pass == PASS_WGRAD) {
    // 64-row tiles: twice the tiles, so half the splits of the reduction axis fill the chip, and half the
    // fp32 partial sums are written and read back (measured over a ResNet-50 step: -1.8 %)
    BM = 64;
  } else if ((long long)((Mg + 127) / 128) * ((Ng + 127) / 128) * splits < 384) {
    // fewer than 1.5 workgroups of 128x128 per CU: 64-row tiles (inside a training step, where the filter
    // gradients of the second stream share the CUs, 384 measured 0.7 % better than 512 and like 256)
    BM = 64;
    // still fewer workgroups than CUs (the 7x7 layers): 64x64, twice as many again
    if ((long long)((Mg + 63) / 64) * ((Ng + 127) / 128) * splits < 256) BN = 64;
  }
}

constexpr int SHORT_NK = 2;

template <int PASS, int FM, int FN>
static void launch_tile(Args& a, int splits, hipStream_t st) {
  constexpr int BM = 2 * FM * 32, BN = 2 * FN * 32;
  a.tiles_m = (a.Mg + BM - 1) / BM;
  a.tiles_n = (a.Ng + BN - 1) / BN;
  a.splits = splits;
  a.stats_rows = BM;
  unsigned blocks_all = grid_blocks(a);
  if (PASS == PASS_DGRAD && a.cls) {  // the four classes side by side, each dealt to the XCDs like a launch of its own
    blocks_all = 0;
    for (int c = 0; c < 4; ++c) {
      Args t = a;
      t.tiles_m = a.cls_tiles_m[c] = (a.cls_Mg[c] + BM - 1) / BM;
      blocks_all += grid_blocks(t);
      a.cls_end[c] = (int)blocks_all;
    }
    a.tiles_m = a.cls_tiles_m[3];
  }
  dim3 grid(blocks_all);
  // GEMMs with at most SHORT_NK k-tiles: no ring, twice the workgroups per CU
  // Ring depth.  LDS decides how many workgroups share a CU (160 KiB); a grid with more workgroups than
  // that keeps the CUs busiest with many short rings, a grid that cannot fill them anyway is better
  // off with the deeper ring its LDS share allows: fewer exposed load latencies per workgroup.
  constexpr int STAGE = (BM + BN) * ROWB;
  constexpr int DEEP2 = 2 * 3 * STAGE <= 160 * 1024 ? 3 : 2;  // two workgroups per CU
  constexpr int DEEP1 = 5 * STAGE <= 160 * 1024 ? 5 : 4;      // one workgroup per CU
  const long long blocks = (PASS == PASS_DGRAD && a.cls) ? (long long)blocks_all : (long long)a.tiles_m * a.tiles_n * splits;
  if (PASS != PASS_WGRAD && a.nk <= SHORT_NK)  // no ring, four workgroups per CU
    hipLaunchKernelGGL((igemm_dma_kernel<PASS, (PASS == PASS_WGRAD ? 2 : 1), 2, 2, FM, FN>), grid, dim3(NT), 0, st, a);
  else if (blocks <= 256 && a.nk_per_split >= 8)
    hipLaunchKernelGGL((igemm_dma_kernel<PASS, DEEP1, 2, 2, FM, FN>), grid, dim3(NT), 0, st, a);
  else if (blocks <= 1024 && DEEP2 == 3)  // measured: up to two rounds of workgroups gain from the third stage, longer grids lose
    hipLaunchKernelGGL((igemm_dma_kernel<PASS, DEEP2, 2, 2, FM, FN>), grid, dim3(NT), 0, st, a);
  else
    hipLaunchKernelGGL((igemm_dma_kernel<PASS, 2, 2, 2, FM, FN>), grid, dim3(NT), 0, st, a);
}

template <int PASS> static void launch_pass(Args& a, int splits, hipStream_t st) {
  int BM, BN;
  igemm_dma_tile(PASS, a.Mg, a.Ng, splits, BM, BN);
  if (BN == 64 && BM == 64) launch_tile<PASS, 1, 1>(a, splits, st);
  else if (BN == 64) launch_tile<PASS, 2, 1>(a, splits, st);
  else if (BM == 64) launch_tile<PASS, 1, 2>(a, splits, st);
  else launch_tile<PASS, 2, 2>(a, splits, st);
}

int igemm_dma_launch(int pass, Args& a, int splits, hipStream_t st) {
  if (pass == PASS_FWD) launch_pass<PASS_FWD>(a, splits, st);
  else if (pass == PASS_DGRAD) launch_pass<PASS_DGRAD>(a, splits, st);
  else launch_pass<PASS_WGRAD>(a, splits, st);
  return launch_status("igemm_dma");
}

}  // namespace s4tf
