// Dense (groups == 1) convolution as implicit GEMM on the gfx950 matrix cores.
//
// The three passes of a convolution are each one GEMM  D[i][j] = sum_k A[i][k] * B[j][k]:
//   forward  y [m=(n,p,q)][ko]      A = im2col(x)      k = (r,s,c)    B[ko][k]  = w[r,s,c,ko]
//   dgrad    dx[m=(n,h,w)][c]       A = gather(dy)     k = (r,s,ko)   B[c][k]   = w[r,s,c,ko]
//   wgrad    dw[i=(r,s,c)][ko]      A = im2col(x)^T    k = (n,p,q)    B[ko][k]  = dy[n,p,q,ko]
// (the op and its pullback in the sense of the paper's Section 2.1; layouts NHWC / RSCK).
// Nothing is materialised: the loaders compute addresses on the fly, stage a BM x BK and a
// BN x BK tile in LDS (k contiguous, padded rows, double buffered) and four wavefronts of 64
// lanes each own a 64x64 sub-tile made of 2x2 MFMA 32x32 blocks.  bf16 uses
// v_mfma_f32_32x32x16_bf16 (8 k-values per lane), fp32 uses v_mfma_f32_32x32x2_f32.
// Operands whose memory is contiguous along the GEMM row instead of along k (filters in the
// forward pass, both operands of wgrad) are transposed in registers on their way into LDS.
#include "s4tf_internal.h"
#include "igemm_args.h"

namespace s4tf {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

template <typename T> struct Cfg;
template <> struct Cfg<float> { static constexpr int VEC = 4, BK = 16, PAD = 1; };
template <> struct Cfg<bf16_t> { static constexpr int VEC = 8, BK = 64, PAD = 8; };

__device__ inline uint4 ldg16(const void* p) { return *reinterpret_cast<const uint4*>(p); }
__device__ inline uint4 zero16() { return make_uint4(0u, 0u, 0u, 0u); }

// ---- element index of operand A / B for (row, k), or -1 when it is padding ------------------
// (the element-wise loaders call these per element: every quotient is a multiply-high by a host-computed
// reciprocal; run-time divisions had made them ~150 instructions, most of a first layer's time)
template <int PASS> __device__ inline long long a_index(const Args& a, int row, int kk) {
  const ConvGeom& g = a.g;
  if (PASS == PASS_FWD) {
    const int t = div_magic(row, a.magicQ, a.shiftQ), q = row - t * g.Q, n = div_magic(t, a.magicP, a.shiftP), p = t - n * g.P;
    const int t2 = div_magic(kk, a.magicC, a.shiftC), c = kk - t2 * g.C, r = div_magic(t2, a.magicS, a.shiftS), s = t2 - r * g.S;
    int h = p * g.stride + r - g.pad, w = q * g.stride + s - g.pad;
    if (h < 0 || h >= g.H || w < 0 || w >= g.W) return -1;
    return (((long long)n * g.H + h) * g.W + w) * g.C + c;
  } else if (PASS == PASS_DGRAD) {
    const int t = div_magic(row, a.magicW, a.shiftW), w = row - t * g.W, n = div_magic(t, a.magicH, a.shiftH), h = t - n * g.H;
    const int t2 = div_magic(kk, a.magicK, a.shiftK), ko = kk - t2 * g.K, r = div_magic(t2, a.magicS, a.shiftS), s = t2 - r * g.S;
    int hp = h + g.pad - r, wp = w + g.pad - s;
    if (hp < 0 || wp < 0) return -1;
    int p = hp / g.stride, q = wp / g.stride;
    if (p * g.stride != hp || q * g.stride != wp || p >= g.P || q >= g.Q) return -1;
    return (((long long)n * g.P + p) * g.Q + q) * g.K + ko;
  } else {
    const int t2 = div_magic(row, a.magicC, a.shiftC), c = row - t2 * g.C, r = div_magic(t2, a.magicS, a.shiftS), s = t2 - r * g.S;
    const int t = div_magic(kk, a.magicQ, a.shiftQ), q = kk - t * g.Q, n = div_magic(t, a.magicP, a.shiftP), p = t - n * g.P;
    int h = p * g.stride + r - g.pad, w = q * g.stride + s - g.pad;
    if (h < 0 || h >= g.H || w < 0 || w >= g.W) return -1;
    return (((long long)n * g.H + h) * g.W + w) * g.C + c;
  }
}
template <int PASS> __device__ inline long long b_index(const Args& a, int col, int kk) {
  const ConvGeom& g = a.g;
  if (PASS == PASS_DGRAD) {
    const int rs = div_magic(kk, a.magicK, a.shiftK), ko = kk - rs * g.K;
    return ((long long)rs * g.C + col) * g.K + ko;
  }
  return (long long)kk * g.K + col;  // filters as [(r,s,c)][ko], dy as [(n,p,q)][ko]
}

// ---- LDS tile stores ---------------------------------------------------------------------------
template <typename T, int STRIDE> __device__ inline void store_kvec(T* tile, int row, int k0, uint4 v) {
  if constexpr (sizeof(T) == 2) {
    *reinterpret_cast<uint4*>(&tile[row * STRIDE + k0]) = v;
  } else {
    uint32_t* p = reinterpret_cast<uint32_t*>(&tile[row * STRIDE + k0]);
    p[0] = v.x; p[1] = v.y; p[2] = v.z; p[3] = v.w;
  }
}
__device__ inline uint32_t dword_of(const uint4& v, int i) {
  return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w;
}
__device__ inline uint32_t half_of(const uint4& v, int e) {  // 16-bit element e of 8
  uint32_t d = dword_of(v, e >> 1);
  return (e & 1) ? (d >> 16) : (d & 0xffffu);
}

// ---- loaders --------------------------------------------------------------------------------
// K-contiguous sources: a thread owns one 16-byte chunk column (kc) of ROWS/64 rows.
template <typename T, int ROWS, int BK_> struct KLoaderBase {
  static constexpr int VEC = Cfg<T>::VEC, BK = BK_, STRIDE = BK + Cfg<T>::PAD;
  static constexpr int CPR = BK / VEC;       // chunks per row
  static constexpr int RPP = NT / CPR;       // rows per pass
  static constexpr int NP = (ROWS + RPP - 1) / RPP;
  uint4 v[NP];
  __device__ void store(T* tile, int tid) const {
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      int row = tid / CPR + i * RPP;
      if (ROWS % RPP == 0 || row < ROWS) store_kvec<T, STRIDE>(tile, row, (tid % CPR) * VEC, v[i]);
    }
  }
};

// forward A: rows are output pixels (n,p,q), k = (r,s,c)
template <typename T, int ROWS, int BK_> struct FwdALoader : KLoaderBase<T, ROWS, BK_> {
  typedef KLoaderBase<T, ROWS, BK_> B_;
  const T* x;
  long long base[B_::NP];
  int h0[B_::NP], w0[B_::NP];
  bool rv[B_::NP];
  int r, s, c;
  __device__ void init(const Args& a, int row0, int tid, int kt0) {
    x = static_cast<const T*>(a.a);
    const ConvGeom& g = a.g;
#pragma unroll
    for (int i = 0; i < B_::NP; ++i) {
      int row = row0 + tid / B_::CPR + i * B_::RPP;
      rv[i] = row < a.Mg && (ROWS % B_::RPP == 0 || tid / B_::CPR + i * B_::RPP < ROWS);
      const int t = div_magic(row, a.magicQ, a.shiftQ), q = row - t * g.Q, n = div_magic(t, a.magicP, a.shiftP), p = t - n * g.P;
      base[i] = (long long)n * g.H * g.W * g.C;
      h0[i] = p * g.stride - g.pad;
      w0[i] = q * g.stride - g.pad;
    }
    int kk = kt0 * B_::BK + (tid % B_::CPR) * B_::VEC;
    const int t2 = div_magic(kk, a.magicC, a.shiftC);
    c = kk - t2 * g.C;
    r = div_magic(t2, a.magicS, a.shiftS);
    s = t2 - r * g.S;
  }
  __device__ void load(const Args& a) {
    const ConvGeom& g = a.g;
#pragma unroll
    for (int i = 0; i < B_::NP; ++i) {
      int h = h0[i] + r, w = w0[i] + s;
      bool ok = rv[i] && r < g.R && h >= 0 && h < g.H && w >= 0 && w < g.W;
      this->v[i] = ok ? ldg16(x + base[i] + ((long long)h * g.W + w) * g.C + c) : zero16();
    }
    c += B_::BK;
    while (c >= g.C) {
      c -= g.C;
      if (++s == g.S) { s = 0; ++r; }
    }
  }
};

// dgrad A: rows are input pixels (n,h,w), k = (r,s,ko); gathers dy
template <typename T, int ROWS, int BK_> struct DgradALoader : KLoaderBase<T, ROWS, BK_> {
  typedef KLoaderBase<T, ROWS, BK_> B_;
  const T* dy;
  long long base[B_::NP];
  int hp0[B_::NP], wp0[B_::NP];
  bool rv[B_::NP];
  int r, s, ko;
  __device__ void init(const Args& a, int row0, int tid, int kt0) {
    dy = static_cast<const T*>(a.a);
    const ConvGeom& g = a.g;
#pragma unroll
    for (int i = 0; i < B_::NP; ++i) {
      int row = row0 + tid / B_::CPR + i * B_::RPP;
      rv[i] = row < a.Mg && (ROWS % B_::RPP == 0 || tid / B_::CPR + i * B_::RPP < ROWS);
      const int t = div_magic(row, a.magicW, a.shiftW), w = row - t * g.W, n = div_magic(t, a.magicH, a.shiftH), h = t - n * g.H;
      base[i] = (long long)n * g.P * g.Q * g.K;
      hp0[i] = h + g.pad;
      wp0[i] = w + g.pad;
    }
    int kk = kt0 * B_::BK + (tid % B_::CPR) * B_::VEC;
    const int t2 = div_magic(kk, a.magicK, a.shiftK);
    ko = kk - t2 * g.K;
    r = div_magic(t2, a.magicS, a.shiftS);
    s = t2 - r * g.S;
  }
  __device__ void load(const Args& a) {
    const ConvGeom& g = a.g;
#pragma unroll
    for (int i = 0; i < B_::NP; ++i) {
      int hp = hp0[i] - r, wp = wp0[i] - s;
      bool ok = rv[i] && r < g.R && hp >= 0 && wp >= 0;
      int p, q;
      if (g.stride == 1) {
        p = hp; q = wp;
      } else if (g.stride == 2) {
        ok = ok && (((hp | wp) & 1) == 0);
        p = hp >> 1; q = wp >> 1;
      } else {
        p = hp / g.stride; q = wp / g.stride;
        ok = ok && p * g.stride == hp && q * g.stride == wp;
      }
      ok = ok && p < g.P && q < g.Q;
      this->v[i] = ok ? ldg16(dy + base[i] + ((long long)p * g.Q + q) * g.K + ko) : zero16();
    }
    ko += B_::BK;
    while (ko >= g.K) {
      ko -= g.K;
      if (++s == g.S) { s = 0; ++r; }
    }
  }
};

// dgrad B: rows are input channels c, k = (r,s,ko); filters are contiguous along ko
template <typename T, int ROWS, int BK_> struct DgradBLoader : KLoaderBase<T, ROWS, BK_> {
  typedef KLoaderBase<T, ROWS, BK_> B_;
  const T* w;
  int cidx[B_::NP];
  bool rv[B_::NP];
  int rs, ko;
  __device__ void init(const Args& a, int row0, int tid, int kt0) {
    w = static_cast<const T*>(a.b);
#pragma unroll
    for (int i = 0; i < B_::NP; ++i) {
      cidx[i] = row0 + tid / B_::CPR + i * B_::RPP;
      rv[i] = cidx[i] < a.Ng && (ROWS % B_::RPP == 0 || tid / B_::CPR + i * B_::RPP < ROWS);
    }
    int kk = kt0 * B_::BK + (tid % B_::CPR) * B_::VEC;
    rs = div_magic(kk, a.magicK, a.shiftK);
    ko = kk - rs * a.g.K;
  }
  __device__ void load(const Args& a) {
    const ConvGeom& g = a.g;
#pragma unroll
    for (int i = 0; i < B_::NP; ++i) {
      bool ok = rv[i] && rs < g.R * g.S;
      this->v[i] = ok ? ldg16(w + ((long long)rs * g.C + cidx[i]) * g.K + ko) : zero16();
    }
    ko += B_::BK;
    while (ko >= g.K) { ko -= g.K; ++rs; }
  }
};

// Row-contiguous sources.  A thread owns VEC adjacent rows at KP consecutive k positions and
// scatters them into the k-contiguous LDS tile (bf16: packs KP values per row into one store).
template <typename T, int ROWS, int BK_> struct RLoaderBase {
  static constexpr int VEC = Cfg<T>::VEC, BK = BK_, STRIDE = BK + Cfg<T>::PAD;
  static constexpr int RC = ROWS / VEC;                       // row chunks
  static constexpr int KG = (NT / RC) < BK ? (NT / RC) : BK;  // k groups
  static constexpr int KP = BK / KG;                          // k positions per thread
  static_assert(KP == 1 || KP == 2 || KP == 4, "unsupported tile shape");
  uint4 v[KP];
  __device__ static bool active(int tid) { return tid < RC * KG; }
  __device__ static int kgroup(int tid) { return tid % KG; }
  __device__ static int rchunk(int tid) { return tid / KG; }
  __device__ void store(T* tile, int tid) const {
    if (!active(tid)) return;
    int row0 = rchunk(tid) * VEC, k0 = kgroup(tid) * KP;
    if constexpr (sizeof(T) == 2) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        T* dst = &tile[(row0 + e) * STRIDE + k0];
        if constexpr (KP == 1) {
          *dst = (T)half_of(v[0], e);
        } else if constexpr (KP == 2) {
          *reinterpret_cast<uint32_t*>(dst) = half_of(v[0], e) | (half_of(v[1], e) << 16);
        } else {
          uint2 o;
          o.x = half_of(v[0], e) | (half_of(v[1], e) << 16);
          o.y = half_of(v[2], e) | (half_of(v[3], e) << 16);
          *reinterpret_cast<uint2*>(dst) = o;
        }
      }
    } else {
#pragma unroll
      for (int u = 0; u < KP; ++u)
#pragma unroll
        for (int e = 0; e < 4; ++e)
          *reinterpret_cast<uint32_t*>(&tile[(row0 + e) * STRIDE + k0 + u]) = dword_of(v[u], e);
    }
  }
};

// plain [k][ld] matrix: filters in the forward pass ([(r,s,c)][ko]) and dy in wgrad ([(n,p,q)][ko])
template <typename T, int ROWS, int BK_> struct PlainRLoader : RLoaderBase<T, ROWS, BK_> {
  typedef RLoaderBase<T, ROWS, BK_> B_;
  const T* src;
  int j0, kk;
  bool rv;
  __device__ void init(const Args& a, int row0, int tid, int kt0) {
    src = static_cast<const T*>(a.b);
    j0 = row0 + B_::rchunk(tid) * B_::VEC;
    rv = B_::active(tid) && j0 < a.Ng;
    kk = kt0 * B_::BK + B_::kgroup(tid) * B_::KP;
  }
  __device__ void load(const Args& a) {
#pragma unroll
    for (int u = 0; u < B_::KP; ++u) {
      bool ok = rv && kk + u < a.Kg;
      this->v[u] = ok ? ldg16(src + (long long)(kk + u) * a.g.K + j0) : zero16();
    }
    kk += B_::BK;
  }
};

// wgrad A: rows are (r,s,c) (contiguous along c), k = output pixel (n,p,q); gathers x
template <typename T, int ROWS, int BK_> struct WgradALoader : RLoaderBase<T, ROWS, BK_> {
  typedef RLoaderBase<T, ROWS, BK_> B_;
  const T* x;
  int r, s, c0;
  bool rv;
  int pn[B_::KP], pp[B_::KP], pq[B_::KP];
  int m;  // pixel index of k position 0
  __device__ void init(const Args& a, int row0, int tid, int kt0) {
    x = static_cast<const T*>(a.a);
    const ConvGeom& g = a.g;
    int i0 = row0 + B_::rchunk(tid) * B_::VEC;
    rv = B_::active(tid) && i0 < a.Mg;
    const int t2 = div_magic(i0, a.magicC, a.shiftC);
    c0 = i0 - t2 * g.C;
    r = div_magic(t2, a.magicS, a.shiftS);
    s = t2 - r * g.S;
    m = kt0 * B_::BK + B_::kgroup(tid) * B_::KP;
#pragma unroll
    for (int u = 0; u < B_::KP; ++u) {
      const int mm = m + u, t = div_magic(mm, a.magicQ, a.shiftQ);
      pq[u] = mm - t * g.Q;
      pn[u] = div_magic(t, a.magicP, a.shiftP);
      pp[u] = t - pn[u] * g.P;
    }
  }
  __device__ void load(const Args& a) {
    const ConvGeom& g = a.g;
#pragma unroll
    for (int u = 0; u < B_::KP; ++u) {
      bool ok = rv && m + u < a.Kg;
      long long idx;
      if (a.simple) {
        idx = (long long)(m + u) * g.C + c0;
      } else {
        int h = pp[u] * g.stride + r - g.pad, w = pq[u] * g.stride + s - g.pad;
        ok = ok && h >= 0 && h < g.H && w >= 0 && w < g.W;
        idx = (((long long)pn[u] * g.H + h) * g.W + w) * g.C + c0;
        pq[u] += B_::BK;
        while (pq[u] >= g.Q) {
          pq[u] -= g.Q;
          if (++pp[u] == g.P) { pp[u] = 0; ++pn[u]; }
        }
      }
      this->v[u] = ok ? ldg16(x + idx) : zero16();
    }
    m += B_::BK;
  }
};

// Element-wise fallback for channel counts that are not a multiple of the vector width
// (first layers with 1 or 3 channels, 6- and 10-wide outputs).  Full index arithmetic per
// element: slow, used only where the tensors are tiny or the layer is a stem.
template <typename T, int PASS, int ROWS, bool IS_A, int BK_> struct ScalarLoader {
  static constexpr int BK = BK_, STRIDE = BK + Cfg<T>::PAD;
  static constexpr int E = ROWS * BK / NT;
  static constexpr bool KFAST = IS_A ? (PASS != PASS_WGRAD) : (PASS == PASS_DGRAD);
  T v[E];
  int row0, kbase;
  __device__ void init(const Args&, int row0_, int, int kt0) {
    row0 = row0_;
    kbase = kt0 * BK;
  }
  __device__ void load(const Args& a, int tid) {
    const T* src = static_cast<const T*>(IS_A ? a.a : a.b);
#pragma unroll
    for (int i = 0; i < E; ++i) {
      int e = tid + i * NT;
      int rl = KFAST ? e / BK : e % ROWS, kl = KFAST ? e % BK : e / ROWS;
      int row = row0 + rl, kk = kbase + kl;
      long long idx = -1;
      if (row < (IS_A ? a.Mg : a.Ng) && kk < a.Kg)
        idx = IS_A ? a_index<PASS>(a, row, kk) : b_index<PASS>(a, row, kk);
      v[i] = idx >= 0 ? src[idx] : (T)0;
    }
    kbase += BK;
  }
  __device__ void store(T* tile, int tid) const {
#pragma unroll
    for (int i = 0; i < E; ++i) {
      int e = tid + i * NT;
      int rl = KFAST ? e / BK : e % ROWS, kl = KFAST ? e % BK : e / ROWS;
      tile[rl * STRIDE + kl] = v[i];
    }
  }
};

template <typename T, int PASS, int ROWS, bool VECMODE, bool IS_A, int BK_> struct LoaderSel;
template <typename T, int ROWS, int BK_> struct LoaderSel<T, PASS_FWD, ROWS, true, true, BK_> { typedef FwdALoader<T, ROWS, BK_> type; };
template <typename T, int ROWS, int BK_> struct LoaderSel<T, PASS_FWD, ROWS, true, false, BK_> { typedef PlainRLoader<T, ROWS, BK_> type; };
template <typename T, int ROWS, int BK_> struct LoaderSel<T, PASS_DGRAD, ROWS, true, true, BK_> { typedef DgradALoader<T, ROWS, BK_> type; };
template <typename T, int ROWS, int BK_> struct LoaderSel<T, PASS_DGRAD, ROWS, true, false, BK_> { typedef DgradBLoader<T, ROWS, BK_> type; };
template <typename T, int ROWS, int BK_> struct LoaderSel<T, PASS_WGRAD, ROWS, true, true, BK_> { typedef WgradALoader<T, ROWS, BK_> type; };
template <typename T, int ROWS, int BK_> struct LoaderSel<T, PASS_WGRAD, ROWS, true, false, BK_> { typedef PlainRLoader<T, ROWS, BK_> type; };

// ---- MFMA over one staged k-tile ----------------------------------------------------------------
template <typename T, int FM, int FN, int STRIDE, int BK>
__device__ inline void mma_tile(const T* As, const T* Bs, int arow, int brow, int lane, f32x16 (&acc)[FM][FN]) {
  if constexpr (sizeof(T) == 2) {
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 af[FM], bf[FN];
#pragma unroll
      for (int i = 0; i < FM; ++i)
        af[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(
                    &As[(arow + i * 32 + (lane & 31)) * STRIDE + ks * 16 + 8 * (lane >> 5)]));
#pragma unroll
      for (int j = 0; j < FN; ++j)
        bf[j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(
                    &Bs[(brow + j * 32 + (lane & 31)) * STRIDE + ks * 16 + 8 * (lane >> 5)]));
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
    }
  } else {
#pragma unroll
    for (int ks = 0; ks < BK / 2; ++ks) {
      float af[FM], bf[FN];
#pragma unroll
      for (int i = 0; i < FM; ++i) af[i] = As[(arow + i * 32 + (lane & 31)) * STRIDE + ks * 2 + (lane >> 5)];
#pragma unroll
      for (int j = 0; j < FN; ++j) bf[j] = Bs[(brow + j * 32 + (lane & 31)) * STRIDE + ks * 2 + (lane >> 5)];
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i], bf[j], acc[i][j], 0, 0, 0);
    }
  }
}

// WM x WN x WK wavefronts, each FM x FN MFMA blocks of 32x32.  With WK > 1 the WK wavefronts that share
// an output sub-tile each multiply a WK-th of every k-tile's depth and their accumulators are added
// through LDS before the epilogue: small output tiles (many workgroups for GEMMs with few rows) that
// still keep four wavefronts busy.  NBUF = 2 stores the next k-tile into a second LDS buffer while the current
// one is multiplied; NBUF = 1 has one buffer and a second barrier per k-tile instead, which lets twice as many
// workgroups share a CU: for GEMMs whose k-loop is a handful of tiles, where what hides the load latency is
// other workgroups and not this one's own pipeline.
template <typename T, int PASS, bool VECMODE, int WM, int WN, int FM, int FN, int BK_, int WK = 1, int NBUF = 2>
__global__ __launch_bounds__(NT) void igemm_kernel(const Args a) {
  static_assert(WM * WN * WK == 4, "four wavefronts");
  static_assert(WK == 1 || sizeof(T) == 4, "the k split over wavefronts is for the fp32 epilogue only");
  constexpr int BM = WM * FM * 32, BN = WN * FN * 32;
  constexpr int BK = BK_, STRIDE = BK + Cfg<T>::PAD;
  constexpr int KW = BK / WK;  // depth of a k-tile one wavefront multiplies
  constexpr int TILE = (BM + BN) * STRIDE;
  static_assert((WK - 1) * FM * FN * 16 * 64 * 4 <= NBUF * TILE * (int)sizeof(T), "accumulators must fit in the tile buffers");
  __shared__ __attribute__((aligned(16))) T smem[NBUF * TILE];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // consecutive workgroup ids land on different XCDs; give each XCD a contiguous run of
  // tiles so that tiles sharing an A row-block share that XCD's L2
  int logical, split;
  if (!block_to_tile(a, logical, split)) return;
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

  const int wk = wave / (WM * WN), wmn = wave % (WM * WN);
  const int arow = (wmn / WN) * FM * 32, brow = (wmn % WN) * FN * 32;
  const int koff = wk * KW;

  if constexpr (VECMODE) {
    typename LoaderSel<T, PASS, BM, true, true, BK>::type la;
    typename LoaderSel<T, PASS, BN, true, false, BK>::type lb;
    la.init(a, m0, tid, kt0);
    lb.init(a, n0, tid, kt0);
    la.load(a);
    lb.load(a);
    la.store(smem, tid);
    lb.store(smem + BM * STRIDE, tid);
    __syncthreads();
    for (int kt = kt0; kt < kt1; ++kt) {
      const int cur = NBUF == 2 ? (kt - kt0) & 1 : 0, nxt = NBUF == 2 ? cur ^ 1 : 0;
      const bool more = kt + 1 < kt1;
      if (more) {
        la.load(a);
        lb.load(a);
      }
      mma_tile<T, FM, FN, STRIDE, KW>(smem + cur * TILE + koff, smem + cur * TILE + BM * STRIDE + koff, arow, brow, lane, acc);
      if (NBUF == 1) __syncthreads();  // everyone is done reading the only buffer
      if (more) {
        la.store(smem + nxt * TILE, tid);
        lb.store(smem + nxt * TILE + BM * STRIDE, tid);
      }
      __syncthreads();
    }
  } else {
    ScalarLoader<T, PASS, BM, true, BK> la;
    ScalarLoader<T, PASS, BN, false, BK> lb;
    la.init(a, m0, tid, kt0);
    lb.init(a, n0, tid, kt0);
    la.load(a, tid);
    lb.load(a, tid);
    la.store(smem, tid);
    lb.store(smem + BM * STRIDE, tid);
    __syncthreads();
    for (int kt = kt0; kt < kt1; ++kt) {
      const int cur = NBUF == 2 ? (kt - kt0) & 1 : 0, nxt = NBUF == 2 ? cur ^ 1 : 0;
      const bool more = kt + 1 < kt1;
      if (more) {
        la.load(a, tid);
        lb.load(a, tid);
      }
      mma_tile<T, FM, FN, STRIDE, KW>(smem + cur * TILE + koff, smem + cur * TILE + BM * STRIDE + koff, arow, brow, lane, acc);
      if (NBUF == 1) __syncthreads();  // everyone is done reading the only buffer
      if (more) {
        la.store(smem + nxt * TILE, tid);
        lb.store(smem + nxt * TILE + BM * STRIDE, tid);
      }
      __syncthreads();
    }
  }

  if constexpr (WK > 1) {
    // the k-loop ended with a barrier: the tile buffers are free.  Wavefronts wk = 1 .. WK-1 hand their
    // accumulators over, wavefront wk = 0 adds them in that order and alone runs the epilogue.
    float* red = reinterpret_cast<float*>(smem);
    if (wk > 0) {
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
          for (int v = 0; v < 16; ++v)
            red[((((wk - 1) * WM * WN + wmn) * FM * FN + i * FN + j) * 16 + v) * 64 + lane] = acc[i][j][v];
    }
    __syncthreads();
    if (wk > 0) return;
#pragma unroll
    for (int k = 0; k < WK - 1; ++k)
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
          for (int v = 0; v < 16; ++v)
            acc[i][j][v] += red[(((k * WM * WN + wmn) * FM * FN + i * FN + j) * 16 + v) * 64 + lane];
  }

  // epilogue.  A 32x32 accumulator block: lane holds column (lane & 31) and, in register v,
  // row 8*(v/4) + 4*(lane >> 5) + (v % 4).
  if constexpr (sizeof(T) == 2 && PASS != PASS_WGRAD && VECMODE) {
    // 16-bit outputs with channel counts that are multiples of 8: stage the fp32 tile in LDS (the k-loop's buffers are free now) so that each
    // lane then writes 8 adjacent outputs (16 bytes) and a wavefront writes whole rows of the tile
    constexpr int CS = BN + 4;  // row stride in floats: rows 4 banks apart, conflict-free column writes
    static_assert(BM * CS * 4 <= NBUF * TILE * (int)sizeof(T), "C tile must fit in the staging buffers");
    float* cs = reinterpret_cast<float*>(smem);
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j) {
        const int col = brow + j * 32 + (lane & 31);
        const float bias = (PASS == PASS_FWD && a.bias && n0 + col < a.Ng) ? a.bias[n0 + col] : 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = arow + i * 32 + 8 * (v / 4) + 4 * (lane >> 5) + (v % 4);
          float val = acc[i][j][v];
          if constexpr (PASS == PASS_FWD) val = act_apply(val + bias, a.act);
          cs[row * CS + col] = val;
        }
      }
    __syncthreads();
    T* out = static_cast<T*>(a.out);
    constexpr int CPR = BN / 8;  // 16-byte chunks per tile row
#pragma unroll
    for (int it = 0; it < BM * CPR / NT; ++it) {
      const int chunk = tid + it * NT;
      const int row = chunk / CPR, col = (chunk % CPR) * 8;
      if (m0 + row >= a.Mg || n0 + col >= a.Ng) continue;
      const float4 lo = *reinterpret_cast<const float4*>(&cs[row * CS + col]);
      const float4 hi = *reinterpret_cast<const float4*>(&cs[row * CS + col + 4]);
      float v8[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
      T* dst = out + (long long)(m0 + row) * a.Ng + n0 + col;
      if (PASS == PASS_DGRAD && a.accumulate) {
        const uint4 old = *reinterpret_cast<const uint4*>(dst);
#pragma unroll
        for (int e = 0; e < 8; ++e) v8[e] += bf16_to_f32((bf16_t)half_of(old, e));
      }
      uint4 o;
      o.x = (uint32_t)f32_to_bf16(v8[0]) | ((uint32_t)f32_to_bf16(v8[1]) << 16);
      o.y = (uint32_t)f32_to_bf16(v8[2]) | ((uint32_t)f32_to_bf16(v8[3]) << 16);
      o.z = (uint32_t)f32_to_bf16(v8[4]) | ((uint32_t)f32_to_bf16(v8[5]) << 16);
      o.w = (uint32_t)f32_to_bf16(v8[6]) | ((uint32_t)f32_to_bf16(v8[7]) << 16);
      *reinterpret_cast<uint4*>(dst) = o;
    }
    return;
  }
  if constexpr (PASS == PASS_FWD && sizeof(T) == 4) {
    // Optional by-product for a BatchNorm that follows (no bias, no activation here): per channel
    // (column) and run of 32 output rows, the sum of the outputs and the sum of their squared deviations
    // from the run's own mean.  Lanes l and l ^ 32 hold the two halves of a column of a 32x32 block.
    // The sums are taken of the deviations from a pivot, the run's first value (which lane l < 32 holds in
    // register 0): sum = s + n*pivot, squared deviations = q - s^2/n with s and q of the size of the
    // channel's spread, so a channel mean of many standard deviations costs no digits.
    if (a.stats) {
#pragma unroll
      for (int i = 0; i < FM; ++i) {
        const int rbase = m0 + arow + i * 32;
        const int cnt = min(max(a.Mg - rbase, 0), 32);
        const long long runs = (a.Mg + 31) / 32;  // the table is channel-major: [sum | squared deviations][column][run]
        float* part = a.stats + rbase / 32;
        const float inv_cnt = cnt > 0 ? 1.f / (float)cnt : 0.f;
#pragma unroll
        for (int j = 0; j < FN; ++j) {
          const float pivot = __shfl(acc[i][j][0], lane & 31, 64);
          float s2[2] = {0.f, 0.f}, q2[2] = {0.f, 0.f};
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int row = rbase + 8 * (v / 4) + 4 * (lane >> 5) + (v % 4);
            const float dev = row < a.Mg ? acc[i][j][v] - pivot : 0.f;
            s2[v & 1] += dev;
            q2[v & 1] = fmaf(dev, dev, q2[v & 1]);
          }
          float s1 = s2[0] + s2[1], q1 = q2[0] + q2[1];
          s1 += __shfl_xor(s1, 32, 64);
          q1 += __shfl_xor(q1, 32, 64);
          const float m2 = fmaxf(q1 - s1 * s1 * inv_cnt, 0.f);
          const int col = n0 + brow + j * 32 + (lane & 31);
          if (lane < 32 && col < a.Ng && cnt > 0) {  // a run with no valid row has no slot
            part[col * runs] = fmaf((float)cnt, pivot, s1);
            part[(a.Ng + col) * runs] = m2;
          }
        }
      }
    }
  }
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j) {
      const int col = n0 + brow + j * 32 + (lane & 31);
      if (col >= a.Ng) continue;
      const float bias = (PASS == PASS_FWD && a.bias) ? a.bias[col] : 0.f;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = m0 + arow + i * 32 + 8 * (v / 4) + 4 * (lane >> 5) + (v % 4);
        if (row >= a.Mg) continue;
        const long long o = (long long)row * a.Ng + col;
        float val = acc[i][j][v];
        if constexpr (PASS == PASS_FWD) {
          T* y = static_cast<T*>(a.out);
          y[o] = from_f32<T>(act_apply(val + bias, a.act));
        } else if constexpr (PASS == PASS_DGRAD) {
          T* dx = static_cast<T*>(a.out);
          if (a.accumulate) val += to_f32<T>(dx[o]);
          dx[o] = from_f32<T>(val);
        } else {
          float* dw = static_cast<float*>(a.out) + (long long)split * a.split_stride;
          dw[o] = val;
        }
      }
    }
}

// out[i] = sum over splits of part[z][i], in a fixed order: ZL lanes stride over the splits of one
// float4 of outputs (each with four running sums), then lane 0 adds the ZL lane totals.
template <int ZL>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float4* __restrict__ part, float4* __restrict__ out,
                                                            long long n4, int splits) {
  constexpr int OL = 256 / ZL;
  __shared__ float4 sh[ZL][OL];
  const int ol = threadIdx.x % OL, zl = threadIdx.x / OL;
  const long long i = (long long)blockIdx.x * OL + ol;
  float4 s[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) s[u] = make_float4(0.f, 0.f, 0.f, 0.f);
  if (i < n4) {
    int z = zl;
    for (; z + 3 * ZL < splits; z += 4 * ZL) {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const float4 v = part[(long long)(z + u * ZL) * n4 + i];
        s[u].x += v.x; s[u].y += v.y; s[u].z += v.z; s[u].w += v.w;
      }
    }
    for (; z < splits; z += ZL) {
      const float4 v = part[(long long)z * n4 + i];
      s[0].x += v.x; s[0].y += v.y; s[0].z += v.z; s[0].w += v.w;
    }
  }
  float4 t;
  t.x = (s[0].x + s[1].x) + (s[2].x + s[3].x);
  t.y = (s[0].y + s[1].y) + (s[2].y + s[3].y);
  t.z = (s[0].z + s[1].z) + (s[2].z + s[3].z);
  t.w = (s[0].w + s[1].w) + (s[2].w + s[3].w);
  if (ZL > 1) {
    sh[zl][ol] = t;
    __syncthreads();
    if (zl == 0) {
#pragma unroll
      for (int l = 1; l < ZL; ++l) {
        const float4 v = sh[l][ol];
        t.x += v.x; t.y += v.y; t.z += v.z; t.w += v.w;
      }
    }
  }
  if (zl == 0 && i < n4) out[i] = t;
}
// the same for output counts that are not multiples of 4
__global__ __launch_bounds__(256) void splitk_reduce_scalar_kernel(const float* __restrict__ part, float* __restrict__ out,
                                                                   long long n, int splits) {
  __shared__ float sh[16][17];
  const int ol = threadIdx.x & 15, zl = threadIdx.x >> 4;
  const long long i = (long long)blockIdx.x * 16 + ol;
  float s = 0.f;
  if (i < n)
    for (int z = zl; z < splits; z += 16) s += part[(long long)z * n + i];
  sh[zl][ol] = s;
  __syncthreads();
  if (zl == 0 && i < n) {
    float t = 0.f;
#pragma unroll
    for (int l = 0; l < 16; ++l) t += sh[l][ol];
    out[i] = t;
  }
}

template <typename T> bool vec_ok(const ConvGeom& g) {
  return g.C % Cfg<T>::VEC == 0 && g.K % Cfg<T>::VEC == 0;
}

// x / d for 0 <= x < 2^31 and d >= 1 as (mulhi(x, magic) + x) >> shift, with shift = ceil(log2 d) and
// magic = ceil(2^(32+shift) / d) - 2^32: the round-up error of the 33-bit multiplier is below d <= 2^shift,
// which makes the quotient exact for every 32-bit x; d == 1 gives magic 0, shift 0, and no special case.
void magic_div(int d, uint32_t& magic, int& shift) {
  if (d < 1) d = 1;
  int s = 0;
  while ((1LL << s) < d) ++s;
  const unsigned __int128 one = 1;
  const unsigned __int128 m = ((one << (32 + s)) + (unsigned)d - 1) / (unsigned)d;
  magic = (uint32_t)(m - (one << 32));
  shift = s;
}

void fill_sizes(Args& a, int pass, int dtype) {
  const ConvGeom& g = a.g;
  const unsigned long long es = dtype_size(dtype);
  const unsigned long long xs = (unsigned long long)g.N * g.H * g.W * g.C * es, ys = (unsigned long long)g.N * g.P * g.Q * g.K * es,
                           ws = (unsigned long long)g.R * g.S * g.C * g.K * es;
  auto clamp = [](unsigned long long v) { return (uint32_t)(v > 0xffffffffULL ? 0xffffffffULL : v); };
  a.a_bytes = clamp(pass == PASS_DGRAD ? ys : xs);
  a.b_bytes = clamp(pass == PASS_WGRAD ? ys : ws);
  magic_div(g.Q, a.magicQ, a.shiftQ);
  magic_div(g.P, a.magicP, a.shiftP);
  magic_div(g.W, a.magicW, a.shiftW);
  magic_div(g.H, a.magicH, a.shiftH);
  magic_div(g.C, a.magicC, a.shiftC);
  magic_div(g.K, a.magicK, a.shiftK);
  magic_div(g.S, a.magicS, a.shiftS);
}

void fill_tiles(Args& a, int BM, int BN, int BK) {
  a.tiles_m = (a.Mg + BM - 1) / BM;
  a.tiles_n = (a.Ng + BN - 1) / BN;
  a.nk = (a.Kg + BK - 1) / BK;
  a.nk_per_split = a.nk;
  a.split_stride = 0;
}

// Tile of the generic fp32 kernel for a GEMM with Mg rows and Ng columns.  The MFMA work of a tile does
// not shrink with the part of it that lies inside the matrix, so a side that fills a small part of
// 128 takes a narrower tile; a narrower tile reads more LDS per MFMA, hence the weights.
void f32_tile(int Mg, int Ng, long long Kg, bool splits_k, int& BM, int& BN) {
  const int bn[3] = {128, 64, 32};
  const float wn[3] = {1.f, 1.15f, 1.4f};
  float best = 0.f;
  BN = 128;
  for (int i = 0; i < 3; ++i) {
    const float cost = (float)((Ng + bn[i] - 1) / bn[i] * bn[i]) * wn[i];
    if (i == 0 || cost < best) { best = cost; BN = bn[i]; }
  }
  BM = 128;
  if (BN >= 64) {
    const float c128 = (float)((Mg + 127) / 128 * 128), c64 = (float)((Mg + 63) / 64 * 64) * 1.15f;
    if (c64 < c128) BM = 64;
  }
  if (splits_k) {  // the filter gradient gets its workgroups from splitting the reduction axis
    if (Mg <= 32) BM = 32;  // few input channels (the first layers of a net): a 32-row tile halves the padding again
    return;
  }
  if ((long long)Mg * Ng * Kg < (1LL << 20)) return;  // too little work for the tile shape to matter
  // fewer tiles than CUs: smaller tiles, down to 32x32 (whose four wavefronts split the k-tile's depth)
  const int bm2[3] = {64, 64, 32}, bn2[3] = {64, 32, 32};
  for (int i = 0; i < 3; ++i) {
    if ((long long)((Mg + BM - 1) / BM) * ((Ng + BN - 1) / BN) >= 256) break;
    if (bm2[i] <= BM && bn2[i] <= BN) { BM = bm2[i]; BN = bn2[i]; }
  }
}

// k-tile depth of the fp32 kernel: 32 for every tile shape whose two double-buffered operand tiles fit into
// 64 KB of LDS with it (all but 128x128), which halves the number of load-wait-multiply rounds of a
// workgroup; 128x128 keeps 16
int f32_bk(int BM, int BN) { return (BM == 128 && BN == 128) ? 16 : ((BN == 32 && BM <= 64) || (BM == 32 && BN == 64)) ? 64 : 32; }

template <typename T, int PASS, int WM, int WN, int FM, int FN, int BK, int WK = 1, int NBUF = 2>
void launch_shape(const Args& a, dim3 grid, hipStream_t st) {
  // Both operands of dgrad are contiguous along the output channels (dy rows, filter rows), and the fp32
  // epilogue stores element by element: there the 16-byte loaders only need K to be a multiple of 4, whatever
  // C is (LeNet's second convolution, 6 -> 16 channels: 66 -> 15 us).
  const bool vec = (sizeof(T) == 4 && PASS == PASS_DGRAD) ? a.g.K % Cfg<T>::VEC == 0 : vec_ok<T>(a.g);
  if (vec)
    hipLaunchKernelGGL((igemm_kernel<T, PASS, true, WM, WN, FM, FN, BK, WK, NBUF>), grid, dim3(NT), 0, st, a);
  else
    hipLaunchKernelGGL((igemm_kernel<T, PASS, false, WM, WN, FM, FN, BK, WK, NBUF>), grid, dim3(NT), 0, st, a);
}

// a.tiles_m / a.tiles_n / a.nk must come from fill_tiles with the tile this picks: 128x128 for bf16,
// f32_tile's (and f32_bk's depth) for fp32
template <typename T, int PASS> int launch(Args& a, int splits, hipStream_t st) {
  if (sizeof(T) == 2 && igemm_dma_ok(PASS, a.g, a)) return igemm_dma_launch(PASS, a, splits, st);
  a.splits = splits;
  dim3 grid(grid_blocks(a));
  if constexpr (sizeof(T) == 4) {
    int BM, BN;
    f32_tile(a.Mg, a.Ng, a.Kg, PASS == PASS_WGRAD, BM, BN);
    if (BM == 128 && BN == 128) launch_shape<T, PASS, 2, 2, 2, 2, 16>(a, grid, st);
    else if (BM == 64 && BN == 32) launch_shape<T, PASS, 2, 1, 1, 1, 64, 2>(a, grid, st);
    else if (BM == 32 && BN == 32) launch_shape<T, PASS, 1, 1, 1, 1, 64, 4>(a, grid, st);
    else if (BM == 32 && BN == 64) launch_shape<T, PASS, 1, 2, 1, 1, 64, 2>(a, grid, st);
    else if (BM == 32 && BN == 128) launch_shape<T, PASS, 1, 4, 1, 1, 32>(a, grid, st);
    else if (BM == 128 && BN == 64) launch_shape<T, PASS, 2, 2, 2, 1, 32>(a, grid, st);
    else if (BM == 128 && BN == 32) launch_shape<T, PASS, 4, 1, 1, 1, 32, 1, 1>(a, grid, st);
    else if (BM == 64 && BN == 128) launch_shape<T, PASS, 2, 2, 1, 2, 32>(a, grid, st);
    else launch_shape<T, PASS, 2, 2, 1, 1, 32>(a, grid, st);
  } else {
    launch_shape<T, PASS, 2, 2, 2, 2, Cfg<bf16_t>::BK>(a, grid, st);
  }
  return launch_status("igemm");
}

void fill_tiles_f32(Args& a, bool splits_k) {
  int BM, BN;
  f32_tile(a.Mg, a.Ng, a.Kg, splits_k, BM, BN);
  fill_tiles(a, BM, BN, f32_bk(BM, BN));
}

// Split of the wgrad reduction axis (output pixels) over workgroups.  The fast bf16 kernel keeps two
// workgroups per CU resident, but each extra split costs a tile of fp32 partials written and read
// again, and these kernels run beside the main stream's: about 320 workgroups of 64x128 measured best
// over a ResNet-50 step (288: +0.5 %, 384: +0.3 %, 512: +0.9 %, 768: +3 %).
void wgrad_split(const ConvGeom& g, int dtype, int& splits, int& nk_per_split) {
  const int Mg = g.R * g.S * g.C;
  const long long Kg = (long long)g.N * g.P * g.Q;
  int BK = Cfg<bf16_t>::BK;
  if (dtype != S4TF_BF16) {
    int BM, BN;
    f32_tile(Mg, g.K, Kg, true, BM, BN);
    BK = f32_bk(BM, BN);
  }
  const long long nk = (Kg + BK - 1) / BK;
  long long want;
  if (dtype == S4TF_BF16 && igemm_dma_geom_ok(PASS_WGRAD, g)) {
    int BM, BN;
    igemm_dma_tile(PASS_WGRAD, Mg, g.K, 1, BM, BN);
    const long long tiles = (long long)((Mg + BM - 1) / BM) * ((g.K + BN - 1) / BN);
    // (at most four tiles: the first layers, whose filter gradients are the tail of a step with nothing
    // left beside them; there more workgroups are simply faster)
    want = (tiles <= 4 ? 512 : 320) / tiles;
  } else {
    int BM = 128, BN = 128;
    if (dtype != S4TF_BF16) f32_tile(Mg, g.K, Kg, true, BM, BN);
    const long long tiles = (long long)((Mg + BM - 1) / BM) * ((g.K + BN - 1) / BN);
    want = (512 + tiles - 1) / tiles;  // measured inside the fp32 training steps: 1024 +1.8 %, 768 +0.8 %, 416 +2 %
  }
  if (want > nk) want = nk;
  if (want < 1) want = 1;
  nk_per_split = (int)((nk + want - 1) / want);
  splits = (int)((nk + nk_per_split - 1) / nk_per_split);
}

}  // namespace

int igemm_fwd(const ConvGeom& g, int dtype, const void* x, const void* w, const float* bias, int act,
              void* y, hipStream_t st, float* stats_part, int* stats_rows) {
  Args a = {};
  a.g = g; a.a = x; a.b = w; a.out = y; a.bias = bias; a.act = act;
  a.Mg = g.N * g.P * g.Q; a.Ng = g.K; a.Kg = g.R * g.S * g.C;
  a.simple = (g.R == 1 && g.S == 1 && g.stride == 1 && g.pad == 0);
  fill_sizes(a, PASS_FWD, dtype);
  if (stats_rows) *stats_rows = 0;
  ProfScope ps(PC_CONV_FWD, st);
  if (dtype == S4TF_BF16) {
    fill_tiles(a, 128, 128, Cfg<bf16_t>::BK);
    if (stats_part && stats_rows && !bias && act == S4TF_ACT_NONE && igemm_dma_ok(PASS_FWD, g, a)) {
      a.stats = stats_part;
      const int rc = igemm_dma_launch(PASS_FWD, a, 1, st);
      *stats_rows = a.stats_rows;
      return rc;
    }
    return launch<bf16_t, PASS_FWD>(a, 1, st);
  }
  const bool with_stats = stats_part && stats_rows && !bias && act == S4TF_ACT_NONE;
  if (patchconv_fwd_ok(g, dtype) && aligned16(x) && aligned16(w) && aligned16(y))  // few channels, 3x3: out of an LDS patch
    return patchconv_fwd(g, x, w, bias, act, y, with_stats ? stats_part : nullptr, with_stats ? stats_rows : nullptr, st);
  if (with_stats) *stats_rows = 32;
  fill_tiles_f32(a, false);
  if (with_stats) a.stats = stats_part;
  return launch<float, PASS_FWD>(a, 1, st);
}

size_t igemm_fwd_stats_bytes(const ConvGeom& g) {  // the finest runs any kernel uses are 32 rows
  const size_t M = (size_t)g.N * g.P * g.Q;
  return (M + 31) / 32 * 2 * g.K * sizeof(float);
}

// Can igemm_dgrad add a (masked) tensor other than the old contents of dx?  Only the stride-1 case of the
// fast bf16 kernel does.
bool igemm_dgrad_adds_other(const ConvGeom& g, int dtype, const void* dy, const void* w, const void* dx,
                            const void* acc_src) {
  if (dtype != S4TF_BF16 || g.stride != 1 || !aligned16(acc_src) || g.C % 8) return false;
  Args a = {};
  a.g = g; a.a = dy; a.b = w; a.out = const_cast<void*>(dx);
  return igemm_dma_ok(PASS_DGRAD, g, a);
}

bool igemm_dgrad_can_add_other(const ConvGeom& g, int dtype) {
  return dtype == S4TF_BF16 && g.stride == 1 && g.C % 8 == 0 && igemm_dma_geom_ok(PASS_DGRAD, g);
}

int igemm_dgrad(const ConvGeom& g, int dtype, const void* dy, const void* w, void* dx, int accumulate,
                hipStream_t st, const void* acc_src, const unsigned char* acc_bits) {
  Args a = {};
  a.g = g; a.a = dy; a.b = w; a.out = dx; a.accumulate = accumulate;
  if (acc_src) {
    if (!igemm_dgrad_adds_other(g, dtype, dy, w, dx, acc_src))
      return fail(S4TF_ERR_UNSUPPORTED, "dgrad: this shape cannot add another tensor");
    a.accumulate = 1;
    a.acc_src = acc_src;
    a.acc_bits = acc_bits;
  }
  a.Mg = g.N * g.H * g.W; a.Ng = g.C; a.Kg = g.R * g.S * g.K;
  a.simple = (g.R == 1 && g.S == 1 && g.stride == 1 && g.pad == 0);
  fill_sizes(a, PASS_DGRAD, dtype);
  ProfScope ps(PC_CONV_DGRAD, st);
  if (dtype == S4TF_BF16 && g.R == 1 && g.S == 1 && g.pad == 0 && g.stride == 2 && igemm_dma_ok(PASS_DGRAD, g, a)) {
    // only pixels (2p, 2q) of dx receive anything: a plain GEMM over the pixels of dy whose rows the
    // epilogue scatters (and, unless it accumulates, surrounds with zeros)
    a.Mg = g.N * g.P * g.Q;
    a.simple = 1;
    a.scatter2 = 1;
    fill_tiles(a, 128, 128, Cfg<bf16_t>::BK);
    return igemm_dma_launch(PASS_DGRAD, a, 1, st);
  }
  if (dtype == S4TF_BF16 && g.stride == 2 && g.R >= 2 && g.S >= 2 && g.K % 64 == 0 && g.H >= 2 && g.W >= 2 &&
      igemm_dma_ok(PASS_DGRAD, g, a)) {
    // An input pixel meets only the taps whose parity matches its own: r = (h + pad) mod 2 (+2, +4, ...),
    // s likewise.  One GEMM per parity class over its pixels and its taps does a quarter of the work of
    // one GEMM over all pixels and all taps, three quarters of which would multiply zeros.
    a.cls = 1;
    int nk_max = 0;
    for (int p = 0; p < 2; ++p) {
      a.cls_r0[p] = a.cls_s0[p] = (p + g.pad) % 2;
      a.cls_Hc[p] = (g.H - p + 1) / 2;
      a.cls_Wc[p] = (g.W - p + 1) / 2;
      magic_div(a.cls_Hc[p], a.cls_magicHc[p], a.cls_shiftHc[p]);
      magic_div(a.cls_Wc[p], a.cls_magicWc[p], a.cls_shiftWc[p]);
    }
    for (int c = 0; c < 4; ++c) {  // slot c: class 3 - c, so that the class with the most taps is dispatched first
      const int ph = (3 - c) >> 1, pw = (3 - c) & 1;
      const int nr = (g.R - a.cls_r0[ph] + 1) / 2, ns = (g.S - a.cls_s0[pw] + 1) / 2;
      a.cls_Mg[c] = g.N * a.cls_Hc[ph] * a.cls_Wc[pw];
      a.cls_nk[c] = nr * ns * g.K / Cfg<bf16_t>::BK;
      if (a.cls_nk[c] > nk_max) nk_max = a.cls_nk[c];
    }
    fill_tiles(a, 128, 128, Cfg<bf16_t>::BK);
    a.nk = a.nk_per_split = nk_max;  // picks the kernel variant; every workgroup takes its class's count
    return igemm_dma_launch(PASS_DGRAD, a, 1, st);
  }
  if (dtype == S4TF_BF16) {
    fill_tiles(a, 128, 128, Cfg<bf16_t>::BK);
    return launch<bf16_t, PASS_DGRAD>(a, 1, st);
  }
  if (patchconv_dgrad_ok(g, dtype) && aligned16(dy) && aligned16(w) && aligned16(dx))
    return patchconv_dgrad(g, dy, w, dx, accumulate, st);
  fill_tiles_f32(a, false);
  return launch<float, PASS_DGRAD>(a, 1, st);
}

size_t igemm_wgrad_workspace(const ConvGeom& g, int dtype) {
  int splits, per;
  if (patchconv_wgrad_ok(g, dtype)) splits = patchconv_wgrad_splits(g);
  else wgrad_split(g, dtype, splits, per);
  if (splits <= 1) return 0;
  return (size_t)splits * g.R * g.S * g.C * g.K * sizeof(float);
}

int igemm_wgrad(const ConvGeom& g, int dtype, const void* x, const void* dy, float* dw, void* ws,
                size_t ws_bytes, hipStream_t st) {
  Args a = {};
  a.g = g; a.a = x; a.b = dy;
  a.Mg = g.R * g.S * g.C; a.Ng = g.K; a.Kg = g.N * g.P * g.Q;
  a.simple = (g.R == 1 && g.S == 1 && g.stride == 1 && g.pad == 0);
  fill_sizes(a, PASS_WGRAD, dtype);
  // few channels, 3x3, small images: out of an LDS patch
  const bool patch = patchconv_wgrad_ok(g, dtype) && aligned16(x) && aligned16(dy) && aligned16(dw) && aligned16(ws);
  int splits, per = 0;
  if (patch) splits = patchconv_wgrad_splits(g);
  else wgrad_split(g, dtype, splits, per);
  const long long n = (long long)a.Mg * a.Ng;
  if (splits > 1 && ws_bytes < (size_t)splits * n * sizeof(float))
    return fail(S4TF_ERR_WORKSPACE, "wgrad needs %zu workspace bytes, got %zu", (size_t)splits * n * sizeof(float), ws_bytes);
  int rc;
  if (patch) {
    ProfScope ps(PC_CONV_WGRAD, st);
    rc = patchconv_wgrad(g, x, dy, splits > 1 ? static_cast<float*>(ws) : dw, splits, st);
  } else {
    if (dtype == S4TF_BF16) fill_tiles(a, 128, 128, Cfg<bf16_t>::BK);
    else fill_tiles_f32(a, true);
    a.nk_per_split = per;
    a.split_stride = n;
    a.out = splits > 1 ? ws : (void*)dw;
    ProfScope ps(PC_CONV_WGRAD, st);
    rc = dtype == S4TF_BF16 ? launch<bf16_t, PASS_WGRAD>(a, splits, st) : launch<float, PASS_WGRAD>(a, splits, st);
  }
  if (rc != S4TF_OK || splits == 1) return rc;
  ProfScope ps(PC_WGRAD_REDUCE, st);
  if (n % 4 == 0 && aligned16(ws) && aligned16(dw)) {
    const long long n4 = n / 4;
    const float4* part = static_cast<const float4*>(ws);
    float4* out = reinterpret_cast<float4*>(dw);
    if (splits >= 32)
      hipLaunchKernelGGL(splitk_reduce_kernel<16>, dim3((unsigned)((n4 + 15) / 16)), dim3(256), 0, st, part, out, n4, splits);
    else if (splits >= 8)
      hipLaunchKernelGGL(splitk_reduce_kernel<4>, dim3((unsigned)((n4 + 63) / 64)), dim3(256), 0, st, part, out, n4, splits);
    else
      hipLaunchKernelGGL(splitk_reduce_kernel<1>, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, st, part, out, n4, splits);
  } else {
    hipLaunchKernelGGL(splitk_reduce_scalar_kernel, dim3((unsigned)((n + 15) / 16)), dim3(256), 0, st,
                       static_cast<const float*>(ws), dw, n, splits);
  }
  return launch_status("splitk_reduce");
}

}  // namespace s4tf
