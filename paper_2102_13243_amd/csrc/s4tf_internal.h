// Internal declarations shared by the HIP translation units of libs4tf.
// Not part of the ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/s4tf.h"

namespace s4tf {

typedef uint16_t bf16_t;  // raw bfloat16 bits

// ---- error reporting --------------------------------------------------------------------
int fail(int status, const char* fmt, ...);
void clear_error();

// ---- bf16 <-> fp32 ----------------------------------------------------------------------
__host__ __device__ inline float bf16_to_f32(bf16_t v) {
  union { uint32_t u; float f; } x;
  x.u = (uint32_t)v << 16;
  return x.f;
}
// round to nearest, ties to even; NaN stays NaN.  Device code takes the hardware conversion of gfx950
// (v_cvt_pk_bf16_f32, two values per instruction when the compiler can pair them).
__host__ __device__ inline bf16_t f32_to_bf16(float f) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __builtin_bit_cast(bf16_t, (__bf16)f);
#else
  union { uint32_t u; float f; } x;
  x.f = f;
  if ((x.u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((x.u >> 16) | 0x40u);
  x.u += 0x7fffu + ((x.u >> 16) & 1u);
  return (bf16_t)(x.u >> 16);
#endif
}
template <typename T> __device__ inline float to_f32(T v);
template <> __device__ inline float to_f32<float>(float v) { return v; }
template <> __device__ inline float to_f32<bf16_t>(bf16_t v) { return bf16_to_f32(v); }
template <typename T> __device__ inline T from_f32(float v);
template <> __device__ inline float from_f32<float>(float v) { return v; }
template <> __device__ inline bf16_t from_f32<bf16_t>(float v) { return f32_to_bf16(v); }

__device__ inline float act_apply(float z, int act) {
  if (act == S4TF_ACT_RELU) return z > 0.f ? z : 0.f;
  if (act == S4TF_ACT_RELU6) return z < 0.f ? 0.f : (z > 6.f ? 6.f : z);
  return z;
}
__device__ inline float act_mask(float y, int act) {
  if (act == S4TF_ACT_RELU) return y > 0.f ? 1.f : 0.f;
  if (act == S4TF_ACT_RELU6) return (y > 0.f && y < 6.f) ? 1.f : 0.f;
  return 1.f;
}

// ---- per-kernel-class timing hook ---------------------------------------------------------
enum ProfClass {
  PC_CONV_FWD = 0, PC_CONV_DGRAD, PC_CONV_WGRAD, PC_WGRAD_REDUCE, PC_DWCONV_FWD, PC_DWCONV_DGRAD,
  PC_DWCONV_WGRAD, PC_BN_STATS, PC_BN_APPLY, PC_BN_VJP_REDUCE, PC_BN_VJP_APPLY, PC_POOL, PC_HEAD,
  PC_SGD, PC_ELEMENTWISE, PC_OTHER
};
struct ProfScope {
  ProfScope(int cls, hipStream_t s);
  ~ProfScope();
  int cls;
  hipStream_t stream;
  void* rec;
};

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline size_t dtype_size(int dtype) { return dtype == S4TF_BF16 ? 2 : 4; }
inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

// ---- internal launchers (arguments already validated) ---------------------------------------
struct ConvGeom {
  int N, H, W, C, K, R, S, stride, pad, P, Q;
};
inline ConvGeom conv_geom(const s4tf_conv_desc& d) {
  ConvGeom g;
  g.N = d.n; g.H = d.h; g.W = d.w; g.C = d.c; g.K = d.k; g.R = d.r; g.S = d.s;
  g.stride = d.stride; g.pad = d.pad;
  g.P = (d.h + 2 * d.pad - d.r) / d.stride + 1;
  g.Q = (d.w + 2 * d.pad - d.s) / d.stride + 1;
  return g;
}

// dense (groups == 1) convolution as implicit GEMM on MFMA
// stats_part (optional, with bias == NULL and act == none): the kernel also writes, for every run of
// *stats_rows consecutive output rows (pixels) r and every channel, the sum of the stored outputs and the
// sum of their squared deviations from that run's own mean, channel-major: stats_part[k*runs + r] and
// stats_part[(K + k)*runs + r] with runs = ceil(N*P*Q / *stats_rows).  *stats_rows comes back 0 when the kernel that ran does not do this.
int igemm_fwd(const ConvGeom& g, int dtype, const void* x, const void* w, const float* bias, int act,
              void* y, hipStream_t st, float* stats_part = nullptr, int* stats_rows = nullptr);
size_t igemm_fwd_stats_bytes(const ConvGeom& g);  // upper bound on the size of stats_part
// fp32 3x3 / stride 1 / padding 1 layers of 16 or 32 channels (and 4 -> 16) whose images are 16 or 32 wide: a
// kernel that multiplies out of an LDS patch (patchconv.hip); igemm_fwd and igemm_dgrad hand such shapes over
bool patchconv_fwd_ok(const ConvGeom& g, int dtype);
bool patchconv_dgrad_ok(const ConvGeom& g, int dtype);
int patchconv_fwd(const ConvGeom& g, const void* x, const void* w, const float* bias, int act, void* y, float* stats,
                  int* stats_rows, hipStream_t st);
int patchconv_dgrad(const ConvGeom& g, const void* dy, const void* w, void* dx, int accumulate, hipStream_t st);
bool patchconv_wgrad_ok(const ConvGeom& g, int dtype);
int patchconv_wgrad_splits(const ConvGeom& g);  // partial filter gradients the kernel leaves for the reduction
int patchconv_wgrad(const ConvGeom& g, const void* x, const void* dy, float* out, int splits, hipStream_t st);
// acc_src (optional; only where igemm_dgrad_adds_other says so): the result is dgrad + acc_src instead of
// dgrad (+ old dx); acc_bits (optional): activation bits as bn_fwd leaves them, one per element of acc_src,
// elements whose bit is clear add nothing.
int igemm_dgrad(const ConvGeom& g, int dtype, const void* dy, const void* w, void* dx, int accumulate,
                hipStream_t st, const void* acc_src = nullptr, const unsigned char* acc_bits = nullptr);
bool igemm_dgrad_adds_other(const ConvGeom& g, int dtype, const void* dy, const void* w, const void* dx,
                            const void* acc_src);
bool igemm_dgrad_can_add_other(const ConvGeom& g, int dtype);  // the same question for 16-byte aligned operands
size_t igemm_wgrad_workspace(const ConvGeom& g, int dtype);
int igemm_wgrad(const ConvGeom& g, int dtype, const void* x, const void* dy, float* dw, void* ws,
                size_t ws_bytes, hipStream_t st);

// depthwise (groups == C == K)
int dwconv_fwd(const ConvGeom& g, int dtype, const void* x, const void* w, const float* bias, int act,
               void* y, hipStream_t st);
int dwconv_dgrad(const ConvGeom& g, int dtype, const void* dy, const void* w, void* dx, int accumulate,
                 hipStream_t st);
size_t dwconv_wgrad_workspace(const ConvGeom& g);
int dwconv_wgrad(const ConvGeom& g, int dtype, const void* x, const void* dy, float* dw, void* ws,
                 hipStream_t st);

// elementwise / reductions
int act_vjp(int dtype, int act, const void* y, const void* dy, void* dz, size_t count, hipStream_t st);
// ws (optional, colsum_workspace(rows, cols) bytes): lets a tall matrix be summed by many blocks in two stages
size_t colsum_workspace(size_t rows, int cols);
int colsum(int dtype, const void* a, size_t rows, int cols, float* out, hipStream_t st, void* ws = nullptr,
           size_t ws_bytes = 0);

// zero-pad / strip the channel axis of [outer][C][inner] tensors
int pad_channels(int dtype, const void* src, void* dst, long long outer, int C, int Cp, int inner, hipStream_t st);
int unpad_channels_f32(const float* src, float* dst, long long outer, int C, int Cp, int inner, hipStream_t st);
// bf16 stride-2 first layer as a stride-1 layer over 2x2 pixel blocks (see pool.hip): the folded batch
// (N, (H+2pad)/2, (W+2pad)/2, 16), the folded filter ((R+1)/2, (S+1)/2, 16, K), and the filter gradient back
int fold2_pixels(const void* x, void* xf, int N, int H, int W, int C, int pad, hipStream_t st);
int fold2_filter(const void* w, void* wf, int R, int S, int C, int K, hipStream_t st);
int unfold2_filter_grad(const float* dwf, float* dw, int R, int S, int C, int K, hipStream_t st);

// batch norm
size_t bn_workspace(size_t M, int C);
size_t bn_mask_bytes(size_t M, int C, int dtype);
// stats_part / stats_rows: per-channel partial sums that the producing convolution left (see igemm_fwd);
// NULL / 0: the statistics are computed here from x.
// maskbits (optional, bn_mask_bytes bytes): the forward pass leaves act'(y) there, one bit per output, and a
// pullback that is given them reads these instead of y (a BatchNorm with a residual cannot rebuild its
// activation mask from x; the bits are a sixteenth of y in bf16).
int bn_fwd(const s4tf_bn_desc& d, const void* x, const void* res, const float* gamma, const float* beta,
           void* y, float* mean, float* invstd, void* ws, hipStream_t st, const float* stats_part = nullptr,
           int stats_rows = 0, unsigned char* maskbits = nullptr);
// inference mode: running statistics instead of batch statistics; their update from a training-mode forward
// pass; folding of an inference-mode BatchNorm into the convolution in front of it
int bn_inference_fwd(const s4tf_bn_desc& d, const void* x, const void* res, const float* gamma, const float* beta,
                     const float* running_mean, const float* running_var, void* y, hipStream_t st);
int bn_update_running(int C, size_t count, float momentum, float eps, const float* mean, const float* invstd,
                      float* rm, float* rv, hipStream_t st);
int bn_fold(int dtype, long long rows, int K, const void* w, const float* bias, const float* gamma, const float* beta,
            const float* rm, const float* rv, float eps, void* w_out, float* bias_out, hipStream_t st);
// bn_fwd with its partial sums in a static device array instead of a workspace: allocates nothing; shapes
// whose partial sums (bn_fwd_scratch_bytes) exceed bn_static_scratch_capacity() are refused
size_t bn_fwd_scratch_bytes(const s4tf_bn_desc& d);
size_t bn_static_scratch_capacity();
int bn_fwd_static(const s4tf_bn_desc& d, const void* x, const void* res, const float* gamma, const float* beta,
                  void* y, float* mean, float* invstd, hipStream_t st);
int bn_vjp(const s4tf_bn_desc& d, const void* x, const void* y, const float* gamma, const float* beta, const float* mean,
           const float* invstd, const void* dy, void* dx, void* dres, float* dgamma, float* dbeta,
           void* ws, hipStream_t st, const unsigned char* maskbits = nullptr);

// pools
// idx (optional, max pool with a channel count that the 16-byte kernels take: pool_saves_positions): one byte per
// output element, written by pool_fwd, the window position of the maximum; pool_vjp given it does not read x
bool pool_saves_positions(const s4tf_pool_desc& d);
int pool_fwd(const s4tf_pool_desc& d, const void* x, void* y, hipStream_t st, unsigned char* idx = nullptr);
int pool_vjp(const s4tf_pool_desc& d, const void* x, const void* dy, void* dx, hipStream_t st, const unsigned char* idx = nullptr);

// head
size_t head_workspace(const s4tf_head_desc& d);
int head_fwd_vjp(const s4tf_head_desc& d, const void* x, const float* W, const float* b,
                 const int32_t* labels, float* loss, void* dx, float* dW, float* db, float* logits,
                 void* ws, hipStream_t st);

// indexing: y[j,:] = x[index[j],:] and its in-place pullback dx[index[j],:] += dy[j,:] (in order of j)
int gather_rows_fwd(const s4tf_gather_desc& d, const void* x, const int32_t* index, void* y, hipStream_t st);
int gather_rows_vjp(const s4tf_gather_desc& d, const void* dy, const int32_t* index, void* dx, hipStream_t st);

// storage-type conversion: dst[i] = bf16(src[i]), round to nearest even
int round_to_bf16(size_t count, const float* src, void* dst, hipStream_t st);

// optimizer
int sgd(size_t count, float* param, float* vel, const float* grad, void* lowp, float lr, float mu,
        hipStream_t st);

// validation shared by the per-op entry points and the whole step
int check_conv_desc(const s4tf_conv_desc* d);
int check_bn_desc(const s4tf_bn_desc* d);
int check_pool_desc(const s4tf_pool_desc* d);
int check_head_desc(const s4tf_head_desc* d);

// argument checks shared by the entry points (api.hip) and the whole-step scheduler (step.hip)
int need(const void* p, const char* name);   // not NULL and 16-byte aligned
int opt(const void* p, const char* name);    // NULL or 16-byte aligned
int check_ws(const void* ws, size_t have, size_t want);
#define CHECK(expr)                 \
  do {                              \
    int rc_ = (expr);               \
    if (rc_ != S4TF_OK) return rc_; \
  } while (0)

// a convolution's three passes, dense or depthwise by the descriptor's groups (api.hip)
int conv_fwd_impl(const s4tf_conv_desc& d, const void* x, const void* w, const float* bias, void* y, hipStream_t st,
                  float* stats_part = nullptr, int* stats_rows = nullptr);
int conv_dgrad_impl(const s4tf_conv_desc& d, const void* w, const void* dz, void* dx, hipStream_t st,
                    const void* acc_src = nullptr, const unsigned char* acc_bits = nullptr);
int conv_param_grads_impl(const s4tf_conv_desc& d, const void* x, const void* dz, float* dw, float* dbias,
                          void* wg_ws, size_t wg_bytes, hipStream_t st);

inline int launch_status(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(S4TF_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
  return S4TF_OK;
}

}  // namespace s4tf
