// The C ABI: argument validation, per-op entry points, and the whole-step scheduler that
// runs forward, pullbacks in reverse op order and the optimizer update on one stream
// (the paper's Section 4.2 training loop; a step is `(inout Model, Minibatch) -> Void`).
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <mutex>
#include <vector>

#include "s4tf_internal.h"

namespace s4tf {

// ---- thread-local error text ----------------------------------------------------------------------
static thread_local char g_err[512] = "";

int fail(int status, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return status;
}
void clear_error() { g_err[0] = 0; }

// ---- per-class kernel timing -----------------------------------------------------------------------
struct ProfRec {
  int cls;
  hipEvent_t e0, e1;
};
static thread_local bool g_prof_on = false;
static thread_local std::vector<ProfRec>* g_prof = nullptr;

ProfScope::ProfScope(int c, hipStream_t s) : cls(c), stream(s), rec(nullptr) {
  if (!g_prof_on) return;
  if (!g_prof) g_prof = new std::vector<ProfRec>();
  ProfRec r;
  r.cls = c;
  if (hipEventCreate(&r.e0) != hipSuccess) return;
  if (hipEventCreate(&r.e1) != hipSuccess) { (void)hipEventDestroy(r.e0); return; }
  (void)hipEventRecord(r.e0, s);
  g_prof->push_back(r);
  rec = reinterpret_cast<void*>(g_prof->size());  // index + 1 of this scope's record
}
ProfScope::~ProfScope() {
  if (rec && g_prof) (void)hipEventRecord((*g_prof)[reinterpret_cast<size_t>(rec) - 1].e1, stream);
}

static const char* kProfNames[S4TF_PROF_CLASSES] = {
    "conv_fwd_igemm", "conv_dgrad_igemm", "conv_wgrad_igemm", "wgrad_splitk_reduce", "dwconv_fwd",
    "dwconv_dgrad", "dwconv_wgrad", "bn_stats", "bn_apply", "bn_vjp_reduce", "bn_vjp_apply", "pool",
    "head", "sgd", "elementwise", "other"};

// ---- validation ---------------------------------------------------------------------------------------
static bool dtype_ok(int t) { return t == S4TF_F32 || t == S4TF_BF16; }
static bool act_ok(int a) { return a == S4TF_ACT_NONE || a == S4TF_ACT_RELU || a == S4TF_ACT_RELU6; }
static const long long kMaxElems = (1LL << 31) - 1;  // per-tensor element limit of the kernels' int math

int check_conv_desc(const s4tf_conv_desc* d) {
  if (!d) return fail(S4TF_ERR_NULL, "conv descriptor is NULL");
  if (!dtype_ok(d->dtype) || !act_ok(d->act)) return fail(S4TF_ERR_DTYPE, "conv: bad dtype %d or act %d", d->dtype, d->act);
  if (d->n <= 0 || d->h <= 0 || d->w <= 0 || d->c <= 0 || d->k <= 0 || d->r <= 0 || d->s <= 0 || d->stride <= 0 ||
      d->pad < 0 || d->groups <= 0)
    return fail(S4TF_ERR_SHAPE, "conv: sizes must be positive (pad >= 0)");
  if (d->h + 2 * d->pad < d->r || d->w + 2 * d->pad < d->s) return fail(S4TF_ERR_SHAPE, "conv: filter larger than padded input");
  if (d->c % d->groups || d->k % d->groups) return fail(S4TF_ERR_SHAPE, "conv: c and k must be multiples of groups");
  if (d->groups != 1 && !(d->groups == d->c && d->k == d->c))
    return fail(S4TF_ERR_UNSUPPORTED, "conv: groups must be 1 or c with k == c (depthwise)");
  // (the depthwise filter gradient keeps one sum per tap in registers; refused here, for every pass, so that a
  // pullback or a training step cannot fail after its first kernels have run)
  if (d->groups != 1 && (d->r > 3 || d->s > 3))
    return fail(S4TF_ERR_UNSUPPORTED, "conv: depthwise filters larger than 3x3 are not supported");
  ConvGeom g = conv_geom(*d);
  if ((long long)d->n * d->h * d->w * d->c > kMaxElems || (long long)d->n * g.P * g.Q * d->k > kMaxElems ||
      (long long)d->r * d->s * d->c * d->k > kMaxElems)
    return fail(S4TF_ERR_SHAPE, "conv: a tensor exceeds 2^31-1 elements");
  return S4TF_OK;
}
int check_bn_desc(const s4tf_bn_desc* d) {
  if (!d) return fail(S4TF_ERR_NULL, "bn descriptor is NULL");
  if (!dtype_ok(d->dtype) || !act_ok(d->act)) return fail(S4TF_ERR_DTYPE, "bn: bad dtype %d or act %d", d->dtype, d->act);
  if (d->n <= 0 || d->h <= 0 || d->w <= 0 || d->c <= 0) return fail(S4TF_ERR_SHAPE, "bn: sizes must be positive");
  if (!(d->eps >= 0.f)) return fail(S4TF_ERR_SHAPE, "bn: eps must be >= 0");
  if ((long long)d->n * d->h * d->w * d->c > kMaxElems) return fail(S4TF_ERR_SHAPE, "bn: tensor exceeds 2^31-1 elements");
  return S4TF_OK;
}
int check_pool_desc(const s4tf_pool_desc* d) {
  if (!d) return fail(S4TF_ERR_NULL, "pool descriptor is NULL");
  if (!dtype_ok(d->dtype)) return fail(S4TF_ERR_DTYPE, "pool: bad dtype %d", d->dtype);
  if (d->kind != S4TF_POOL_AVG2 && d->kind != S4TF_POOL_MAX3S2) return fail(S4TF_ERR_DTYPE, "pool: bad kind %d", d->kind);
  if (d->n <= 0 || d->h <= 0 || d->w <= 0 || d->c <= 0) return fail(S4TF_ERR_SHAPE, "pool: sizes must be positive");
  if (d->kind == S4TF_POOL_AVG2 && (d->h < 2 || d->w < 2)) return fail(S4TF_ERR_SHAPE, "avg pool needs h, w >= 2");
  if ((long long)d->n * d->h * d->w * d->c > kMaxElems) return fail(S4TF_ERR_SHAPE, "pool: tensor exceeds 2^31-1 elements");
  return S4TF_OK;
}
int check_head_desc(const s4tf_head_desc* d) {
  if (!d) return fail(S4TF_ERR_NULL, "head descriptor is NULL");
  if (!dtype_ok(d->dtype)) return fail(S4TF_ERR_DTYPE, "head: bad dtype %d", d->dtype);
  if (d->n <= 0 || d->h <= 0 || d->w <= 0 || d->c <= 0 || d->classes <= 0) return fail(S4TF_ERR_SHAPE, "head: sizes must be positive");
  if ((long long)d->n * d->h * d->w * d->c > kMaxElems || (long long)d->c * d->classes > kMaxElems)
    return fail(S4TF_ERR_SHAPE, "head: tensor exceeds 2^31-1 elements");
  return S4TF_OK;
}

int need(const void* p, const char* name) {
  if (!p) return fail(S4TF_ERR_NULL, "%s is NULL", name);
  if (!aligned16(p)) return fail(S4TF_ERR_ALIGN, "%s is not 16-byte aligned", name);
  return S4TF_OK;
}
int opt(const void* p, const char* name) {
  if (p && !aligned16(p)) return fail(S4TF_ERR_ALIGN, "%s is not 16-byte aligned", name);
  return S4TF_OK;
}
int check_ws(const void* ws, size_t have, size_t want) {
  if (want == 0) return S4TF_OK;
  if (!ws) return fail(S4TF_ERR_WORKSPACE, "workspace of %zu bytes required", want);
  if (!aligned16(ws)) return fail(S4TF_ERR_ALIGN, "workspace is not 16-byte aligned");
  if (have < want) return fail(S4TF_ERR_WORKSPACE, "workspace too small: %zu < %zu bytes", have, want);
  return S4TF_OK;
}

// ---- conv dispatch (dense vs depthwise) ---------------------------------------------------------------
static size_t conv_vjp_ws_parts(const s4tf_conv_desc& d, size_t* dz_bytes) {
  ConvGeom g = conv_geom(d);
  size_t dz = d.act != S4TF_ACT_NONE ? align_up((size_t)g.N * g.P * g.Q * g.K * dtype_size(d.dtype), 256) : 0;
  if (dz_bytes) *dz_bytes = dz;
  size_t wg = d.groups == 1 ? igemm_wgrad_workspace(g, d.dtype) : dwconv_wgrad_workspace(g);
  const size_t cs = colsum_workspace((size_t)g.N * g.P * g.Q, g.K);  // bias gradient: used before the filter gradient, same bytes
  if (cs > wg) wg = cs;
  return dz + align_up(wg, 256);
}

int conv_fwd_impl(const s4tf_conv_desc& d, const void* x, const void* w, const float* bias, void* y, hipStream_t st,
                  float* stats_part, int* stats_rows) {
  ConvGeom g = conv_geom(d);
  if (stats_rows) *stats_rows = 0;
  if (d.groups == 1) return igemm_fwd(g, d.dtype, x, w, bias, d.act, y, st, stats_part, stats_rows);
  return dwconv_fwd(g, d.dtype, x, w, bias, d.act, y, st);
}
// dz: cotangent after the activation pullback
// The pullback's two halves are independent given dz: the input cotangent, and the parameter gradients.
int conv_dgrad_impl(const s4tf_conv_desc& d, const void* w, const void* dz, void* dx, hipStream_t st,
                    const void* acc_src, const unsigned char* acc_bits) {
  ConvGeom g = conv_geom(d);
  if (d.groups == 1) return igemm_dgrad(g, d.dtype, dz, w, dx, d.accumulate_dx, st, acc_src, acc_bits);
  return dwconv_dgrad(g, d.dtype, dz, w, dx, d.accumulate_dx, st);
}
int conv_param_grads_impl(const s4tf_conv_desc& d, const void* x, const void* dz, float* dw, float* dbias,
                          void* wg_ws, size_t wg_bytes, hipStream_t st) {
  ConvGeom g = conv_geom(d);
  if (dbias) CHECK(colsum(d.dtype, dz, (size_t)g.N * g.P * g.Q, g.K, dbias, st, wg_ws, wg_bytes));
  if (d.groups == 1) return igemm_wgrad(g, d.dtype, x, dz, dw, wg_ws, wg_bytes, st);
  return dwconv_wgrad(g, d.dtype, x, dz, dw, wg_ws, st);
}
static int conv_vjp_impl(const s4tf_conv_desc& d, const void* x, const void* w, const void* dz, void* dx, float* dw,
                         float* dbias, void* wg_ws, size_t wg_bytes, hipStream_t st) {
  if (dx) CHECK(conv_dgrad_impl(d, w, dz, dx, st));
  return conv_param_grads_impl(d, x, dz, dw, dbias, wg_ws, wg_bytes, st);
}

// What s4tf_profile_bracket_overhead brackets: one wavefront that waits until the constant-rate (100 MHz)
// real-time counter has advanced by `ticks`; the iteration cap ends it whatever the counter does.
__global__ void prof_spin_kernel(unsigned long long ticks) {
  const unsigned long long t0 = __builtin_amdgcn_s_memrealtime();
  for (int i = 0; i < (1 << 20); ++i) {
    if (__builtin_amdgcn_s_memrealtime() - t0 >= ticks) break;
    __builtin_amdgcn_s_sleep(4);
  }
}

}  // namespace s4tf

using namespace s4tf;

extern "C" {

const char* s4tf_last_error(void) { return g_err; }

// ---- conv ----------------------------------------------------------------------------------------------
size_t s4tf_conv2d_fwd_workspace_bytes(const s4tf_conv_desc* d) {
  clear_error();
  (void)check_conv_desc(d);
  return 0;
}
size_t s4tf_conv2d_vjp_workspace_bytes(const s4tf_conv_desc* d) {
  clear_error();
  if (check_conv_desc(d) != S4TF_OK) return 0;
  return conv_vjp_ws_parts(*d, nullptr);
}

int s4tf_conv2d_fwd(const s4tf_conv_desc* d, const void* x, const void* w, const float* bias, void* y,
                    void* workspace, size_t workspace_bytes, void* stream) {
  clear_error();
  (void)workspace; (void)workspace_bytes;
  CHECK(check_conv_desc(d));
  CHECK(need(x, "x")); CHECK(need(w, "w")); CHECK(need(y, "y")); CHECK(opt(bias, "bias"));
  return conv_fwd_impl(*d, x, w, bias, y, (hipStream_t)stream);
}

int s4tf_conv2d_vjp(const s4tf_conv_desc* d, const void* x, const void* w, const void* y, const void* dy,
                    void* dx, float* dw, float* dbias, void* workspace, size_t workspace_bytes, void* stream) {
  clear_error();
  CHECK(check_conv_desc(d));
  CHECK(need(x, "x")); CHECK(need(w, "w")); CHECK(need(dy, "dy")); CHECK(need(dw, "dw"));
  CHECK(opt(dx, "dx")); CHECK(opt(dbias, "dbias"));
  if (d->act != S4TF_ACT_NONE) CHECK(need(y, "y (required when act != NONE)"));
  size_t dz_bytes = 0;
  size_t want = conv_vjp_ws_parts(*d, &dz_bytes);
  CHECK(check_ws(workspace, workspace_bytes, want));
  hipStream_t st = (hipStream_t)stream;
  const void* dz = dy;
  char* wsb = static_cast<char*>(workspace);
  if (d->act != S4TF_ACT_NONE) {
    ConvGeom g = conv_geom(*d);
    CHECK(act_vjp(d->dtype, d->act, y, dy, wsb, (size_t)g.N * g.P * g.Q * g.K, st));
    dz = wsb;
  }
  return conv_vjp_impl(*d, x, w, dz, dx, dw, dbias, wsb ? wsb + dz_bytes : nullptr, want - dz_bytes, st);
}

// ---- batch norm ------------------------------------------------------------------------------------------
size_t s4tf_bn_relu_workspace_bytes(const s4tf_bn_desc* d) {
  clear_error();
  if (check_bn_desc(d) != S4TF_OK) return 0;
  return bn_workspace((size_t)d->n * d->h * d->w, d->c);
}
int s4tf_bn_relu_fwd(const s4tf_bn_desc* d, const void* x, const void* residual, const float* gamma,
                     const float* beta, void* y, float* save_mean, float* save_invstd, void* workspace,
                     size_t workspace_bytes, void* stream) {
  clear_error();
  CHECK(check_bn_desc(d));
  CHECK(need(x, "x")); CHECK(need(gamma, "gamma")); CHECK(need(beta, "beta")); CHECK(need(y, "y"));
  CHECK(need(save_mean, "save_mean")); CHECK(need(save_invstd, "save_invstd")); CHECK(opt(residual, "residual"));
  CHECK(check_ws(workspace, workspace_bytes, bn_workspace((size_t)d->n * d->h * d->w, d->c)));
  return bn_fwd(*d, x, residual, gamma, beta, y, save_mean, save_invstd, workspace, (hipStream_t)stream);
}
int s4tf_bn_relu_fwd_static(const s4tf_bn_desc* d, const void* x, const void* residual, const float* gamma,
                            const float* beta, void* y, float* save_mean, float* save_invstd, void* stream) {
  clear_error();
  CHECK(check_bn_desc(d));
  CHECK(need(x, "x")); CHECK(need(gamma, "gamma")); CHECK(need(beta, "beta")); CHECK(need(y, "y"));
  CHECK(need(save_mean, "save_mean")); CHECK(need(save_invstd, "save_invstd")); CHECK(opt(residual, "residual"));
  return bn_fwd_static(*d, x, residual, gamma, beta, y, save_mean, save_invstd, (hipStream_t)stream);
}
size_t s4tf_bn_relu_fwd_static_limit(const s4tf_bn_desc* d, size_t* needed) {
  clear_error();
  if (needed) *needed = 0;
  if (d && check_bn_desc(d) == S4TF_OK && needed) *needed = bn_fwd_scratch_bytes(*d);
  return bn_static_scratch_capacity();
}
int s4tf_bn_relu_vjp(const s4tf_bn_desc* d, const void* x, const void* y, const float* gamma, const float* beta,
                     const float* save_mean, const float* save_invstd, const void* dy, void* dx, void* dresidual,
                     float* dgamma, float* dbeta, void* workspace, size_t workspace_bytes, void* stream) {
  clear_error();
  CHECK(check_bn_desc(d));
  CHECK(need(x, "x")); CHECK(need(gamma, "gamma")); CHECK(need(save_mean, "save_mean"));
  CHECK(need(save_invstd, "save_invstd")); CHECK(need(dy, "dy")); CHECK(need(dx, "dx"));
  CHECK(need(dgamma, "dgamma")); CHECK(need(dbeta, "dbeta")); CHECK(opt(dresidual, "dresidual"));
  CHECK(opt(beta, "beta"));
  if (d->act != S4TF_ACT_NONE && !(beta && !dresidual)) CHECK(need(y, "y (required when act != NONE, unless beta is given and there is no residual)"));
  CHECK(check_ws(workspace, workspace_bytes, bn_workspace((size_t)d->n * d->h * d->w, d->c)));
  return bn_vjp(*d, x, y, gamma, beta, save_mean, save_invstd, dy, dx, dresidual, dgamma, dbeta, workspace, (hipStream_t)stream);
}

// ---- batch norm, inference mode ------------------------------------------------------------------------------
int s4tf_bn_inference_fwd(const s4tf_bn_desc* d, const void* x, const void* residual, const float* gamma,
                          const float* beta, const float* running_mean, const float* running_var, void* y, void* stream) {
  clear_error();
  CHECK(check_bn_desc(d));
  CHECK(need(x, "x")); CHECK(need(gamma, "gamma")); CHECK(need(beta, "beta")); CHECK(need(y, "y"));
  CHECK(need(running_mean, "running_mean")); CHECK(need(running_var, "running_var")); CHECK(opt(residual, "residual"));
  return bn_inference_fwd(*d, x, residual, gamma, beta, running_mean, running_var, y, (hipStream_t)stream);
}
int s4tf_bn_update_running(int32_t c, size_t count, float momentum, float eps, const float* save_mean,
                           const float* save_invstd, float* running_mean, float* running_var, void* stream) {
  clear_error();
  if (c <= 0 || count == 0) return fail(S4TF_ERR_SHAPE, "bn_update_running: c and count must be positive");
  if (!(momentum >= 0.f && momentum <= 1.f) || !(eps >= 0.f)) return fail(S4TF_ERR_SHAPE, "bn_update_running: momentum in [0,1], eps >= 0");
  CHECK(need(save_mean, "save_mean")); CHECK(need(save_invstd, "save_invstd"));
  CHECK(need(running_mean, "running_mean")); CHECK(need(running_var, "running_var"));
  return bn_update_running(c, count, momentum, eps, save_mean, save_invstd, running_mean, running_var, (hipStream_t)stream);
}
int s4tf_bn_fold_into_conv(const s4tf_conv_desc* d, const void* w, const float* bias, const float* gamma,
                           const float* beta, const float* running_mean, const float* running_var, float eps,
                           void* w_out, float* bias_out, void* stream) {
  clear_error();
  CHECK(check_conv_desc(d));
  if (!(eps >= 0.f)) return fail(S4TF_ERR_SHAPE, "bn_fold: eps must be >= 0");
  CHECK(need(w, "w")); CHECK(need(gamma, "gamma")); CHECK(need(beta, "beta")); CHECK(need(running_mean, "running_mean"));
  CHECK(need(running_var, "running_var")); CHECK(need(w_out, "w_out")); CHECK(need(bias_out, "bias_out")); CHECK(opt(bias, "bias"));
  return bn_fold(d->dtype, (long long)d->r * d->s * (d->c / d->groups), d->k, w, bias, gamma, beta, running_mean, running_var, eps,
                 w_out, bias_out, (hipStream_t)stream);
}

// ---- pooling ----------------------------------------------------------------------------------------------
int s4tf_pool2d_fwd(const s4tf_pool_desc* d, const void* x, void* y, void* stream) {
  clear_error();
  CHECK(check_pool_desc(d));
  CHECK(need(x, "x")); CHECK(need(y, "y"));
  return pool_fwd(*d, x, y, (hipStream_t)stream);
}
int s4tf_pool2d_vjp(const s4tf_pool_desc* d, const void* x, const void* dy, void* dx, void* stream) {
  clear_error();
  CHECK(check_pool_desc(d));
  CHECK(need(dy, "dy")); CHECK(need(dx, "dx"));
  if (d->kind == S4TF_POOL_MAX3S2) CHECK(need(x, "x (required for max pool)"));
  return pool_vjp(*d, x, dy, dx, (hipStream_t)stream);
}

// ---- head ---------------------------------------------------------------------------------------------------
size_t s4tf_pool_dense_xent_workspace_bytes(const s4tf_head_desc* d) {
  clear_error();
  if (check_head_desc(d) != S4TF_OK) return 0;
  return head_workspace(*d);
}
int s4tf_pool_dense_xent_fwd_vjp(const s4tf_head_desc* d, const void* x, const float* W, const float* b,
                                 const int32_t* labels, float* loss, void* dx, float* dW, float* db, float* logits,
                                 void* workspace, size_t workspace_bytes, void* stream) {
  clear_error();
  CHECK(check_head_desc(d));
  CHECK(need(x, "x")); CHECK(need(W, "W")); CHECK(need(b, "b")); CHECK(need(labels, "labels"));
  CHECK(need(loss, "loss")); CHECK(need(dW, "dW")); CHECK(need(db, "db")); CHECK(opt(dx, "dx")); CHECK(opt(logits, "logits"));
  CHECK(check_ws(workspace, workspace_bytes, head_workspace(*d)));
  return head_fwd_vjp(*d, x, W, b, labels, loss, dx, dW, db, logits, workspace, (hipStream_t)stream);
}

// ---- optimizer ------------------------------------------------------------------------------------------------
int s4tf_sgd_momentum(size_t count, float* param, float* velocity, const float* grad, void* param_lowp, float lr,
                      float momentum, void* stream) {
  clear_error();
  if (count == 0) return S4TF_OK;
  CHECK(need(param, "param")); CHECK(need(velocity, "velocity")); CHECK(need(grad, "grad")); CHECK(opt(param_lowp, "param_lowp"));
  return sgd(count, param, velocity, grad, param_lowp, lr, momentum, (hipStream_t)stream);
}

// ---- indexing -------------------------------------------------------------------------------------------------
static int check_gather_desc(const s4tf_gather_desc* d) {
  if (!d) return fail(S4TF_ERR_NULL, "gather descriptor is NULL");
  if (!dtype_ok(d->dtype)) return fail(S4TF_ERR_DTYPE, "gather: bad dtype %d", d->dtype);
  if (d->rows <= 0 || d->cols <= 0 || d->count < 0) return fail(S4TF_ERR_SHAPE, "gather: rows and cols must be positive, count >= 0");
  if ((long long)d->rows * d->cols > kMaxElems || (long long)d->count * d->cols > kMaxElems)
    return fail(S4TF_ERR_SHAPE, "gather: tensor exceeds 2^31-1 elements");
  return S4TF_OK;
}
int s4tf_gather_rows_fwd(const s4tf_gather_desc* d, const void* x, const int32_t* index, void* y, void* stream) {
  clear_error();
  CHECK(check_gather_desc(d));
  if (d->count == 0) return S4TF_OK;
  CHECK(need(x, "x")); CHECK(need(index, "index")); CHECK(need(y, "y"));
  return gather_rows_fwd(*d, x, index, y, (hipStream_t)stream);
}
int s4tf_gather_rows_vjp(const s4tf_gather_desc* d, const void* dy, const int32_t* index, void* dx, void* stream) {
  clear_error();
  CHECK(check_gather_desc(d));
  if (d->count == 0) return S4TF_OK;
  CHECK(need(dy, "dy")); CHECK(need(index, "index")); CHECK(need(dx, "dx"));
  return gather_rows_vjp(*d, dy, index, dx, (hipStream_t)stream);
}

int s4tf_round_to_bf16(size_t count, const float* src, void* dst, void* stream) {
  clear_error();
  if (count == 0) return S4TF_OK;
  CHECK(need(src, "src")); CHECK(need(dst, "dst"));
  return round_to_bf16(count, src, dst, (hipStream_t)stream);
}

// ---- measurement hook ------------------------------------------------------------------------------------------------
int s4tf_profile_enable(int on) {
  g_prof_on = on != 0;
  return S4TF_OK;
}
int s4tf_profile_collect(double* ms, int64_t* launches) {
  clear_error();
  if (!ms || !launches) return fail(S4TF_ERR_NULL, "ms or launches is NULL");
  for (int i = 0; i < S4TF_PROF_CLASSES; ++i) { ms[i] = 0.0; launches[i] = 0; }
  if (!g_prof) return S4TF_OK;
  int rc = S4TF_OK;
  for (ProfRec& r : *g_prof) {
    float t = 0.f;
    if (hipEventSynchronize(r.e1) != hipSuccess || hipEventElapsedTime(&t, r.e0, r.e1) != hipSuccess)
      rc = fail(S4TF_ERR_DEVICE, "profile: event read failed");
    else if (r.cls >= 0 && r.cls < S4TF_PROF_CLASSES) { ms[r.cls] += (double)t; launches[r.cls] += 1; }
    (void)hipEventDestroy(r.e0);
    (void)hipEventDestroy(r.e1);
  }
  g_prof->clear();
  return rc;
}
int s4tf_profile_bracket_overhead(void* stream, int reps, double* ms_per_pair) {
  clear_error();
  if (!ms_per_pair) return fail(S4TF_ERR_NULL, "ms_per_pair is NULL");
  if (reps < 1 || reps > 4096) return fail(S4TF_ERR_SHAPE, "reps must be in 1..4096");
  hipStream_t st = static_cast<hipStream_t>(stream);
  const unsigned long long kSpinTicks = 2000;  // 20 us: the length of a typical kernel of the step
  std::vector<hipEvent_t> ev(2 * (size_t)reps, nullptr);
  int rc = S4TF_OK;
  for (hipEvent_t& e : ev)
    if (hipEventCreate(&e) != hipSuccess) { rc = fail(S4TF_ERR_DEVICE, "profile: event create failed"); break; }
  if (rc == S4TF_OK) {
    hipLaunchKernelGGL(s4tf::prof_spin_kernel, dim3(1), dim3(64), 0, st, kSpinTicks);  // first launch: loads the code
    (void)hipStreamSynchronize(st);
    for (int i = 0; i < reps; ++i) {
      (void)hipEventRecord(ev[2 * i], st);
      hipLaunchKernelGGL(s4tf::prof_spin_kernel, dim3(1), dim3(64), 0, st, kSpinTicks);
      (void)hipEventRecord(ev[2 * i + 1], st);
    }
    double sum = 0.0;
    if (hipStreamSynchronize(st) != hipSuccess) rc = fail(S4TF_ERR_DEVICE, "profile: synchronize failed");
    for (int i = 0; i < reps && rc == S4TF_OK; ++i) {
      float t = 0.f;
      if (hipEventElapsedTime(&t, ev[2 * i], ev[2 * i + 1]) != hipSuccess) rc = fail(S4TF_ERR_DEVICE, "profile: event read failed");
      sum += (double)t;
    }
    if (rc == S4TF_OK) *ms_per_pair = sum / reps - (double)kSpinTicks * 1e-5;  // 100 MHz: 1e-5 ms per tick
  }
  for (hipEvent_t e : ev)
    if (e) (void)hipEventDestroy(e);
  return rc;
}
const char* s4tf_profile_class_name(int cls) {
  return (cls >= 0 && cls < S4TF_PROF_CLASSES) ? kProfNames[cls] : "";
}

}  // extern "C"
