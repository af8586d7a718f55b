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

static int need(const void* p, const char* name) {
  if (!p) return fail(S4TF_ERR_NULL, "%s is NULL", name);
  if (!aligned16(p)) return fail(S4TF_ERR_ALIGN, "%s is not 16-byte aligned", name);
  return S4TF_OK;
}
static int opt(const void* p, const char* name) {
  if (p && !aligned16(p)) return fail(S4TF_ERR_ALIGN, "%s is not 16-byte aligned", name);
  return S4TF_OK;
}
#define CHECK(expr)                \
  do {                             \
    int rc_ = (expr);              \
    if (rc_ != S4TF_OK) return rc_; \
  } while (0)

static int check_ws(const void* ws, size_t have, size_t want) {
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

static int conv_fwd_impl(const s4tf_conv_desc& d, const void* x, const void* w, const float* bias, void* y, hipStream_t st,
                         float* stats_part = nullptr, int* stats_rows = nullptr) {
  ConvGeom g = conv_geom(d);
  if (stats_rows) *stats_rows = 0;
  if (d.groups == 1) return igemm_fwd(g, d.dtype, x, w, bias, d.act, y, st, stats_part, stats_rows);
  return dwconv_fwd(g, d.dtype, x, w, bias, d.act, y, st);
}
// dz: cotangent after the activation pullback
// The pullback's two halves are independent given dz: the input cotangent, and the parameter gradients.
static int conv_dgrad_impl(const s4tf_conv_desc& d, const void* w, const void* dz, void* dx, hipStream_t st,
                           const void* acc_src = nullptr, const unsigned char* acc_bits = nullptr) {
  ConvGeom g = conv_geom(d);
  if (d.groups == 1) return igemm_dgrad(g, d.dtype, dz, w, dx, d.accumulate_dx, st, acc_src, acc_bits);
  return dwconv_dgrad(g, d.dtype, dz, w, dx, d.accumulate_dx, st);
}
static int conv_param_grads_impl(const s4tf_conv_desc& d, const void* x, const void* dz, float* dw, float* dbias,
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

// ---- second stream of the train step -------------------------------------------------------------------
// Parameter gradients of the convolutions are needed only by the optimizer at the end of the step, while
// the chain of input cotangents (dgrad, BatchNorm pullback) is latency and bandwidth bound and leaves
// the matrix cores idle: the step forks the filter-gradient kernels onto a stream of the library's own
// (default priority) and joins it before the optimizer.  One stream and two events per device, created
// on first use and kept for the life of the process.
struct SideStream {
  hipStream_t stream = nullptr;
  hipEvent_t fork = nullptr, join = nullptr;
  hipEvent_t back[8] = {};  // side -> main dependencies inside a step (side branches), used round-robin
};
static std::mutex g_side_mutex;
static SideStream g_side[64];
static int side_stream(SideStream** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return fail(S4TF_ERR_DEVICE, "cannot tell the current device");
  std::lock_guard<std::mutex> lock(g_side_mutex);
  SideStream& s = g_side[dev];
  if (!s.stream) {
    hipStream_t st = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (hipStreamCreateWithFlags(&st, hipStreamNonBlocking) != hipSuccess ||
        hipEventCreateWithFlags(&e0, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&e1, hipEventDisableTiming) != hipSuccess)
      return fail(S4TF_ERR_DEVICE, "cannot create the second stream of the train step: %s", hipGetErrorString(hipGetLastError()));
    for (int k = 0; k < 8; ++k)
      if (hipEventCreateWithFlags(&s.back[k], hipEventDisableTiming) != hipSuccess)
        return fail(S4TF_ERR_DEVICE, "cannot create the events of the train step: %s", hipGetErrorString(hipGetLastError()));
    s.stream = st; s.fork = e0; s.join = e1;
  }
  *out = &s;
  return S4TF_OK;
}

// ---- whole-step planning -------------------------------------------------------------------------------
struct TensorPlan {
  int n, h, w, c;
  size_t elems;
  size_t act_off, grad_off;  // bytes into the workspace
  int consumers;
  int alias_of;  // flatten: shares buffers with this tensor, else -1
  int root;      // the tensor whose buffers this one uses (itself unless an alias chain); 0 = the batch
};
struct NetPlan {
  std::vector<TensorPlan> t;
  std::vector<int64_t> poff, psize;  // 2 per op
  // per BatchNorm op with activation bits whose residual input has one other consumer, a plain convolution of
  // the main branch (an identity shortcut): that convolution's op index, else -1.  The pullback of such a
  // BatchNorm need not write its residual cotangent dz = act'(y) dy: the convolution's dgrad adds it from dy
  // and the bits in its epilogue (same values, one tensor less written).
  std::vector<int> defer_conv;
  std::vector<size_t> mask_off;      // per op: activation bits of a BatchNorm with residual and activation (0: none)
  std::vector<size_t> stat_off;      // per op: save_mean/invstd (BN); max pool: the saved window positions (one byte per output)
  // a convolution on the batch itself whose channel count is not a multiple of 8 (bf16) or 4 (fp32) runs
  // on zero-padded copies of the batch and of its filter (pad_c channels), see train step
  std::vector<int> pad_c;
  std::vector<size_t> xpad_off, wpad_off, dwpad_off;
  size_t param_count;
  size_t scratch_off, scratch_bytes, total_bytes;
  size_t wscratch_off, wscratch_bytes;  // scratch of the filter-gradient kernels, which run on a stream of their own
  // Side branches: a convolution + BatchNorm pair whose only use is as the residual input of a later
  // BatchNorm (the projection shortcut of a residual block), while other ops lie between the pair and
  // the op that made its input.  Forward, the pair runs on the second stream as soon as its input
  // exists, beside the main branch; its pullback runs there too.  branch_of[op]: the pair's number or
  // -1; start_after[op]: the pair to start once op is queued; needs[op]: the pair whose output op reads.
  std::vector<int> branch_of, start_after, needs;
  std::vector<int> branch_conv;         // per pair: its convolution's op index
  size_t sscratch_off;                  // scratch of the side branches (as large as the main scratch)
  // A step whose convolutions add up to little arithmetic is a chain of kernels of a few microseconds each:
  // there a hand-over between streams (5-10 us) costs more than the overlap can return, and the whole step
  // runs on the caller's stream.
  bool one_stream;
};

static int plan_net(const s4tf_net_desc* net, NetPlan& pl) {
  if (!net) return fail(S4TF_ERR_NULL, "net descriptor is NULL");
  if (!net->ops || net->n_ops <= 0) return fail(S4TF_ERR_NULL, "net has no ops");
  if (!dtype_ok(net->dtype)) return fail(S4TF_ERR_DTYPE, "net: bad dtype %d", net->dtype);
  if (net->n <= 0 || net->h <= 0 || net->w <= 0 || net->c <= 0) return fail(S4TF_ERR_SHAPE, "net: batch sizes must be positive");
  const int nops = net->n_ops;
  const size_t es = dtype_size(net->dtype);
  pl.t.assign(nops + 1, TensorPlan());
  pl.poff.assign(2 * nops, 0);
  pl.psize.assign(2 * nops, 0);
  pl.stat_off.assign(nops, 0);
  pl.mask_off.assign(nops, 0);
  pl.defer_conv.assign(nops, -1);
  pl.pad_c.assign(nops, 0);
  pl.xpad_off.assign(nops, 0);
  pl.wpad_off.assign(nops, 0);
  pl.dwpad_off.assign(nops, 0);
  pl.t[0] = TensorPlan{net->n, net->h, net->w, net->c, (size_t)net->n * net->h * net->w * net->c, 0, 0, 0, -1, 0};
  size_t pcount = 0, off = 0, scratch = 0, wscratch = 0;
  auto add_param = [&](int op, int slot, size_t n) {
    pl.poff[2 * op + slot] = (int64_t)pcount;
    pl.psize[2 * op + slot] = (int64_t)n;
    pcount += align_up(n, 8);
  };
  for (int i = 0; i < nops; ++i) {
    const s4tf_op& op = net->ops[i];
    if (op.in < 0 || op.in > i) return fail(S4TF_ERR_SHAPE, "op %d: input tensor %d is not an earlier tensor", i, op.in);
    if ((i == nops - 1) != (op.kind == S4TF_OP_HEAD)) return fail(S4TF_ERR_SHAPE, "op %d: the head must be the last op and only there", i);
    const TensorPlan in = pl.t[op.in];
    pl.t[op.in].consumers++;
    TensorPlan out = TensorPlan{in.n, in.h, in.w, in.c, 0, 0, 0, 0, -1, i + 1};
    switch (op.kind) {
      case S4TF_OP_CONV: {
        s4tf_conv_desc d = {in.n, in.h, in.w, in.c, op.k, op.r, op.s, op.stride, op.pad, op.groups, net->dtype, op.act, 0};
        int rc = check_conv_desc(&d);
        if (rc != S4TF_OK) return rc;
        ConvGeom g = conv_geom(d);
        out.h = g.P; out.w = g.Q; out.c = op.k;
        add_param(i, 0, (size_t)op.r * op.s * (in.c / op.groups) * op.k);
        if (op.has_bias) add_param(i, 1, (size_t)op.k);
        // channel count of the batch not a multiple of the 16-byte loaders' vector (8 bf16, 4 fp32): padded copies
        const int vecw = net->dtype == S4TF_BF16 ? 8 : 4;
        // (fp32: only where the convolution is big enough to repay the two copy launches)
        if (in.root == 0 && op.groups == 1 && in.c % vecw != 0 &&
            (net->dtype == S4TF_BF16 || (op.k % 4 == 0 && (long long)g.N * g.P * g.Q >= 32768))) {
          pl.pad_c[i] = (int)align_up((size_t)in.c, vecw);
          g.C = pl.pad_c[i];
        }
        size_t ws = op.groups == 1 ? igemm_wgrad_workspace(g, net->dtype) : dwconv_wgrad_workspace(g);
        if (ws > wscratch) wscratch = ws;
        if (op.has_bias) {
          ws = colsum_workspace((size_t)g.N * g.P * g.Q, g.K);
          if (ws > wscratch) wscratch = ws;
        }
        // a BatchNorm right behind takes its statistics from partial sums the convolution leaves in scratch
        // (right behind on its stream: a projection shortcut's two ops, which run on the second stream, may lie between)
        for (int k = i + 1; k < nops && k <= i + 3 && op.groups == 1; ++k)
          if (net->ops[k].kind == S4TF_OP_BN && net->ops[k].in == i + 1) {
            ws = igemm_fwd_stats_bytes(g);
            if (ws > scratch) scratch = ws;
          }
        break;
      }
      case S4TF_OP_BN: {
        s4tf_bn_desc d = {in.n, in.h, in.w, in.c, op.eps, op.act, net->dtype, 0};
        int rc = check_bn_desc(&d);
        if (rc != S4TF_OK) return rc;
        if (in.root == 0) return fail(S4TF_ERR_UNSUPPORTED, "op %d: BatchNorm directly on the batch is not supported", i);
        if (op.res >= 0) {
          if (op.res > i) return fail(S4TF_ERR_SHAPE, "op %d: residual tensor %d is not an earlier tensor", i, op.res);
          const TensorPlan& r = pl.t[op.res];
          if (r.n != in.n || r.h != in.h || r.w != in.w || r.c != in.c) return fail(S4TF_ERR_SHAPE, "op %d: residual shape differs", i);
          pl.t[op.res].consumers++;
        }
        add_param(i, 0, (size_t)in.c);
        add_param(i, 1, (size_t)in.c);
        size_t ws = bn_workspace((size_t)in.n * in.h * in.w, in.c);
        if (ws > scratch) scratch = ws;
        break;
      }
      case S4TF_OP_AVGPOOL2:
      case S4TF_OP_MAXPOOL3S2: {
        s4tf_pool_desc d = {in.n, in.h, in.w, in.c, op.kind == S4TF_OP_AVGPOOL2 ? S4TF_POOL_AVG2 : S4TF_POOL_MAX3S2, net->dtype, 0};
        int rc = check_pool_desc(&d);
        if (rc != S4TF_OK) return rc;
        if (op.kind == S4TF_OP_AVGPOOL2) { out.h = in.h / 2; out.w = in.w / 2; }
        else { out.h = (in.h - 1) / 2 + 1; out.w = (in.w - 1) / 2 + 1; }
        break;
      }
      case S4TF_OP_FLATTEN:
        out.c = in.h * in.w * in.c; out.h = 1; out.w = 1;
        out.alias_of = op.in;
        out.root = in.root;
        break;
      case S4TF_OP_HEAD: {
        s4tf_head_desc d = {in.n, in.h, in.w, in.c, op.k, net->dtype};
        int rc = check_head_desc(&d);
        if (rc != S4TF_OK) return rc;
        add_param(i, 0, (size_t)in.c * op.k);
        add_param(i, 1, (size_t)op.k);
        size_t ws = head_workspace(d);
        if (ws > scratch) scratch = ws;
        out.h = 1; out.w = 1; out.c = op.k;
        break;
      }
      default:
        return fail(S4TF_ERR_DTYPE, "op %d: unknown kind %d", i, op.kind);
    }
    out.elems = (size_t)out.n * out.h * out.w * out.c;
    pl.t[i + 1] = out;
  }
  // consumers: every tensor except the head's output needs one; BN inputs and flatten inputs exactly one
  for (int i = 0; i < nops; ++i) {
    const s4tf_op& op = net->ops[i];
    if (i + 1 < nops && pl.t[i + 1].consumers == 0) return fail(S4TF_ERR_SHAPE, "tensor %d (output of op %d) has no consumer", i + 1, i);
    if ((op.kind == S4TF_OP_BN || op.kind == S4TF_OP_FLATTEN) && pl.t[op.in].root != 0 && pl.t[op.in].consumers != 1)
      return fail(S4TF_ERR_UNSUPPORTED, "op %d: the input of a BN/flatten op must have no other consumer", i);
  }
  // workspace: activations, cotangents, BN statistics, shared scratch
  for (int i = 1; i < nops; ++i) {  // tensor nops is the head's (virtual) output
    TensorPlan& t = pl.t[i];
    if (t.root != i) {  // an alias: buffers of its root (none if the root is the batch)
      t.act_off = pl.t[t.root].act_off;
      t.grad_off = pl.t[t.root].grad_off;
      continue;
    }
    t.act_off = off; off += align_up(t.elems * es, 256);
    t.grad_off = off; off += align_up(t.elems * es, 256);
  }
  for (int i = 0; i < nops; ++i)
    if (net->ops[i].kind == S4TF_OP_BN) {
      pl.stat_off[i] = off;
      off += align_up((size_t)2 * pl.t[net->ops[i].in].c * sizeof(float), 256);
      // A BatchNorm with residual and activation leaves act'(y) as bits for its pullback, which then need not
      // read y: where a pixel's bits are at least 32 adjacent bytes (narrower rows make scattered byte accesses
      // that cost more than the reads they save: ResNet-56, +0.9 %; ResNet-50: -1.7 %).  off > 0 here: 0 = none.
      const TensorPlan& bt = pl.t[net->ops[i].in];
      if (net->ops[i].res >= 0 && net->ops[i].act != S4TF_ACT_NONE && bn_mask_bytes(1, bt.c, net->dtype) >= 32) {
        pl.mask_off[i] = off;
        off += align_up(bn_mask_bytes((size_t)bt.n * bt.h * bt.w, bt.c, net->dtype), 256);
      }
    } else if (net->ops[i].kind == S4TF_OP_MAXPOOL3S2) {
      pl.stat_off[i] = off;
      off += align_up(pl.t[i + 1].elems, 256);
    }
  for (int i = 0; i < nops; ++i)
    if (pl.pad_c[i]) {
      const s4tf_op& op = net->ops[i];
      const TensorPlan& in = pl.t[op.in];
      pl.xpad_off[i] = off; off += align_up((size_t)in.n * in.h * in.w * pl.pad_c[i] * es, 256);
      pl.wpad_off[i] = off; off += align_up((size_t)op.r * op.s * pl.pad_c[i] * op.k * es, 256);
      pl.dwpad_off[i] = off; off += align_up((size_t)op.r * op.s * pl.pad_c[i] * op.k * sizeof(float), 256);
    }
  double conv_flops = 0.0;  // forward pass
  for (int i = 0; i < nops; ++i)
    if (net->ops[i].kind == S4TF_OP_CONV) {
      const s4tf_op& op = net->ops[i];
      conv_flops += 2.0 * (double)pl.t[i + 1].elems * op.r * op.s * pl.t[op.in].c / op.groups;
    }
  pl.one_stream = conv_flops < 0.5e9;
  pl.scratch_off = off;
  pl.scratch_bytes = align_up(scratch, 256);
  pl.wscratch_off = pl.scratch_off + pl.scratch_bytes;
  pl.wscratch_bytes = align_up(wscratch, 256);
  pl.sscratch_off = pl.wscratch_off + pl.wscratch_bytes;
  pl.total_bytes = pl.sscratch_off + pl.scratch_bytes;
  // side branches
  pl.branch_of.assign(nops, -1);
  pl.start_after.assign(nops, -1);
  pl.needs.assign(nops, -1);
  pl.branch_conv.clear();
  for (int j = 0; j + 2 < nops; ++j) {
    const s4tf_op& cv = net->ops[j];
    const s4tf_op& bn = net->ops[j + 1];
    if (cv.kind != S4TF_OP_CONV || cv.groups != 1 || pl.pad_c[j] || bn.kind != S4TF_OP_BN || bn.in != j + 1 || bn.res >= 0) continue;
    const int X = cv.in;
    if (X <= 0 || pl.t[X].root != X || X >= j) continue;             // its input: a tensor of its own, made at least one op earlier
    if (pl.t[j + 2].consumers != 1) continue;
    int user = -1;
    for (int r = j + 2; r < nops; ++r)
      if (net->ops[r].kind == S4TF_OP_BN && net->ops[r].res == j + 2) { user = r; break; }
    if (user < 0 || pl.start_after[X - 1] >= 0 || pl.needs[user] >= 0) continue;
    const int id = (int)pl.branch_conv.size();
    pl.branch_conv.push_back(j);
    pl.branch_of[j] = pl.branch_of[j + 1] = id;
    pl.start_after[X - 1] = id;
    pl.needs[user] = id;
  }
  // identity shortcuts whose residual cotangent the consuming convolution's dgrad can add by itself
  for (int i = 0; i < nops; ++i) {
    const s4tf_op& bn = net->ops[i];
    if (bn.kind != S4TF_OP_BN || bn.res <= 0 || !pl.mask_off[i] || pl.branch_of[i] >= 0) continue;
    const int R = bn.res;
    if (pl.t[R].root != R || pl.t[R].consumers != 2) continue;
    int conv = -1;
    for (int j = 0; j < i; ++j)
      if (net->ops[j].in == R && j != i) { conv = j; break; }
    if (conv < 0) continue;
    const s4tf_op& cv = net->ops[conv];
    if (cv.kind != S4TF_OP_CONV || cv.groups != 1 || cv.stride != 1 || cv.act != S4TF_ACT_NONE || pl.pad_c[conv] ||
        pl.branch_of[conv] >= 0)
      continue;
    pl.defer_conv[i] = conv;
  }
  pl.param_count = pcount;
  return S4TF_OK;
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

int s4tf_round_to_bf16(size_t count, const float* src, void* dst, void* stream) {
  clear_error();
  if (count == 0) return S4TF_OK;
  CHECK(need(src, "src")); CHECK(need(dst, "dst"));
  return round_to_bf16(count, src, dst, (hipStream_t)stream);
}

// ---- whole step ---------------------------------------------------------------------------------------------------
size_t s4tf_net_param_count(const s4tf_net_desc* net) {
  clear_error();
  NetPlan pl;
  if (plan_net(net, pl) != S4TF_OK) return 0;
  return pl.param_count;
}
int s4tf_net_param_layout(const s4tf_net_desc* net, int64_t* offsets, int64_t* sizes) {
  clear_error();
  NetPlan pl;
  CHECK(plan_net(net, pl));
  for (size_t i = 0; i < pl.poff.size(); ++i) {
    if (offsets) offsets[i] = pl.poff[i];
    if (sizes) sizes[i] = pl.psize[i];
  }
  return S4TF_OK;
}
int s4tf_net_tensor_layout(const s4tf_net_desc* net, int64_t* act_off, int64_t* grad_off, int32_t* shape,
                           int64_t* stat_off) {
  clear_error();
  NetPlan pl;
  CHECK(plan_net(net, pl));
  for (int t = 0; t < net->n_ops; ++t) {
    const TensorPlan& tp = pl.t[t];
    const bool has = tp.root != 0;
    if (act_off) act_off[t] = has ? (int64_t)tp.act_off : -1;
    if (grad_off) grad_off[t] = has ? (int64_t)tp.grad_off : -1;
    if (shape) { shape[4 * t] = tp.n; shape[4 * t + 1] = tp.h; shape[4 * t + 2] = tp.w; shape[4 * t + 3] = tp.c; }
  }
  if (stat_off)
    for (int i = 0; i < net->n_ops; ++i) stat_off[i] = net->ops[i].kind == S4TF_OP_BN ? (int64_t)pl.stat_off[i] : -1;
  return S4TF_OK;
}
size_t s4tf_train_step_workspace_bytes(const s4tf_net_desc* net) {
  clear_error();
  NetPlan pl;
  if (plan_net(net, pl) != S4TF_OK) return 0;
  return pl.total_bytes;
}

int s4tf_train_step(const s4tf_net_desc* net, s4tf_params* params, const s4tf_batch* batch, float lr) {
  clear_error();
  NetPlan pl;
  CHECK(plan_net(net, pl));
  if (!params || !batch) return fail(S4TF_ERR_NULL, "params or batch is NULL");
  CHECK(need(params->master, "params.master")); CHECK(need(params->velocity, "params.velocity"));
  CHECK(need(params->grad, "params.grad")); CHECK(opt(params->lowp, "params.lowp"));
  const bool bf16 = net->dtype == S4TF_BF16;
  if (bf16 && !params->lowp) return fail(S4TF_ERR_NULL, "params.lowp is required for a bf16 net");
  if (params->count != pl.param_count)
    return fail(S4TF_ERR_SHAPE, "params.count is %zu, the net needs %zu", params->count, pl.param_count);
  CHECK(need(batch->x, "batch.x")); CHECK(need(batch->labels, "batch.labels")); CHECK(need(batch->loss, "batch.loss"));
  CHECK(check_ws(batch->workspace, batch->workspace_bytes, pl.total_bytes));

  hipStream_t st = (hipStream_t)batch->stream;
  char* ws = static_cast<char*>(batch->workspace);
  const int nops = net->n_ops;
  const int dt = net->dtype;
  void* scratch = ws + pl.scratch_off;
  void* wscratch = ws + pl.wscratch_off;
  SideStream* side = nullptr;
  CHECK(side_stream(&side));
  const bool one_stream = pl.one_stream;               // small steps: everything in order on `st`
  const hipStream_t side_st = one_stream ? st : side->stream;
  // Whatever way this function returns, `st` ends up waiting for what the side stream was given, so
  // that in stream order on `st` the step is over (and its workspace free) when its last kernel is.
  struct Join {
    SideStream* s; hipStream_t st; bool forked = false;
    int now() {
      if (!forked) return S4TF_OK;
      forked = false;
      if (hipEventRecord(s->join, s->stream) != hipSuccess || hipStreamWaitEvent(st, s->join, 0) != hipSuccess)
        return fail(S4TF_ERR_DEVICE, "train step: stream join failed");
      return S4TF_OK;
    }
    ~Join() { (void)now(); }
  } join{side, st};
  // everything `st` has queued so far (the previous step's optimizer included) precedes the side stream's work
  auto fork = [&]() -> int {
    if (one_stream) return S4TF_OK;
    join.forked = true;
    if (hipEventRecord(side->fork, st) != hipSuccess || hipStreamWaitEvent(side->stream, side->fork, 0) != hipSuccess)
      return fail(S4TF_ERR_DEVICE, "train step: stream fork failed");
    return S4TF_OK;
  };
  auto act_ptr = [&](int t) -> const void* { return pl.t[t].root == 0 ? batch->x : (const void*)(ws + pl.t[t].act_off); };
  auto out_ptr = [&](int t) -> void* { return ws + pl.t[t].act_off; };
  auto grad_ptr = [&](int t) -> void* { return ws + pl.t[t].grad_off; };
  auto conv_w = [&](int op) -> const void* {
    return bf16 ? (const void*)(static_cast<bf16_t*>(params->lowp) + pl.poff[2 * op])
                : (const void*)(params->master + pl.poff[2 * op]);
  };
  auto conv_desc = [&](int i, int accumulate) {
    const s4tf_op& op = net->ops[i];
    const TensorPlan& in = pl.t[op.in];
    s4tf_conv_desc d = {in.n, in.h, in.w, in.c, op.k, op.r, op.s, op.stride, op.pad, op.groups, dt, op.act, accumulate};
    return d;
  };

  // ---- forward ----
  void* sscratch = ws + pl.sscratch_off;
  // side -> main dependencies: the event a side branch's output (forward) or a tensor's cotangent
  // (backward) is ready at; `st` waits for it where it first touches that data
  int back_next = 0;
  std::vector<int> branch_event(pl.branch_conv.size(), -1);
  auto side_done = [&](int& slot) -> int {  // marks what the side stream has been given so far
    if (one_stream) return S4TF_OK;
    slot = back_next++ % 8;
    if (hipEventRecord(side->back[slot], side->stream) != hipSuccess) return fail(S4TF_ERR_DEVICE, "train step: event record failed");
    return S4TF_OK;
  };
  auto wait_side = [&](int& slot) -> int {
    if (slot < 0) return S4TF_OK;
    if (hipStreamWaitEvent(st, side->back[slot], 0) != hipSuccess) return fail(S4TF_ERR_DEVICE, "train step: event wait failed");
    slot = -1;
    return S4TF_OK;
  };
  // one forward op on stream s with scratch scr; stats_rows: in, what the op before left in scr; out, what this one leaves
  auto fwd_op = [&](int i, hipStream_t s, void* scr, int& stats_rows) -> int {
    const s4tf_op& op = net->ops[i];
    const TensorPlan& in = pl.t[op.in];
    const int prev_stats_rows = stats_rows;
    stats_rows = 0;
    switch (op.kind) {
      case S4TF_OP_CONV: {
        s4tf_conv_desc d = conv_desc(i, 0);
        const float* bias = op.has_bias ? params->master + pl.poff[2 * i + 1] : nullptr;
        // the next op on this stream is a BatchNorm of this convolution's output (ops of a side branch, which run on
        // the other stream with a scratch of their own, may lie between in op order)
        bool bn_next = false;
        for (int k = i + 1; k < nops && k <= i + 3 && op.groups == 1; ++k) {
          if (net->ops[k].kind == S4TF_OP_BN && net->ops[k].in == i + 1) { bn_next = true; break; }
          if (pl.branch_of[k] < 0 || pl.branch_of[i] >= 0) break;
        }
        float* sp = bn_next ? static_cast<float*>(scr) : nullptr;
        int* sr = bn_next ? &stats_rows : nullptr;
        if (pl.pad_c[i]) {  // zero-padded channels contribute nothing: same result, 16-byte loaders
          CHECK(pad_channels(dt, act_ptr(op.in), ws + pl.xpad_off[i], (long long)in.n * in.h * in.w, in.c, pl.pad_c[i], 1, s));
          CHECK(pad_channels(dt, conv_w(i), ws + pl.wpad_off[i], (long long)op.r * op.s, in.c, pl.pad_c[i], op.k, s));
          d.c = pl.pad_c[i];
          CHECK(conv_fwd_impl(d, ws + pl.xpad_off[i], ws + pl.wpad_off[i], bias, out_ptr(i + 1), s, sp, sr));
          break;
        }
        CHECK(conv_fwd_impl(d, act_ptr(op.in), conv_w(i), bias, out_ptr(i + 1), s, sp, sr));
        break;
      }
      case S4TF_OP_BN: {
        s4tf_bn_desc d = {in.n, in.h, in.w, in.c, op.eps, op.act, dt, 0};
        float* stats = reinterpret_cast<float*>(ws + pl.stat_off[i]);
        CHECK(bn_fwd(d, act_ptr(op.in), op.res >= 0 ? act_ptr(op.res) : nullptr, params->master + pl.poff[2 * i],
                     params->master + pl.poff[2 * i + 1], out_ptr(i + 1), stats, stats + in.c, scr, s,
                     prev_stats_rows > 0 ? static_cast<const float*>(scr) : nullptr, prev_stats_rows,
                     pl.mask_off[i] ? reinterpret_cast<unsigned char*>(ws + pl.mask_off[i]) : nullptr));
        break;
      }
      case S4TF_OP_AVGPOOL2:
      case S4TF_OP_MAXPOOL3S2: {
        s4tf_pool_desc d = {in.n, in.h, in.w, in.c, op.kind == S4TF_OP_AVGPOOL2 ? S4TF_POOL_AVG2 : S4TF_POOL_MAX3S2, dt, 0};
        unsigned char* pos = pool_saves_positions(d) ? reinterpret_cast<unsigned char*>(ws + pl.stat_off[i]) : nullptr;
        CHECK(pool_fwd(d, act_ptr(op.in), out_ptr(i + 1), s, pos));
        break;
      }
      default:
        break;  // flatten: a reinterpretation
    }
    return S4TF_OK;
  };
  int stats_rows = 0;  // > 0: the previous op, a convolution, left partial statistics of its output in scratch
  for (int i = 0; i < nops - 1; ++i) {
    if (pl.branch_of[i] >= 0) continue;  // ran on the side stream when its input appeared (and left `scratch` alone)
    if (pl.needs[i] >= 0) CHECK(wait_side(branch_event[pl.needs[i]]));
    CHECK(fwd_op(i, st, scratch, stats_rows));
    if (pl.start_after[i] >= 0) {  // the input of a side branch is queued: the branch starts beside what follows
      const int b = pl.start_after[i], j = pl.branch_conv[b];
      CHECK(fork());
      int sr = 0;
      CHECK(fwd_op(j, side_st, sscratch, sr));
      CHECK(fwd_op(j + 1, side_st, sscratch, sr));
      CHECK(side_done(branch_event[b]));
    }
  }
  auto resolve = [&](int t) -> int { return pl.t[t].root; };

  // ---- head: loss and the first cotangent ----
  std::vector<char> written(nops + 1, 0);
  {
    const s4tf_op& op = net->ops[nops - 1];
    const TensorPlan& in = pl.t[op.in];
    s4tf_head_desc d = {in.n, in.h, in.w, in.c, op.k, dt};
    const int src = resolve(op.in);
    void* dx = src == 0 ? nullptr : grad_ptr(src);
    CHECK(head_fwd_vjp(d, act_ptr(op.in), params->master + pl.poff[2 * (nops - 1)],
                       params->master + pl.poff[2 * (nops - 1) + 1], batch->labels, batch->loss, dx,
                       params->grad + pl.poff[2 * (nops - 1)], params->grad + pl.poff[2 * (nops - 1) + 1], nullptr,
                       scratch, st));
    written[src] = 1;
  }
  // ---- pullbacks in reverse op order ----
  // Ops of a side branch run on the side stream (after the op that feeds them their cotangent, which
  // the fork orders); a cotangent they write is waited for where the main stream first touches it.
  std::vector<int> grad_event(nops + 1, -1);   // per tensor: pending side-stream write of its cotangent
  std::vector<int> deferred(nops + 1, -1);     // per tensor: the BatchNorm whose residual cotangent its consumer's dgrad adds
  std::vector<char> branch_forked(pl.branch_conv.size(), 0);
  int early_join = -1;  // event slot: everything the side stream got before the first op's filter gradient
  // Filter (and bias) gradient of convolution j, on the second stream.
  auto param_grads = [&](int j) -> int {
    const s4tf_op& cv = net->ops[j];
    const TensorPlan& cin = pl.t[cv.in];
    s4tf_conv_desc d = conv_desc(j, 0);
    void* dyj = grad_ptr(j + 1);
    float* dbias = cv.has_bias ? params->grad + pl.poff[2 * j + 1] : nullptr;
    if (pl.pad_c[j]) {  // the batch has no cotangent; the filter gradient of the padded channels is dropped
      d.c = pl.pad_c[j];
      float* dwp = reinterpret_cast<float*>(ws + pl.dwpad_off[j]);
      CHECK(conv_param_grads_impl(d, ws + pl.xpad_off[j], dyj, dwp, dbias, wscratch, pl.wscratch_bytes, side_st));
      return unpad_channels_f32(dwp, params->grad + pl.poff[2 * j], (long long)cv.r * cv.s, cin.c, pl.pad_c[j], cv.k, side_st);
    }
    return conv_param_grads_impl(d, act_ptr(pl.t[cv.in].root), dyj, params->grad + pl.poff[2 * j], dbias, wscratch,
                                 pl.wscratch_bytes, side_st);
  };
  // A hand-over to the second stream costs the first one 5-7 us (measured: an event record between two kernels
  // 2.9 us, more once another stream waits on it), so the filter gradients of the main branch are handed over
  // FORK_EVERY convolutions at a time: cotangent buffers are never reused, so a filter gradient can start any
  // time after its convolution's output cotangent is final.
  constexpr int FORK_EVERY = 3;
  std::vector<int> pending;
  std::vector<int> convs_before(nops, 0);  // main-branch convolutions with a smaller op index
  for (int k = 1; k < nops; ++k)
    convs_before[k] = convs_before[k - 1] + (net->ops[k - 1].kind == S4TF_OP_CONV && pl.branch_of[k - 1] < 0 ? 1 : 0);
  auto flush_pending = [&]() -> int {
    if (pending.empty()) return S4TF_OK;
    CHECK(fork());
    for (int j : pending) {
      // The first op's filter gradient is the last piece of side-stream work: mark the point before it, so that
      // the optimizer can start on every other parameter while that gradient is still being computed.
      if (j == 0 && pl.poff[0] == 0) CHECK(side_done(early_join));
      CHECK(param_grads(j));
    }
    pending.clear();
    return S4TF_OK;
  };
  for (int i = nops - 2; i >= 0; --i) {
    const s4tf_op& op = net->ops[i];
    const TensorPlan& in = pl.t[op.in];
    const int src = resolve(op.in);
    const bool want_dx = src != 0;
    void* dy = grad_ptr(i + 1);
    const int br = pl.branch_of[i];
    const bool on_side = br >= 0;
    hipStream_t s = on_side ? side_st : st;
    void* scr = on_side ? sscratch : scratch;
    if (on_side) {
      if (!branch_forked[br]) {  // everything queued on `st` so far (its cotangent's producer included) comes first
        CHECK(fork());
        branch_forked[br] = 1;
      }
    } else {
      CHECK(wait_side(grad_event[resolve(i + 1)]));
      if (want_dx) CHECK(wait_side(grad_event[src]));
    }
    switch (op.kind) {
      case S4TF_OP_CONV: {
        s4tf_conv_desc d = conv_desc(i, written[src] ? 1 : 0);
        if (op.act != S4TF_ACT_NONE)  // in place: dy is not needed once dz exists
          CHECK(act_vjp(dt, op.act, out_ptr(i + 1), dy, dy, pl.t[i + 1].elems, s));
        // dz is final.  The input cotangent is computed first; the parameter gradients go to the side
        // stream and start when it is done, so that they run beside the bandwidth-bound BatchNorm pullback
        // of the layer before rather than beside this layer's other matrix kernel (measured: 2 % of the step).
        if (want_dx && !pl.pad_c[i] && deferred[src] >= 0) {
          const int b = deferred[src];  // dx = dgrad + the residual cotangent of BatchNorm b, from its dy and bits
          if (written[src]) return fail(S4TF_ERR_UNSUPPORTED, "train step: deferred residual cotangent of tensor %d already written", src);
          CHECK(conv_dgrad_impl(d, conv_w(i), dy, grad_ptr(src), s, grad_ptr(b + 1),
                                reinterpret_cast<const unsigned char*>(ws + pl.mask_off[b])));
          deferred[src] = -1;
          written[src] = 1;
        } else if (want_dx && !pl.pad_c[i]) {
          CHECK(conv_dgrad_impl(d, conv_w(i), dy, grad_ptr(src), s));
          written[src] = 1;
          if (on_side) CHECK(side_done(grad_event[src]));
        }
        if (on_side) {
          CHECK(param_grads(i));
        } else {
          pending.push_back(i);
          // (the last few of the pass one by one: whatever is still queued when the main stream runs out of work
          // is the tail of the step)
          // A big filter gradient (gigaflops, contracted over tens of thousands of pixels: 50-130 us on the second
          // stream, behind main-stream kernels that are as long) is worth a hand-over of its own: started as early
          // as possible, the second stream is not what the end of the step waits for (ResNet-50: -1 %; the small
          // layers of the fp32 nets lose 1-2 % when handed over singly).
          const TensorPlan& ot = pl.t[i + 1];
          const double wflops = 2.0 * (double)ot.elems * op.r * op.s * in.c / op.groups;
          const bool big = wflops >= 5e9 && (double)ot.n * ot.h * ot.w >= 40000.0;
          if ((int)pending.size() >= FORK_EVERY || convs_before[i] < 6 || big) CHECK(flush_pending());
        }
        break;
      }
      case S4TF_OP_BN: {
        const int rsrc = op.res >= 0 ? resolve(op.res) : -1;
        if (!on_side && rsrc > 0) CHECK(wait_side(grad_event[rsrc]));
        s4tf_bn_desc d = {in.n, in.h, in.w, in.c, op.eps, op.act, dt, (rsrc > 0 && written[rsrc]) ? 1 : 0};
        float* stats = reinterpret_cast<float*>(ws + pl.stat_off[i]);
        void* dxb = grad_ptr(src);  // src != 0: checked when the net was planned
        void* dres = rsrc > 0 ? grad_ptr(rsrc) : nullptr;
        if (pl.defer_conv[i] >= 0 && !on_side && !written[rsrc]) {
          // identity shortcut: the dgrad of the block's first convolution will add dz = act'(y) dy itself
          const int j = pl.defer_conv[i];
          s4tf_conv_desc cd = conv_desc(j, 0);
          if (igemm_dgrad_adds_other(conv_geom(cd), dt, grad_ptr(j + 1), conv_w(j), dres, dy)) {
            deferred[rsrc] = i;
            dres = nullptr;
          }
        }
        // no residual in the forward pass: the pullback rebuilds the activation mask from x and skips y
        const float* beta = op.res < 0 ? params->master + pl.poff[2 * i + 1] : nullptr;
        CHECK(bn_vjp(d, act_ptr(src), out_ptr(i + 1), params->master + pl.poff[2 * i], beta, stats, stats + in.c, dy, dxb,
                     dres, params->grad + pl.poff[2 * i], params->grad + pl.poff[2 * i + 1], scr, s,
                     pl.mask_off[i] ? reinterpret_cast<const unsigned char*>(ws + pl.mask_off[i]) : nullptr));
        written[src] = 1;
        if (rsrc > 0 && dres) written[rsrc] = 1;
        break;
      }
      case S4TF_OP_AVGPOOL2:
      case S4TF_OP_MAXPOOL3S2: {
        if (!want_dx) break;
        s4tf_pool_desc d = {in.n, in.h, in.w, in.c, op.kind == S4TF_OP_AVGPOOL2 ? S4TF_POOL_AVG2 : S4TF_POOL_MAX3S2, dt,
                            written[src] ? 1 : 0};
        const unsigned char* pos = pool_saves_positions(d) ? reinterpret_cast<const unsigned char*>(ws + pl.stat_off[i]) : nullptr;
        CHECK(pool_vjp(d, act_ptr(src), dy, grad_ptr(src), s, pos));
        written[src] = 1;
        break;
      }
      default:  // flatten shares its buffers (and its cotangent) with its input
        break;
    }
  }
  CHECK(flush_pending());
  // ---- optimizer: one launch over the whole arena, once the side stream's gradients are in ----
  if (early_join >= 0) {  // all parameters but the first op's, then, after the join, those
    const s4tf_op& op0 = net->ops[0];  // its parameters lie at the start of the arena, padded to 8 elements each
    const size_t head = op0.has_bias ? (size_t)pl.poff[1] + align_up((size_t)pl.psize[1], 8) : align_up((size_t)pl.psize[0], 8);
    CHECK(wait_side(early_join));
    CHECK(sgd(params->count - head, params->master + head, params->velocity + head, params->grad + head,
              bf16 ? (void*)(static_cast<bf16_t*>(params->lowp) + head) : nullptr, lr, net->momentum, st));
    CHECK(join.now());
    return sgd(head, params->master, params->velocity, params->grad, bf16 ? params->lowp : nullptr, lr, net->momentum, st);
  }
  CHECK(join.now());
  return sgd(params->count, params->master, params->velocity, params->grad, bf16 ? params->lowp : nullptr, lr,
             net->momentum, st);
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
