// The whole training step: forward, pullbacks in reverse op order and the optimizer update (the paper's
// Section 4.2 training loop; a step is `(inout Model, Minibatch) -> Void`).
//
// A network is planned ONCE: shapes, parameter and workspace layout, which ops run on the second stream,
// which cotangent is accumulated into which, where an event hands data from one stream to the other.  The
// result is a flat schedule, a list of commands (one per kernel family launch or stream operation) that a
// step replays with the caller's pointers.  Plans are kept in a cache keyed by a hash of the descriptor, so
// that the descriptor form of s4tf_train_step plans a net the first time it sees it and only replays
// afterwards: the role the trace-hash cache of compiled programs plays in the paper's Section 3.4, without a
// trace or a compiler.  s4tf_net_create hands the same plan to callers that want to own it.
#include <string.h>

#include <memory>
#include <mutex>
#include <vector>

#include "s4tf_internal.h"
#include "igemm_args.h"

namespace s4tf {
namespace {

// ---- second stream of the train step -------------------------------------------------------------------
// Parameter gradients of the convolutions are needed only by the optimizer at the end of the step, while
// the chain of input cotangents (dgrad, BatchNorm pullback) is latency and bandwidth bound and leaves
// the matrix cores idle: the step forks the filter-gradient kernels onto a stream of the library's own
// (default priority) and joins it before the optimizer.  One stream and ten events per device, created
// on first use and kept for the life of the process.  A two-stream step holds the device's lock while it
// enqueues, so that steps issued from several host threads do not interleave their use of the events.
struct SideStream {
  hipStream_t stream = nullptr;
  hipEvent_t fork = nullptr, join = nullptr;
  hipEvent_t back[8] = {};  // side -> main dependencies inside a step (side branches), used round-robin
  std::mutex step_mutex;
};
std::mutex g_side_mutex;
SideStream g_side[64];

int side_stream(SideStream** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return fail(S4TF_ERR_DEVICE, "cannot tell the current device");
  std::lock_guard<std::mutex> lock(g_side_mutex);
  SideStream& s = g_side[dev];
  if (!s.stream) {
    hipStream_t st = nullptr;
    hipEvent_t ev[10] = {};
    bool ok = hipStreamCreateWithFlags(&st, hipStreamNonBlocking) == hipSuccess;
    for (int k = 0; ok && k < 10; ++k) ok = hipEventCreateWithFlags(&ev[k], hipEventDisableTiming) == hipSuccess;
    if (!ok) {  // nothing half-made is kept
      const char* why = hipGetErrorString(hipGetLastError());
      for (hipEvent_t e : ev)
        if (e) (void)hipEventDestroy(e);
      if (st) (void)hipStreamDestroy(st);
      return fail(S4TF_ERR_DEVICE, "cannot create the second stream of the train step: %s", why);
    }
    s.fork = ev[0];
    s.join = ev[1];
    for (int k = 0; k < 8; ++k) s.back[k] = ev[2 + k];
    s.stream = st;
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
  // on zero-padded copies of the batch and of its filter (pad_c channels)
  std::vector<int> pad_c;
  // ... or, bf16 with stride 2, an odd filter and at most 4 channels, as a stride-1 convolution over 2x2 pixel
  // blocks of 16 channels (fold[op] = 1, pad_c = 16; fold2_pixels and its companions): a shorter reduction axis
  // than channel padding gives, and every 16-byte operand chunk holds two pixels
  std::vector<char> fold;
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

bool dtype_ok(int t) { return t == S4TF_F32 || t == S4TF_BF16; }

// The stride-1 geometry over 2x2 pixel blocks that stands for a stride-2 convolution of geometry g (see fold2_pixels)
ConvGeom folded_geom(const ConvGeom& g, int pad) {
  ConvGeom f = g;
  f.H = (g.H + 2 * pad) / 2; f.W = (g.W + 2 * pad) / 2; f.C = 16;
  f.R = (g.R + 1) / 2; f.S = (g.S + 1) / 2; f.stride = 1; f.pad = 0;
  f.P = f.H - f.R + 1; f.Q = f.W - f.S + 1;
  return f;
}
s4tf_conv_desc folded_desc(const s4tf_conv_desc& d) {
  s4tf_conv_desc f = d;
  f.h = (d.h + 2 * d.pad) / 2; f.w = (d.w + 2 * d.pad) / 2; f.c = 16;
  f.r = (d.r + 1) / 2; f.s = (d.s + 1) / 2; f.stride = 1; f.pad = 0;
  return f;
}

int plan_net(const s4tf_net_desc* net, NetPlan& pl) {
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
  pl.fold.assign(nops, 0);
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
          if (net->dtype == S4TF_BF16 && op.stride == 2 && in.c <= 4 && op.r >= 3 && op.s >= 3 && (op.r & 1) && (op.s & 1) &&
              (in.h + 2 * op.pad) % 2 == 0 && (in.w + 2 * op.pad) % 2 == 0 && op.k % 8 == 0) {
            const ConvGeom gf = folded_geom(g, op.pad);
            if (gf.P == g.P && gf.Q == g.Q && igemm_dma_geom_ok(PASS_FWD, gf) && igemm_dma_geom_ok(PASS_WGRAD, gf)) {
              pl.fold[i] = 1;
              pl.pad_c[i] = 16;
              g = gf;
            }
          }
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
      // folded: (h + 2 pad)/2 x (w + 2 pad)/2 pixels of 16 channels, (r+1)/2 x (s+1)/2 taps
      const size_t px = pl.fold[i] ? (size_t)in.n * ((in.h + 2 * op.pad) / 2) * ((in.w + 2 * op.pad) / 2) : (size_t)in.n * in.h * in.w;
      const size_t taps = pl.fold[i] ? (size_t)((op.r + 1) / 2) * ((op.s + 1) / 2) : (size_t)op.r * op.s;
      pl.xpad_off[i] = off; off += align_up(px * pl.pad_c[i] * es, 256);
      pl.wpad_off[i] = off; off += align_up(taps * pl.pad_c[i] * op.k * es, 256);
      pl.dwpad_off[i] = off; off += align_up(taps * pl.pad_c[i] * op.k * sizeof(float), 256);
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
    const TensorPlan& ci = pl.t[cv.in];
    s4tf_conv_desc cd = {ci.n, ci.h, ci.w, ci.c, cv.k, cv.r, cv.s, cv.stride, cv.pad, cv.groups, net->dtype, cv.act, 0};
    if (!igemm_dgrad_can_add_other(conv_geom(cd), net->dtype)) continue;
    pl.defer_conv[i] = conv;
  }
  pl.param_count = pcount;
  return S4TF_OK;
}

// ---- the schedule -------------------------------------------------------------------------------------------
enum CmdKind : uint8_t {
  K_FORK, K_JOIN, K_SIDE_DONE, K_WAIT_SIDE,        // stream operations (a: event slot)
  K_CONV_FWD, K_BN_FWD, K_POOL_FWD, K_HEAD,        // forward (conv: a = 1 when it emits statistics partial sums)
  K_ACT_VJP, K_DGRAD, K_PARAM_GRADS, K_BN_VJP,     // pullbacks (dgrad: a = accumulate, b = BatchNorm whose residual
  K_POOL_VJP, K_SGD                                //  cotangent it adds or -1; bn: a = accumulate into dres, b = 1 when
};                                                 //  dres is left to that dgrad; pool: a = accumulate; sgd: a = part)
struct Cmd {
  uint8_t kind;
  uint8_t side;  // 1: the library's second stream, 0: the caller's
  uint8_t scr;   // 1: the side branches' scratch, 0: the main scratch
  int op, a, b;
};

}  // namespace
}  // namespace s4tf

// The handle behind s4tf_net_create (global namespace: the C header declares `struct s4tf_net`).
struct s4tf_net {
  s4tf_net_desc desc;  // desc.ops points at `ops`
  std::vector<s4tf_op> ops;
  s4tf::NetPlan pl;
  std::vector<s4tf::Cmd> cmds;
  uint64_t hash;
};

namespace s4tf {
namespace {

// Walks the net once, in the order a step runs it, and writes the schedule down.  Everything that can make a
// step impossible is decided here, before any step launches anything.
int record_schedule(s4tf_net& N) {
  const s4tf_net_desc* net = &N.desc;
  const NetPlan& pl = N.pl;
  std::vector<Cmd>& out = N.cmds;
  out.clear();
  const int nops = net->n_ops;
  const bool one_stream = pl.one_stream;
  auto emit = [&](uint8_t kind, bool side, bool scr, int op, int a = 0, int b = -1) {
    out.push_back(Cmd{kind, (uint8_t)((side && !one_stream) ? 1 : 0), (uint8_t)(scr ? 1 : 0), op, a, b});
  };
  auto resolve = [&](int t) -> int { return pl.t[t].root; };
  // side -> main dependencies: the event slot a side branch's output (forward) or a tensor's cotangent
  // (backward) is ready at; the main stream waits for it where it first touches that data
  int back_next = 0;
  auto fork = [&]() { if (!one_stream) emit(K_FORK, false, false, -1); };
  auto side_done = [&](int& slot) {
    if (one_stream) return;
    slot = back_next++ % 8;
    emit(K_SIDE_DONE, true, false, -1, slot);
  };
  auto wait_side = [&](int& slot) {
    if (slot < 0) return;
    emit(K_WAIT_SIDE, false, false, -1, slot);
    slot = -1;
  };
  // ---- forward ----
  std::vector<int> branch_event(pl.branch_conv.size(), -1);
  auto fwd_op = [&](int i, bool side) {
    const s4tf_op& op = net->ops[i];
    switch (op.kind) {
      case S4TF_OP_CONV: {
        // the next op on this stream is a BatchNorm of this convolution's output (ops of a side branch, which run on
        // the other stream with a scratch of their own, may lie between in op order)
        bool bn_next = false;
        for (int k = i + 1; k < nops && k <= i + 3 && op.groups == 1; ++k) {
          if (net->ops[k].kind == S4TF_OP_BN && net->ops[k].in == i + 1) { bn_next = true; break; }
          if (pl.branch_of[k] < 0 || pl.branch_of[i] >= 0) break;
        }
        emit(K_CONV_FWD, side, side, i, bn_next ? 1 : 0);
        break;
      }
      case S4TF_OP_BN: emit(K_BN_FWD, side, side, i); break;
      case S4TF_OP_AVGPOOL2:
      case S4TF_OP_MAXPOOL3S2: emit(K_POOL_FWD, side, side, i); break;
      default: break;  // flatten: a reinterpretation
    }
  };
  for (int i = 0; i < nops - 1; ++i) {
    if (pl.branch_of[i] >= 0) continue;  // runs on the side stream when its input appears
    if (pl.needs[i] >= 0) wait_side(branch_event[pl.needs[i]]);
    fwd_op(i, false);
    if (pl.start_after[i] >= 0) {  // the input of a side branch is queued: the branch starts beside what follows
      const int b = pl.start_after[i], j = pl.branch_conv[b];
      fork();
      fwd_op(j, true);
      fwd_op(j + 1, true);
      side_done(branch_event[b]);
    }
  }
  // ---- head: loss and the first cotangent ----
  std::vector<char> written(nops + 1, 0);
  {
    const int src = resolve(net->ops[nops - 1].in);
    emit(K_HEAD, false, false, nops - 1, src);
    written[src] = 1;
  }
  // ---- pullbacks in reverse op order ----
  // Ops of a side branch run on the side stream (after the op that feeds them their cotangent, which
  // the fork orders); a cotangent they write is waited for where the main stream first touches it.
  std::vector<int> grad_event(nops + 1, -1);   // per tensor: pending side-stream write of its cotangent
  std::vector<int> deferred(nops + 1, -1);     // per tensor: the BatchNorm whose residual cotangent its consumer's dgrad adds
  std::vector<char> branch_forked(pl.branch_conv.size(), 0);
  int early_join = -1;  // event slot: everything the side stream got before the first op's filter gradient
  // A hand-over to the second stream costs the first one 5-7 us (measured: an event record between two kernels
  // 2.9 us, more once another stream waits on it), so the filter gradients of the main branch are handed over
  // FORK_EVERY convolutions at a time: cotangent buffers are never reused, so a filter gradient can start any
  // time after its convolution's output cotangent is final.
  constexpr int FORK_EVERY = 3;
  std::vector<int> pending;
  std::vector<int> convs_before(nops, 0);  // main-branch convolutions with a smaller op index
  for (int k = 1; k < nops; ++k)
    convs_before[k] = convs_before[k - 1] + (net->ops[k - 1].kind == S4TF_OP_CONV && pl.branch_of[k - 1] < 0 ? 1 : 0);
  auto flush_pending = [&]() {
    if (pending.empty()) return;
    fork();
    for (int j : pending) {
      // The first op's filter gradient is the last piece of side-stream work: mark the point before it, so that
      // the optimizer can start on every other parameter while that gradient is still being computed.
      if (j == 0 && pl.poff[0] == 0) side_done(early_join);
      emit(K_PARAM_GRADS, true, false, j);
    }
    pending.clear();
  };
  for (int i = nops - 2; i >= 0; --i) {
    const s4tf_op& op = net->ops[i];
    const TensorPlan& in = pl.t[op.in];
    const int src = resolve(op.in);
    const bool want_dx = src != 0;
    const int br = pl.branch_of[i];
    const bool on_side = br >= 0;
    if (on_side) {
      if (!branch_forked[br]) {  // everything queued on the main stream so far (its cotangent's producer included) comes first
        fork();
        branch_forked[br] = 1;
      }
    } else {
      wait_side(grad_event[resolve(i + 1)]);
      if (want_dx) wait_side(grad_event[src]);
    }
    switch (op.kind) {
      case S4TF_OP_CONV: {
        if (op.act != S4TF_ACT_NONE) emit(K_ACT_VJP, on_side, on_side, i);  // in place: dy is not needed once dz exists
        // dz is final.  The input cotangent is computed first; the parameter gradients go to the side
        // stream and start when it is done, so that they run beside the bandwidth-bound BatchNorm pullback
        // of the layer before rather than beside this layer's other matrix kernel (measured: 2 % of the step).
        if (want_dx && !pl.pad_c[i] && deferred[src] >= 0) {
          const int b = deferred[src];  // dx = dgrad + the residual cotangent of BatchNorm b, from its dy and bits
          if (written[src]) return fail(S4TF_ERR_UNSUPPORTED, "deferred residual cotangent of tensor %d already written", src);
          emit(K_DGRAD, on_side, on_side, i, 0, b);
          deferred[src] = -1;
          written[src] = 1;
        } else if (want_dx && !pl.pad_c[i]) {
          emit(K_DGRAD, on_side, on_side, i, written[src] ? 1 : 0, -1);
          written[src] = 1;
          if (on_side) side_done(grad_event[src]);
        }
        if (on_side) {
          emit(K_PARAM_GRADS, true, false, i);
        } else {
          pending.push_back(i);
          // A big filter gradient (gigaflops, contracted over tens of thousands of pixels: 50-130 us on the second
          // stream, behind main-stream kernels that are as long) is worth a hand-over of its own: started as early
          // as possible, the second stream is not what the end of the step waits for (ResNet-50: -1 %; the small
          // layers of the fp32 nets lose 1-2 % when handed over singly).  The last few of the pass go one by one
          // too: whatever is still queued when the main stream runs out of work is the tail of the step.
          const TensorPlan& ot = pl.t[i + 1];
          const double wflops = 2.0 * (double)ot.elems * op.r * op.s * in.c / op.groups;
          const bool big = wflops >= 5e9 && (double)ot.n * ot.h * ot.w >= 40000.0;
          if ((int)pending.size() >= FORK_EVERY || convs_before[i] < 6 || big) flush_pending();
        }
        break;
      }
      case S4TF_OP_BN: {
        const int rsrc = op.res >= 0 ? resolve(op.res) : -1;
        if (!on_side && rsrc > 0) wait_side(grad_event[rsrc]);
        const int acc_dres = (rsrc > 0 && written[rsrc]) ? 1 : 0;
        int leave_dres = 0;
        if (pl.defer_conv[i] >= 0 && !on_side && rsrc > 0 && !written[rsrc]) {
          // identity shortcut: the dgrad of the block's first convolution will add dz = act'(y) dy itself
          deferred[rsrc] = i;
          leave_dres = 1;
        }
        emit(K_BN_VJP, on_side, on_side, i, acc_dres, leave_dres);
        written[src] = 1;
        if (rsrc > 0 && !leave_dres) written[rsrc] = 1;
        break;
      }
      case S4TF_OP_AVGPOOL2:
      case S4TF_OP_MAXPOOL3S2:
        if (!want_dx) break;
        emit(K_POOL_VJP, on_side, on_side, i, written[src] ? 1 : 0);
        written[src] = 1;
        break;
      default:  // flatten shares its buffers (and its cotangent) with its input
        break;
    }
  }
  flush_pending();
  for (int t = 1; t < nops; ++t)
    if (deferred[t] >= 0) return fail(S4TF_ERR_UNSUPPORTED, "residual cotangent of tensor %d left without a convolution to add it", t);
  // ---- optimizer: one launch over the whole arena, once the side stream's gradients are in ----
  if (early_join >= 0) {  // all parameters but the first op's, then, after the join, those
    wait_side(early_join);
    emit(K_SGD, false, false, -1, 1);
    if (!one_stream) emit(K_JOIN, false, false, -1);
    emit(K_SGD, false, false, -1, 2);
  } else {
    if (!one_stream) emit(K_JOIN, false, false, -1);
    emit(K_SGD, false, false, -1, 0);
  }
  return S4TF_OK;
}

uint64_t hash_desc(const s4tf_net_desc* d) {  // FNV-1a over the scalar fields and the op records
  uint64_t h = 1469598103934665603ull;
  auto mix = [&](const void* p, size_t n) {
    const unsigned char* b = static_cast<const unsigned char*>(p);
    for (size_t i = 0; i < n; ++i) { h ^= b[i]; h *= 1099511628211ull; }
  };
  const int32_t head[6] = {d->n, d->h, d->w, d->c, d->dtype, d->n_ops};
  mix(head, sizeof head);
  mix(&d->momentum, sizeof d->momentum);
  for (int i = 0; i < d->n_ops; ++i) {
    const s4tf_op& o = d->ops[i];
    const int32_t f[11] = {o.kind, o.in, o.res, o.k, o.r, o.s, o.stride, o.pad, o.groups, o.has_bias, o.act};
    mix(f, sizeof f);
    mix(&o.eps, sizeof o.eps);
  }
  return h;
}
bool same_op(const s4tf_op& a, const s4tf_op& b) {
  return a.kind == b.kind && a.in == b.in && a.res == b.res && a.k == b.k && a.r == b.r && a.s == b.s && a.stride == b.stride &&
         a.pad == b.pad && a.groups == b.groups && a.has_bias == b.has_bias && a.act == b.act &&
         memcmp(&a.eps, &b.eps, sizeof a.eps) == 0;
}
bool same_desc(const s4tf_net_desc& a, const s4tf_net_desc* b) {
  if (a.n != b->n || a.h != b->h || a.w != b->w || a.c != b->c || a.dtype != b->dtype || a.n_ops != b->n_ops ||
      memcmp(&a.momentum, &b->momentum, sizeof a.momentum) != 0)
    return false;
  for (int i = 0; i < a.n_ops; ++i)
    if (!same_op(a.ops[i], b->ops[i])) return false;
  return true;
}

// plans a net (the caller checked desc and desc->ops for NULL)
int build_net(const s4tf_net_desc* desc, std::unique_ptr<s4tf_net>& out) {
  std::unique_ptr<s4tf_net> N(new s4tf_net());
  CHECK(plan_net(desc, N->pl));
  N->ops.assign(desc->ops, desc->ops + desc->n_ops);
  N->desc = *desc;
  N->desc.ops = N->ops.data();
  N->hash = hash_desc(desc);
  CHECK(record_schedule(*N));
  out = std::move(N);
  return S4TF_OK;
}

// Plans kept for the descriptor form of the calls, most recently made last.
constexpr size_t kCacheEntries = 32;
std::mutex g_cache_mutex;
std::vector<std::shared_ptr<s4tf_net>> g_cache;

int cached_net(const s4tf_net_desc* desc, std::shared_ptr<s4tf_net>& out) {
  if (!desc) return fail(S4TF_ERR_NULL, "net descriptor is NULL");
  if (!desc->ops || desc->n_ops <= 0) return fail(S4TF_ERR_NULL, "net has no ops");
  const uint64_t h = hash_desc(desc);
  std::lock_guard<std::mutex> lock(g_cache_mutex);
  for (size_t i = g_cache.size(); i-- > 0;)
    if (g_cache[i]->hash == h && same_desc(g_cache[i]->desc, desc)) {
      out = g_cache[i];
      return S4TF_OK;
    }
  std::unique_ptr<s4tf_net> N;
  CHECK(build_net(desc, N));
  if (g_cache.size() >= kCacheEntries) g_cache.erase(g_cache.begin());
  g_cache.emplace_back(std::move(N));
  out = g_cache.back();
  return S4TF_OK;
}

// Replays the schedule with the caller's pointers.
int run_step(const s4tf_net& N, s4tf_params* params, const s4tf_batch* batch, float lr) {
  const s4tf_net_desc* net = &N.desc;
  const NetPlan& pl = N.pl;
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
  SideStream* side = nullptr;
  std::unique_lock<std::mutex> device_lock;
  if (!pl.one_stream) {
    CHECK(side_stream(&side));
    device_lock = std::unique_lock<std::mutex>(side->step_mutex);
  }
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
  void* scratch_of[2] = {ws + pl.scratch_off, ws + pl.sscratch_off};
  void* wscratch = ws + pl.wscratch_off;
  int stats_rows[2] = {0, 0};  // per scratch: > 0 when the op before, a convolution, left partial statistics there

  for (const Cmd& c : N.cmds) {
    const hipStream_t s = c.side ? side->stream : st;
    void* scr = scratch_of[c.scr];
    const int i = c.op;
    switch (c.kind) {
      case K_FORK:  // everything `st` has queued so far (the previous step's optimizer included) precedes the side stream's work
        join.forked = true;
        if (hipEventRecord(side->fork, st) != hipSuccess || hipStreamWaitEvent(side->stream, side->fork, 0) != hipSuccess)
          return fail(S4TF_ERR_DEVICE, "train step: stream fork failed");
        break;
      case K_JOIN:
        CHECK(join.now());
        break;
      case K_SIDE_DONE:  // marks what the side stream has been given so far
        if (hipEventRecord(side->back[c.a], side->stream) != hipSuccess) return fail(S4TF_ERR_DEVICE, "train step: event record failed");
        break;
      case K_WAIT_SIDE:
        if (hipStreamWaitEvent(st, side->back[c.a], 0) != hipSuccess) return fail(S4TF_ERR_DEVICE, "train step: event wait failed");
        break;
      case K_CONV_FWD: {
        const s4tf_op& op = net->ops[i];
        const TensorPlan& in = pl.t[op.in];
        stats_rows[c.scr] = 0;
        s4tf_conv_desc d = conv_desc(i, 0);
        const float* bias = op.has_bias ? params->master + pl.poff[2 * i + 1] : nullptr;
        float* sp = c.a ? static_cast<float*>(scr) : nullptr;
        int* sr = c.a ? &stats_rows[c.scr] : nullptr;
        if (pl.fold[i]) {
          CHECK(fold2_pixels(act_ptr(op.in), ws + pl.xpad_off[i], in.n, in.h, in.w, in.c, op.pad, s));
          CHECK(fold2_filter(conv_w(i), ws + pl.wpad_off[i], op.r, op.s, in.c, op.k, s));
          CHECK(conv_fwd_impl(folded_desc(d), ws + pl.xpad_off[i], ws + pl.wpad_off[i], bias, out_ptr(i + 1), s, sp, sr));
          break;
        }
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
      case K_BN_FWD: {
        const s4tf_op& op = net->ops[i];
        const TensorPlan& in = pl.t[op.in];
        const int prev_rows = stats_rows[c.scr];
        stats_rows[c.scr] = 0;
        s4tf_bn_desc d = {in.n, in.h, in.w, in.c, op.eps, op.act, dt, 0};
        float* stats = reinterpret_cast<float*>(ws + pl.stat_off[i]);
        CHECK(bn_fwd(d, act_ptr(op.in), op.res >= 0 ? act_ptr(op.res) : nullptr, params->master + pl.poff[2 * i],
                     params->master + pl.poff[2 * i + 1], out_ptr(i + 1), stats, stats + in.c, scr, s,
                     prev_rows > 0 ? static_cast<const float*>(scr) : nullptr, prev_rows,
                     pl.mask_off[i] ? reinterpret_cast<unsigned char*>(ws + pl.mask_off[i]) : nullptr));
        break;
      }
      case K_POOL_FWD: {
        const s4tf_op& op = net->ops[i];
        const TensorPlan& in = pl.t[op.in];
        stats_rows[c.scr] = 0;
        s4tf_pool_desc d = {in.n, in.h, in.w, in.c, op.kind == S4TF_OP_AVGPOOL2 ? S4TF_POOL_AVG2 : S4TF_POOL_MAX3S2, dt, 0};
        unsigned char* pos = pool_saves_positions(d) ? reinterpret_cast<unsigned char*>(ws + pl.stat_off[i]) : nullptr;
        CHECK(pool_fwd(d, act_ptr(op.in), out_ptr(i + 1), s, pos));
        break;
      }
      case K_HEAD: {
        const s4tf_op& op = net->ops[i];
        const TensorPlan& in = pl.t[op.in];
        s4tf_head_desc d = {in.n, in.h, in.w, in.c, op.k, dt};
        void* dx = c.a == 0 ? nullptr : grad_ptr(c.a);
        CHECK(head_fwd_vjp(d, act_ptr(op.in), params->master + pl.poff[2 * i], params->master + pl.poff[2 * i + 1],
                           batch->labels, batch->loss, dx, params->grad + pl.poff[2 * i], params->grad + pl.poff[2 * i + 1],
                           nullptr, scr, s));
        break;
      }
      case K_ACT_VJP:
        CHECK(act_vjp(dt, net->ops[i].act, out_ptr(i + 1), grad_ptr(i + 1), grad_ptr(i + 1), pl.t[i + 1].elems, s));
        break;
      case K_DGRAD: {
        const int src = pl.t[net->ops[i].in].root;
        s4tf_conv_desc d = conv_desc(i, c.a);
        if (c.b >= 0)
          CHECK(conv_dgrad_impl(d, conv_w(i), grad_ptr(i + 1), grad_ptr(src), s, grad_ptr(c.b + 1),
                                reinterpret_cast<const unsigned char*>(ws + pl.mask_off[c.b])));
        else
          CHECK(conv_dgrad_impl(d, conv_w(i), grad_ptr(i + 1), grad_ptr(src), s));
        break;
      }
      case K_PARAM_GRADS: {  // filter (and bias) gradient of convolution i
        const s4tf_op& cv = net->ops[i];
        const TensorPlan& cin = pl.t[cv.in];
        s4tf_conv_desc d = conv_desc(i, 0);
        void* dyj = grad_ptr(i + 1);
        float* dbias = cv.has_bias ? params->grad + pl.poff[2 * i + 1] : nullptr;
        if (pl.fold[i]) {  // on the folded batch the forward pass left; the gradient of the folded filter is unfolded
          float* dwp = reinterpret_cast<float*>(ws + pl.dwpad_off[i]);
          CHECK(conv_param_grads_impl(folded_desc(d), ws + pl.xpad_off[i], dyj, dwp, dbias, wscratch, pl.wscratch_bytes, s));
          CHECK(unfold2_filter_grad(dwp, params->grad + pl.poff[2 * i], cv.r, cv.s, cin.c, cv.k, s));
          break;
        }
        if (pl.pad_c[i]) {  // the batch has no cotangent; the filter gradient of the padded channels is dropped
          d.c = pl.pad_c[i];
          float* dwp = reinterpret_cast<float*>(ws + pl.dwpad_off[i]);
          CHECK(conv_param_grads_impl(d, ws + pl.xpad_off[i], dyj, dwp, dbias, wscratch, pl.wscratch_bytes, s));
          CHECK(unpad_channels_f32(dwp, params->grad + pl.poff[2 * i], (long long)cv.r * cv.s, cin.c, pl.pad_c[i], cv.k, s));
          break;
        }
        CHECK(conv_param_grads_impl(d, act_ptr(cin.root), dyj, params->grad + pl.poff[2 * i], dbias, wscratch,
                                    pl.wscratch_bytes, s));
        break;
      }
      case K_BN_VJP: {
        const s4tf_op& op = net->ops[i];
        const TensorPlan& in = pl.t[op.in];
        const int src = in.root;
        const int rsrc = op.res >= 0 ? pl.t[op.res].root : -1;
        s4tf_bn_desc d = {in.n, in.h, in.w, in.c, op.eps, op.act, dt, c.a};
        float* stats = reinterpret_cast<float*>(ws + pl.stat_off[i]);
        void* dres = (rsrc > 0 && c.b != 1) ? grad_ptr(rsrc) : nullptr;
        // no residual in the forward pass: the pullback rebuilds the activation mask from x and skips y
        const float* beta = op.res < 0 ? params->master + pl.poff[2 * i + 1] : nullptr;
        CHECK(bn_vjp(d, act_ptr(src), out_ptr(i + 1), params->master + pl.poff[2 * i], beta, stats, stats + in.c,
                     grad_ptr(i + 1), grad_ptr(src), dres, params->grad + pl.poff[2 * i], params->grad + pl.poff[2 * i + 1], scr, s,
                     pl.mask_off[i] ? reinterpret_cast<const unsigned char*>(ws + pl.mask_off[i]) : nullptr));
        break;
      }
      case K_POOL_VJP: {
        const s4tf_op& op = net->ops[i];
        const TensorPlan& in = pl.t[op.in];
        const int src = in.root;
        s4tf_pool_desc d = {in.n, in.h, in.w, in.c, op.kind == S4TF_OP_AVGPOOL2 ? S4TF_POOL_AVG2 : S4TF_POOL_MAX3S2, dt, c.a};
        const unsigned char* pos = pool_saves_positions(d) ? reinterpret_cast<const unsigned char*>(ws + pl.stat_off[i]) : nullptr;
        CHECK(pool_vjp(d, act_ptr(src), grad_ptr(i + 1), grad_ptr(src), s, pos));
        break;
      }
      case K_SGD: {
        // the first op's parameters lie at the start of the arena, padded to 8 elements each
        const s4tf_op& op0 = net->ops[0];
        const size_t head = op0.has_bias ? (size_t)pl.poff[1] + align_up((size_t)pl.psize[1], 8) : align_up((size_t)pl.psize[0], 8);
        size_t lo = 0, hi = params->count;
        if (c.a == 1) lo = head;
        if (c.a == 2) hi = head;
        CHECK(sgd(hi - lo, params->master + lo, params->velocity + lo, params->grad + lo,
                  bf16 ? (void*)(static_cast<bf16_t*>(params->lowp) + lo) : nullptr, lr, net->momentum, st));
        break;
      }
      default:
        return fail(S4TF_ERR_UNSUPPORTED, "train step: unknown command %d", (int)c.kind);
    }
  }
  (void)nops;
  return join.now();
}

}  // namespace
}  // namespace s4tf

using namespace s4tf;

extern "C" {

int s4tf_net_create(const s4tf_net_desc* desc, s4tf_net** out) {
  clear_error();
  if (!out) return fail(S4TF_ERR_NULL, "out is NULL");
  *out = nullptr;
  if (!desc) return fail(S4TF_ERR_NULL, "net descriptor is NULL");
  if (!desc->ops || desc->n_ops <= 0) return fail(S4TF_ERR_NULL, "net has no ops");
  std::unique_ptr<s4tf_net> N;
  CHECK(build_net(desc, N));
  *out = N.release();
  return S4TF_OK;
}
void s4tf_net_destroy(s4tf_net* net) { delete net; }

size_t s4tf_net_schedule_length(const s4tf_net* net) { return net ? net->cmds.size() : 0; }
uint64_t s4tf_net_hash(const s4tf_net* net) { return net ? net->hash : 0; }

int s4tf_net_train_step(const s4tf_net* net, s4tf_params* params, const s4tf_batch* batch, float lr) {
  clear_error();
  if (!net) return fail(S4TF_ERR_NULL, "net is NULL");
  return run_step(*net, params, batch, lr);
}

size_t s4tf_net_param_count(const s4tf_net_desc* net) {
  clear_error();
  std::shared_ptr<s4tf_net> N;
  if (cached_net(net, N) != S4TF_OK) return 0;
  return N->pl.param_count;
}
int s4tf_net_param_layout(const s4tf_net_desc* net, int64_t* offsets, int64_t* sizes) {
  clear_error();
  std::shared_ptr<s4tf_net> N;
  CHECK(cached_net(net, N));
  for (size_t i = 0; i < N->pl.poff.size(); ++i) {
    if (offsets) offsets[i] = N->pl.poff[i];
    if (sizes) sizes[i] = N->pl.psize[i];
  }
  return S4TF_OK;
}
int s4tf_net_tensor_layout(const s4tf_net_desc* net, int64_t* act_off, int64_t* grad_off, int32_t* shape,
                           int64_t* stat_off) {
  clear_error();
  std::shared_ptr<s4tf_net> N;
  CHECK(cached_net(net, N));
  const NetPlan& pl = N->pl;
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
  std::shared_ptr<s4tf_net> N;
  if (cached_net(net, N) != S4TF_OK) return 0;
  return N->pl.total_bytes;
}

int s4tf_train_step(const s4tf_net_desc* net, s4tf_params* params, const s4tf_batch* batch, float lr) {
  clear_error();
  std::shared_ptr<s4tf_net> N;
  CHECK(cached_net(net, N));
  return run_step(*N, params, batch, lr);
}

}  // extern "C"
