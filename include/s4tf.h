/*
 * s4tf.h -- C ABI of the MI355X (gfx950) training-step library.
 *
 * The library computes one differentiated training step of a convolutional network:
 * forward pass, the pullbacks of every op in reverse order, and an in-place
 * SGD-momentum update.  That is the loop the paper writes in Section 4.2 (figure
 * "Training LeNet on a simple dataset"): `gradient(at: model) { softmaxCrossEntropy(
 * logits: model(batch.data), labels: batch.label) }` followed by
 * `optimizer.update(&model, along: gradients)`.  Every `*_vjp` entry point is one
 * pullback in the sense of Section 2.1: it maps the cotangent of an op's output to the
 * cotangents of its inputs and parameters; the tensors a pullback "captures" are passed
 * back in by the caller.  The step has the type `(inout Model, Minibatch) -> Void` of
 * Section 4.2: parameters and velocities are updated in place, no second copy of the
 * model is made.
 *
 * General rules (all entry points)
 *  - Every data pointer is a DEVICE pointer (HIP global memory) unless marked "host".
 *    Descriptor structs are host memory and are read before the call returns.
 *  - Layouts: activations NHWC; filters (R,S,C/groups,K) (the paper's
 *    `filterShape: (5, 5, 1, 6)` = (H,W,Cin,Cout)); dense weights [in,out], y = xW + b.
 *    Convolution is cross-correlation with symmetric zero padding,
 *    P = floor((H + 2*pad - R)/stride) + 1.
 *  - dtype is the storage type of activations, activation cotangents and the working
 *    copy of conv filters: S4TF_F32 (float) or S4TF_BF16 (bfloat16, round to nearest
 *    even on store, fp32 accumulation).  Parameter gradients, BatchNorm statistics,
 *    gamma/beta, biases, the whole head, master weights and velocities are always fp32.
 *  - Ownership: the caller allocates and frees every buffer, including workspaces.  The
 *    library keeps no pointer after the work it enqueued has completed.
 *  - Execution: all work is enqueued on `stream` (a hipStream_t passed as void*, NULL is
 *    the default stream).  No entry point synchronises the host.
 *  - Errors: every entry point returns an s4tf_status.  Arguments, shapes and everything a
 *    network's plan decides are validated before anything is launched: after any status but
 *    S4TF_ERR_DEVICE nothing was written.  S4TF_ERR_DEVICE (a launch, event or stream call
 *    failed half way) leaves the outputs, and for a train step the workspace, gradients and
 *    parameters, undefined.  A message is available from s4tf_last_error() (thread-local).
 *    No exception crosses the ABI.
 *  - Alignment: device pointers must be 16-byte aligned.  Outputs must not alias inputs
 *    except where documented (param/velocity of s4tf_sgd_momentum, the in-place update
 *    of s4tf_train_step).
 *  - Workspaces: each op that needs scratch memory has a `*_workspace_bytes` query; the
 *    caller passes at least that many bytes (16-byte aligned).  Contents are undefined
 *    on entry and on return.
 */
#ifndef S4TF_H
#define S4TF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  S4TF_OK = 0,
  S4TF_ERR_NULL = -1,        /* a required pointer is NULL */
  S4TF_ERR_SHAPE = -2,       /* non-positive size, empty output, inconsistent shapes */
  S4TF_ERR_DTYPE = -3,       /* unknown dtype / activation code */
  S4TF_ERR_UNSUPPORTED = -4, /* valid but not implemented (e.g. 1 < groups < C) */
  S4TF_ERR_WORKSPACE = -5,   /* workspace missing or too small */
  S4TF_ERR_DEVICE = -6,      /* HIP launch error */
  S4TF_ERR_ALIGN = -7        /* pointer not 16-byte aligned */
} s4tf_status;

typedef enum { S4TF_F32 = 0, S4TF_BF16 = 1 } s4tf_dtype;
typedef enum { S4TF_ACT_NONE = 0, S4TF_ACT_RELU = 1, S4TF_ACT_RELU6 = 2 } s4tf_act;

/* Convolution.  x is (n,h,w,c), w is (r,s,c/groups,k), y is (n,p,q,k).  groups must be 1
 * or c (depthwise, which also needs k == c and a filter of at most 3x3; anything else is refused
 * with S4TF_ERR_UNSUPPORTED before anything runs).  act is applied to conv + bias in the
 * forward pass (the `activation: relu` of the paper's Conv2D/Dense layers).
 * accumulate_dx != 0 makes the pullback ADD the input cotangent to what dx already holds
 * (the `inout` formulation of a pullback, Section 4.3) instead of overwriting it. */
typedef struct {
  int32_t n, h, w, c, k, r, s, stride, pad, groups;
  int32_t dtype; /* s4tf_dtype */
  int32_t act;   /* s4tf_act */
  int32_t accumulate_dx;
} s4tf_conv_desc;

/* BatchNorm (training mode, biased variance, eps inside the square root) + optional
 * residual add + activation over an (n,h,w,c) tensor. */
typedef struct {
  int32_t n, h, w, c;
  float eps;
  int32_t act;   /* s4tf_act */
  int32_t dtype; /* s4tf_dtype */
  int32_t accumulate_dres; /* pullback adds into dresidual instead of overwriting */
  int32_t accumulate_dx;   /* pullback adds into dx instead of overwriting (Section 4.3) */
} s4tf_bn_desc;

/* Head: global average pool over (h,w), dense c -> classes, mean softmax cross-entropy. */
typedef struct {
  int32_t n, h, w, c, classes;
  int32_t dtype; /* storage type of x and dx; W, b, loss and their gradients are fp32 */
  int32_t accumulate_dx; /* the pullback adds into dx instead of overwriting (Section 4.3) */
} s4tf_head_desc;

typedef enum { S4TF_POOL_AVG2 = 0, S4TF_POOL_MAX3S2 = 1 } s4tf_pool_kind;
/* AVG2: 2x2 window, stride 2, no padding (the paper's AvgPool2D(poolSize: (2,2),
 * strides: (2,2))).  MAX3S2: 3x3 window, stride 2, padding 1, padding never wins. */
typedef struct {
  int32_t n, h, w, c;
  int32_t kind;  /* s4tf_pool_kind */
  int32_t dtype; /* s4tf_dtype */
  int32_t accumulate_dx;
} s4tf_pool_desc;

/* Thread-local message for the last non-OK status returned on this thread ("" if none).
 * Host pointer to static storage; valid until the next library call on the thread. */
const char* s4tf_last_error(void);

/* ---- conv2d (Conv2D / Dense of the paper's Section 4.1 figure) -------------------------
 * fwd:  y[n,p,q,k] = act(bias[k] + sum_{r,s,c} x[n,p*stride+r-pad,q*stride+s-pad,c] w[r,s,c,k])
 * vjp:  dz = dy * act'(y)  (act' evaluated on the stored output: 0<y for relu, 0<y<6 for relu6)
 *       dx[n,h,w,c] (+)= sum_{r,s,k} dz[n,p,q,k] w[r,s,c,k]  over (p,q) with p*stride+r-pad = h ...
 *       dw[r,s,c,k]  = sum_{n,p,q} x[n,p*stride+r-pad,q*stride+s-pad,c] dz[n,p,q,k]   (fp32)
 *       dbias[k]     = sum_{n,p,q} dz[n,p,q,k]                                          (fp32)
 * x, w, y, dy, dx have the descriptor's dtype.  bias/dbias may be NULL.  y may be NULL in
 * vjp when act is NONE.  dx may be NULL (no consumer, e.g. the first layer).  dw and dbias
 * are overwritten.  A dense layer is the case h = w = r = s = 1. */
size_t s4tf_conv2d_fwd_workspace_bytes(const s4tf_conv_desc* d);
size_t s4tf_conv2d_vjp_workspace_bytes(const s4tf_conv_desc* d);
int s4tf_conv2d_fwd(const s4tf_conv_desc* d, const void* x, const void* w, const float* bias, void* y,
                    void* workspace, size_t workspace_bytes, void* stream);
int s4tf_conv2d_vjp(const s4tf_conv_desc* d, const void* x, const void* w, const void* y,
                    const void* dy, void* dx, float* dw, float* dbias, void* workspace,
                    size_t workspace_bytes, void* stream);

/* ---- BatchNorm + residual + activation ------------------------------------------------
 * fwd:  per channel over m = n*h*w: mean, var (biased), invstd = 1/sqrt(var + eps);
 *       xhat = (x - mean)*invstd;  z = gamma*xhat + beta (+ residual);  y = act(z);
 *       save_mean[c], save_invstd[c] are written for the pullback.
 * vjp:  dz = dy*act'(y);  dresidual (+)= dz;  dbeta = sum dz;  dgamma = sum dz*xhat;
 *       dx = gamma*invstd*(dz - dbeta/m - xhat*dgamma/m)
 * residual / dresidual may be NULL.  gamma, beta, statistics and their gradients are fp32
 * arrays of c elements.  y may be NULL in vjp when act is NONE.
 * beta in vjp is optional (NULL: act'(y) is read off y).  Give it only if the forward call had
 * no residual: with beta given and dresidual NULL the pullback rebuilds z = gamma*xhat + beta
 * from x with the forward pass's own arithmetic, takes act' from it and does not read y (which
 * may then be NULL): one tensor less to fetch. */
size_t s4tf_bn_relu_workspace_bytes(const s4tf_bn_desc* d);
int s4tf_bn_relu_fwd(const s4tf_bn_desc* d, const void* x, const void* residual, const float* gamma,
                     const float* beta, void* y, float* save_mean, float* save_invstd,
                     void* workspace, size_t workspace_bytes, void* stream);
/* s4tf_bn_relu_fwd for callers that cannot allocate device memory or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments without the
 * workspace, same kernels, same results bit for bit.  The statistics kernels' partial sums live in a
 * device array that is part of the library itself (1 MiB per GPU, held until the process ends); the call
 * allocates nothing, frees nothing and clears nothing.  A shape whose partial sums need more than that
 * (roughly: more than 131 072 channel x pixel-chunk pairs, e.g. 512 channels over 200 000 pixels) is
 * refused with S4TF_ERR_WORKSPACE before anything is launched; s4tf_bn_relu_fwd_static_limit returns the
 * capacity in bytes and, through `needed` (host, nullable), what the descriptor's shape needs.  All calls
 * on one GPU share the array: calls that overlap in time on one GPU (different streams or threads) race;
 * calls in one stream are ordered and need no care, nothing carries over from one call to the next. */
int s4tf_bn_relu_fwd_static(const s4tf_bn_desc* d, const void* x, const void* residual, const float* gamma,
                            const float* beta, void* y, float* save_mean, float* save_invstd, void* stream);
size_t s4tf_bn_relu_fwd_static_limit(const s4tf_bn_desc* d, size_t* needed);
int s4tf_bn_relu_vjp(const s4tf_bn_desc* d, const void* x, const void* y, const float* gamma,
                     const float* beta, const float* save_mean, const float* save_invstd, const void* dy, void* dx,
                     void* dresidual, float* dgamma, float* dbeta, void* workspace,
                     size_t workspace_bytes, void* stream);

/* ---- BatchNorm in inference mode ----------------------------------------------------------
 * For models that start from trained parameters (the paper's Section 1 motivates fine-tuning from
 * a checkpoint): running statistics take the place of batch statistics.
 *   s4tf_bn_inference_fwd   y = act(gamma (x - running_mean)/sqrt(running_var + eps) + beta (+ residual));
 *                           descriptor as for s4tf_bn_relu_fwd (eps from it), no workspace, nothing saved.
 *   s4tf_bn_update_running  after a training-mode forward pass over `count` = n*h*w samples per channel:
 *                           running_mean <- (1-momentum) running_mean + momentum save_mean
 *                           running_var  <- (1-momentum) running_var  + momentum var count/(count-1)
 *                           with var = 1/save_invstd^2 - eps the biased batch variance (so the running
 *                           variance averages unbiased estimates).  In place on the two running arrays.
 *   s4tf_bn_fold_into_conv  the convolution that equals "convolution (w, bias), then inference-mode
 *                           BatchNorm": w_out[r,s,c,k] = w[r,s,c,k] s_k, bias_out[k] = beta_k + (bias_k -
 *                           running_mean_k) s_k, s_k = gamma_k/sqrt(running_var_k + eps).  w, w_out have the
 *                           descriptor's dtype (w_out rounded on store) and shape (r,s,c/groups,k); bias is
 *                           nullable; bias_out is fp32 [k].  s4tf_conv2d_fwd with (w_out, bias_out) and the
 *                           BatchNorm's activation then runs the pair as one kernel.
 * gamma, beta and the statistics are fp32 arrays of c (fold: k) elements. */
int s4tf_bn_inference_fwd(const s4tf_bn_desc* d, const void* x, const void* residual, const float* gamma,
                          const float* beta, const float* running_mean, const float* running_var, void* y,
                          void* stream);
int s4tf_bn_update_running(int32_t c, size_t count, float momentum, float eps, const float* save_mean,
                           const float* save_invstd, float* running_mean, float* running_var, void* stream);
int s4tf_bn_fold_into_conv(const s4tf_conv_desc* d, const void* w, const float* bias, const float* gamma,
                           const float* beta, const float* running_mean, const float* running_var, float eps,
                           void* w_out, float* bias_out, void* stream);

/* ---- pooling ---------------------------------------------------------------------------
 * AVG2 fwd: mean of the window; vjp: dy/4 to each of the four inputs.
 * MAX3S2 fwd: maximum of the in-range window; vjp: the whole dy goes to the first maximum
 * in row-major window order (needs x). x may be NULL in vjp for AVG2. */
int s4tf_pool2d_fwd(const s4tf_pool_desc* d, const void* x, void* y, void* stream);
int s4tf_pool2d_vjp(const s4tf_pool_desc* d, const void* x, const void* dy, void* dx, void* stream);

/* ---- head: global-avg-pool + dense + softmax cross-entropy, value and pullback --------
 * (`softmaxCrossEntropy(logits:labels:)` of the paper's training loop, reduced to the
 * scalar `gradient(at:in:)` requires by a mean over the batch.)
 *   pbar[n,c] = mean_{h,w} x[n,h,w,c];  z = pbar W + b;
 *   loss = -(1/n) sum_n log softmax(z_n)[labels[n]]      (max-subtracted, fp32)
 *   dz = (softmax(z) - onehot(labels))/n;  dW = pbar^T dz;  db = sum_n dz;
 *   dx[n,h,w,c] = (dz W^T)[n,c] / (h*w)
 * W is fp32 [c,classes], b fp32 [classes], labels int32 [n] in [0,classes) (a label out
 * of range contributes no -1 term and no loss; it is the caller's error).  loss is one
 * fp32 device scalar.  dx may be NULL.  logits (nullable) receives z as fp32 [n,classes]. */
size_t s4tf_pool_dense_xent_workspace_bytes(const s4tf_head_desc* d);
int s4tf_pool_dense_xent_fwd_vjp(const s4tf_head_desc* d, const void* x, const float* W, const float* b,
                                 const int32_t* labels, float* loss, void* dx, float* dW, float* db,
                                 float* logits, void* workspace, size_t workspace_bytes,
                                 void* stream);

/* ---- indexing (gather of rows) and its pullback in the `inout` formulation ------------------
 * The paper's Section 4.3 (and its Appendix B listing) takes `x[i]` as the example: a pullback of
 * type (T) -> [T] must build a whole array of zeros to hold one value, O(n) per use, whereas the
 * formulation (T, inout [T]) -> Void adds the cotangent in place, O(1) per use.
 *   fwd:  y[j, :] = x[index[j], :]                      j = 0..count-1, rows of `cols` elements
 *   vjp:  dx[index[j], :] += dy[j, :]                   in order of j (deterministic also when an
 *         index repeats); dx is inout and only the gathered rows are touched: the work is
 *         count * cols, whatever the number of rows of x.
 * x, y, dy, dx have `dtype`; index is int32 [count] on the device with 0 <= index[j] < rows (an index
 * out of range is skipped in both directions: y[j,:] = 0, no update).  count may be 0. */
typedef struct {
  int32_t rows, cols, count;
  int32_t dtype; /* s4tf_dtype */
} s4tf_gather_desc;
int s4tf_gather_rows_fwd(const s4tf_gather_desc* d, const void* x, const int32_t* index, void* y, void* stream);
int s4tf_gather_rows_vjp(const s4tf_gather_desc* d, const void* dy, const int32_t* index, void* dx, void* stream);

/* ---- SGD with momentum, in place (`optimizer.update(&model, along: gradients)`) -------
 *   velocity <- momentum*velocity + grad;   param <- param - lr*velocity
 *   param_lowp[i] <- bf16(param[i])  when param_lowp is not NULL (working copy)
 * count may be 0 (no-op). param and velocity are updated in place. */
int s4tf_sgd_momentum(size_t count, float* param, float* velocity, const float* grad, void* param_lowp,
                      float lr, float momentum, void* stream);

/* ---- storage-type conversion --------------------------------------------------------------
 * dst[i] = bfloat16(src[i]), round to nearest even (NaN stays NaN): how a caller that holds fp32 data
 * produces the bf16 tensors this library reads (a batch, the initial working copy of the parameters),
 * with the same rounding the library applies to everything it stores in bf16.  src: count floats,
 * dst: count bf16 values, both device memory; count may be 0. */
int s4tf_round_to_bf16(size_t count, const float* src, void* dst, void* stream);

/* ---- whole step -------------------------------------------------------------------------
 * A network is a static list of ops in topological order; op i produces tensor i+1,
 * tensor 0 is the batch.  `in`/`res` name earlier tensors.  The last op must be the head
 * and every other tensor needs at least one consumer. */
typedef enum {
  S4TF_OP_CONV = 0,       /* uses k,r,s,stride,pad,groups,has_bias,act */
  S4TF_OP_BN = 1,         /* uses res (-1: none), act, eps */
  S4TF_OP_AVGPOOL2 = 2,
  S4TF_OP_MAXPOOL3S2 = 3,
  S4TF_OP_FLATTEN = 4,    /* (n,h,w,c) -> (n,1,1,h*w*c), a reinterpretation, no copy */
  S4TF_OP_HEAD = 5        /* uses k = classes */
} s4tf_op_kind;

typedef struct {
  int32_t kind; /* s4tf_op_kind */
  int32_t in;   /* input tensor id */
  int32_t res;  /* residual tensor id for BN, else -1 */
  int32_t k, r, s, stride, pad, groups, has_bias;
  int32_t act;  /* s4tf_act */
  float eps;
} s4tf_op;

typedef struct {
  int32_t n, h, w, c;   /* batch tensor shape */
  int32_t dtype;        /* s4tf_dtype of activations */
  int32_t n_ops;
  const s4tf_op* ops;   /* host array */
  float momentum;
} s4tf_net_desc;

/* Parameters live in one flat fp32 arena; each op's tensors sit at the offsets
 * s4tf_net_param_layout reports (op order; conv: filter then bias; BN: gamma then beta;
 * head: W then b; every tensor starts at a multiple of 8 elements, padding is zero and
 * stays zero).  grad has the same layout and is overwritten by the step.  lowp is the
 * bf16 working copy of the arena (same offsets); required when dtype is BF16 (it must
 * hold bf16(master) on entry and is refreshed by the update), ignored otherwise. */
typedef struct {
  float* master;   /* inout */
  float* velocity; /* inout */
  float* grad;     /* out */
  void* lowp;      /* inout, bf16, nullable for F32 nets */
  size_t count;    /* elements in each arena, = s4tf_net_param_count */
} s4tf_params;

typedef struct {
  const void* x;         /* (n,h,w,c) in the net's dtype */
  const int32_t* labels; /* int32 [n] */
  float* loss;           /* out: one fp32 device scalar */
  void* workspace;       /* activation stash, cotangents, scratch */
  size_t workspace_bytes;
  void* stream;
} s4tf_batch;

/* Host-side queries.  offsets/sizes (host arrays, 2 entries per op, nullable) receive the
 * arena offset and element count of the op's first and second parameter tensor (size 0 if
 * absent).  Return 0 / write nothing if the descriptor is invalid (see s4tf_last_error). */
size_t s4tf_net_param_count(const s4tf_net_desc* net);
int s4tf_net_param_layout(const s4tf_net_desc* net, int64_t* offsets, int64_t* sizes);
size_t s4tf_train_step_workspace_bytes(const s4tf_net_desc* net);

/* Where the step keeps its intermediates inside the workspace, for inspection and tests.
 * All arguments after `net` are nullable host arrays.  For tensor t in 0..n_ops-1 (the head's
 * output has no buffer): act_off[t] / grad_off[t] = byte offset of the activation / of its
 * cotangent, -1 for the batch and reinterpretations of it; shape[4t..4t+3] = n,h,w,c.
 * stat_off[i] (n_ops entries) = byte offset of BatchNorm op i's save_mean (c floats, followed
 * by save_invstd), -1 for other ops.  After a step every buffer still holds its final value. */
int s4tf_net_tensor_layout(const s4tf_net_desc* net, int64_t* act_off, int64_t* grad_off, int32_t* shape,
                           int64_t* stat_off);

/* One training step: forward, loss, pullbacks in reverse op order (cotangents of a tensor
 * with several consumers are summed in reverse consumer order), then one SGD-momentum
 * update of the whole arena.  Enqueues on batch->stream; never synchronises the host.
 * The parameter-gradient kernels of the convolutions run on a second stream that the
 * library creates once per device (default priority, kept until the process ends); the
 * step orders it after the work already queued on batch->stream and makes batch->stream
 * wait for it before the update, also when the step fails half way, so in stream order on
 * batch->stream the step is complete (and its workspace reusable) when its last kernel is.
 * Steps on the same device share that second stream (and take turns enqueuing).  A net whose convolutions add up to
 * less than 0.5 GFLOP per forward pass runs on batch->stream alone.  The step allocates no
 * memory, issues no memset and no synchronisation, so once the second stream exists (after
 * the first call on the device) a caller may capture a step in a HIP graph of its own:
 * the second stream is forked from batch->stream and joined back into it inside the call. */
int s4tf_train_step(const s4tf_net_desc* net, s4tf_params* params, const s4tf_batch* batch, float lr);

/* ---- planned networks ---------------------------------------------------------------------
 * A network is planned once: shapes, the parameter and workspace layout, which ops run beside
 * each other on the second stream, which cotangent accumulates into which, and the flat list
 * of launches and stream operations (the schedule) that a step then replays with the caller's
 * pointers.  The descriptor form of the calls above keeps its plans in a cache inside the
 * library, keyed by a hash of the descriptor (scalar fields and op records; the 32 most
 * recently planned nets are kept): the role the cache of compiled traces, keyed by a hash of
 * the trace, plays in the paper's Section 3.4, so that only the first step of a net pays for
 * planning.  s4tf_net_create gives a caller a plan of its own: *out (host pointer) is valid
 * until s4tf_net_destroy, independent of the cache and of the descriptor's memory, and may
 * be used by several threads at once (a step does not modify it).  s4tf_net_train_step is
 * s4tf_train_step on such a plan: same arguments, same kernels in the same order, bit-identical
 * results.  Every reason a net cannot be run (S4TF_ERR_SHAPE / _UNSUPPORTED / _DTYPE) is
 * reported by s4tf_net_create, respectively by the first descriptor call, before any launch.
 * Two-stream steps on one device are serialised by a lock held while a step is enqueued, so
 * several host threads may step (different workspaces) on one device.
 * s4tf_net_schedule_length: commands in the schedule; s4tf_net_hash: the cache key. */
typedef struct s4tf_net s4tf_net;
int s4tf_net_create(const s4tf_net_desc* desc, s4tf_net** out);
void s4tf_net_destroy(s4tf_net* net); /* NULL is allowed */
int s4tf_net_train_step(const s4tf_net* net, s4tf_params* params, const s4tf_batch* batch, float lr);
size_t s4tf_net_schedule_length(const s4tf_net* net);
uint64_t s4tf_net_hash(const s4tf_net* net);

/* ---- measurement hook -------------------------------------------------------------------
 * While enabled, every kernel launch made by this thread's calls is bracketed by a pair of
 * HIP events on its stream.  s4tf_profile_collect synchronises those events and adds up
 * elapsed milliseconds and launch counts per kernel class into host arrays of
 * S4TF_PROF_CLASSES entries, then clears the record. Class names: s4tf_profile_class_name. */
#define S4TF_PROF_CLASSES 16
int s4tf_profile_enable(int on);
int s4tf_profile_collect(double* ms, int64_t* launches);
/* What one such pair of events adds to the kernel between them: the mean elapsed time, in
 * milliseconds, of `reps` (1..4096) pairs around a one-wavefront kernel that waits 20 us on
 * the device's real-time counter, less those 20 us, on `stream` (a device stream handle as
 * void*, NULL = the default stream), written to *ms_per_pair (host).  Synchronises the
 * stream.  A kernel trace sees a kernel's execution only; the events also see its dispatch,
 * so elapsed - this is what compares with a trace. */
int s4tf_profile_bracket_overhead(void* stream, int reps, double* ms_per_pair);
const char* s4tf_profile_class_name(int cls);

#ifdef __cplusplus
}
#endif
#endif /* S4TF_H */
