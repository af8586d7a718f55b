"""CPU oracle: Python front end of `s4tf_oracle.c` and the whole-step interpreter.

TEST INFRASTRUCTURE ONLY.  Only tests, the smoke check and the bench's `cpu_baseline`
leg may import this module; the product path never does.  It shares no code with the
GPU library.

`train_step` follows the paper's training loop (Section 4.2, figure "Training LeNet on
a simple dataset"): forward through the op list, the scalar mean softmax cross-entropy,
the pullbacks in reverse order (each op's VJP maps the output cotangent to input and
parameter cotangents, Section 2.1), then the optimizer update.  All arithmetic is
float64.  For bf16 workloads every tensor that the GPU library stores in bf16
(activations, activation cotangents, working copies of conv filters) is rounded to the
bf16 grid at the same places; everything else (statistics, parameter gradients, the
head, master weights, velocities) stays float64.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "s4tf_oracle.c")
_LIB = os.path.join(_HERE, "liborc.so")
_ACT = {"none": 0, "relu": 1, "relu6": 2}


def build(force=False):
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O3", "-march=x86-64-v3", "-fopenmp", "-fPIC", "-shared",
                               "-std=c11", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.orc_num_threads.restype = ctypes.c_int
    return _lib


def num_threads():
    return int(lib().orc_num_threads())


def _d(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double)) if a is not None else None


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


_ci = ctypes.c_int
_cs = ctypes.c_size_t
_cd = ctypes.c_double


def round_bf16(a, inplace=False, slow=False):
    out = _f64(a)
    if not inplace or out is not a:
        out = out.copy()
    (lib().orc_round_bf16_slow if slow else lib().orc_round_bf16)(_d(out), _cs(out.size))
    return out


def conv2d_fwd(x, w, bias, stride, pad, groups=1):
    x, w = _f64(x), _f64(w)
    n, h, wd, c = x.shape
    r, s, cg, k = w.shape
    assert cg * groups == c and k % groups == 0
    p = (h + 2 * pad - r) // stride + 1
    q = (wd + 2 * pad - s) // stride + 1
    y = np.empty((n, p, q, k), np.float64)
    b = _f64(bias) if bias is not None else None
    lib().orc_conv2d_fwd(_d(x), _d(w), _d(b), _d(y), _ci(n), _ci(h), _ci(wd), _ci(c), _ci(k),
                         _ci(r), _ci(s), _ci(stride), _ci(pad), _ci(groups))
    return y


def conv2d_vjp(x, w, dy, stride, pad, groups=1, need_dx=True, need_db=False):
    x, w, dy = _f64(x), _f64(w), _f64(dy)
    n, h, wd, c = x.shape
    r, s, cg, k = w.shape
    dx = np.empty_like(x) if need_dx else None
    dw = np.empty_like(w)
    db = np.empty(k, np.float64) if need_db else None
    lib().orc_conv2d_vjp(_d(x), _d(w), _d(dy), _d(dx), _d(dw), _d(db), _ci(n), _ci(h), _ci(wd),
                         _ci(c), _ci(k), _ci(r), _ci(s), _ci(stride), _ci(pad), _ci(groups))
    return dx, dw, db


def bias_act_fwd(x, bias, act):
    x = _f64(x)
    c = x.shape[-1]
    y = np.empty_like(x)
    b = _f64(bias) if bias is not None else None
    lib().orc_bias_act_fwd(_d(x), _d(b), _d(y), _cs(x.size // c), _ci(c), _ci(_ACT[act]))
    return y


def bias_act_vjp(y, dy, act, need_db=True):
    y, dy = _f64(y), _f64(dy)
    c = y.shape[-1]
    dx = np.empty_like(y)
    db = np.empty(c, np.float64) if need_db else None
    lib().orc_bias_act_vjp(_d(y), _d(dy), _d(dx), _d(db), _cs(y.size // c), _ci(c), _ci(_ACT[act]))
    return dx, db


def bn_act_fwd(x, res, gamma, beta, eps, act):
    x, gamma, beta = _f64(x), _f64(gamma), _f64(beta)
    res = _f64(res) if res is not None else None
    c = x.shape[-1]
    y = np.empty_like(x)
    mean = np.empty(c, np.float64)
    invstd = np.empty(c, np.float64)
    lib().orc_bn_act_fwd(_d(x), _d(res), _d(gamma), _d(beta), _d(y), _d(mean), _d(invstd),
                         _cs(x.size // c), _ci(c), _cd(eps), _ci(_ACT[act]))
    return y, mean, invstd


def bn_act_vjp(x, y, gamma, mean, invstd, dy, act, need_dres):
    x, y, gamma, dy = _f64(x), _f64(y), _f64(gamma), _f64(dy)
    c = x.shape[-1]
    dx = np.empty_like(x)
    dres = np.empty_like(x) if need_dres else None
    dgamma = np.empty(c, np.float64)
    dbeta = np.empty(c, np.float64)
    lib().orc_bn_act_vjp(_d(x), _d(y), _d(gamma), _d(_f64(mean)), _d(_f64(invstd)), _d(dy), _d(dx),
                         _d(dres), _d(dgamma), _d(dbeta), _cs(x.size // c), _ci(c), _ci(_ACT[act]))
    return dx, dres, dgamma, dbeta


def avgpool2_fwd(x):
    x = _f64(x)
    n, h, w, c = x.shape
    y = np.empty((n, h // 2, w // 2, c), np.float64)
    lib().orc_avgpool2_fwd(_d(x), _d(y), _ci(n), _ci(h), _ci(w), _ci(c))
    return y


def avgpool2_vjp(dy, x_shape):
    dy = _f64(dy)
    n, h, w, c = x_shape
    dx = np.empty(x_shape, np.float64)
    lib().orc_avgpool2_vjp(_d(dy), _d(dx), _ci(n), _ci(h), _ci(w), _ci(c))
    return dx


def maxpool3s2_fwd(x):
    x = _f64(x)
    n, h, w, c = x.shape
    y = np.empty((n, (h - 1) // 2 + 1, (w - 1) // 2 + 1, c), np.float64)
    lib().orc_maxpool3s2_fwd(_d(x), _d(y), _ci(n), _ci(h), _ci(w), _ci(c))
    return y


def maxpool3s2_vjp(x, dy):
    x, dy = _f64(x), _f64(dy)
    n, h, w, c = x.shape
    dx = np.empty_like(x)
    lib().orc_maxpool3s2_vjp(_d(x), _d(dy), _d(dx), _ci(n), _ci(h), _ci(w), _ci(c))
    return dx


def head_fwd_vjp(x, W, b, labels, need_dx=True):
    x, W, b = _f64(x), _f64(W), _f64(b)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    n, h, w, c = x.shape
    classes = W.shape[1]
    loss = ctypes.c_double(0.0)
    dx = np.empty_like(x) if need_dx else None
    dW = np.empty_like(W)
    db = np.empty_like(b)
    logits = np.empty((n, classes), np.float64)
    lib().orc_head_fwd_vjp(_d(x), _d(W), _d(b), labels.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                           ctypes.byref(loss), _d(dx), _d(dW), _d(db), _d(logits), _ci(n), _ci(h),
                           _ci(w), _ci(c), _ci(classes))
    return float(loss.value), dx, dW, db, logits


def sgd_momentum(param, velocity, grad, lr, momentum):
    """In place on float64 arrays."""
    assert param.dtype == np.float64 and velocity.dtype == np.float64
    g = _f64(grad)
    lib().orc_sgd_momentum(_cs(param.size), _d(param), _d(velocity), _d(g), _cd(lr), _cd(momentum))


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def gather_rows_fwd(x, index):
    """y[j,:] = x[index[j],:] for a 2-D x."""
    x = _f64(x)
    idx, ip = _i32(index)
    y = np.empty((idx.size, x.shape[1]), np.float64)
    lib().orc_gather_rows_fwd(_d(x), ip, _d(y), _ci(x.shape[0]), _ci(x.shape[1]), _ci(idx.size))
    return y


def gather_rows_vjp(dy, index, dx):
    """In place on the float64 array dx: dx[index[j],:] += dy[j,:], in order of j."""
    assert dx.dtype == np.float64 and dx.flags["C_CONTIGUOUS"]
    dy = _f64(dy)
    idx, ip = _i32(index)
    lib().orc_gather_rows_vjp(_d(dy), ip, _d(dx), _ci(dx.shape[0]), _ci(dx.shape[1]), _ci(idx.size))


def bn_inference_fwd(x, res, gamma, beta, running_mean, running_var, eps, act):
    x = _f64(x)
    res = _f64(res) if res is not None else None
    c = x.shape[-1]
    y = np.empty_like(x)
    lib().orc_bn_inference_fwd(_d(x), _d(res), _d(_f64(gamma)), _d(_f64(beta)), _d(_f64(running_mean)),
                               _d(_f64(running_var)), _d(y), _cs(x.size // c), _ci(c), _cd(eps), _ci(_ACT[act]))
    return y


def bn_update_running(mean, invstd, running_mean, running_var, count, momentum, eps):
    """Returns the updated (running_mean, running_var); count = samples per channel of the batch."""
    rm, rv = _f64(running_mean).copy(), _f64(running_var).copy()
    lib().orc_bn_update_running(_d(_f64(mean)), _d(_f64(invstd)), _d(rm), _d(rv), _ci(rm.size), _cs(count),
                                _cd(momentum), _cd(eps))
    return rm, rv


def bn_fold(w, bias, gamma, beta, running_mean, running_var, eps):
    """Filter and bias of the convolution that equals conv(w, bias) followed by inference-mode BatchNorm."""
    w = _f64(w)
    k = w.shape[-1]
    w_out, b_out = np.empty_like(w), np.empty(k, np.float64)
    b = _f64(bias) if bias is not None else None
    lib().orc_bn_fold(_d(w), _d(b), _d(_f64(gamma)), _d(_f64(beta)), _d(_f64(running_mean)), _d(_f64(running_var)),
                      _d(w_out), _d(b_out), _cs(w.size // k), _ci(k), _cd(eps))
    return w_out, b_out


# --------------------------------------------------------------------------------------
# whole step
# --------------------------------------------------------------------------------------
def forward(net, x, params, keep=True):
    """Forward pass only.  Returns (tensors, saved) where tensors[t] is tensor t (the last
    entry is the head's input; the head itself is evaluated in `train_step`)."""
    rnd = (lambda a: round_bf16(a, inplace=True)) if net["dtype"] == "bf16" else (lambda a: a)
    tensors = [_f64(x)]
    saved = []
    for op, p in zip(net["ops"], params):
        kind = op["kind"]
        xin = tensors[op["in"]]
        sv = None
        if kind == "conv":
            w_used = round_bf16(p[0]) if net["dtype"] == "bf16" else _f64(p[0])
            bias = _f64(p[1]) if op["bias"] else None
            y = conv2d_fwd(xin, w_used, bias, op["stride"], op["pad"], op["groups"])
            if op["act"] != "none":
                y = bias_act_fwd(y, None, op["act"])
            y = rnd(y)
            sv = w_used
        elif kind == "bn":
            res = tensors[op["res"]] if op["res"] >= 0 else None
            y, mean, invstd = bn_act_fwd(xin, res, p[0], p[1], op["eps"], op["act"])
            y = rnd(y)
            sv = (mean, invstd)
        elif kind == "avgpool2":
            y = rnd(avgpool2_fwd(xin))
        elif kind == "maxpool3s2":
            y = maxpool3s2_fwd(xin)
        elif kind == "flatten":
            y = xin.reshape(xin.shape[0], 1, 1, -1)
        elif kind == "head":
            y = None
        else:
            raise ValueError(kind)
        tensors.append(y)
        saved.append(sv)
    return tensors, saved


def train_step(net, x, labels, params, velocity=None, lr=None, momentum=None, keep_cotangents=False):
    """One differentiated training step.  `params` is the nested list of arrays from the
    workload generator (any float dtype); nothing is modified in place.  Returns a dict:
    loss, logits, grads, params (updated), velocity (updated), tensors and, when
    keep_cotangents is set, cotangents: {tensor id: the finished cotangent its producer's
    pullback received} (otherwise each is dropped once it has been used)."""
    lr = net["lr"] if lr is None else lr
    momentum = net["momentum"] if momentum is None else momentum
    rnd = (lambda a: round_bf16(a, inplace=True)) if net["dtype"] == "bf16" else (lambda a: a)
    ops = net["ops"]
    assert ops[-1]["kind"] == "head"
    tensors, saved = forward(net, x, params)
    grads = [[None] * len(p) for p in params]
    cot = {}
    kept = {}

    def contribute(t, g):
        if t == 0 or g is None:
            return
        cot[t] = rnd(cot[t] + g) if t in cot else rnd(g)

    hop = ops[-1]
    loss, dx, dW, db, logits = head_fwd_vjp(tensors[hop["in"]], params[-1][0], params[-1][1], labels,
                                            need_dx=hop["in"] != 0)
    grads[-1] = [dW, db]
    contribute(hop["in"], dx)
    for i in range(len(ops) - 2, -1, -1):
        op, p = ops[i], params[i]
        kind = op["kind"]
        tin = op["in"]
        dy = cot.pop(i + 1, None)
        if dy is None:
            raise ValueError("op %d output has no consumer" % i)
        if keep_cotangents:
            kept[i + 1] = dy
        xin, y = tensors[tin], tensors[i + 1]
        if kind == "conv":
            dz, dbias = dy, None
            if op["act"] != "none":
                dz, _ = bias_act_vjp(y, dy, op["act"], need_db=False)
            dxi, dw, dbias = conv2d_vjp(xin, saved[i], dz, op["stride"], op["pad"], op["groups"],
                                        need_dx=tin != 0, need_db=op["bias"])
            grads[i] = [dw] + ([dbias] if op["bias"] else [])
            contribute(tin, dxi)
        elif kind == "bn":
            mean, invstd = saved[i]
            dxi, dres, dgamma, dbeta = bn_act_vjp(xin, y, p[0], mean, invstd, dy, op["act"],
                                                  need_dres=op["res"] >= 0)
            grads[i] = [dgamma, dbeta]
            # the residual tensor was consumed after this op's input in forward order, so its
            # cotangent is contributed first
            if op["res"] >= 0:
                contribute(op["res"], dres)
            contribute(tin, dxi)
        elif kind == "avgpool2":
            contribute(tin, avgpool2_vjp(dy, xin.shape))
        elif kind == "maxpool3s2":
            contribute(tin, maxpool3s2_vjp(xin, dy))
        elif kind == "flatten":
            contribute(tin, dy.reshape(xin.shape))
    new_params, new_vel = [], []
    for i, p in enumerate(params):
        np_, nv_ = [], []
        for j, a in enumerate(p):
            th = _f64(a).copy()
            v = _f64(velocity[i][j]).copy() if velocity is not None else np.zeros_like(th)
            sgd_momentum(th.reshape(-1), v.reshape(-1), grads[i][j].reshape(-1), lr, momentum)
            np_.append(th)
            nv_.append(v)
        new_params.append(np_)
        new_vel.append(nv_)
    return {"loss": loss, "logits": logits, "grads": grads, "params": new_params,
            "velocity": new_vel, "tensors": tensors, "cotangents": kept}
