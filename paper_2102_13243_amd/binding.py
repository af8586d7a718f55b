"""ctypes binding of libs4tf.so: the same entry points as include/s4tf.h, argument marshalling
only.  PyTorch is used for device memory and streams; every step of the path runs in the
library's HIP kernels.  There is no CPU fallback: if the library cannot be loaded, importing
the entry points raises."""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libs4tf.so")

S4TF_F32, S4TF_BF16 = 0, 1
ACT = {"none": 0, "relu": 1, "relu6": 2}
POOL_AVG2, POOL_MAX3S2 = 0, 1
OP_CONV, OP_BN, OP_AVGPOOL2, OP_MAXPOOL3S2, OP_FLATTEN, OP_HEAD = range(6)
PROF_CLASSES = 16

c_i32, c_f32, c_vp, c_sz = ctypes.c_int32, ctypes.c_float, ctypes.c_void_p, ctypes.c_size_t


class ConvDesc(ctypes.Structure):
    _fields_ = [(n, c_i32) for n in ("n", "h", "w", "c", "k", "r", "s", "stride", "pad", "groups", "dtype",
                                     "act", "accumulate_dx")]


class BnDesc(ctypes.Structure):
    _fields_ = [("n", c_i32), ("h", c_i32), ("w", c_i32), ("c", c_i32), ("eps", c_f32), ("act", c_i32),
                ("dtype", c_i32), ("accumulate_dres", c_i32), ("accumulate_dx", c_i32)]


class HeadDesc(ctypes.Structure):
    _fields_ = [(n, c_i32) for n in ("n", "h", "w", "c", "classes", "dtype", "accumulate_dx")]


class GatherDesc(ctypes.Structure):
    _fields_ = [(n, c_i32) for n in ("rows", "cols", "count", "dtype")]


class PoolDesc(ctypes.Structure):
    _fields_ = [(n, c_i32) for n in ("n", "h", "w", "c", "kind", "dtype", "accumulate_dx")]


class Op(ctypes.Structure):
    _fields_ = [(n, c_i32) for n in ("kind", "in_", "res", "k", "r", "s", "stride", "pad", "groups", "has_bias",
                                     "act")] + [("eps", c_f32)]


class NetDesc(ctypes.Structure):
    _fields_ = [("n", c_i32), ("h", c_i32), ("w", c_i32), ("c", c_i32), ("dtype", c_i32), ("n_ops", c_i32),
                ("ops", ctypes.POINTER(Op)), ("momentum", c_f32)]


class Params(ctypes.Structure):
    _fields_ = [("master", c_vp), ("velocity", c_vp), ("grad", c_vp), ("lowp", c_vp), ("count", c_sz)]


class Batch(ctypes.Structure):
    _fields_ = [("x", c_vp), ("labels", c_vp), ("loss", c_vp), ("workspace", c_vp), ("workspace_bytes", c_sz),
                ("stream", c_vp)]


_lib = None


class S4tfError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("s4tf status %d: %s" % (status, message))
        self.status = status


def lib():
    """Load libs4tf.so (building it first only if it has never been built)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from . import build as _build
        _build.build()
    L = ctypes.CDLL(LIB_PATH)
    P = ctypes.POINTER
    L.s4tf_last_error.restype = ctypes.c_char_p
    L.s4tf_last_error.argtypes = []
    for name in ("s4tf_conv2d_fwd_workspace_bytes", "s4tf_conv2d_vjp_workspace_bytes"):
        getattr(L, name).restype = c_sz
        getattr(L, name).argtypes = [P(ConvDesc)]
    L.s4tf_bn_relu_workspace_bytes.restype = c_sz
    L.s4tf_bn_relu_workspace_bytes.argtypes = [P(BnDesc)]
    L.s4tf_pool_dense_xent_workspace_bytes.restype = c_sz
    L.s4tf_pool_dense_xent_workspace_bytes.argtypes = [P(HeadDesc)]
    L.s4tf_conv2d_fwd.argtypes = [P(ConvDesc), c_vp, c_vp, c_vp, c_vp, c_vp, c_sz, c_vp]
    L.s4tf_conv2d_vjp.argtypes = [P(ConvDesc), c_vp, c_vp, c_vp, c_vp, c_vp, c_vp, c_vp, c_vp, c_sz, c_vp]
    L.s4tf_bn_relu_fwd.argtypes = [P(BnDesc), c_vp, c_vp, c_vp, c_vp, c_vp, c_vp, c_vp, c_vp, c_sz, c_vp]
    L.s4tf_bn_relu_vjp.argtypes = [P(BnDesc)] + [c_vp] * 12 + [c_sz, c_vp]
    L.s4tf_bn_relu_fwd_static.argtypes = [P(BnDesc)] + [c_vp] * 8
    L.s4tf_bn_relu_fwd_static.restype = ctypes.c_int
    L.s4tf_bn_relu_fwd_static_limit.argtypes = [P(BnDesc), P(c_sz)]
    L.s4tf_bn_relu_fwd_static_limit.restype = c_sz
    L.s4tf_pool2d_fwd.argtypes = [P(PoolDesc), c_vp, c_vp, c_vp]
    L.s4tf_pool2d_vjp.argtypes = [P(PoolDesc), c_vp, c_vp, c_vp, c_vp]
    L.s4tf_pool_dense_xent_fwd_vjp.argtypes = [P(HeadDesc)] + [c_vp] * 10 + [c_sz, c_vp]
    L.s4tf_sgd_momentum.argtypes = [c_sz, c_vp, c_vp, c_vp, c_vp, c_f32, c_f32, c_vp]
    L.s4tf_bn_inference_fwd.argtypes = [P(BnDesc)] + [c_vp] * 8
    L.s4tf_bn_inference_fwd.restype = ctypes.c_int
    L.s4tf_bn_update_running.argtypes = [c_i32, c_sz, c_f32, c_f32, c_vp, c_vp, c_vp, c_vp, c_vp]
    L.s4tf_bn_update_running.restype = ctypes.c_int
    L.s4tf_bn_fold_into_conv.argtypes = [P(ConvDesc)] + [c_vp] * 6 + [c_f32, c_vp, c_vp, c_vp]
    L.s4tf_bn_fold_into_conv.restype = ctypes.c_int
    L.s4tf_gather_rows_fwd.argtypes = [P(GatherDesc), c_vp, c_vp, c_vp, c_vp]
    L.s4tf_gather_rows_fwd.restype = ctypes.c_int
    L.s4tf_gather_rows_vjp.argtypes = [P(GatherDesc), c_vp, c_vp, c_vp, c_vp]
    L.s4tf_gather_rows_vjp.restype = ctypes.c_int
    L.s4tf_round_to_bf16.argtypes = [c_sz, c_vp, c_vp, c_vp]
    L.s4tf_round_to_bf16.restype = ctypes.c_int
    L.s4tf_net_param_count.restype = c_sz
    L.s4tf_net_param_count.argtypes = [P(NetDesc)]
    L.s4tf_net_param_layout.argtypes = [P(NetDesc), P(ctypes.c_int64), P(ctypes.c_int64)]
    L.s4tf_net_tensor_layout.argtypes = [P(NetDesc), P(ctypes.c_int64), P(ctypes.c_int64), P(c_i32), P(ctypes.c_int64)]
    L.s4tf_net_tensor_layout.restype = ctypes.c_int
    L.s4tf_train_step_workspace_bytes.restype = c_sz
    L.s4tf_train_step_workspace_bytes.argtypes = [P(NetDesc)]
    L.s4tf_train_step.argtypes = [P(NetDesc), P(Params), P(Batch), c_f32]
    L.s4tf_net_create.argtypes = [P(NetDesc), P(c_vp)]
    L.s4tf_net_create.restype = ctypes.c_int
    L.s4tf_net_destroy.argtypes = [c_vp]
    L.s4tf_net_destroy.restype = None
    L.s4tf_net_train_step.argtypes = [c_vp, P(Params), P(Batch), c_f32]
    L.s4tf_net_train_step.restype = ctypes.c_int
    L.s4tf_net_schedule_length.argtypes = [c_vp]
    L.s4tf_net_schedule_length.restype = c_sz
    L.s4tf_net_hash.argtypes = [c_vp]
    L.s4tf_net_hash.restype = ctypes.c_uint64
    L.s4tf_profile_enable.argtypes = [ctypes.c_int]
    L.s4tf_profile_collect.argtypes = [P(ctypes.c_double), P(ctypes.c_int64)]
    L.s4tf_profile_bracket_overhead.argtypes = [ctypes.c_void_p, ctypes.c_int, P(ctypes.c_double)]
    L.s4tf_profile_class_name.restype = ctypes.c_char_p
    L.s4tf_profile_class_name.argtypes = [ctypes.c_int]
    for name in ("s4tf_conv2d_fwd", "s4tf_conv2d_vjp", "s4tf_bn_relu_fwd", "s4tf_bn_relu_vjp", "s4tf_pool2d_fwd",
                 "s4tf_pool2d_vjp", "s4tf_pool_dense_xent_fwd_vjp", "s4tf_sgd_momentum", "s4tf_net_param_layout",
                 "s4tf_train_step", "s4tf_profile_enable", "s4tf_profile_collect"):
        getattr(L, name).restype = ctypes.c_int
    _lib = L
    return L


def last_error():
    return lib().s4tf_last_error().decode()


def _check(status):
    if status != 0:
        raise S4tfError(status, last_error())


def _p(t):
    """Device pointer of a torch tensor (or pass through ints / None)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


# ---- entry points, named as in s4tf.h ----------------------------------------------------------------
def s4tf_conv2d_fwd_workspace_bytes(d):
    return int(lib().s4tf_conv2d_fwd_workspace_bytes(ctypes.byref(d)))


def s4tf_conv2d_vjp_workspace_bytes(d):
    return int(lib().s4tf_conv2d_vjp_workspace_bytes(ctypes.byref(d)))


def s4tf_conv2d_fwd(d, x, w, bias, y, workspace=None, stream=None):
    _check(lib().s4tf_conv2d_fwd(ctypes.byref(d), _p(x), _p(w), _p(bias), _p(y), _p(workspace), _nbytes(workspace),
                                 _stream(stream)))


def s4tf_conv2d_vjp(d, x, w, y, dy, dx, dw, dbias, workspace=None, stream=None):
    _check(lib().s4tf_conv2d_vjp(ctypes.byref(d), _p(x), _p(w), _p(y), _p(dy), _p(dx), _p(dw), _p(dbias),
                                 _p(workspace), _nbytes(workspace), _stream(stream)))


def s4tf_bn_relu_workspace_bytes(d):
    return int(lib().s4tf_bn_relu_workspace_bytes(ctypes.byref(d)))


def s4tf_bn_relu_fwd(d, x, residual, gamma, beta, y, save_mean, save_invstd, workspace, stream=None):
    _check(lib().s4tf_bn_relu_fwd(ctypes.byref(d), _p(x), _p(residual), _p(gamma), _p(beta), _p(y), _p(save_mean),
                                  _p(save_invstd), _p(workspace), _nbytes(workspace), _stream(stream)))


def s4tf_bn_relu_fwd_static(d, x, residual, gamma, beta, y, save_mean, save_invstd, stream=None):
    _check(lib().s4tf_bn_relu_fwd_static(ctypes.byref(d), _p(x), _p(residual), _p(gamma), _p(beta), _p(y), _p(save_mean),
                                         _p(save_invstd), _stream(stream)))


def s4tf_bn_relu_fwd_static_limit(d):
    """(capacity of the static scratch in bytes, bytes the descriptor's shape needs)"""
    needed = c_sz(0)
    cap = lib().s4tf_bn_relu_fwd_static_limit(ctypes.byref(d), ctypes.byref(needed))
    return int(cap), int(needed.value)


def s4tf_bn_relu_vjp(d, x, y, gamma, beta, save_mean, save_invstd, dy, dx, dresidual, dgamma, dbeta, workspace,
                     stream=None):
    _check(lib().s4tf_bn_relu_vjp(ctypes.byref(d), _p(x), _p(y), _p(gamma), _p(beta), _p(save_mean), _p(save_invstd), _p(dy),
                                  _p(dx), _p(dresidual), _p(dgamma), _p(dbeta), _p(workspace), _nbytes(workspace),
                                  _stream(stream)))


def s4tf_pool2d_fwd(d, x, y, stream=None):
    _check(lib().s4tf_pool2d_fwd(ctypes.byref(d), _p(x), _p(y), _stream(stream)))


def s4tf_pool2d_vjp(d, x, dy, dx, stream=None):
    _check(lib().s4tf_pool2d_vjp(ctypes.byref(d), _p(x), _p(dy), _p(dx), _stream(stream)))


def s4tf_pool_dense_xent_workspace_bytes(d):
    return int(lib().s4tf_pool_dense_xent_workspace_bytes(ctypes.byref(d)))


def s4tf_pool_dense_xent_fwd_vjp(d, x, W, b, labels, loss, dx, dW, db, logits, workspace, stream=None):
    _check(lib().s4tf_pool_dense_xent_fwd_vjp(ctypes.byref(d), _p(x), _p(W), _p(b), _p(labels), _p(loss), _p(dx),
                                              _p(dW), _p(db), _p(logits), _p(workspace), _nbytes(workspace),
                                              _stream(stream)))


def s4tf_sgd_momentum(count, param, velocity, grad, param_lowp, lr, momentum, stream=None):
    _check(lib().s4tf_sgd_momentum(count, _p(param), _p(velocity), _p(grad), _p(param_lowp), lr, momentum,
                                   _stream(stream)))


def s4tf_bn_inference_fwd(d, x, residual, gamma, beta, running_mean, running_var, y, stream=None):
    _check(lib().s4tf_bn_inference_fwd(ctypes.byref(d), _p(x), _p(residual), _p(gamma), _p(beta), _p(running_mean),
                                       _p(running_var), _p(y), _stream(stream)))


def s4tf_bn_update_running(c, count, momentum, eps, save_mean, save_invstd, running_mean, running_var, stream=None):
    _check(lib().s4tf_bn_update_running(c, count, momentum, eps, _p(save_mean), _p(save_invstd), _p(running_mean),
                                        _p(running_var), _stream(stream)))


def s4tf_bn_fold_into_conv(d, w, bias, gamma, beta, running_mean, running_var, eps, w_out, bias_out, stream=None):
    _check(lib().s4tf_bn_fold_into_conv(ctypes.byref(d), _p(w), _p(bias), _p(gamma), _p(beta), _p(running_mean),
                                        _p(running_var), eps, _p(w_out), _p(bias_out), _stream(stream)))


def s4tf_gather_rows_fwd(d, x, index, y, stream=None):
    _check(lib().s4tf_gather_rows_fwd(ctypes.byref(d), _p(x), _p(index), _p(y), _stream(stream)))


def s4tf_gather_rows_vjp(d, dy, index, dx, stream=None):
    _check(lib().s4tf_gather_rows_vjp(ctypes.byref(d), _p(dy), _p(index), _p(dx), _stream(stream)))


def s4tf_round_to_bf16(count, src, dst, stream=None):
    _check(lib().s4tf_round_to_bf16(count, _p(src), _p(dst), _stream(stream)))


def to_bf16_device(t):
    """A bf16 device tensor with the values of the fp32 device tensor t, rounded by the library's kernel
    (torch only allocates the destination)."""
    import torch
    src = t.contiguous()
    dst = torch.empty(src.shape, dtype=torch.bfloat16, device=src.device)
    s4tf_round_to_bf16(src.numel(), src, dst)
    return dst


def s4tf_net_param_count(net_desc):
    return int(lib().s4tf_net_param_count(ctypes.byref(net_desc)))


def s4tf_net_param_layout(net_desc):
    n = 2 * net_desc.n_ops
    off = (ctypes.c_int64 * n)()
    size = (ctypes.c_int64 * n)()
    _check(lib().s4tf_net_param_layout(ctypes.byref(net_desc), off, size))
    return list(off), list(size)


def s4tf_net_tensor_layout(net_desc):
    n = net_desc.n_ops
    act, grad, stat = (ctypes.c_int64 * n)(), (ctypes.c_int64 * n)(), (ctypes.c_int64 * n)()
    shape = (c_i32 * (4 * n))()
    _check(lib().s4tf_net_tensor_layout(ctypes.byref(net_desc), act, grad, shape, stat))
    return list(act), list(grad), [tuple(shape[4 * t:4 * t + 4]) for t in range(n)], list(stat)


def s4tf_train_step_workspace_bytes(net_desc):
    return int(lib().s4tf_train_step_workspace_bytes(ctypes.byref(net_desc)))


def s4tf_train_step(net_desc, params, batch, lr):
    _check(lib().s4tf_train_step(ctypes.byref(net_desc), ctypes.byref(params), ctypes.byref(batch), lr))


def s4tf_net_create(net_desc):
    """Returns the handle (an integer address) of a plan of the net."""
    out = c_vp()
    _check(lib().s4tf_net_create(ctypes.byref(net_desc), ctypes.byref(out)))
    return out.value


def s4tf_net_destroy(handle):
    lib().s4tf_net_destroy(handle)


def s4tf_net_train_step(handle, params, batch, lr):
    _check(lib().s4tf_net_train_step(handle, ctypes.byref(params), ctypes.byref(batch), lr))


def s4tf_net_schedule_length(handle):
    return int(lib().s4tf_net_schedule_length(handle))


def s4tf_net_hash(handle):
    return int(lib().s4tf_net_hash(handle))


def s4tf_profile_enable(on):
    _check(lib().s4tf_profile_enable(1 if on else 0))


def s4tf_profile_bracket_overhead(stream=None, reps=256):
    ms = ctypes.c_double(0.0)
    _check(lib().s4tf_profile_bracket_overhead(stream, int(reps), ctypes.byref(ms)))
    return ms.value


def s4tf_profile_collect():
    ms = (ctypes.c_double * PROF_CLASSES)()
    cnt = (ctypes.c_int64 * PROF_CLASSES)()
    _check(lib().s4tf_profile_collect(ms, cnt))
    return {lib().s4tf_profile_class_name(i).decode(): (ms[i], cnt[i]) for i in range(PROF_CLASSES) if cnt[i]}


# ---- marshalling helpers --------------------------------------------------------------------------------
def make_net_desc(net):
    """s4tf_net_desc from the plain-dict description used by the workload generator.  Returns
    (desc, keepalive) -- keep `keepalive` referenced as long as desc is used."""
    ops = (Op * len(net["ops"]))()
    for o, src in zip(ops, net["ops"]):
        kind = src["kind"]
        o.in_ = src["in"]
        o.res = -1
        o.groups, o.stride = 1, 1
        if kind == "conv":
            o.kind = OP_CONV
            o.k, o.r, o.s, o.stride, o.pad, o.groups = src["k"], src["r"], src["s"], src["stride"], src["pad"], src["groups"]
            o.has_bias = 1 if src["bias"] else 0
            o.act = ACT[src["act"]]
        elif kind == "bn":
            o.kind = OP_BN
            o.res = src["res"]
            o.act = ACT[src["act"]]
            o.eps = src["eps"]
        elif kind == "avgpool2":
            o.kind = OP_AVGPOOL2
        elif kind == "maxpool3s2":
            o.kind = OP_MAXPOOL3S2
        elif kind == "flatten":
            o.kind = OP_FLATTEN
        elif kind == "head":
            o.kind = OP_HEAD
            o.k = src["classes"]
        else:
            raise ValueError(kind)
    n, h, w, c = net["input"]
    d = NetDesc(n, h, w, c, S4TF_BF16 if net["dtype"] == "bf16" else S4TF_F32, len(net["ops"]), ops, net["momentum"])
    return d, ops


class TrainState:
    """Device buffers of one network: parameter arenas, workspace, loss scalar.  Marshalling
    only: packs/unpacks the nested parameter lists of the workload generator into the flat
    arena layout the library reports."""

    def __init__(self, net, params, device="cuda:0"):
        import torch
        self.torch = torch
        self.net = net
        self.device = device
        self.desc, self._keep = make_net_desc(net)
        self.count = s4tf_net_param_count(self.desc)
        if self.count == 0:
            raise S4tfError(-2, last_error())
        self.offsets, self.sizes = s4tf_net_param_layout(self.desc)
        self.shapes = [[a.shape for a in p] for p in params]
        arena = self.pack(params)
        self.master = torch.from_numpy(arena).to(device)
        self.velocity = torch.zeros(self.count, dtype=torch.float32, device=device)
        self.grad = torch.zeros(self.count, dtype=torch.float32, device=device)
        self.lowp = None
        if net["dtype"] == "bf16":
            self.lowp = to_bf16_device(self.master)
        self.ws_bytes = s4tf_train_step_workspace_bytes(self.desc)
        self.workspace = torch.empty(max(self.ws_bytes, 16), dtype=torch.uint8, device=device)
        self.loss = torch.zeros(4, dtype=torch.float32, device=device)

    def pack(self, params):
        arena = np.zeros(self.count, np.float32)
        for i, p in enumerate(params):
            for j, a in enumerate(p):
                off, size = self.offsets[2 * i + j], self.sizes[2 * i + j]
                assert size == a.size, (i, j, size, a.size)
                arena[off:off + size] = np.asarray(a, np.float32).reshape(-1)
        return arena

    def unpack(self, arena):
        arena = np.asarray(arena)
        out = []
        for i, shp in enumerate(self.shapes):
            out.append([arena[self.offsets[2 * i + j]:self.offsets[2 * i + j] + self.sizes[2 * i + j]].reshape(s)
                        for j, s in enumerate(shp)])
        return out

    def upload_batch(self, x, labels):
        torch = self.torch
        xt = torch.from_numpy(np.ascontiguousarray(x, np.float32)).to(self.device)
        if self.net["dtype"] == "bf16":
            xt = to_bf16_device(xt)
        return xt, torch.from_numpy(np.ascontiguousarray(labels, np.int32)).to(self.device)

    def step(self, x_dev, labels_dev, lr=None, stream=None, handle=None):
        """One training step; with `handle` (from s4tf_net_create) through the planned-network entry point."""
        lr = self.net["lr"] if lr is None else lr
        p = Params(_p(self.master), _p(self.velocity), _p(self.grad), _p(self.lowp), self.count)
        b = Batch(_p(x_dev), _p(labels_dev), _p(self.loss), _p(self.workspace), self.ws_bytes, _stream(stream))
        if handle is not None:
            s4tf_net_train_step(handle, p, b, lr)
        else:
            s4tf_train_step(self.desc, p, b, lr)

    def _view(self, off, shape, dtype):
        torch = self.torch
        n = int(np.prod(shape))
        es = 2 if dtype == torch.bfloat16 else 4
        return self.workspace[off:off + n * es].view(dtype).view(*shape)

    def tensor(self, t, cotangent=False):
        """float64 host copy of the step's activation t (or of its cotangent) from the workspace."""
        if not hasattr(self, "_layout"):
            self._layout = s4tf_net_tensor_layout(self.desc)
        act, grad, shape, _ = self._layout
        off = (grad if cotangent else act)[t]
        if off < 0:
            raise ValueError("tensor %d has no buffer" % t)
        dt = self.torch.bfloat16 if self.net["dtype"] == "bf16" else self.torch.float32
        self.torch.cuda.synchronize()
        return self._view(off, shape[t], dt).to(self.torch.float32).cpu().numpy().astype(np.float64)

    def bn_stats(self, op):
        if not hasattr(self, "_layout"):
            self._layout = s4tf_net_tensor_layout(self.desc)
        _, _, shape, stat = self._layout
        c = shape[self.net["ops"][op]["in"]][3]
        self.torch.cuda.synchronize()
        v = self._view(stat[op], (2, c), self.torch.float32).cpu().numpy().astype(np.float64)
        return v[0], v[1]

    def results(self):
        """Synchronise and download loss, gradients, parameters and velocities (nested lists)."""
        self.torch.cuda.synchronize()
        return {"loss": float(self.loss[0].item()), "grads": self.unpack(self.grad.cpu().numpy()),
                "params": self.unpack(self.master.cpu().numpy()),
                "velocity": self.unpack(self.velocity.cpu().numpy())}
