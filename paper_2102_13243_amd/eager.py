"""Op-by-op execution of a training step through the per-op entry points of s4tf.h.

The paper runs a step either eagerly, one pre-compiled kernel per Tensor op dispatched by
the host as the program reaches it (Section 3.3, "Eager mode"), or as one fused, traced
program (Section 3.4, LazyTensor + XLA); its Table 3 compares the two on ResNet-56.  The
fused side of this library is `s4tf_train_step`.  This module is the eager side: the host
walks the op list, calls one entry point per op (conv2d_fwd, bn_relu_fwd, ..., then the
pullbacks in reverse order, then one SGD call per parameter tensor) and, with `sync=True`,
waits for the device after every call, as a host program that looks at each result would.
With `sync=False` the calls are only enqueued (the asynchronous dispatch the paper
describes for its eager mode).

Argument marshalling and op sequencing only: every number is computed by the library's
kernels.  Used by the eager-versus-fused ablation of bench.py and by the parity tests.
"""
import numpy as np

from . import binding as B


class EagerState(B.TrainState):
    """Same parameter arenas and `results()` as TrainState; `step` dispatches op by op."""

    def __init__(self, net, params, device="cuda:0", sync=True):
        super().__init__(net, params, device)
        torch = self.torch
        self.sync = sync
        self.workspace = None  # the fused step's stash is not used here
        self.ws_bytes = 0
        bf16 = net["dtype"] == "bf16"
        self.dt = torch.bfloat16 if bf16 else torch.float32
        code = B.S4TF_BF16 if bf16 else B.S4TF_F32
        _, _, shapes, _ = B.s4tf_net_tensor_layout(self.desc)
        ops = net["ops"]
        self.acts = [None] * (len(ops) + 1)
        self.cots = [None] * (len(ops) + 1)
        self.descs, self.stats = [], []
        ws = 16
        for i, op in enumerate(ops):
            n, h, w, c = shapes[op["in"]]
            kind, d = op["kind"], None
            if kind == "conv":
                d = B.ConvDesc(n, h, w, c, op["k"], op["r"], op["s"], op["stride"], op["pad"], op["groups"], code,
                               B.ACT[op["act"]], 0)
                ws = max(ws, B.s4tf_conv2d_fwd_workspace_bytes(d), B.s4tf_conv2d_vjp_workspace_bytes(d))
            elif kind == "bn":
                d = B.BnDesc(n, h, w, c, op["eps"], B.ACT[op["act"]], code, 0)
                ws = max(ws, B.s4tf_bn_relu_workspace_bytes(d))
            elif kind in ("avgpool2", "maxpool3s2"):
                d = B.PoolDesc(n, h, w, c, B.POOL_AVG2 if kind == "avgpool2" else B.POOL_MAX3S2, code, 0)
            elif kind == "head":
                d = B.HeadDesc(n, h, w, c, op["classes"], code)
                ws = max(ws, B.s4tf_pool_dense_xent_workspace_bytes(d))
            self.descs.append(d)
            self.stats.append(torch.empty((2, c), dtype=torch.float32, device=device) if kind == "bn" else None)
            if kind == "flatten":  # a reinterpretation: output and cotangent share the input's storage
                continue
            if kind != "head":
                self.acts[i + 1] = torch.empty(tuple(shapes[i + 1]), dtype=self.dt, device=device)
        # cotangents: one buffer per tensor that has a producer (the batch needs none)
        for t in range(1, len(ops)):
            if ops[t - 1]["kind"] != "flatten":
                self.cots[t] = torch.empty(tuple(shapes[t]), dtype=self.dt, device=device)
        for i, op in enumerate(ops):
            if op["kind"] == "flatten":
                self.acts[i + 1] = self.acts[op["in"]].view(tuple(shapes[i + 1]))
                self.cots[i + 1] = self.cots[op["in"]].view(tuple(shapes[i + 1]))
        self.op_ws = torch.empty(ws, dtype=torch.uint8, device=device)

    # ---- helpers ---------------------------------------------------------------------------------------
    def _call(self, fn, *args):
        fn(*args)
        if self.sync:
            self.torch.cuda.synchronize()

    def _param(self, arena, i, j):
        off, size = self.offsets[2 * i + j], self.sizes[2 * i + j]
        return arena[off:off + size] if size else None

    def _weights(self, i):
        """Filter of conv i in the net's storage type (the bf16 working copy for bf16 nets)."""
        return self._param(self.lowp if self.lowp is not None else self.master, i, 0)

    # ---- one step --------------------------------------------------------------------------------------
    def step(self, x_dev, labels_dev, lr=None, stream=None):
        lr = self.net["lr"] if lr is None else lr
        ops, acts, cots = self.net["ops"], self.acts, self.cots
        if self.net["ops"][0]["kind"] == "flatten":
            raise ValueError("the first op reinterprets the batch: give the batch in that shape instead")
        acts[0] = x_dev
        # forward, in op order
        for i, op in enumerate(ops):
            kind, d, x = op["kind"], self.descs[i], acts[op["in"]]
            if kind == "conv":
                self._call(B.s4tf_conv2d_fwd, d, x, self._weights(i), self._param(self.master, i, 1), acts[i + 1],
                           self.op_ws, stream)
            elif kind == "bn":
                res = acts[op["res"]] if op["res"] >= 0 else None
                self._call(B.s4tf_bn_relu_fwd, d, x, res, self._param(self.master, i, 0), self._param(self.master, i, 1),
                           acts[i + 1], self.stats[i][0], self.stats[i][1], self.op_ws, stream)
            elif kind in ("avgpool2", "maxpool3s2"):
                self._call(B.s4tf_pool2d_fwd, d, x, acts[i + 1], stream)
            elif kind == "head":  # value and pullback in one call, as in the header
                self._call(B.s4tf_pool_dense_xent_fwd_vjp, d, x, self._param(self.master, i, 0),
                           self._param(self.master, i, 1), labels_dev, self.loss, cots[op["in"]],
                           self._param(self.grad, i, 0), self._param(self.grad, i, 1), None, self.op_ws, stream)
        # pullbacks, in reverse order.  A tensor with several consumers gets its first contribution
        # written and the later ones added (the accumulate flags of the descriptors).
        written = [False] * (len(ops) + 1)
        written[ops[-1]["in"]] = True
        for i in range(len(ops) - 2, -1, -1):
            op = ops[i]
            kind, d, t = op["kind"], self.descs[i], op["in"]
            x, dy = acts[t], cots[i + 1]
            if not written[i + 1]:
                raise ValueError("tensor %d has no consumer" % (i + 1))
            if kind == "flatten":
                if written[t]:
                    raise NotImplementedError("a flattened tensor with another consumer")
                written[t] = True
                continue
            dx = cots[t] if t > 0 else None
            if kind == "conv":
                d.accumulate_dx = 1 if (dx is not None and written[t]) else 0
                y = acts[i + 1] if op["act"] != "none" else None
                self._call(B.s4tf_conv2d_vjp, d, x, self._weights(i), y, dy, dx, self._param(self.grad, i, 0),
                           self._param(self.grad, i, 1), self.op_ws, stream)
            elif kind == "bn":
                if t == 0 or written[t]:
                    raise NotImplementedError("BatchNorm on the batch or on a tensor with another consumer")
                r = op["res"]
                dres = cots[r] if r > 0 else None
                d.accumulate_dres = 1 if (dres is not None and written[r]) else 0
                # without a residual the pullback rebuilds the activation mask from x (beta given, y not read)
                beta = self._param(self.master, i, 1) if (r < 0 and op["act"] != "none") else None
                self._call(B.s4tf_bn_relu_vjp, d, x, acts[i + 1], self._param(self.master, i, 0), beta,
                           self.stats[i][0], self.stats[i][1], dy, dx, dres, self._param(self.grad, i, 0),
                           self._param(self.grad, i, 1), self.op_ws, stream)
                if r > 0:
                    written[r] = True
            else:  # pools
                if dx is not None:
                    d.accumulate_dx = 1 if written[t] else 0
                    self._call(B.s4tf_pool2d_vjp, d, x, dy, dx, stream)
            written[t] = True
        # optimizer: one update per parameter tensor
        for i in range(len(ops)):
            for j in range(2):
                size = self.sizes[2 * i + j]
                if size:
                    self._call(B.s4tf_sgd_momentum, size, self._param(self.master, i, j), self._param(self.velocity, i, j),
                               self._param(self.grad, i, j),
                               self._param(self.lowp, i, j) if self.lowp is not None else None, lr,
                               self.net["momentum"], stream)

    # ---- inspection (same interface as TrainState) ---------------------------------------------------------
    def tensor(self, t, cotangent=False):
        buf = (self.cots if cotangent else self.acts)[t]
        if buf is None:
            raise ValueError("tensor %d has no buffer" % t)
        self.torch.cuda.synchronize()
        return buf.to(self.torch.float32).cpu().numpy().astype(np.float64)

    def bn_stats(self, op):
        self.torch.cuda.synchronize()
        v = self.stats[op].cpu().numpy().astype(np.float64)
        return v[0], v[1]
