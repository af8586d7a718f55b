"""Local consistency of one finished GPU training step against the CPU oracle.

A deep ReLU network is chaotic in the numerical sense: two correct implementations that differ
only in summation order drift apart layer by layer (a rounding difference flips a ReLU mask or a
bf16 rounding, the flipped element changes everything downstream).  Comparing the two end to end
therefore measures that drift, not correctness.  This checker instead takes every op of the step
on its own: the op's INPUTS are the tensors the GPU itself produced (read back from the step's
workspace), its expected OUTPUT is the oracle's op applied to those inputs, and that is compared
with what the GPU stored.  A chain of steps that are each correct is correct as a whole, and each
comparison is as tight as a single-op test.  Big convolutions are checked on sampled output
pixels / filter slices, each computed from the plain definition; everything else in full
(`full_flops=float("inf")` checks every convolution in full: the full-size headline workload does).
Every comparison is norm-wise (relative L2, the gate; relative max-norm reported) and element by
element (parity_metrics.py), so that a wrong row inside a large tensor cannot hide in the norm.
"""
import numpy as np

from oracle import oracle as orc
from parity_metrics import rel_l2, rel_inf, check_tensor, elementwise_f32

FULL_FLOPS = 3e9   # convolutions cheaper than this are checked on every output element


def _act(z, act):
    if act == "relu":
        return np.maximum(z, 0.0)
    if act == "relu6":
        return np.clip(z, 0.0, 6.0)
    return z


def _mask(y, act):
    if act == "relu":
        return (y > 0).astype(np.float64)
    if act == "relu6":
        return ((y > 0) & (y < 6)).astype(np.float64)
    return np.ones_like(y)


def conv_rows_fwd(x, w, bias, op, pos):
    """y[n,p,q,:] from the definition for each (n,p,q) in pos."""
    r_, s_, cg, k_ = w.shape
    st, pad, dw = op["stride"], op["pad"], op["groups"] > 1
    out = np.zeros((len(pos), k_))
    _, h_, w_, c_ = x.shape
    for i, (n, p, q) in enumerate(pos):
        acc = np.zeros(k_) if bias is None else np.array(bias, np.float64)
        for r in range(r_):
            hh = p * st + r - pad
            if hh < 0 or hh >= h_:
                continue
            for s in range(s_):
                ww = q * st + s - pad
                if ww < 0 or ww >= w_:
                    continue
                acc = acc + (x[n, hh, ww] * w[r, s, 0] if dw else x[n, hh, ww] @ w[r, s])
        out[i] = acc
    return out


def conv_rows_dgrad(dz, w, op, xshape, pos):
    """dx[n,h,w,:] from the definition for each (n,h,w) in pos."""
    r_, s_, cg, k_ = w.shape
    st, pad, dw = op["stride"], op["pad"], op["groups"] > 1
    _, p_, q_, _ = dz.shape
    out = np.zeros((len(pos), xshape[3]))
    for i, (n, h, ww) in enumerate(pos):
        acc = np.zeros(xshape[3])
        for r in range(r_):
            hp = h + pad - r
            if hp < 0 or hp % st or hp // st >= p_:
                continue
            for s in range(s_):
                wp = ww + pad - s
                if wp < 0 or wp % st or wp // st >= q_:
                    continue
                d = dz[n, hp // st, wp // st]
                acc = acc + (d * w[r, s, 0] if dw else w[r, s] @ d)
        out[i] = acc
    return out


class LocalChecker:
    def __init__(self, net, wl, state, samples=192, seed=0, full_flops=None, progress=None):
        self.net, self.wl, self.st = net, wl, state
        self.full_flops = full_flops
        self.progress = progress or (lambda msg: None)
        self.ops = net["ops"]
        self.bf16 = net["dtype"] == "bf16"
        self.rnd = (lambda a: orc.round_bf16(a)) if self.bf16 else (lambda a: a)
        self.tol_act = 5e-3 if self.bf16 else 3e-5
        self.tol_par = 2e-3 if self.bf16 else 2e-4
        self.samples = samples
        self.rng = np.random.default_rng(seed)
        self.x = np.asarray(wl["x"], np.float64)
        self.report = []
        self.detail = []   # (what, rel-L2, bound, rel-inf, element-wise summary) of every tensor comparison
        # resolve flatten aliases
        self.root = [0]
        for i, op in enumerate(self.ops):
            self.root.append(self.root[op["in"]] if op["kind"] == "flatten" else i + 1)
        self.shapes = None

    # -- data access -----------------------------------------------------------------------------
    def act(self, t):
        r = self.root[t]
        a = self.x if r == 0 else self.st.tensor(r)
        if r != t:
            a = a.reshape(a.shape[0], 1, 1, -1) if self.ops[t - 1]["kind"] == "flatten" else a
        return a

    def cot(self, t):
        return self.st.tensor(self.root[t], cotangent=True)

    def note(self, what, err, tol):
        """A scalar measure against its bound."""
        self.report.append((what, err, tol))
        assert err <= tol, "%s: %.3g > %.3g" % (what, err, tol)

    def tensor_check(self, what, got, ref, tol, lowp=None, atol=None, atol_extra=None, operand_scale=None):
        """A tensor against the oracle's: relative L2 against tol, and every element (lowp: the tensor is
        stored in bf16, ref is already rounded; default: the net's storage type)."""
        rec = check_tensor(what, got, ref, self.bf16 if lowp is None else lowp, tol, atol, atol_extra, operand_scale)
        self.report.append((rec[0], rec[1], rec[2]))
        self.detail.append(rec)

    def conv_w(self, i):
        w = np.asarray(self.wl["params"][i][0], np.float64)
        return orc.round_bf16(w) if self.bf16 else w

    def conv_is_small(self, op, xshape, yshape):
        flops = 2.0 * yshape[0] * yshape[1] * yshape[2] * yshape[3] * op["r"] * op["s"] * xshape[3] / op["groups"]
        return flops <= (FULL_FLOPS if self.full_flops is None else self.full_flops) or op["groups"] > 1

    # -- forward -----------------------------------------------------------------------------------
    def check_forward(self):
        for i, op in enumerate(self.ops[:-1]):
            kind = op["kind"]
            if kind == "flatten":
                continue
            self.progress("%s: checking the forward pass, op %d of %d" % (self.net["name"], i, len(self.ops)))
            x = self.act(op["in"])
            y = self.act(i + 1)
            p = self.wl["params"][i]
            if kind == "conv":
                w = self.conv_w(i)
                bias = np.asarray(p[1], np.float64) if op["bias"] else None
                if self.conv_is_small(op, x.shape, y.shape):
                    ref = self.rnd(_act(orc.conv2d_fwd(x, w, bias, op["stride"], op["pad"], op["groups"]), op["act"]))
                    self.tensor_check("op %d conv fwd" % i, y, ref, self.tol_act)
                else:
                    n_, p_, q_, _ = y.shape
                    pos = np.stack([self.rng.integers(0, n_, self.samples), self.rng.integers(0, p_, self.samples),
                                    self.rng.integers(0, q_, self.samples)], 1)
                    pos[0] = (0, 0, 0)
                    pos[1] = (n_ - 1, p_ - 1, q_ - 1)
                    ref = self.rnd(_act(conv_rows_fwd(x, w, bias, op, pos), op["act"]))
                    got = y[pos[:, 0], pos[:, 1], pos[:, 2]]
                    self.tensor_check("op %d conv fwd (sampled)" % i, got, ref, self.tol_act)
            elif kind == "bn":
                res = self.act(op["res"]) if op["res"] >= 0 else None
                ref, mean, invstd = orc.bn_act_fwd(x, res, p[0], p[1], op["eps"], op["act"])
                gm, gi = self.st.bn_stats(i)
                # in units of the channel's standard deviation (a mean can be exactly zero: BatchNorm
                # without activation followed by a 1x1 convolution)
                self.note("op %d bn mean" % i, float(np.max(np.abs(gm - mean) * invstd)), 2e-5)
                self.note("op %d bn invstd" % i, float(np.max(np.abs(gi - invstd) / invstd)), 5e-5)
                self.tensor_check("op %d bn fwd" % i, y, self.rnd(ref), self.tol_act)
            elif kind == "avgpool2":
                self.tensor_check("op %d avgpool fwd" % i, y, self.rnd(orc.avgpool2_fwd(x)), self.tol_act)
            elif kind == "maxpool3s2":
                assert np.array_equal(y, orc.maxpool3s2_fwd(x)), "op %d maxpool fwd: not bit-exact" % i
                self.report.append(("op %d maxpool fwd" % i, 0.0, 0.0))

    # -- head + backward ------------------------------------------------------------------------------
    def check_backward(self, results):
        ops, n_ops = self.ops, len(self.ops)
        grads = results["grads"]
        contrib = {}   # root tensor -> list of contributions (full tensors or sampled rows), reverse consumer order
        # a tensor that feeds a big convolution is checked on sampled pixels, every other one in full
        pos_of = {}
        for i, op in enumerate(ops[:-1]):
            t_in = self.root[op["in"]]
            if op["kind"] == "conv" and t_in != 0 and t_in not in pos_of and t_in == op["in"]:
                xs, ys = self.act(op["in"]).shape, self.act(i + 1).shape
                if not self.conv_is_small(op, xs, ys):
                    s = self.samples
                    pos = np.stack([self.rng.integers(0, xs[0], s), self.rng.integers(0, xs[1], s),
                                    self.rng.integers(0, xs[2], s)], 1)
                    pos[0] = (0, 0, 0)
                    pos[1] = (xs[0] - 1, xs[1] - 1, xs[2] - 1)
                    pos_of[t_in] = pos

        def pick(t, full):
            pos = pos_of.get(t)
            full = np.asarray(full).reshape(self.act(t).shape)
            return full if pos is None else full[pos[:, 0], pos[:, 1], pos[:, 2]]

        def add(t, arr):
            if t != 0:
                contrib.setdefault(t, []).append(arr)

        hop = ops[-1]
        xh = self.act(hop["in"])
        Wh, bh = self.wl["params"][-1]
        l_ref, dx_ref, dW_ref, db_ref, _ = orc.head_fwd_vjp(xh, Wh, bh, self.wl["labels"])
        self.note("head loss", abs(results["loss"] - l_ref) / abs(l_ref), 2e-5)
        self.tensor_check("head dW", grads[-1][0], dW_ref, 1e-4, lowp=False)
        self.tensor_check("head db", grads[-1][1], db_ref, 1e-4, lowp=False)
        rt = self.root[hop["in"]]
        if rt != 0:
            add(rt, pick(rt, dx_ref))
        for i in range(n_ops - 2, -1, -1):
            op = ops[i]
            kind = op["kind"]
            if kind == "flatten":
                continue
            self.progress("%s: checking the backward pass, op %d of %d" % (self.net["name"], i, len(self.ops)))
            t_in = self.root[op["in"]]
            x = self.act(op["in"])
            y = self.act(i + 1)
            dy = self.cot(i + 1)
            # The finished cotangent of this op's output is what the GPU fed to its pullback; check it
            # against the contributions its consumers made (computed from the GPU's own tensors).  A conv
            # with a fused activation applies the activation pullback to that buffer in place.
            post = _mask(y, op["act"]) if kind == "conv" and op["act"] != "none" else None
            self._check_cotangent(i + 1, contrib, pos_of, dy, post)
            p = self.wl["params"][i]
            if kind == "conv":
                w = self.conv_w(i)
                dz = dy * _mask(y, op["act"])
                want_dx = t_in != 0
                if self.conv_is_small(op, x.shape, y.shape):
                    dxr, dwr, dbr = orc.conv2d_vjp(x, w, dz, op["stride"], op["pad"], op["groups"], need_dx=want_dx,
                                                   need_db=op["bias"])
                    self.tensor_check("op %d conv dw" % i, grads[i][0], dwr, self.tol_par, lowp=False,
                                      atol_extra=self._dw_allowance(x, dz, op["groups"]))
                    if op["bias"]:
                        self.sum_check("op %d conv db" % i, grads[i][1], dbr, np.abs(dz), self.tol_par)
                    if want_dx:
                        add(t_in, pick(t_in, dxr))
                else:
                    c_ = x.shape[3]
                    cs = np.sort(self.rng.choice(c_, size=min(4, c_), replace=False))
                    _, dwr, _ = orc.conv2d_vjp(np.ascontiguousarray(x[..., cs]), np.ascontiguousarray(w[:, :, cs, :]), dz,
                                               op["stride"], op["pad"], 1, need_dx=False)
                    self.tensor_check("op %d conv dw (channel slice)" % i, grads[i][0][:, :, cs, :], dwr, self.tol_par, lowp=False,
                                      atol_extra=self._dw_allowance(x[..., cs], dz, 1))
                    if want_dx and pos_of.get(t_in) is not None:
                        add(t_in, conv_rows_dgrad(dz, w, op, x.shape, pos_of[t_in]))
                    elif want_dx:   # a reinterpreted (flattened) input: small, checked in full
                        add(t_in, pick(t_in, orc.conv2d_vjp(x, w, dz, op["stride"], op["pad"], op["groups"])[0]))
            elif kind == "bn":
                # the pullback's inputs include the statistics its forward pass saved (fp32; checked against the
                # oracle's in check_forward): the oracle's pullback is evaluated at those
                mean, invstd = self.st.bn_stats(i)
                dxr, dres, dg, db = orc.bn_act_vjp(x, y, p[0], mean, invstd, dy, op["act"], op["res"] >= 0)
                dza = np.abs(dy) if op["act"] == "none" else np.abs(dy) * _mask(y, op["act"])
                self.sum_check("op %d bn dbeta" % i, grads[i][1], db, dza, 2e-4)
                dza *= np.abs(x - mean)
                dza *= invstd
                self.sum_check("op %d bn dgamma" % i, grads[i][0], dg, dza, 2e-4)
                del dza
                if op["res"] >= 0:
                    add(self.root[op["res"]], pick(self.root[op["res"]], dres))
                add(t_in, pick(t_in, dxr))
            elif kind == "avgpool2":
                add(t_in, pick(t_in, orc.avgpool2_vjp(dy, x.shape)))
            elif kind == "maxpool3s2":
                add(t_in, pick(t_in, orc.maxpool3s2_vjp(x, dy)))

    @staticmethod
    def _dw_allowance(x, dz, groups):
        """dw[r,s,c,k] = sum over pixels of x[..c] dz[..k]: an fp32 accumulation errs by about 1e-7 of the
        magnitude of its terms and partial sums, whatever the sum cancels down to (activations with a large
        mean against a cotangent that sums to zero).  Allowance per (c, k): 1e-6 ||x_c||_2 ||dz_k||_2, which
        bounds 1e-6 sum |x| |dz| (Cauchy-Schwarz; borders and strides only remove terms)."""
        xn = np.sqrt((x.reshape(-1, x.shape[-1]) ** 2).sum(axis=0))
        dn = np.sqrt((dz.reshape(-1, dz.shape[-1]) ** 2).sum(axis=0))
        if groups > 1:   # depthwise: (r, s, 1, c)
            return 1e-6 * (xn * dn)[None, None, None, :]
        return 1e-6 * (xn[:, None] * dn[None, :])[None, None, :, :]

    def sum_check(self, what, got, ref, terms_abs, tol):
        """A per-channel sum of cotangent terms (bias gradient, dbeta, dgamma) whose terms may cancel, even
        exactly (the beta of a BatchNorm that feeds a convolution followed by BatchNorm has gradient zero).
        Its error is measured against the sum of the magnitudes of its terms S[c] = sum |term|:
        norm-wise, relative L2 <= tol unless the whole difference is below 1e-6 max S (both sides are then
        rounding noise around a sum that cancels); element-wise, |got - ref| <= 1e-4 |ref| + 2e-6 S[c]."""
        S = terms_abs.reshape(-1, terms_abs.shape[-1]).sum(axis=0)
        d = np.abs(np.asarray(got, np.float64) - ref)
        e2 = 0.0 if float(d.max()) <= 1e-6 * float(S.max()) else rel_l2(got, ref)
        self.note(what, e2, tol)
        worst = float((d / (1e-4 * np.abs(ref) + 2e-6 * S + 1e-300)).max())
        assert worst <= 1.0, "%s: element-wise check failed (worst element %.3g of its bound)" % (what, worst)
        self.detail.append((what, e2, tol, rel_inf(got, ref), "worst element %.3g of its bound" % worst))

    def _check_cotangent(self, t, contrib, pos_of, dy_gpu, post=None):
        t = self.root[t]
        parts = contrib.pop(t, None)
        assert parts, "tensor %d has no cotangent contribution" % t
        pos = pos_of.get(t)
        sel = (lambda a: a) if pos is None else (lambda a: a[pos[:, 0], pos[:, 1], pos[:, 2]])
        got = sel(dy_gpu)
        exp = self.rnd(np.array(parts[0], np.float64).reshape(got.shape))
        scale = None
        for extra in parts[1:]:   # a rounded sum of stored values: grid spacing at the largest operand
            e = np.asarray(extra, np.float64).reshape(got.shape)
            scale = np.maximum(np.abs(exp), np.abs(e)) if scale is None else np.maximum(scale, np.abs(e))
            exp = self.rnd(exp + e)
        if post is not None:
            exp = exp * sel(post)
        tol = self.tol_act * (1.0 + 0.5 * (len(parts) - 1))
        self.tensor_check("tensor %d cotangent (%d contribution%s%s)" % (t, len(parts), "s" if len(parts) > 1 else "",
                                                                        "" if pos is None else ", sampled"),
                          got, exp, tol, operand_scale=scale if self.bf16 else None)

    def check_update(self, results, lr, momentum):
        """velocity = momentum*0 + grad and param = param0 - lr*velocity for a first step."""
        for i, p in enumerate(self.wl["params"]):
            for j, a in enumerate(p):
                g = results["grads"][i][j]
                assert np.array_equal(results["velocity"][i][j], g), (i, j)
                ref = np.asarray(a, np.float64) - lr * g
                assert rel_l2(results["params"][i][j], ref) <= 2e-7, (i, j)

    def run(self):
        results = self.st.results()
        self.check_forward()
        self.check_backward(results)
        self.check_update(results, self.net["lr"], self.net["momentum"])
        worst = sorted(self.report, key=lambda r: -(r[1] / r[2] if r[2] > 0 else r[1]))[:3]
        return results, worst
