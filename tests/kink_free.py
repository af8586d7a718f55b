"""Workloads on which an end-to-end gradient comparison is well posed.

The gradient of a ReLU network is discontinuous where a pre-activation z crosses 0 (or 6 for ReLU6)
and where two entries of a max-pool window swap ranks.  Two correct implementations that differ by
rounding agree on every such decision as long as every z stays further from its kinks than their
rounding difference (fp32 against fp64: about 1e-6 of the spread of z).  `make_kink_free` takes a
seeded workload and moves each channel's additive parameter (the beta of a BatchNorm, the bias of a
convolution with an activation) by the smallest multiple of margin * std(z) that leaves every
pre-activation of that channel at least margin * std(z) away from its kinks, layer by layer in op
order, using the oracle's own forward ops.  The shifts are a few 1e-4 of a standard deviation: the
workload keeps its shapes and distributions.  `kink_margins` measures what a workload has.

Test infrastructure; uses the oracle, never the GPU library.
"""
import numpy as np

from oracle import oracle as orc


def _kinks(act):
    return (0.0,) if act == "relu" else (0.0, 6.0) if act == "relu6" else ()


def _channel_std(v):
    sd = v.reshape(-1, v.shape[-1]).std(axis=0)
    return np.where(sd > 0, sd, 1.0)


def _min_distance(z, act, sd):
    """Per channel: the smallest |z - kink| / std over all elements and kinks."""
    z2 = z.reshape(-1, z.shape[-1])
    m = np.full(z2.shape[1], np.inf)
    for k in _kinks(act):
        m = np.minimum(m, np.abs(z2 - k).min(axis=0) / sd)
    return m


def _maxpool_gap(x):
    """Smallest gap (in units of the tensor's per-channel std) between the largest and the second
    largest entry of a 3x3/2 window whose maximum is positive (ties among zeros after a ReLU are
    harmless: their cotangent is masked upstream)."""
    n, h, w, c = x.shape
    xp = np.full((n, h + 2, w + 2, c), -np.inf)
    xp[:, 1:-1, 1:-1] = x
    p, q = (h - 1) // 2 + 1, (w - 1) // 2 + 1
    win = np.stack([xp[:, r:r + 2 * p:2, s:s + 2 * q:2] for r in range(3) for s in range(3)], -1)
    win = np.sort(win, -1)
    gap = (win[..., -1] - win[..., -2]) / _channel_std(x)
    pos = win[..., -1] > 0
    return float(gap[pos].min()) if pos.any() else float("inf")


def _walk(net, wl, margin):
    """Forward pass with the oracle's ops.  margin > 0: adjusts the shifts in a copy of the parameters.
    Returns (params, report) with report = list of (op, what, smallest margin, elements)."""
    assert net["dtype"] == "f32", "only fp32 workloads can be made kink free (bf16 roundings move z by ~1e-3 std)"
    params = [[np.array(a, np.float32) for a in p] for p in wl["params"]]
    tensors = [np.asarray(wl["x"], np.float64)]
    report = []
    for i, op in enumerate(net["ops"]):
        kind = op["kind"]
        x = tensors[op["in"]]
        p = params[i]
        act = op.get("act", "none")
        y = None
        if kind == "conv":
            v = orc.conv2d_fwd(x, p[0], None, op["stride"], op["pad"], op["groups"])
            if op["bias"]:
                if act != "none":
                    p[1] = _settle(v, p[1], act, margin)
                v = v + np.asarray(p[1], np.float64)
            if act != "none":
                report.append((i, "conv+" + act, float(_min_distance(v, act, _channel_std(v)).min()), v.size))
                y = orc.bias_act_fwd(v, None, act)
            else:
                y = v
        elif kind == "bn":
            res = tensors[op["res"]] if op["res"] >= 0 else None
            if act != "none":
                zero = np.zeros_like(p[1])
                v, _, _ = orc.bn_act_fwd(x, res, p[0], zero, op["eps"], "none")   # z without beta
                p[1] = _settle(v, p[1], act, margin)
            z, _, _ = orc.bn_act_fwd(x, res, p[0], p[1], op["eps"], "none")
            if act != "none":
                report.append((i, "bn+" + act, float(_min_distance(z, act, _channel_std(z)).min()), z.size))
            y, _, _ = orc.bn_act_fwd(x, res, p[0], p[1], op["eps"], act)
        elif kind == "avgpool2":
            y = orc.avgpool2_fwd(x)
        elif kind == "maxpool3s2":
            report.append((i, "maxpool", _maxpool_gap(x), x.size))
            y = orc.maxpool3s2_fwd(x)
        elif kind == "flatten":
            y = x.reshape(x.shape[0], 1, 1, -1)
        tensors.append(y)
    return params, report


def layer_margin(margin, samples_per_channel):
    """The margin asked of a layer: `margin` where a channel has thousands of samples (the gaps between
    neighbouring samples are then a few 1e-4 std wide), more where it has few (late layers: up to 1e-2
    std, which costs nothing there and covers the rounding differences that have built up by then)."""
    return float(min(1e-2, max(margin, 0.1 / max(samples_per_channel, 1)))) if margin > 0 else 0.0


def _settle(v, shift, act, margin):
    """New per-channel shifts b' = b + t*step (step = 2*m*std, |t| as small as possible) such that every
    |v + b' - kink| >= m*std, m = layer_margin(margin, samples).  v: the pre-activations without the shift, (..., C)."""
    if margin <= 0:
        return shift
    v2 = v.reshape(-1, v.shape[-1])
    margin = layer_margin(margin, v2.shape[0])
    sd = _channel_std(v)
    b0 = np.asarray(shift, np.float64)
    out = b0.copy()
    todo = np.arange(v2.shape[1])
    for t in range(0, 2000):
        for sign in ((1,) if t == 0 else (1, -1)):
            if todo.size == 0:
                break
            cand = b0[todo] + sign * t * 2.0 * margin * sd[todo]
            # the float32 value the libraries will see decides
            cand = cand.astype(np.float32).astype(np.float64)
            ok = _min_distance(v2[:, todo] + cand, act, sd[todo]) >= margin
            out[todo[ok]] = cand[ok]
            todo = todo[~ok]
    assert todo.size == 0, "no kink-free shift found for %d channels" % todo.size
    return out.astype(np.float32)


def kink_margins(net, wl):
    """[(op, what, smallest distance of a pre-activation to a kink in std units, elements)]"""
    return _walk(net, wl, 0.0)[1]


def make_kink_free(net, wl, margin=1e-4):
    """Copy of the workload with kink-free shifts; second result: the margins it then has."""
    params, report = _walk(net, wl, margin)
    out = dict(wl, params=params)
    return out, report
