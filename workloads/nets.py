"""Seeded synthetic workloads: network descriptions, initial parameters and batches.

This module is the only thing the CPU oracle and the GPU library have in common.  It
holds no arithmetic of the method: it lists the ops of each network (a static op list,
the role `sequenced(through:)` plays in the paper's LeNet figure, Section 4.1) and
draws inputs, labels and initial parameters from one NumPy generator per workload.
Neither side's shape inference, rounding or kernels live here.

A network is a dict:
  name, dtype ("f32" | "bf16"), input (N,H,W,C), classes, lr, momentum, seed,
  ops: list of dicts, op i produces tensor i+1 (tensor 0 is the batch):
    {"kind": "conv", "in": t, "k": K, "r": R, "s": S, "stride": s, "pad": p,
     "groups": g, "bias": bool, "act": "none"|"relu"|"relu6"}
    {"kind": "bn", "in": t, "res": t2 | -1, "act": ..., "eps": 1e-5}
    {"kind": "avgpool2", "in": t}      2x2 stride 2
    {"kind": "maxpool3s2", "in": t}    3x3 stride 2 pad 1
    {"kind": "flatten", "in": t}       (N,H,W,C) -> (N,1,1,H*W*C), NHWC order
    {"kind": "head", "in": t, "classes": n}   global avg pool + dense + softmax-CE
Parameters are a list (one entry per op) of lists of float32 arrays:
  conv: [w (R,S,C/groups,K)] (+ [bias (K)]);  bn: [gamma (C), beta (C)];
  head: [W (C,classes), b (classes)];  others: [].
Layouts: activations NHWC, filters (R,S,Cin/groups,Cout) as in the paper's
`filterShape: (5, 5, 1, 6)`, dense weights [in,out].
"""
import numpy as np

ACTS = ("none", "relu", "relu6")


def _conv(t, k, r, stride=1, pad=0, groups=1, bias=False, act="none"):
    return {"kind": "conv", "in": t, "k": k, "r": r, "s": r, "stride": stride, "pad": pad,
            "groups": groups, "bias": bias, "act": act}


def _bn(t, act="none", res=-1):
    return {"kind": "bn", "in": t, "res": res, "act": act, "eps": 1e-5}


class _Builder:
    def __init__(self):
        self.ops = []

    def add(self, op):
        self.ops.append(op)
        return len(self.ops)  # id of the tensor this op produces


def tiny_block(batch=8):
    b = _Builder()
    t = b.add(_conv(0, 16, 3, pad=1))
    t = b.add(_bn(t, "relu"))
    b.add({"kind": "head", "in": t, "classes": 10})
    return dict(name="tiny", dtype="f32", input=(batch, 16, 16, 3), classes=10, lr=0.1,
                momentum=0.9, seed=1001, init="he", x_dist="normal", ops=b.ops)


def lenet5(batch=128):
    """The LeNet-5 variant of the paper's Section 4.1 figure: conv1 is `.same` (pad 2),
    conv2 has no padding argument (valid), so 28 -> 28 -> 14 -> 10 -> 5 and 16*5*5 = 400."""
    b = _Builder()
    t = b.add(_conv(0, 6, 5, pad=2, bias=True, act="relu"))
    t = b.add({"kind": "avgpool2", "in": t})
    t = b.add(_conv(t, 16, 5, pad=0, bias=True, act="relu"))
    t = b.add({"kind": "avgpool2", "in": t})
    t = b.add({"kind": "flatten", "in": t})
    t = b.add(_conv(t, 120, 1, bias=True, act="relu"))
    t = b.add(_conv(t, 84, 1, bias=True, act="relu"))
    b.add({"kind": "head", "in": t, "classes": 10})
    return dict(name="lenet5", dtype="f32", input=(batch, 28, 28, 1), classes=10, lr=0.01,
                momentum=0.0, seed=1002, init="glorot", x_dist="uniform", ops=b.ops)


def resnet56(batch=128, blocks_per_stage=9, hw=32):
    b = _Builder()
    t = b.add(_conv(0, 16, 3, pad=1))
    t = b.add(_bn(t, "relu"))
    cin = 16
    for stage, cout in enumerate((16, 32, 64)):
        for blk in range(blocks_per_stage):
            stride = 2 if (stage > 0 and blk == 0) else 1
            skip = t
            u = b.add(_conv(t, cout, 3, stride=stride, pad=1))
            u = b.add(_bn(u, "relu"))
            u = b.add(_conv(u, cout, 3, pad=1))
            if stride != 1 or cin != cout:
                s = b.add(_conv(skip, cout, 1, stride=stride))
                skip = b.add(_bn(s, "none"))
            t = b.add(_bn(u, "relu", res=skip))
            cin = cout
    b.add({"kind": "head", "in": t, "classes": 10})
    return dict(name="resnet56", dtype="f32", input=(batch, hw, hw, 3), classes=10, lr=0.1,
                momentum=0.9, seed=1003, init="he", x_dist="normal", ops=b.ops)


def resnet50(batch=64, hw=224, stages=(3, 4, 6, 3), classes=1000, dtype="bf16"):
    """Bottleneck ResNet, stride on the 3x3 of the first block of stages 2-4, projection
    (1x1 conv + BN) on the first block of every stage."""
    b = _Builder()
    t = b.add(_conv(0, 64, 7, stride=2, pad=3))
    t = b.add(_bn(t, "relu"))
    t = b.add({"kind": "maxpool3s2", "in": t})
    cin = 64
    for stage, nblk in enumerate(stages):
        width = 64 << stage
        cout = width * 4
        for blk in range(nblk):
            stride = 2 if (stage > 0 and blk == 0) else 1
            skip = t
            u = b.add(_conv(t, width, 1))
            u = b.add(_bn(u, "relu"))
            u = b.add(_conv(u, width, 3, stride=stride, pad=1))
            u = b.add(_bn(u, "relu"))
            u = b.add(_conv(u, cout, 1))
            if blk == 0:
                s = b.add(_conv(skip, cout, 1, stride=stride))
                skip = b.add(_bn(s, "none"))
            t = b.add(_bn(u, "relu", res=skip))
            cin = cout
    b.add({"kind": "head", "in": t, "classes": classes})
    return dict(name="resnet50", dtype=dtype, input=(batch, hw, hw, 3), classes=classes, lr=0.1,
                momentum=0.9, seed=1004, init="he", x_dist="normal", ops=b.ops)


def mobilenetv2(batch=32, hw=224, classes=1000):
    b = _Builder()
    t = b.add(_conv(0, 32, 3, stride=2, pad=1))
    t = b.add(_bn(t, "relu6"))
    cin = 32
    schedule = ((1, 16, 1, 1), (6, 24, 2, 2), (6, 32, 3, 2), (6, 64, 4, 2), (6, 96, 3, 1),
                (6, 160, 3, 2), (6, 320, 1, 1))
    for expand, cout, reps, first_stride in schedule:
        for i in range(reps):
            stride = first_stride if i == 0 else 1
            skip = t
            u = t
            hidden = cin * expand
            if expand != 1:
                u = b.add(_conv(u, hidden, 1))
                u = b.add(_bn(u, "relu6"))
            u = b.add(_conv(u, hidden, 3, stride=stride, pad=1, groups=hidden))
            u = b.add(_bn(u, "relu6"))
            u = b.add(_conv(u, cout, 1))
            if stride == 1 and cin == cout:
                t = b.add(_bn(u, "none", res=skip))
            else:
                t = b.add(_bn(u, "none"))
            cin = cout
    t = b.add(_conv(t, 1280, 1))
    t = b.add(_bn(t, "relu6"))
    b.add({"kind": "head", "in": t, "classes": classes})
    return dict(name="mobilenetv2", dtype="f32", input=(batch, hw, hw, 3), classes=classes, lr=0.1,
                momentum=0.9, seed=1005, init="he", x_dist="normal", ops=b.ops)


CONFIGS = {"tiny": tiny_block, "lenet5": lenet5, "resnet56": resnet56, "resnet50": resnet50,
           "mobilenetv2": mobilenetv2}


def tensor_shapes(net):
    """Shapes (N,H,W,C) of tensor 0..n_ops.  Bookkeeping for the generator only (it needs
    channel counts to size the parameter arrays)."""
    shapes = [tuple(net["input"])]
    for op in net["ops"]:
        n, h, w, c = shapes[op["in"]]
        kind = op["kind"]
        if kind == "conv":
            p = (h + 2 * op["pad"] - op["r"]) // op["stride"] + 1
            q = (w + 2 * op["pad"] - op["s"]) // op["stride"] + 1
            shapes.append((n, p, q, op["k"]))
        elif kind == "bn":
            shapes.append((n, h, w, c))
        elif kind == "avgpool2":
            shapes.append((n, h // 2, w // 2, c))
        elif kind == "maxpool3s2":
            shapes.append((n, (h + 2 - 3) // 2 + 1, (w + 2 - 3) // 2 + 1, c))
        elif kind == "flatten":
            shapes.append((n, 1, 1, h * w * c))
        elif kind == "head":
            shapes.append((n, 1, 1, op["classes"]))
        else:
            raise ValueError(kind)
    return shapes


def to_bf16_grid(a):
    """Round float32 values to the nearest bf16-representable value (ties to even) and
    return them as float32.  Used only to make the *inputs* of bf16 workloads exactly
    representable, so that both sides start from identical numbers."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(np.shape(a))


def make_workload(net, perturb=False):
    """Draw x, labels, then the parameters in op order from default_rng(net['seed']).

    perturb=True additionally draws non-trivial BatchNorm gamma/beta and biases (after
    everything else, so the default stream is unchanged); used by parity tests so that
    a mistake in how those enter the arithmetic cannot hide behind gamma=1, beta=0.
    perturb="shifted": inputs and activations far from zero mean, so that every convolution output
    has a per-channel mean of several standard deviations (x ~ N(12,1) resp. U[0,1)+12; BatchNorms
    with an activation get gamma ~ 0.25, beta ~ 4, i.e. outputs of mean 4 and spread 0.25): the
    workload on which one-pass variance formulas lose digits.
    """
    rng = np.random.default_rng(net["seed"])
    n, h, w, c = net["input"]
    if net["x_dist"] == "normal":
        x = rng.standard_normal((n, h, w, c), dtype=np.float32)
    else:
        x = rng.random((n, h, w, c), dtype=np.float32)
    if net["dtype"] == "bf16":
        x = to_bf16_grid(x)
    labels = rng.integers(0, net["classes"], size=n, dtype=np.int32)
    shapes = tensor_shapes(net)
    params = []
    for op in net["ops"]:
        cin = shapes[op["in"]][3]
        kind = op["kind"]
        if kind == "conv":
            r, s, k, g = op["r"], op["s"], op["k"], op["groups"]
            fan_in, fan_out = r * s * cin // g, r * s * k // g
            shape = (r, s, cin // g, k)
            if net["init"] == "he":
                wgt = (rng.standard_normal(shape, dtype=np.float32)
                       * np.float32(np.sqrt(2.0 / fan_in)))
            else:
                lim = np.sqrt(6.0 / (fan_in + fan_out))
                wgt = ((rng.random(shape, dtype=np.float32) * 2 - 1) * np.float32(lim))
            p = [wgt.astype(np.float32)]
            if op["bias"]:
                p.append(np.zeros(k, np.float32))
            params.append(p)
        elif kind == "bn":
            params.append([np.ones(cin, np.float32), np.zeros(cin, np.float32)])
        elif kind == "head":
            k = op["classes"]
            if net["init"] == "he":
                wgt = rng.standard_normal((cin, k), dtype=np.float32) * np.float32(np.sqrt(2.0 / cin))
            else:
                lim = np.sqrt(6.0 / (cin + k))
                wgt = (rng.random((cin, k), dtype=np.float32) * 2 - 1) * np.float32(lim)
            params.append([wgt.astype(np.float32), np.zeros(k, np.float32)])
        else:
            params.append([])
    if perturb:
        shifted = perturb == "shifted"
        if shifted:
            x = x + np.float32(12.0)
            if net["dtype"] == "bf16":
                x = to_bf16_grid(x)
        for op, p in zip(net["ops"], params):
            if op["kind"] == "bn":
                p[0] = (1.0 + 0.3 * rng.standard_normal(p[0].shape)).astype(np.float32)
                p[1] = (0.2 * rng.standard_normal(p[1].shape)).astype(np.float32)
                if shifted and op["act"] != "none":
                    p[0] = (0.25 * p[0]).astype(np.float32)
                    p[1] = (p[1] + 4.0).astype(np.float32)
            elif op["kind"] in ("conv", "head") and len(p) == 2:
                p[1] = (0.1 * rng.standard_normal(p[1].shape)).astype(np.float32)
    return {"x": x, "labels": labels, "params": params}


def param_count(params):
    return int(sum(a.size for p in params for a in p))
