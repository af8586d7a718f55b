"""Pins of the CPU oracle against things other than itself: brute force, finite differences,
adjoint identities, closed forms, invariants and library routines.  CPU only."""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import oracle as orc
from workloads import nets

RNG = np.random.default_rng(7)


def fd_grad(f, a, h=1e-6, idx=None):
    """Central finite differences of scalar f with respect to array a (all entries or idx)."""
    g = np.zeros_like(a)
    flat = a.reshape(-1)
    gf = g.reshape(-1)
    for i in (range(flat.size) if idx is None else idx):
        old = flat[i]
        flat[i] = old + h
        fp = f()
        flat[i] = old - h
        fm = f()
        flat[i] = old
        gf[i] = (fp - fm) / (2 * h)
    return g


def brute_conv(x, w, b, stride, pad, groups):
    """Direct convolution from the definition, pure Python loops, written independently."""
    n_, h_, w_, c_ = x.shape
    r_, s_, cg, k_ = w.shape
    kg = k_ // groups
    p_ = (h_ + 2 * pad - r_) // stride + 1
    q_ = (w_ + 2 * pad - s_) // stride + 1
    y = np.zeros((n_, p_, q_, k_))
    for n, p, q, k in itertools.product(range(n_), range(p_), range(q_), range(k_)):
        g = k // kg
        acc = 0.0 if b is None else b[k]
        for r, s, c in itertools.product(range(r_), range(s_), range(cg)):
            hh, ww = p * stride + r - pad, q * stride + s - pad
            if 0 <= hh < h_ and 0 <= ww < w_:
                acc += x[n, hh, ww, g * cg + c] * w[r, s, c, k]
        y[n, p, q, k] = acc
    return y


CONV_CASES = [
    # n h w c k r stride pad groups
    (2, 5, 5, 3, 4, 3, 1, 1, 1),
    (2, 6, 5, 3, 4, 3, 2, 1, 1),
    (1, 7, 7, 2, 3, 5, 2, 2, 1),
    (2, 5, 6, 4, 6, 3, 1, 0, 2),
    (2, 6, 6, 4, 4, 3, 2, 1, 4),   # depthwise
    (1, 4, 4, 3, 5, 1, 2, 0, 1),   # strided 1x1 projection
    (2, 5, 5, 2, 3, 3, 1, 2, 1),   # pad larger than needed for "same"
]


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_fwd_brute_force(case):
    n, h, w, c, k, r, stride, pad, groups = case
    x = RNG.standard_normal((n, h, w, c))
    wt = RNG.standard_normal((r, r, c // groups, k))
    b = RNG.standard_normal(k)
    y = orc.conv2d_fwd(x, wt, b, stride, pad, groups)
    np.testing.assert_allclose(y, brute_conv(x, wt, b, stride, pad, groups), rtol=1e-12, atol=1e-12)


def test_conv_special_cases():
    x = RNG.standard_normal((3, 6, 5, 7))
    # 1x1 stride 1 is a plain matmul over pixels
    w1 = RNG.standard_normal((1, 1, 7, 4))
    np.testing.assert_allclose(orc.conv2d_fwd(x, w1, None, 1, 0), x @ w1[0, 0], rtol=1e-12, atol=1e-12)
    # filter as large as the image, no padding: a dense layer over the flattened (h,w,c) input
    wf = RNG.standard_normal((6, 5, 7, 3))
    np.testing.assert_allclose(orc.conv2d_fwd(x, wf, None, 1, 0).reshape(3, 3),
                               x.reshape(3, -1) @ wf.reshape(-1, 3), rtol=1e-12, atol=1e-12)
    # delta filter at the centre of a 3x3 with pad 1 is the identity per channel
    wd = np.zeros((3, 3, 7, 7))
    wd[1, 1] = np.eye(7)
    np.testing.assert_allclose(orc.conv2d_fwd(x, wd, None, 1, 1), x, rtol=0, atol=0)
    # delta at (0,0) shifts the image by (+1,+1) with zero fill (cross-correlation, no flip)
    ws = np.zeros((3, 3, 7, 7))
    ws[0, 0] = np.eye(7)
    y = orc.conv2d_fwd(x, ws, None, 1, 1)
    np.testing.assert_array_equal(y[:, 1:, 1:], x[:, :-1, :-1])
    assert np.all(y[:, 0] == 0) and np.all(y[:, :, 0] == 0)
    # depthwise equals per-channel single-channel convolutions
    wdw = RNG.standard_normal((3, 3, 1, 7))
    ydw = orc.conv2d_fwd(x, wdw, None, 1, 1, groups=7)
    for ch in range(7):
        yc = orc.conv2d_fwd(x[..., ch:ch + 1], wdw[..., ch:ch + 1], None, 1, 1)
        np.testing.assert_allclose(ydw[..., ch:ch + 1], yc, rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_vjp_finite_differences_and_adjoint(case):
    n, h, w, c, k, r, stride, pad, groups = case
    x = RNG.standard_normal((n, h, w, c))
    wt = RNG.standard_normal((r, r, c // groups, k))
    b = RNG.standard_normal(k)
    y = orc.conv2d_fwd(x, wt, b, stride, pad, groups)
    dy = RNG.standard_normal(y.shape)
    dx, dw, db = orc.conv2d_vjp(x, wt, dy, stride, pad, groups, need_dx=True, need_db=True)

    def f():
        return float(np.sum(orc.conv2d_fwd(x, wt, b, stride, pad, groups) * dy))

    np.testing.assert_allclose(dx, fd_grad(f, x), rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(dw, fd_grad(f, wt), rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(db, fd_grad(f, b), rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(db, dy.sum(axis=(0, 1, 2)), rtol=1e-12)
    # conv is bilinear: <conv(x,w), dy> = <x, dx> = <w, dw>
    lin = float(np.sum(orc.conv2d_fwd(x, wt, None, stride, pad, groups) * dy))
    assert abs(lin - np.sum(x * dx)) <= 1e-10 * max(1.0, abs(lin))
    assert abs(lin - np.sum(wt * dw)) <= 1e-10 * max(1.0, abs(lin))


def test_conv_dgrad_stride1_is_flipped_forward():
    x = RNG.standard_normal((2, 6, 7, 3))
    wt = RNG.standard_normal((3, 3, 3, 5))
    dy = RNG.standard_normal((2, 6, 7, 5))
    dx, _, _ = orc.conv2d_vjp(x, wt, dy, 1, 1)
    wflip = np.ascontiguousarray(wt[::-1, ::-1].transpose(0, 1, 3, 2))
    np.testing.assert_allclose(dx, orc.conv2d_fwd(dy, wflip, None, 1, 3 - 1 - 1), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("act,use_res", [("none", False), ("relu", False), ("relu", True), ("relu6", True)])
def test_bn_forward_invariants_and_vjp(act, use_res):
    m_shape, c = (3, 4, 5), 6
    x = RNG.standard_normal(m_shape + (c,)) * 2.0 + 1.5
    res = RNG.standard_normal(x.shape) if use_res else None
    gamma = 1.0 + 0.3 * RNG.standard_normal(c)
    beta = 0.2 * RNG.standard_normal(c) + (3.0 if act == "relu6" else 0.0)
    eps = 1e-5
    y, mean, invstd = orc.bn_act_fwd(x, res, gamma, beta, eps, act)
    xf = x.reshape(-1, c)
    np.testing.assert_allclose(mean, xf.mean(0), rtol=1e-12)
    np.testing.assert_allclose(invstd, 1 / np.sqrt(xf.var(0) + eps), rtol=1e-12)
    # gamma=1, beta=0, no act: output mean 0 and variance var/(var+eps)
    y0, _, _ = orc.bn_act_fwd(x, None, np.ones(c), np.zeros(c), eps, "none")
    y0f = y0.reshape(-1, c)
    np.testing.assert_allclose(y0f.mean(0), 0, atol=1e-13)
    np.testing.assert_allclose(y0f.var(0), xf.var(0) / (xf.var(0) + eps), rtol=1e-12)
    # invariance to per-channel affine maps of the input (a > 0), up to the eps term
    a = 0.5 + RNG.random(c)
    y1, _, _ = orc.bn_act_fwd(x * a + 3.0, None, np.ones(c), np.zeros(c), 0.0, "none")
    y2, _, _ = orc.bn_act_fwd(x, None, np.ones(c), np.zeros(c), 0.0, "none")
    np.testing.assert_allclose(y1, y2, rtol=1e-10, atol=1e-10)
    # pullback
    dy = RNG.standard_normal(x.shape)
    dx, dres, dgamma, dbeta = orc.bn_act_vjp(x, y, gamma, mean, invstd, dy, act, use_res)

    def f():
        yy, _, _ = orc.bn_act_fwd(x, res, gamma, beta, eps, act)
        return float(np.sum(yy * dy))

    np.testing.assert_allclose(dx, fd_grad(f, x), rtol=2e-6, atol=1e-7)
    np.testing.assert_allclose(dgamma, fd_grad(f, gamma), rtol=2e-6, atol=1e-7)
    np.testing.assert_allclose(dbeta, fd_grad(f, beta), rtol=2e-6, atol=1e-7)
    if use_res:
        np.testing.assert_allclose(dres, fd_grad(f, res), rtol=2e-6, atol=1e-7)
    # the input cotangent is orthogonal to the shift and scale directions of each channel
    xhat = (xf - mean) * invstd
    dxf = dx.reshape(-1, c)
    np.testing.assert_allclose(dxf.sum(0), 0, atol=1e-12)
    # ... exactly so for eps = 0; with eps the scale direction leaves gamma*invstd*dgamma*eps*invstd^2
    np.testing.assert_allclose((dxf * xhat).sum(0), gamma * invstd * dgamma * eps * invstd ** 2,
                               rtol=1e-7, atol=1e-12)
    # masks use strict inequalities on the stored output
    mask = (y > 0) if act == "relu" else ((y > 0) & (y < 6)) if act == "relu6" else np.ones_like(y, bool)
    if use_res:
        np.testing.assert_array_equal(dres, dy * mask)


def test_activation_masks_at_kinks():
    y = np.array([[0.0, 6.0, 3.0, -0.0]])
    dy = np.ones_like(y)
    dx, _ = orc.bias_act_vjp(y, dy, "relu")
    np.testing.assert_array_equal(dx, [[0, 1, 1, 0]])
    dx, _ = orc.bias_act_vjp(y, dy, "relu6")
    np.testing.assert_array_equal(dx, [[0, 0, 1, 0]])
    x = np.array([[-1.0, 7.0, 2.0]])
    np.testing.assert_array_equal(orc.bias_act_fwd(x, np.array([0.5, 0.5, 0.5]), "relu6"), [[0, 6, 2.5]])


def test_bias_act_vjp_fd():
    x = RNG.standard_normal((4, 3, 5))
    b = RNG.standard_normal(5)
    dy = RNG.standard_normal(x.shape)
    y = orc.bias_act_fwd(x, b, "relu")
    dx, db = orc.bias_act_vjp(y, dy, "relu")
    f = lambda: float(np.sum(orc.bias_act_fwd(x, b, "relu") * dy))
    np.testing.assert_allclose(dx, fd_grad(f, x), rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(db, fd_grad(f, b), rtol=1e-6, atol=1e-8)


def test_pools():
    x = RNG.standard_normal((2, 6, 8, 3))
    y = orc.avgpool2_fwd(x)
    np.testing.assert_allclose(y, x.reshape(2, 3, 2, 4, 2, 3).mean(axis=(2, 4)), rtol=1e-13)
    dy = RNG.standard_normal(y.shape)
    dx = orc.avgpool2_vjp(dy, x.shape)
    np.testing.assert_allclose(dx, np.repeat(np.repeat(dy, 2, 1), 2, 2) / 4, rtol=1e-13)
    assert abs(dx.sum() - dy.sum()) < 1e-12
    # max pool 3x3/2 pad 1 against a padded sliding-window maximum
    for shape in [(2, 7, 7, 3), (1, 8, 6, 2)]:
        x = RNG.standard_normal(shape)
        y = orc.maxpool3s2_fwd(x)
        n, h, w, c = shape
        xp = np.full((n, h + 2, w + 2, c), -np.inf)
        xp[:, 1:-1, 1:-1] = x
        p, q = y.shape[1:3]
        ref = np.stack([np.stack([xp[:, 2 * i:2 * i + 3, 2 * j:2 * j + 3].max(axis=(1, 2))
                                  for j in range(q)], 1) for i in range(p)], 1)
        np.testing.assert_array_equal(y, ref)
        dy = RNG.standard_normal(y.shape)
        dx = orc.maxpool3s2_vjp(x, dy)
        f = lambda: float(np.sum(orc.maxpool3s2_fwd(x) * dy))
        np.testing.assert_allclose(dx, fd_grad(f, x, h=1e-7), rtol=1e-5, atol=1e-7)
        assert abs(dx.sum() - dy.sum()) < 1e-12


def test_maxpool_tie_goes_to_first_in_window_order():
    x = np.zeros((1, 4, 4, 1))
    dy = np.arange(1, 5, dtype=np.float64).reshape(1, 2, 2, 1)
    dx = orc.maxpool3s2_vjp(x, dy)
    # window (p,q) covers rows 2p-1..2p+1; its first in-range element in row-major order:
    # (0,0)->(0,0)  (0,1)->(0,1)  (1,0)->(1,0)  (1,1)->(1,1)
    expect = np.zeros((4, 4))
    expect[0, 0], expect[0, 1], expect[1, 0], expect[1, 1] = 1, 2, 3, 4
    np.testing.assert_array_equal(dx[0, :, :, 0], expect)


def test_head_closed_forms():
    n, h, w, c, k = 6, 3, 2, 5, 10
    x = RNG.standard_normal((n, h, w, c))
    labels = np.array([0, 3, 3, 9, 1, 3], np.int32)
    # W = 0, b = 0: loss = ln(classes), db = 1/classes - frequency of each label
    loss, dx, dW, db, _ = orc.head_fwd_vjp(x, np.zeros((c, k)), np.zeros(k), labels)
    assert abs(loss - math.log(10)) < 1e-14
    freq = np.bincount(labels, minlength=k) / n
    np.testing.assert_allclose(db, 1.0 / k - freq, atol=1e-15)
    assert np.all(dx == 0)
    W = RNG.standard_normal((c, k))
    b = RNG.standard_normal(k)
    loss, dx, dW, db, logits = orc.head_fwd_vjp(x, W, b, labels)
    pbar = x.mean(axis=(1, 2))
    z = pbar @ W + b
    np.testing.assert_allclose(logits, z, rtol=1e-12)
    sm = np.exp(z - z.max(1, keepdims=True))
    sm /= sm.sum(1, keepdims=True)
    dz = sm.copy()
    dz[np.arange(n), labels] -= 1
    dz /= n
    np.testing.assert_allclose(loss, -np.mean(np.log(sm[np.arange(n), labels])), rtol=1e-12)
    np.testing.assert_allclose(db, dz.sum(0), rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(dW, pbar.T @ dz, rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(dx, np.broadcast_to(((dz @ W.T) / (h * w))[:, None, None, :], x.shape),
                               rtol=1e-11, atol=1e-14)
    f = lambda: orc.head_fwd_vjp(x, W, b, labels)[0]
    np.testing.assert_allclose(dx, fd_grad(f, x), rtol=1e-6, atol=1e-9)
    np.testing.assert_allclose(dW, fd_grad(f, W), rtol=1e-6, atol=1e-9)
    np.testing.assert_allclose(db, fd_grad(f, b), rtol=1e-6, atol=1e-9)
    # large logits do not overflow (max-subtracted)
    loss_big = orc.head_fwd_vjp(x, W * 1e3, b, labels)[0]
    assert np.isfinite(loss_big)


def test_sgd_closed_form():
    g = RNG.standard_normal(5)
    th0 = RNG.standard_normal(5)
    th, v = th0.copy(), np.zeros(5)
    mu, lr, steps = 0.9, 0.1, 7
    for _ in range(steps):
        orc.sgd_momentum(th, v, g, lr, mu)
    np.testing.assert_allclose(v, g * (1 - mu ** steps) / (1 - mu), rtol=1e-12)
    vsum = sum(g * (1 - mu ** i) / (1 - mu) for i in range(1, steps + 1))
    np.testing.assert_allclose(th, th0 - lr * vsum, rtol=1e-12)
    th, v = th0.copy(), np.zeros(5)
    orc.sgd_momentum(th, v, g, lr, 0.0)
    np.testing.assert_allclose(th, th0 - lr * g, rtol=1e-15)


def test_bf16_rounding_against_library_and_known_values():
    torch = pytest.importorskip("torch")
    a = RNG.standard_normal(20000).astype(np.float32) * np.float32(10.0) ** RNG.integers(-30, 30, 20000).astype(np.float32)
    a = np.concatenate([a, np.array([0.0, -0.0, 1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1e-40, 3e38, 3.39e38],
                                    np.float32)])
    ref = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    got = orc.round_bf16(a.astype(np.float64))
    np.testing.assert_array_equal(got.astype(np.float32), ref)
    np.testing.assert_array_equal(orc.round_bf16(a.astype(np.float64), slow=True).astype(np.float32), ref)
    # doubles that are not float32-representable: fast (bit pattern) and slow (frexp) paths agree
    d = RNG.standard_normal(20000) * 10.0 ** RNG.integers(-45, 40, 20000)
    np.testing.assert_array_equal(orc.round_bf16(d), orc.round_bf16(d, slow=True))
    # ties to even on hand-computed cases (8 significant bits)
    np.testing.assert_array_equal(orc.round_bf16(np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 + 2.0 ** -8 + 2.0 ** -30])),
                                  [1.0, 1 + 2.0 ** -6, 1 + 2.0 ** -7])
    np.testing.assert_array_equal(nets.to_bf16_grid(a), ref)


# ---------------------------------------------------------------------------------------
# whole networks
# ---------------------------------------------------------------------------------------
def test_parameter_counts_and_lenet_shapes():
    counts = {"tiny": 634, "lenet5": 61706, "resnet56": 855770, "resnet50": 25557032, "mobilenetv2": 3504872}
    for name, expect in counts.items():
        net = nets.CONFIGS[name](batch=1)
        shapes = nets.tensor_shapes(net)
        total = 0
        for op in net["ops"]:
            cin = shapes[op["in"]][3]
            if op["kind"] == "conv":
                total += op["r"] * op["s"] * cin // op["groups"] * op["k"] + (op["k"] if op["bias"] else 0)
            elif op["kind"] == "bn":
                total += 2 * cin
            elif op["kind"] == "head":
                total += cin * op["classes"] + op["classes"]
        assert total == expect, name
    golden = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "lenet_shapes.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            key, val = line.split(":")
            golden[key.strip()] = [int(t) for t in val.split()]
    net = nets.lenet5(batch=2)
    wl = nets.make_workload(net)
    tensors, _ = orc.forward(net, wl["x"], wl["params"])
    got = [t.shape[1:] for t in tensors[:-1]]
    names = ["input", "conv1", "pool1", "conv2", "pool2", "flatten", "fc1", "fc2"]
    for nm, shp in zip(names, got):
        assert list(shp) == golden[nm], nm
    assert nets.param_count(wl["params"]) == golden["params"][0]
    assert wl["params"][-1][0].shape == (84, 10)


def _loss_only(net, x, labels, params):
    tensors, _ = orc.forward(net, x, params)
    return orc.head_fwd_vjp(tensors[net["ops"][-1]["in"]], params[-1][0], params[-1][1], labels, need_dx=False)[0]


@pytest.mark.parametrize("name,kw", [
    ("tiny", dict(batch=4)),
    ("lenet5", dict(batch=3)),
    ("resnet56", dict(batch=3, blocks_per_stage=2, hw=8)),
    ("resnet50", dict(batch=4, hw=32, stages=(2, 1, 1, 1), classes=7, dtype="f32")),
    ("mobilenetv2", dict(batch=4, hw=64, classes=5)),
])
def test_whole_step_gradient_by_finite_differences(name, kw):
    """The interpreter's reverse chaining (residual fan-in, projections, pools, flatten) is
    pinned by differentiating the whole loss numerically at a few coordinates of every
    parameter tensor."""
    net = nets.CONFIGS[name](**kw)
    wl = nets.make_workload(net, perturb=True)
    params = [[a.astype(np.float64) for a in p] for p in wl["params"]]
    out = orc.train_step(net, wl["x"], wl["labels"], params)
    rng = np.random.default_rng(3)
    worst = 0.0
    for i, p in enumerate(params):
        for j, a in enumerate(p):
            idx = rng.choice(a.size, size=min(2, a.size), replace=False)
            f = lambda: _loss_only(net, wl["x"], wl["labels"], params)
            ref = out["grads"][i][j].reshape(-1)[idx]
            # ReLU/ReLU6/max-pool kinks make a single step size unreliable: a kink crossing
            # spoils one h, a wrong gradient spoils all of them
            err = np.full(len(idx), np.inf)
            for h in (1e-5, 1e-6, 3e-7):
                g = fd_grad(f, a, h=h, idx=idx).reshape(-1)[idx]
                err = np.minimum(err, np.abs(g - ref))
            # (a beta that feeds a 1x1 conv + BatchNorm has an exactly zero gradient: absolute floor)
            scale = np.abs(out["grads"][i][j]).max() + 1e-3
            worst = max(worst, float(np.max(err) / scale))
    assert worst < 2e-5, worst
    # update: theta' = theta - lr * (mu*0 + g)
    for i, p in enumerate(params):
        for j, a in enumerate(p):
            np.testing.assert_allclose(out["params"][i][j], a - net["lr"] * out["grads"][i][j], rtol=1e-12, atol=1e-15)
            np.testing.assert_allclose(out["velocity"][i][j], out["grads"][i][j], rtol=0, atol=0)


def test_initial_loss_is_near_log_classes():
    for name, kw in [("tiny", {}), ("lenet5", dict(batch=16))]:
        net = nets.CONFIGS[name](**kw)
        wl = nets.make_workload(net)
        loss = _loss_only(net, wl["x"], wl["labels"], wl["params"])
        assert abs(loss - math.log(net["classes"])) < 1.5, (name, loss)


def test_lenet_loss_falls_over_ten_steps_and_step_is_functional():
    net = nets.lenet5(batch=16)
    wl = nets.make_workload(net)
    params = wl["params"]
    snapshot = [[a.copy() for a in p] for p in params]
    vel, losses = None, []
    for _ in range(10):
        out = orc.train_step(net, wl["x"], wl["labels"], params, vel)
        params, vel = out["params"], out["velocity"]
        losses.append(out["loss"])
    assert losses[-1] < losses[0]
    assert all(b <= a + 1e-9 for a, b in zip(losses, losses[1:]))
    # the inputs of the first step were not modified: the step is a pure function of them
    for p, q in zip(snapshot, wl["params"]):
        for a, b in zip(p, q):
            np.testing.assert_array_equal(a, b)


def test_bf16_step_rounds_stored_tensors_only():
    net = nets.resnet50(batch=2, hw=32, stages=(1, 1, 1, 1), classes=5)
    wl = nets.make_workload(net)
    out = orc.train_step(net, wl["x"], wl["labels"], wl["params"])
    for t in out["tensors"][:-1]:
        np.testing.assert_array_equal(t, orc.round_bf16(t))
    # parameter gradients are not rounded to bf16
    g = out["grads"][0][0]
    assert not np.array_equal(g, orc.round_bf16(g))
    assert np.isfinite(out["loss"])


@pytest.mark.parametrize("act", ["none", "relu", "relu6"])
def test_bn_forward_output_closed_form_with_every_input_nontrivial(act):
    """y = act(gamma (x - mean)/sqrt(var + eps) + beta + residual), written out with NumPy: gamma, beta, the
    residual and the clamp all enter (a dropped or doubled term, a residual added after the activation or a
    gamma applied to the residual would each fail)."""
    x = RNG.standard_normal((3, 5, 4, 7)) * 1.7 - 0.8
    res = RNG.standard_normal(x.shape) * 2.0 + 1.0
    gamma = 1.0 + 0.5 * RNG.standard_normal(7)
    beta = RNG.standard_normal(7) + 2.5
    eps = 1e-3
    xf = x.reshape(-1, 7)
    z = gamma * (x - xf.mean(0)) / np.sqrt(((xf - xf.mean(0)) ** 2).mean(0) + eps) + beta + res
    want = z if act == "none" else np.maximum(z, 0.0) if act == "relu" else np.minimum(np.maximum(z, 0.0), 6.0)
    if act == "relu6":
        assert (z > 6).any() and (z < 0).any()   # both clamps are exercised
    y, _, _ = orc.bn_act_fwd(x, res, gamma, beta, eps, act)
    np.testing.assert_allclose(y, want, rtol=1e-12, atol=1e-12)
    y_nores, _, _ = orc.bn_act_fwd(x, None, gamma, beta, eps, "none")
    np.testing.assert_allclose(y_nores, z - res, rtol=1e-12, atol=1e-12)


def test_bf16_fan_in_sums_cotangents_in_reverse_consumer_order_rounding_after_each_addition():
    """A tensor with two consumers (a convolution and, later, the residual input of a BatchNorm): in a bf16
    workload its cotangent is round(round(residual cotangent) + convolution's input cotangent), i.e. the later
    consumer contributes first and the sum is rounded to bf16 after every addition.  Rebuilt here from the
    oracle's per-op pullbacks and an independent rounding routine (the workload generator's, NumPy integer
    arithmetic); the other order gives different bits."""
    ops = [dict(kind="conv", **{"in": 0}, k=8, r=3, s=3, stride=1, pad=1, groups=1, bias=False, act="none"),
           dict(kind="bn", **{"in": 1}, res=-1, act="relu", eps=1e-5),                    # tensor 2: two consumers
           dict(kind="conv", **{"in": 2}, k=8, r=3, s=3, stride=1, pad=1, groups=1, bias=False, act="none"),
           dict(kind="bn", **{"in": 3}, res=2, act="relu", eps=1e-5),
           dict(kind="head", **{"in": 4}, classes=5)]
    net = dict(name="fanin", dtype="bf16", input=(4, 6, 6, 8), classes=5, lr=0.1, momentum=0.9, seed=77, init="he",
               x_dist="normal", ops=ops)
    wl = nets.make_workload(net, perturb=True)
    out = orc.train_step(net, wl["x"], wl["labels"], wl["params"], keep_cotangents=True)
    t, cot = out["tensors"], out["cotangents"]
    r32 = lambda a: nets.to_bf16_grid(np.asarray(a, np.float32)).astype(np.float64)   # noqa: E731
    # pullback of the second BatchNorm (op 3) from the cotangent the oracle fed it
    _, mean, invstd = orc.bn_act_fwd(t[3], t[2], wl["params"][3][0], wl["params"][3][1], 1e-5, "relu")
    dx3, dres, _, _ = orc.bn_act_vjp(t[3], t[4], wl["params"][3][0], mean, invstd, cot[4], "relu", True)
    np.testing.assert_array_equal(cot[3], r32(dx3))
    w2 = r32(wl["params"][2][0])
    dconv, _, _ = orc.conv2d_vjp(t[2], w2, cot[3], 1, 1)
    in_order = r32(r32(dres) + dconv)          # the later consumer (the residual input) first
    np.testing.assert_array_equal(cot[2], in_order)
    assert not np.array_equal(in_order, r32(r32(dconv) + dres))


def test_gather_rows_and_its_inout_pullback():
    """Indexing against NumPy's fancy indexing and np.add.at (repeated indices included), the adjoint identity
    <gather(x), dy> = <x, scatter(dy)>, accumulation into what dx already holds, and the point of the inout
    formulation (Section 4.3): rows that are not named are not touched."""
    x = RNG.standard_normal((50, 7))
    idx = np.array([3, 49, 3, 0, 17, 3], np.int32)
    y = orc.gather_rows_fwd(x, idx)
    np.testing.assert_array_equal(y, x[idx])
    dy = RNG.standard_normal(y.shape)
    base = RNG.standard_normal(x.shape)
    dx = base.copy()
    orc.gather_rows_vjp(dy, idx, dx)
    want = base.copy()
    np.add.at(want, idx, dy)
    np.testing.assert_allclose(dx, want, rtol=1e-15, atol=1e-15)
    untouched = np.setdiff1d(np.arange(50), idx)
    np.testing.assert_array_equal(dx[untouched], base[untouched])
    zero = np.zeros_like(x)
    orc.gather_rows_vjp(dy, idx, zero)
    np.testing.assert_allclose(np.sum(y * dy), np.sum(x * zero), rtol=1e-13)
    # an index out of range reads zeros and writes nothing
    bad = np.array([2, -1, 50], np.int32)
    yb = orc.gather_rows_fwd(x, bad)
    np.testing.assert_array_equal(yb[1:], 0.0)
    dxb = base.copy()
    orc.gather_rows_vjp(dy[:3], bad, dxb)
    np.testing.assert_array_equal(np.delete(dxb, 2, axis=0), np.delete(base, 2, axis=0))


@pytest.mark.parametrize("act,use_res,use_bias", [("none", False, False), ("relu", True, True), ("relu6", False, True)])
def test_bn_inference_update_and_fold(act, use_res, use_bias):
    """Inference-mode BatchNorm written out with NumPy; the running-statistics update against NumPy's unbiased
    variance (momentum 1 from any start gives the batch statistics themselves); folding: the convolution with
    folded filter and bias IS the convolution followed by inference-mode BatchNorm."""
    x = RNG.standard_normal((2, 6, 5, 3))
    w = RNG.standard_normal((3, 3, 3, 4)) * 0.4
    bias = RNG.standard_normal(4) if use_bias else None
    gamma, beta = 1.0 + 0.4 * RNG.standard_normal(4), RNG.standard_normal(4) + 2.0
    rm, rv = RNG.standard_normal(4), 0.5 + RNG.random(4)
    eps = 1e-3
    u = orc.conv2d_fwd(x, w, bias, 1, 1)
    res = RNG.standard_normal(u.shape) if use_res else None
    z = gamma * (u - rm) / np.sqrt(rv + eps) + beta + (res if use_res else 0.0)
    want = z if act == "none" else np.maximum(z, 0) if act == "relu" else np.clip(z, 0, 6)
    y = orc.bn_inference_fwd(u, res, gamma, beta, rm, rv, eps, act)
    np.testing.assert_allclose(y, want, rtol=1e-12, atol=1e-12)
    # running statistics
    _, mean, invstd = orc.bn_act_fwd(u, None, gamma, beta, eps, "none")
    uf = u.reshape(-1, 4)
    m = uf.shape[0]
    rm1, rv1 = orc.bn_update_running(mean, invstd, rm, rv, m, 0.1, eps)
    np.testing.assert_allclose(rm1, 0.9 * rm + 0.1 * uf.mean(0), rtol=1e-12)
    np.testing.assert_allclose(rv1, 0.9 * rv + 0.1 * uf.var(0, ddof=1), rtol=1e-9)
    rm2, rv2 = orc.bn_update_running(mean, invstd, rm, rv, m, 1.0, eps)
    np.testing.assert_allclose(rm2, uf.mean(0), rtol=1e-12)
    np.testing.assert_allclose(rv2, uf.var(0, ddof=1), rtol=1e-9)
    # folding
    wf, bf = orc.bn_fold(w, bias, gamma, beta, rm, rv, eps)
    folded = orc.conv2d_fwd(x, wf, bf, 1, 1)
    if use_res:
        folded = folded + res
    folded = orc.bias_act_fwd(folded, None, act)
    np.testing.assert_allclose(folded, y, rtol=1e-11, atol=1e-11)
