"""GPU parity: every entry point of the C ABI against the CPU oracle on the same seeded inputs.

Tolerances.  Relative L2 error per tensor, ||gpu - oracle||_2 / ||oracle||_2.
 fp32 storage: the GPU accumulates in fp32, the oracle in fp64; per-op outputs agree to ~1e-6,
   the bound used is 2e-5 (1e-4 for long reductions).  Whole steps use the workload's stated
   bounds: 1e-4 on the loss, 1e-3 on every gradient and updated parameter.
 bf16 storage: both sides round the same tensors to bf16 (ties to even) but accumulate in
   different precisions, so a few outputs land on the other side of a rounding boundary
   (one bf16 ulp = 2^-8 relative).  Per-op bound 4e-3 for bf16 outputs, 2e-3 for fp32
   outputs computed from bf16 inputs; whole steps 5e-3 on the loss, 2e-2 on gradients.
 A gradient that is exactly zero in exact arithmetic (the beta of a BatchNorm that feeds a
 1x1 convolution followed by BatchNorm) is compared on an absolute scale instead.
"""
import numpy as np
import pytest

from oracle import oracle as orc
from workloads import nets

torch = pytest.importorskip("torch")
from paper_2102_13243_amd import binding as B  # noqa: E402
from local_check import LocalChecker  # noqa: E402

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def to_dev(a, bf16=False, dtype=None):
    if a is None:
        return None
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32 if dtype is None else dtype))
    if bf16:
        t = t.to(torch.bfloat16)
    return t.to(DEV)


def to_host(t):
    torch.cuda.synchronize()
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def empty(shape, bf16=False):
    return torch.full(tuple(shape), float("nan"), dtype=torch.bfloat16 if bf16 else torch.float32, device=DEV)


def ws(nbytes):
    return torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device=DEV)


def rel_l2(a, b):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    den = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / den) if den > 0 else float(np.linalg.norm(a - b))


def grid(a, bf16):
    """Input values on the storage grid (bf16 inputs must be exactly representable)."""
    a = np.asarray(a, np.float32)
    return nets.to_bf16_grid(a) if bf16 else a


RNG = np.random.default_rng(11)

# n h w c k r stride pad
CONV_SHAPES = [
    (2, 9, 9, 8, 16, 3, 1, 1),        # single tile, vector path
    (3, 17, 13, 16, 24, 3, 1, 1),     # ragged M, N < tile
    (2, 16, 16, 32, 160, 3, 2, 1),    # two N tiles with a tail, stride 2
    (4, 14, 14, 64, 64, 1, 1, 0),     # 1x1: plain GEMM fast path
    (2, 15, 15, 40, 48, 1, 2, 0),     # strided 1x1 projection, odd extent
    (2, 12, 12, 24, 8, 5, 1, 2),      # 5x5
    (2, 23, 23, 3, 16, 3, 1, 1),      # 3 input channels: element-wise loader
    (2, 28, 28, 1, 6, 5, 1, 2),       # LeNet conv1 shape
    (2, 14, 14, 6, 16, 5, 1, 0),      # LeNet conv2 shape
    (5, 1, 1, 400, 120, 1, 1, 0),     # dense layer
    (130, 1, 1, 84, 10, 1, 1, 0),     # dense, ragged everything
    (1, 35, 35, 8, 8, 7, 2, 3),       # 7x7 stride 2 (stem-like), N = 1
    (2, 8, 8, 128, 256, 3, 1, 1),     # deep K loop (1152), two N tiles
    (2, 6, 6, 16, 16, 3, 1, 2),       # pad wider than "same"
    (2, 15, 15, 64, 128, 1, 2, 0),    # strided 1x1, odd extent, fast path: dgrad scatters rows and zero-fills
    (2, 16, 16, 128, 64, 1, 2, 0),    # strided 1x1, even extent, 64-wide output
    (3, 20, 20, 64, 64, 3, 1, 1),     # 64-wide GEMMs in all three passes, several ragged row tiles
    (2, 30, 30, 64, 256, 1, 1, 0),    # one k-tile forward (no ring), two in dgrad
    (2, 9, 9, 256, 64, 1, 1, 0),      # four k-tiles forward, one in dgrad
    (2, 16, 16, 64, 128, 3, 2, 1),    # strided 3x3, fast path: dgrad as one GEMM per parity class of input pixels
    (2, 15, 13, 128, 64, 3, 2, 1),    # ... odd extents: the four classes differ in size
    (1, 11, 11, 64, 64, 5, 2, 2),     # ... 5x5: two or three taps per axis and class
    (2, 14, 14, 64, 64, 3, 2, 0),     # ... no padding: the last input row and column meet no output pixel
    (2, 64, 64, 32, 64, 3, 1, 1),     # fp32: enough work and few enough tiles for the 64x32 and 32x32 tiles
]


@pytest.mark.parametrize("bf16", [False, True], ids=["f32", "bf16"])
@pytest.mark.parametrize("shape", CONV_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_conv2d_fwd_and_vjp(shape, bf16):
    n, h, w, c, k, r, stride, pad = shape
    x = grid(RNG.standard_normal((n, h, w, c)), bf16)
    wt = grid(RNG.standard_normal((r, r, c, k)) * np.sqrt(2.0 / (r * r * c)), bf16)
    bias = RNG.standard_normal(k).astype(np.float32)
    d = B.ConvDesc(n, h, w, c, k, r, r, stride, pad, 1, B.S4TF_BF16 if bf16 else B.S4TF_F32, B.ACT["relu"], 0)
    p = (h + 2 * pad - r) // stride + 1
    q = (w + 2 * pad - r) // stride + 1
    xd, wd, bd = to_dev(x, bf16), to_dev(wt, bf16), to_dev(bias)
    y = empty((n, p, q, k), bf16)
    B.s4tf_conv2d_fwd(d, xd, wd, bd, y)
    y_ref = orc.bias_act_fwd(orc.conv2d_fwd(x, wt, bias, stride, pad), None, "relu")
    if bf16:
        y_ref = orc.round_bf16(y_ref)
    y_gpu = to_host(y)
    assert np.isfinite(y_gpu).all()
    assert rel_l2(y_gpu, y_ref) < (4e-3 if bf16 else 2e-5)
    # pullback, from the oracle's y so that both sides use the same activation mask
    dy = grid(RNG.standard_normal((n, p, q, k)), bf16)
    dz_ref, _ = orc.bias_act_vjp(y_ref, dy, "relu", need_db=False)
    dx_ref, dw_ref, db_ref = orc.conv2d_vjp(x, wt, dz_ref, stride, pad, need_dx=True, need_db=True)
    dx = empty((n, h, w, c), bf16)
    dx.fill_(float("nan"))   # every element must be written, also those no output pixel reads
    dw, db = empty((r, r, c, k)), empty((k,))
    wsp = ws(B.s4tf_conv2d_vjp_workspace_bytes(d))
    B.s4tf_conv2d_vjp(d, xd, wd, to_dev(y_ref, bf16), to_dev(dy, bf16), dx, dw, db, wsp)
    tol_act = 4e-3 if bf16 else 2e-5
    tol_par = 2e-3 if bf16 else 1e-4
    assert rel_l2(to_host(dx), orc.round_bf16(dx_ref) if bf16 else dx_ref) < tol_act
    assert rel_l2(to_host(dw), dw_ref) < tol_par
    assert rel_l2(to_host(db), db_ref) < tol_par
    # accumulate into an existing cotangent, no bias gradient, no dx
    d.accumulate_dx = 1
    base = grid(RNG.standard_normal((n, h, w, c)), bf16)
    dx2 = to_dev(base, bf16)
    B.s4tf_conv2d_vjp(d, xd, wd, to_dev(y_ref, bf16), to_dev(dy, bf16), dx2, dw, None, wsp)
    want = base + dx_ref
    assert rel_l2(to_host(dx2), orc.round_bf16(want) if bf16 else want) < tol_act
    dw.fill_(float("nan"))
    B.s4tf_conv2d_vjp(d, xd, wd, to_dev(y_ref, bf16), to_dev(dy, bf16), None, dw, None, wsp)
    assert rel_l2(to_host(dw), dw_ref) < tol_par


# n h w c r stride pad
DW_SHAPES = [(2, 14, 14, 32, 3, 1, 1), (2, 15, 15, 96, 3, 2, 1), (1, 7, 7, 960, 3, 1, 1), (3, 9, 9, 6, 3, 1, 1),
             (2, 28, 28, 144, 3, 2, 1),
             (2, 13, 18, 24, 3, 1, 1),      # not square, widths that leave a ragged last strip
             (2, 13, 18, 24, 3, 2, 1),
             (2, 12, 17, 40, 3, 2, 1),      # even height, odd width, stride 2
             (8, 15, 64, 1024, 3, 1, 1),    # enough threads for the longest row walk (14 rows), last chunk of one row
             (8, 29, 128, 1024, 3, 2, 1),   # ... and for 7-row walks at stride 2
             (2, 9, 9, 16, 3, 1, 0),        # no padding: the general kernels
             (2, 11, 11, 8, 2, 2, 0)]       # 2x2 filter


@pytest.mark.parametrize("bf16", [False, True], ids=["f32", "bf16"])
@pytest.mark.parametrize("shape", DW_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_depthwise_conv(shape, bf16):
    n, h, w, c, r, stride, pad = shape
    x = grid(RNG.standard_normal((n, h, w, c)), bf16)
    wt = grid(RNG.standard_normal((r, r, 1, c)) * np.sqrt(2.0 / (r * r)), bf16)
    d = B.ConvDesc(n, h, w, c, c, r, r, stride, pad, c, B.S4TF_BF16 if bf16 else B.S4TF_F32, B.ACT["none"], 0)
    p = (h + 2 * pad - r) // stride + 1
    q = (w + 2 * pad - r) // stride + 1
    xd, wd = to_dev(x, bf16), to_dev(wt, bf16)
    y = empty((n, p, q, c), bf16)
    B.s4tf_conv2d_fwd(d, xd, wd, None, y)
    y_ref = orc.conv2d_fwd(x, wt, None, stride, pad, groups=c)
    assert rel_l2(to_host(y), orc.round_bf16(y_ref) if bf16 else y_ref) < (4e-3 if bf16 else 2e-5)
    dy = grid(RNG.standard_normal((n, p, q, c)), bf16)
    dx_ref, dw_ref, _ = orc.conv2d_vjp(x, wt, dy, stride, pad, groups=c)
    dx, dw = empty((n, h, w, c), bf16), empty((r, r, 1, c))
    wsp = ws(B.s4tf_conv2d_vjp_workspace_bytes(d))
    B.s4tf_conv2d_vjp(d, xd, wd, None, to_dev(dy, bf16), dx, dw, None, wsp)
    assert rel_l2(to_host(dx), orc.round_bf16(dx_ref) if bf16 else dx_ref) < (4e-3 if bf16 else 2e-5)
    assert rel_l2(to_host(dw), dw_ref) < (2e-3 if bf16 else 1e-4)
    if n * h * w * c > 4_000_000:
        return
    # bias and activation in the forward pass; the pullback accumulating into an existing cotangent
    bias = RNG.standard_normal(c).astype(np.float32)
    d2 = B.ConvDesc(n, h, w, c, c, r, r, stride, pad, c, B.S4TF_BF16 if bf16 else B.S4TF_F32, B.ACT["relu6"], 0)
    B.s4tf_conv2d_fwd(d2, xd, wd, to_dev(bias), y)
    y2_ref = orc.bias_act_fwd(orc.conv2d_fwd(x, wt, bias, stride, pad, groups=c), None, "relu6")
    assert rel_l2(to_host(y), orc.round_bf16(y2_ref) if bf16 else y2_ref) < (4e-3 if bf16 else 2e-5)
    base = grid(RNG.standard_normal((n, h, w, c)), bf16)
    d3 = B.ConvDesc(n, h, w, c, c, r, r, stride, pad, c, B.S4TF_BF16 if bf16 else B.S4TF_F32, B.ACT["none"], 1)
    dx2 = to_dev(base, bf16)
    B.s4tf_conv2d_vjp(d3, xd, wd, None, to_dev(dy, bf16), dx2, dw, None, wsp)
    want = base + dx_ref
    assert rel_l2(to_host(dx2), orc.round_bf16(want) if bf16 else want) < (4e-3 if bf16 else 2e-5)


BN_SHAPES = [(2, 5, 7, 16), (4, 16, 16, 64), (3, 9, 9, 6), (2, 7, 7, 960), (64, 8, 8, 32), (1, 1, 3, 8)]


@pytest.mark.parametrize("bf16", [False, True], ids=["f32", "bf16"])
@pytest.mark.parametrize("act,use_res", [("none", False), ("relu", False), ("relu", True), ("relu6", True)])
@pytest.mark.parametrize("shape", BN_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_bn_relu_fwd_and_vjp(shape, act, use_res, bf16):
    n, h, w, c = shape
    x = grid(RNG.standard_normal(shape) * 2.0 + 3.0, bf16)   # mean well away from zero
    res = grid(RNG.standard_normal(shape), bf16) if use_res else None
    gamma = (1.0 + 0.3 * RNG.standard_normal(c)).astype(np.float32)
    beta = (0.2 * RNG.standard_normal(c) + (3.0 if act == "relu6" else 0.0)).astype(np.float32)
    d = B.BnDesc(n, h, w, c, 1e-5, B.ACT[act], B.S4TF_BF16 if bf16 else B.S4TF_F32, 0)
    wsp = ws(B.s4tf_bn_relu_workspace_bytes(d))
    xd, rd, gd, bd = to_dev(x, bf16), to_dev(res, bf16), to_dev(gamma), to_dev(beta)
    y, mean, invstd = empty(shape, bf16), empty((c,)), empty((c,))
    B.s4tf_bn_relu_fwd(d, xd, rd, gd, bd, y, mean, invstd, wsp)
    y_ref, mean_ref, invstd_ref = orc.bn_act_fwd(x, res, gamma, beta, 1e-5, act)
    if bf16:
        y_ref = orc.round_bf16(y_ref)
    assert rel_l2(to_host(mean), mean_ref) < 2e-6
    assert rel_l2(to_host(invstd), invstd_ref) < 2e-5
    assert rel_l2(to_host(y), y_ref) < (4e-3 if bf16 else 2e-5)
    dy = grid(RNG.standard_normal(shape), bf16)
    dx_ref, dres_ref, dg_ref, db_ref = orc.bn_act_vjp(x, y_ref, gamma, mean_ref, invstd_ref, dy, act, use_res)
    dx, dres = empty(shape, bf16), (empty(shape, bf16) if use_res else None)
    dg, db = empty((c,)), empty((c,))
    B.s4tf_bn_relu_vjp(d, xd, to_dev(y_ref, bf16), gd, None, to_dev(mean_ref), to_dev(invstd_ref), to_dev(dy, bf16), dx,
                       dres, dg, db, wsp)
    assert rel_l2(to_host(dg), dg_ref) < 1e-4
    assert rel_l2(to_host(db), db_ref) < 1e-4
    assert rel_l2(to_host(dx), orc.round_bf16(dx_ref) if bf16 else dx_ref) < (6e-3 if bf16 else 5e-5)
    if not use_res and act != "none":
        # beta given, no residual: the activation mask is rebuilt from x with the statistics the GPU's own
        # forward pass saved, y is not read (NULL).  An element whose z rounds to the other side of 0 (or 6)
        # than the oracle's may differ; the tolerances are those of the first call.
        dx.fill_(float("nan"))
        B.s4tf_bn_relu_vjp(d, xd, None, gd, bd, mean, invstd, to_dev(dy, bf16), dx, None, dg, db, wsp)
        assert rel_l2(to_host(dg), dg_ref) < 1e-4
        assert rel_l2(to_host(db), db_ref) < 1e-4
        assert rel_l2(to_host(dx), orc.round_bf16(dx_ref) if bf16 else dx_ref) < (6e-3 if bf16 else 5e-5)
    if use_res:
        assert rel_l2(to_host(dres), dres_ref) == 0.0
        d.accumulate_dres = 1
        base = grid(RNG.standard_normal(shape), bf16)
        dres2 = to_dev(base, bf16)
        B.s4tf_bn_relu_vjp(d, xd, to_dev(y_ref, bf16), gd, None, to_dev(mean_ref), to_dev(invstd_ref), to_dev(dy, bf16), dx,
                           dres2, dg, db, wsp)
        want = base + dres_ref
        assert rel_l2(to_host(dres2), orc.round_bf16(want) if bf16 else want) < (4e-3 if bf16 else 1e-6)


@pytest.mark.parametrize("bf16", [False, True], ids=["f32", "bf16"])
@pytest.mark.parametrize("kind,shape", [(B.POOL_AVG2, (3, 10, 10, 16)), (B.POOL_AVG2, (2, 28, 28, 6)),
                                        (B.POOL_AVG2, (2, 7, 9, 5)), (B.POOL_MAX3S2, (2, 16, 16, 64)),
                                        (B.POOL_MAX3S2, (3, 9, 11, 7)), (B.POOL_MAX3S2, (1, 2, 2, 3))])
def test_pool2d(kind, shape, bf16):
    n, h, w, c = shape
    x = grid(RNG.standard_normal(shape), bf16)
    if kind == B.POOL_MAX3S2:
        x = np.maximum(x, 0)   # ties among zeros, as after a ReLU
    d = B.PoolDesc(n, h, w, c, kind, B.S4TF_BF16 if bf16 else B.S4TF_F32, 0)
    y_ref = orc.avgpool2_fwd(x) if kind == B.POOL_AVG2 else orc.maxpool3s2_fwd(x)
    xd = to_dev(x, bf16)
    y = empty(y_ref.shape, bf16)
    B.s4tf_pool2d_fwd(d, xd, y)
    if kind == B.POOL_MAX3S2:
        np.testing.assert_array_equal(to_host(y), y_ref)
    else:
        assert rel_l2(to_host(y), orc.round_bf16(y_ref) if bf16 else y_ref) < (4e-3 if bf16 else 1e-6)
    dy = grid(RNG.standard_normal(y_ref.shape), bf16)
    dx_ref = orc.avgpool2_vjp(dy, x.shape) if kind == B.POOL_AVG2 else orc.maxpool3s2_vjp(x, dy)
    dx = empty(shape, bf16)
    B.s4tf_pool2d_vjp(d, xd, to_dev(dy, bf16), dx)
    assert rel_l2(to_host(dx), orc.round_bf16(dx_ref) if bf16 else dx_ref) < (4e-3 if bf16 else 1e-6)
    d.accumulate_dx = 1
    base = grid(RNG.standard_normal(shape), bf16)
    dx2 = to_dev(base, bf16)
    B.s4tf_pool2d_vjp(d, xd, to_dev(dy, bf16), dx2)
    want = base + dx_ref
    assert rel_l2(to_host(dx2), orc.round_bf16(want) if bf16 else want) < (4e-3 if bf16 else 1e-6)


@pytest.mark.parametrize("bf16", [False, True], ids=["f32", "bf16"])
@pytest.mark.parametrize("shape", [(8, 16, 16, 16, 10), (128, 1, 1, 84, 10), (6, 7, 7, 256, 1000), (3, 2, 3, 20, 7)],
                         ids=lambda s: "x".join(map(str, s)))
def test_head(shape, bf16):
    n, h, w, c, k = shape
    x = grid(RNG.standard_normal((n, h, w, c)), bf16)
    W = (RNG.standard_normal((c, k)) * np.sqrt(2.0 / c)).astype(np.float32)
    b = (0.1 * RNG.standard_normal(k)).astype(np.float32)
    labels = RNG.integers(0, k, n).astype(np.int32)
    d = B.HeadDesc(n, h, w, c, k, B.S4TF_BF16 if bf16 else B.S4TF_F32)
    wsp = ws(B.s4tf_pool_dense_xent_workspace_bytes(d))
    loss, dx, dW, db, logits = empty((4,)), empty((n, h, w, c), bf16), empty((c, k)), empty((k,)), empty((n, k))
    B.s4tf_pool_dense_xent_fwd_vjp(d, to_dev(x, bf16), to_dev(W), to_dev(b), to_dev(labels, dtype=np.int32), loss, dx, dW,
                                   db, logits, wsp)
    l_ref, dx_ref, dW_ref, db_ref, z_ref = orc.head_fwd_vjp(x, W, b, labels)
    assert rel_l2(to_host(logits), z_ref) < 2e-5
    assert abs(to_host(loss)[0] - l_ref) < 1e-5 * abs(l_ref)
    assert rel_l2(to_host(dW), dW_ref) < 5e-5
    assert rel_l2(to_host(db), db_ref) < 5e-5
    assert rel_l2(to_host(dx), orc.round_bf16(dx_ref) if bf16 else dx_ref) < (4e-3 if bf16 else 5e-5)
    # W = 0, b = 0: loss = ln(classes)
    B.s4tf_pool_dense_xent_fwd_vjp(d, to_dev(x, bf16), to_dev(np.zeros_like(W)), to_dev(np.zeros_like(b)),
                                   to_dev(labels, dtype=np.int32), loss, None, dW, db, None, wsp)
    assert abs(to_host(loss)[0] - np.log(k)) < 1e-6 * np.log(k)


@pytest.mark.parametrize("count", [1, 3, 4, 634, 100003])
def test_sgd_momentum(count):
    p = RNG.standard_normal(count).astype(np.float32)
    v = RNG.standard_normal(count).astype(np.float32)
    g = RNG.standard_normal(count).astype(np.float32)
    pd, vd, gd = to_dev(p), to_dev(v), to_dev(g)
    low = torch.zeros(count + 8, dtype=torch.bfloat16, device=DEV)
    B.s4tf_sgd_momentum(count, pd, vd, gd, low, 0.1, 0.9)
    p64, v64 = p.astype(np.float64), v.astype(np.float64)
    orc.sgd_momentum(p64, v64, g, 0.1, 0.9)
    assert rel_l2(to_host(vd), v64) < 1e-6 and rel_l2(to_host(pd), p64) < 1e-6
    # the bf16 working copy is the rounded fp32 master (same precision on both sides)
    np.testing.assert_array_equal(to_host(low)[:count], orc.round_bf16(to_host(pd)))
    assert float(low[count:].abs().max()) == 0.0
    # constant gradient, several steps: closed form v_k = g (1 - mu^k)/(1 - mu)
    pd, vd = to_dev(p), to_dev(np.zeros_like(v))
    for _ in range(5):
        B.s4tf_sgd_momentum(count, pd, vd, gd, None, 0.1, 0.9)
    assert rel_l2(to_host(vd), g.astype(np.float64) * (1 - 0.9 ** 5) / 0.1) < 1e-6


# ---------------------------------------------------------------------------------------------------
# whole steps
# ---------------------------------------------------------------------------------------------------
def oracle_step_with_conditioning(net, wl, jitter=1e-7):
    """The oracle's step, plus for every parameter gradient how far it moves (relative L2) when the
    oracle's own convolution outputs are perturbed by a relative `jitter` at the fp32 rounding level.
    Gradients that are sums of almost cancelling terms (the beta of a BatchNorm whose consumer is a
    convolution followed by another BatchNorm) move by orders of magnitude more than the jitter;
    no two implementations can agree on them end to end more closely than that."""
    ref = orc.train_step(net, wl["x"], wl["labels"], wl["params"])
    rng = np.random.default_rng(99)
    fwd0 = orc.conv2d_fwd
    try:
        orc.conv2d_fwd = lambda *a, **k: (lambda y: y * (1.0 + jitter * rng.standard_normal(y.shape)))(fwd0(*a, **k))
        jit = orc.train_step(net, wl["x"], wl["labels"], wl["params"])
    finally:
        orc.conv2d_fwd = fwd0
    ref["sensitivity"] = [[rel_l2(x, y) for x, y in zip(p, q)] for p, q in zip(jit["grads"], ref["grads"])]
    return ref


def compare_step(net, gpu, ref, loss_tol, grad_tol, param_tol):
    """End-to-end comparison.  Bound per gradient tensor: grad_tol, widened to 100x the tensor's own
    sensitivity to a 1e-7 jitter where that is larger (see oracle_step_with_conditioning).  When a
    ReLU decision differs between the two forward passes the gradients are only reported: the two
    runs then differentiate different piecewise-linear functions, and the step has already been
    verified op by op by the local checks."""
    assert abs(gpu["loss"] - ref["loss"]) <= loss_tol * abs(ref["loss"]), (gpu["loss"], ref["loss"])
    flips = count_mask_flips(net, gpu, ref) if "state" in gpu and "tensors" in ref else 0
    elems = sum(t.size for t in ref["tensors"][1:-1]) if "tensors" in ref else 1
    assert flips <= max(3, 2e-6 * elems), ("activation decisions differ in too many places", flips, elems)
    if flips:
        errs = [rel_l2(a, b) for pg, pr in zip(gpu["grads"], ref["grads"]) for a, b in zip(pg, pr)]
        print("\n%s: loss gpu %.7g oracle %.7g; %d of %d activation decisions differ, gradients not compared end to "
              "end (median rel-L2 %.2g, max %.2g)" % (net["name"], gpu["loss"], ref["loss"], flips, elems,
                                                      float(np.median(errs)), max(errs)))
        return
    gmax = max(float(np.abs(g).max()) for p in ref["grads"] for g in p)
    sens = ref.get("sensitivity")
    worst = {"grad": (0.0, None), "param": (0.0, None)}
    widened, total = 0, 0
    for i, (pg, pr) in enumerate(zip(gpu["grads"], ref["grads"])):
        for j, (a, b) in enumerate(zip(pg, pr)):
            assert np.isfinite(a).all(), (i, j)
            total += 1
            e = rel_l2(a, b)
            if e > grad_tol and (float(np.abs(a - b).max()) <= 1e-6 * gmax or (sens is not None and sens[i][j] > 0.5)):
                # a gradient that is exactly zero in exact arithmetic (the oracle's own value is rounding
                # noise): both sides must be negligible on the scale of the net's gradients
                assert float(np.abs(a).max()) <= 1e-4 * gmax and float(np.abs(b).max()) <= 1e-4 * gmax, (i, j)
                continue
            bound = grad_tol
            if sens is not None and 100.0 * sens[i][j] > grad_tol:
                bound = 100.0 * sens[i][j]
                widened += 1
            assert e <= bound, ("gradient", i, j, net["ops"][i]["kind"], e, bound)
            assert rel_l2(gpu["velocity"][i][j], ref["velocity"][i][j]) <= bound, ("velocity", i, j)
            if bound == grad_tol and e > worst["grad"][0]:
                worst["grad"] = (e, (i, j, net["ops"][i]["kind"]))
            ep = rel_l2(gpu["params"][i][j], ref["params"][i][j])
            if ep > worst["param"][0]:
                worst["param"] = (ep, (i, j))
            assert ep <= max(param_tol, bound), ("param", i, j, ep)
    print("\n%s: loss gpu %.7g oracle %.7g; worst rel-L2 grad %.3g at %s, param %.3g; %d of %d gradient tensors compared with a bound widened by their conditioning"
          % (net["name"], gpu["loss"], ref["loss"], worst["grad"][0], worst["grad"][1], worst["param"][0], widened, total))


def run_gpu_steps(net, wl, steps=1, local=False):
    st = B.TrainState(net, wl["params"], DEV)
    xd, ld = st.upload_batch(wl["x"], wl["labels"])
    losses = []
    for _ in range(steps):
        st.step(xd, ld)
        torch.cuda.synchronize()
        losses.append(float(st.loss[0].item()))
    if local:   # every op of the finished step against the oracle op applied to the GPU's own inputs
        ck = LocalChecker(net, wl, st)
        out, worst = ck.run()
        print("\n%s: %d local checks passed; closest to their bounds: %s"
              % (net["name"], len(ck.report), "; ".join("%s %.2g/%.2g" % w for w in worst)))
    else:
        out = st.results()
    out["losses"] = losses
    out["state"] = st
    return out


def count_mask_flips(net, gpu, ref):
    """Elements whose ReLU / ReLU6 / max-pool decision differs between the GPU's and the oracle's
    forward pass (one side sits at a kink, the other a rounding error away from it).  A single such
    element changes the gradients downstream by about 1/sqrt(elements of its tensor)."""
    st, flips = gpu["state"], 0
    for i, op in enumerate(net["ops"][:-1]):
        act = op.get("act", "none")
        if op["kind"] in ("conv", "bn") and act != "none":
            a, b = st.tensor(i + 1), ref["tensors"][i + 1]
            flips += int(((a > 0) != (b > 0)).sum())
            if act == "relu6":
                flips += int(((a < 6) != (b < 6)).sum())
    return flips


SMALL_NETS = [
    ("tiny", dict()),
    ("lenet5", dict(batch=16)),
    ("resnet56", dict(batch=8, blocks_per_stage=2, hw=16)),
    ("resnet50", dict(batch=4, hw=64, stages=(2, 1, 1, 1), classes=24, dtype="f32")),
    ("mobilenetv2", dict(batch=4, hw=64, classes=16)),
]


@pytest.mark.parametrize("perturb", [False, True], ids=["init", "perturbed"])
@pytest.mark.parametrize("name,kw", SMALL_NETS, ids=[n for n, _ in SMALL_NETS])
def test_train_step_small_fp32(name, kw, perturb):
    net = nets.CONFIGS[name](**kw)
    wl = nets.make_workload(net, perturb=perturb)
    ref = oracle_step_with_conditioning(net, wl)
    gpu = run_gpu_steps(net, wl, local=True)
    compare_step(net, gpu, ref, 1e-4, 1e-3, 1e-3)


@pytest.mark.parametrize("name,kw", [("resnet50", dict(batch=8, hw=64, stages=(2, 2, 1, 1), classes=40)),
                                     ("mobilenetv2", dict(batch=4, hw=64, classes=16)),
                                     ("lenet5", dict(batch=16))], ids=["resnet50", "mobilenetv2", "lenet5"])
def test_train_step_small_bf16(name, kw):
    """bf16 storage.  Every op is checked locally; end to end only the loss is compared, and loosely:
    these nets are tiny (BatchNorm over as few as 16 samples in the last stage), so two
    differently-rounded runs drift apart by percents (see test_local_check_cpu.py).  The full-size
    workload, whose statistics average over thousands of samples, is held to 5e-3."""
    net = dict(nets.CONFIGS[name](**kw), dtype="bf16")
    wl = nets.make_workload(net, perturb=True)
    wl["x"] = nets.to_bf16_grid(wl["x"])
    ref = orc.train_step(net, wl["x"], wl["labels"], wl["params"])
    gpu = run_gpu_steps(net, wl, local=True)
    assert abs(gpu["loss"] - ref["loss"]) <= 5e-2 * abs(ref["loss"]), (gpu["loss"], ref["loss"])


def test_train_step_is_deterministic_and_in_place_equals_functional():
    net = nets.resnet56(batch=8, blocks_per_stage=1, hw=16)
    wl = nets.make_workload(net)
    a = run_gpu_steps(net, wl)
    b = run_gpu_steps(net, wl)
    assert a["loss"] == b["loss"]
    for pa, pb in zip(a["grads"], b["grads"]):
        for x, y in zip(pa, pb):
            np.testing.assert_array_equal(x, y)
    # the caller's host copies of the parameters were not touched; the step updated the device
    # arena in place and its result equals the oracle's pure-function step
    ref = oracle_step_with_conditioning(net, wl)
    compare_step(net, a, ref, 1e-4, 1e-3, 1e-3)


def test_config1_tiny_block():
    net = nets.tiny_block()
    wl = nets.make_workload(net)
    ref = oracle_step_with_conditioning(net, wl)
    compare_step(net, run_gpu_steps(net, wl, local=True), ref, 1e-4, 1e-3, 1e-3)


def test_config2_lenet_ten_steps():
    net = nets.lenet5()
    wl = nets.make_workload(net)
    params, vel, ref_losses = wl["params"], None, []
    for _ in range(10):
        ref = orc.train_step(net, wl["x"], wl["labels"], params, vel)
        params, vel = ref["params"], ref["velocity"]
        ref_losses.append(ref["loss"])
    gpu = run_gpu_steps(net, wl, steps=10)
    assert gpu["losses"][-1] < gpu["losses"][0]
    np.testing.assert_allclose(gpu["losses"], ref_losses, rtol=1e-4)
    gpu["loss"] = gpu["losses"][-1]
    compare_step(net, gpu, ref, 1e-4, 1e-3, 1e-3)
    run_gpu_steps(net, wl, steps=1, local=True)


def test_config3_resnet56():
    net = nets.resnet56()
    wl = nets.make_workload(net)
    ref = oracle_step_with_conditioning(net, wl)
    compare_step(net, run_gpu_steps(net, wl, local=True), ref, 1e-4, 1e-3, 1e-3)


def test_config5_mobilenetv2():
    net = nets.mobilenetv2()
    wl = nets.make_workload(net)
    ref = oracle_step_with_conditioning(net, wl)
    compare_step(net, run_gpu_steps(net, wl, local=True), ref, 1e-4, 1e-3, 1e-3)


def test_config4_resnet50_bf16():
    """Full size (batch 64, 224x224), the launch configuration the benchmark times."""
    net = nets.resnet50()
    wl = nets.make_workload(net)
    gpu = run_gpu_steps(net, wl, local=True)
    tensors, _ = orc.forward(net, wl["x"], wl["params"])
    ref_loss = orc.head_fwd_vjp(tensors[net["ops"][-1]["in"]], wl["params"][-1][0], wl["params"][-1][1], wl["labels"],
                                need_dx=False)[0]
    print("resnet50 bf16 loss: gpu %.6f oracle %.6f" % (gpu["loss"], ref_loss))
    assert abs(gpu["loss"] - ref_loss) <= 5e-3 * abs(ref_loss)


# ---- the same step dispatched op by op (the paper's eager mode, Section 3.3) ---------------------------
def run_eager_steps(net, wl, sync, steps=1):
    from paper_2102_13243_amd.eager import EagerState
    st = EagerState(net, wl["params"], DEV, sync=sync)
    xd, ld = st.upload_batch(wl["x"], wl["labels"])
    losses = []
    for _ in range(steps):
        st.step(xd, ld)
        torch.cuda.synchronize()
        losses.append(float(st.loss[0].item()))
    out = st.results()
    out["losses"] = losses
    out["state"] = st
    return out


@pytest.mark.parametrize("name,kw,sync", [(n, kw, i % 2 == 0) for i, (n, kw) in enumerate(SMALL_NETS)],
                         ids=[n for n, _ in SMALL_NETS])
def test_eager_step_small_fp32(name, kw, sync):
    """One entry point per op, pullbacks in reverse order with the accumulate flags doing the gradient
    fan-in, one SGD call per parameter tensor: the result is the oracle's step, to the fused step's bar,
    and the two ways of running the step agree on the loss."""
    net = nets.CONFIGS[name](**kw)
    wl = nets.make_workload(net, perturb=True)
    ref = oracle_step_with_conditioning(net, wl)
    eager = run_eager_steps(net, wl, sync)
    compare_step(net, eager, ref, 1e-4, 1e-3, 1e-3)
    fused = run_gpu_steps(net, wl)
    assert abs(eager["loss"] - fused["loss"]) <= 2e-5 * abs(fused["loss"]), (eager["loss"], fused["loss"])


def test_eager_lenet_ten_steps_and_bf16_loss():
    net = nets.lenet5(batch=16)
    wl = nets.make_workload(net)
    eager = run_eager_steps(net, wl, sync=False, steps=10)
    fused = run_gpu_steps(net, wl, steps=10)
    np.testing.assert_allclose(eager["losses"], fused["losses"], rtol=1e-4)
    # bf16 storage: the working copy of the parameters is refreshed by the per-tensor SGD calls
    net = dict(nets.resnet50(batch=8, hw=64, stages=(2, 2, 1, 1), classes=40), dtype="bf16")
    wl = nets.make_workload(net, perturb=True)
    wl["x"] = nets.to_bf16_grid(wl["x"])
    ref = orc.train_step(net, wl["x"], wl["labels"], wl["params"])
    eager = run_eager_steps(net, wl, sync=True, steps=2)
    assert abs(eager["losses"][0] - ref["loss"]) <= 5e-2 * abs(ref["loss"]), (eager["losses"], ref["loss"])
    assert np.isfinite(eager["losses"][1])
    st = eager["state"]
    np.testing.assert_array_equal(st.lowp.float().cpu().numpy(), st.master.to(torch.bfloat16).float().cpu().numpy())


@pytest.mark.parametrize("name,kw", [("lenet5", dict(batch=16)),
                                     ("resnet50", dict(batch=4, hw=64, stages=(2, 1, 1, 1), classes=24, dtype="f32"))],
                         ids=["one_stream", "two_streams"])
def test_train_step_captured_in_a_graph_replays_like_direct_calls(name, kw):
    """The step allocates nothing, clears nothing with memset calls and synchronises nothing, and its second
    stream is forked from and joined back into the caller's: a caller may capture it in a HIP graph.  Every
    replay (with other work and a synchronisation between replays) must give the loss of the same step
    made by a direct call, bit for bit, since each replay trains the parameters one step further."""
    net = nets.CONFIGS[name](**kw)
    wl = nets.make_workload(net, perturb=True)
    ref = B.TrainState(net, wl["params"], DEV)
    xr, lr_ = ref.upload_batch(wl["x"], wl["labels"])
    want = []
    for _ in range(5):
        ref.step(xr, lr_)
        torch.cuda.synchronize()
        want.append(float(ref.loss[0].item()))
    st = B.TrainState(net, wl["params"], DEV)
    xd, ld = st.upload_batch(wl["x"], wl["labels"])
    st.step(xd, ld)   # the first call on a device creates the library's second stream: not under capture
    torch.cuda.synchronize()
    got = [float(st.loss[0].item())]
    graph, stream = torch.cuda.CUDAGraph(), torch.cuda.Stream()
    with torch.cuda.graph(graph, stream=stream):
        st.step(xd, ld)
    torch.cuda.synchronize()
    for _ in range(4):
        graph.replay()
        torch.cuda.synchronize()
        got.append(float(st.loss[0].item()))
        assert float(xd.float().abs().sum().item()) > 0   # unrelated work on the default stream in between
    assert got == want, (got, want)
    a, b = st.results(), ref.results()
    for pa, pb in zip(a["params"], b["params"]):
        for x, y in zip(pa, pb):
            np.testing.assert_array_equal(x, y)
