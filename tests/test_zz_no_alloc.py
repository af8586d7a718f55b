"""The allocation-free BatchNorm forward entry point (s4tf_bn_relu_fwd_static) against the plain entry point.

Same kernels, partial sums in the library's static device array instead of a caller workspace: results must
be those of s4tf_bn_relu_fwd bit for bit (well inside the parity bar), on two calls in a row, the second with
a smaller input (nothing may carry over in the shared array), and also against the CPU oracle.  A shape whose
partial sums do not fit is refused before anything is launched."""
import ctypes

import numpy as np
import pytest

from oracle import oracle as orc
from workloads import nets

torch = pytest.importorskip("torch")
from paper_2102_13243_amd import binding as B  # noqa: E402
from parity_metrics import check_tensor  # noqa: E402

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _run(shape, act, use_res, bf16, rng):
    n, h, w, c = shape
    f32 = lambda a: np.ascontiguousarray(a, np.float32)  # noqa: E731
    x = f32(rng.standard_normal(shape) * 2.0 + 3.0)
    res = f32(rng.standard_normal(shape)) if use_res else None
    if bf16:
        x = nets.to_bf16_grid(x)
        res = nets.to_bf16_grid(res) if use_res else None
    gamma = f32(1.0 + 0.3 * rng.standard_normal(c))
    beta = f32(0.2 * rng.standard_normal(c))
    dt = torch.bfloat16 if bf16 else torch.float32
    dev = lambda a: None if a is None else torch.from_numpy(a).to(DEV)  # noqa: E731
    xd = dev(x).to(dt)
    rd = dev(res).to(dt) if use_res else None
    gd, bd = dev(gamma), dev(beta)
    d = B.BnDesc(n, h, w, c, 1e-5, B.ACT[act], B.S4TF_BF16 if bf16 else B.S4TF_F32, 0)
    cap, needed = B.s4tf_bn_relu_fwd_static_limit(d)
    assert 0 < needed <= cap == 1 << 20

    def outputs():
        return (torch.full(shape, float("nan"), dtype=dt, device=DEV), torch.full((c,), float("nan"), device=DEV),
                torch.full((c,), float("nan"), device=DEV))

    y0, m0, i0 = outputs()
    wsp = torch.empty(max(B.s4tf_bn_relu_workspace_bytes(d), 16), dtype=torch.uint8, device=DEV)
    B.s4tf_bn_relu_fwd(d, xd, rd, gd, bd, y0, m0, i0, wsp)
    y1, m1, i1 = outputs()   # allocated before the call under test: the call itself allocates nothing
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    B.s4tf_bn_relu_fwd_static(d, xd, rd, gd, bd, y1, m1, i1)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    host = lambda t: t.float().cpu().numpy().astype(np.float64)  # noqa: E731
    np.testing.assert_array_equal(host(m1), host(m0))
    np.testing.assert_array_equal(host(i1), host(i0))
    np.testing.assert_array_equal(host(y1), host(y0))
    # and against the oracle, at the parity bar of the plain entry point's test
    y_ref, mean_ref, invstd_ref = orc.bn_act_fwd(x, res, gamma, beta, 1e-5, act)
    assert float(np.max(np.abs(host(m1) - mean_ref) * invstd_ref)) < 5e-6
    assert float(np.max(np.abs(host(i1) - invstd_ref) / invstd_ref)) < 2e-5
    check_tensor("bn y (static scratch)", host(y1), orc.round_bf16(y_ref) if bf16 else y_ref, bf16, 4e-3 if bf16 else 2e-5)


@pytest.mark.parametrize("bf16", [False, True], ids=["f32", "bf16"])
def test_static_scratch_forward_matches_the_workspace_forward_on_two_calls_in_a_row(bf16):
    rng = np.random.default_rng(21)
    _run((64, 56, 56, 64), "relu", True, bf16, rng)    # hundreds of pixel chunks: 200-400 KB of the static array are written
    _run((2, 5, 7, 16), "relu6", False, bf16, rng)     # then a much smaller input: stale partial sums must not matter
    _run((3, 9, 9, 6), "none", True, bf16, rng)        # channel count that takes the element-wise kernels


def test_static_scratch_forward_refuses_shapes_beyond_its_capacity():
    d = B.BnDesc(64, 56, 56, 512, 1e-5, B.ACT["relu"], B.S4TF_BF16, 0)
    cap, needed = B.s4tf_bn_relu_fwd_static_limit(d)
    assert needed > cap
    x = torch.zeros(16, dtype=torch.uint8, device=DEV)   # never touched: the refusal comes before any launch
    rc = B.lib().s4tf_bn_relu_fwd_static(ctypes.byref(d), x.data_ptr(), None, x.data_ptr(), x.data_ptr(), x.data_ptr(),
                                         x.data_ptr(), x.data_ptr(), None)
    assert rc == -5 and "static scratch" in B.last_error()
    assert not bool(x.any())
