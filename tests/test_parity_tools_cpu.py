"""CPU tests of the parity tooling: the element-wise error measures, the kink-free workloads, the
end-to-end comparators (fed by the oracle against a perturbed copy of itself, mistakes planted on the
CPU), and the oracle built under AddressSanitizer / UndefinedBehaviorSanitizer."""
import os
import shutil
import subprocess

import numpy as np
import pytest

from oracle import oracle as orc
from workloads import nets
import kink_free as KF
import parity_metrics as PM
import step_compare as SC

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
RNG = np.random.default_rng(3)


# ---- element-wise measures ---------------------------------------------------------------------------
def test_bf16_ulp_is_the_grid_spacing():
    v = np.array([1.0, 1.5, 1.9921875, 2.0, 3.0, 0.75, -5.0, 100.0])
    # next value on the bf16 grid above |v|: |v| + ulp must itself be a bf16 value, |v| + ulp/2 must not round to |v|'s neighbour
    u = PM.bf16_ulp(v)
    np.testing.assert_array_equal(u, [2.0 ** -7, 2.0 ** -7, 2.0 ** -7, 2.0 ** -6, 2.0 ** -6, 2.0 ** -8, 2.0 ** -5, 2.0 ** -1])
    up = np.abs(v) + u
    np.testing.assert_array_equal(nets.to_bf16_grid(up.astype(np.float32)).astype(np.float64), up)


def test_bf16_elementwise_accepts_rounding_flips_and_rejects_a_wrong_row():
    b = orc.round_bf16(RNG.standard_normal((64, 512)) * 3.0)
    a = b.copy()
    idx = RNG.choice(a.size, size=a.size // 50, replace=False)     # 2 % of the elements one ulp off
    a.reshape(-1)[idx] += PM.bf16_ulp(b.reshape(-1)[idx])
    ok, frac, mx = PM.elementwise_bf16(a, b)
    assert ok and frac == 1.0 and mx <= 1.0
    PM.check_tensor("flips", a, b, True, 4e-3)
    bad = b.copy()
    bad[17, :128] = orc.round_bf16(bad[17, :128] * 1.05 + 0.01)   # one wrong row segment of a 32k tensor
    assert PM.rel_l2(bad, b) < 4e-3                                # the norm does not see it
    with pytest.raises(AssertionError):
        PM.check_tensor("wrong row", bad, b, True, 4e-3)
    # more than 0.1 % of the elements two ulps off: each within the everywhere-bound, together too many
    a2 = b.copy()
    idx = RNG.choice(a2.size, size=a2.size // 200, replace=False)
    a2.reshape(-1)[idx] += 2 * PM.bf16_ulp(b.reshape(-1)[idx])
    assert not PM.elementwise_bf16(a2, b)[0]


def test_f32_elementwise_allows_cancellation_noise_only():
    b = RNG.standard_normal(100000)
    b[:10] = 1e-9                                   # elements that cancellation left at zero
    a = b * (1 + 3e-6 * RNG.standard_normal(b.size)) + 1e-6 * RNG.standard_normal(b.size)
    assert PM.elementwise_f32(a, b)[0]
    a[5] += 1e-3                                    # a thousandth of the tensor's scale on one element
    assert PM.rel_l2(a, b) < 2e-5
    assert not PM.elementwise_f32(a, b)[0]
    z = np.zeros(8)
    assert PM.elementwise_f32(z, z)[0] and not PM.elementwise_f32(z + 1e-30, z)[0]


# ---- kink-free workloads and the strict comparator ----------------------------------------------------
SMALL = [("tiny", dict()), ("lenet5", dict(batch=16)), ("resnet56", dict(batch=8, blocks_per_stage=2, hw=16)),
         ("resnet50", dict(batch=4, hw=64, stages=(2, 1, 1, 1), classes=24, dtype="f32")),
         ("mobilenetv2", dict(batch=4, hw=64, classes=16))]


class _State:
    def __init__(self, tensors):
        self.tensors = tensors

    def tensor(self, t, cotangent=False):
        return self.tensors[t]


def _perturbed_step(net, wl, jitter, seed=5):
    """The oracle's step with a relative perturbation of every convolution output: a stand-in for an
    implementation that accumulates in another precision (fp32 against fp64 is about 1e-7)."""
    rng = np.random.default_rng(seed)
    fwd0 = orc.conv2d_fwd
    orc.conv2d_fwd = lambda *a, **k: (lambda y: y * (1.0 + jitter * rng.standard_normal(y.shape)))(fwd0(*a, **k))
    try:
        out = orc.train_step(net, wl["x"], wl["labels"], wl["params"])
    finally:
        orc.conv2d_fwd = fwd0
    out["state"] = _State(out["tensors"])
    return out


@pytest.mark.parametrize("name,kw", SMALL, ids=[n for n, _ in SMALL])
def test_kink_free_workloads_make_the_end_to_end_comparison_well_posed(name, kw):
    net = nets.CONFIGS[name](**kw)
    wl0 = nets.make_workload(net, perturb=True)
    wl, report = KF.make_kink_free(net, wl0, 1e-4)
    assert min(m for _, what, m, _ in report if what != "maxpool") >= 1e-4
    assert min(m for _, _, m, _ in KF.kink_margins(net, wl)) == min(m for _, _, m, _ in report)
    # the shifts moved by a few 1e-4 standard deviations at most (late layers with few samples: 1e-2)
    moved = max(float(np.abs(np.asarray(a, np.float64) - b).max()) for p, q in zip(wl0["params"], wl["params"])
                for a, b in zip(p, q))
    assert moved < 0.05, moved
    assert np.array_equal(wl["x"], wl0["x"]) and np.array_equal(wl["labels"], wl0["labels"])
    ref = orc.train_step(net, wl["x"], wl["labels"], wl["params"], keep_cotangents=True)
    other = _perturbed_step(net, wl, 2e-7)
    SC.compare_step_strict(net, wl, other, ref)
    # planted mistakes (on the CPU, in a copy): a gradient tensor 0.3 % off, and one flipped activation decision
    convs = [i for i, o in enumerate(net["ops"]) if o["kind"] == "conv"]
    i = convs[len(convs) // 2]
    bad = dict(other, grads=[[np.array(g) for g in p] for p in other["grads"]])
    bad["grads"][i][0] = bad["grads"][i][0] * 1.003
    with pytest.raises(AssertionError):
        SC.compare_step_strict(net, wl, bad, ref)
    acts = [t for t, o in enumerate(net["ops"][:-1], start=1) if o.get("act", "none") != "none"]
    tensors = list(other["tensors"])
    flipped = np.array(tensors[acts[0]])
    j = int(np.argmax(flipped.reshape(-1) > 0))
    flipped.reshape(-1)[j] = 0.0
    tensors[acts[0]] = flipped
    with pytest.raises(AssertionError, match="activation decisions"):
        SC.compare_step_strict(net, wl, dict(other, state=_State(tensors)), ref)


def test_without_the_margin_the_same_comparison_is_ill_posed():
    """The seeded workload as drawn: some pre-activation lies within 1e-5 std of a kink, and a perturbation of
    that size flips it; the full-size comparator counts the flip, the strict one refuses."""
    net = nets.resnet50(batch=4, hw=64, stages=(2, 1, 1, 1), classes=24, dtype="f32")
    wl = nets.make_workload(net, perturb=True)
    assert min(m for _, what, m, _ in KF.kink_margins(net, wl) if what != "maxpool") < 1e-5
    ref = orc.train_step(net, wl["x"], wl["labels"], wl["params"], keep_cotangents=True)
    other = _perturbed_step(net, wl, 1e-5)
    assert SC.count_mask_flips(net, other, ref) > 0
    with pytest.raises(AssertionError):
        SC.compare_step_strict(net, wl, other, ref)


def test_full_size_comparator_bounds_flips_and_medians():
    net = nets.resnet56(batch=8, blocks_per_stage=2, hw=16)
    wl = nets.make_workload(net)
    ref = orc.train_step(net, wl["x"], wl["labels"], wl["params"])
    good = _perturbed_step(net, wl, 1e-7)
    SC.compare_step_full_size(net, good, ref, 1e-4, 1e-3)
    bad = dict(good, grads=[[np.array(g) * 1.01 for g in p] for p in good["grads"]])
    with pytest.raises(AssertionError, match="median gradient"):
        SC.compare_step_full_size(net, bad, ref, 1e-4, 1e-3)
    tensors = [None if t is None else np.array(t) for t in good["tensors"]]
    t2 = tensors[2]
    t2[t2 > 0] = 0.0                                 # a whole layer's decisions differ
    with pytest.raises(AssertionError, match="activation decisions"):
        SC.compare_step_full_size(net, dict(good, state=_State(tensors)), ref, 1e-4, 1e-3)


# ---- the oracle under sanitizers -------------------------------------------------------------------------
def test_oracle_is_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    if not shutil.which("gcc") or not os.path.exists(subprocess.run(
            ["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()):
        pytest.skip("gcc or its sanitizer runtime is not available")
    exe = str(tmp_path / "orc_sanitized")
    subprocess.check_call(["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=all", "-fopenmp", "-std=c11", "-o", exe,
                           os.path.join(ROOT, "oracle", "s4tf_oracle.c"), os.path.join(ROOT, "oracle", "sanitize_driver.c"),
                           "-lm"])
    env = dict(os.environ)
    # (the link-order check is off so that a library preloaded by the environment does not stop the run)
    env.update(OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert res.returncode == 0 and res.stdout.strip() == "ok", res.stdout + res.stderr
