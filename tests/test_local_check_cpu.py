"""CPU tests of the test infrastructure itself.

1. The local-consistency checker (local_check.py) accepts a step computed by the oracle and
   rejects steps with a planted mistake (planted on the CPU, in a copy of the oracle's results).
2. Why whole-step gradient comparisons are not the parity gate for deep nets: two runs of the
   ORACLE that differ by a relative jitter of 1e-6 on convolution outputs (far below any
   accumulation-order effect) end up with parameter gradients that differ by much more than the
   per-op error of either run, because ReLU masks / bf16 roundings flip and the flips propagate.
"""
import numpy as np
import pytest

from oracle import oracle as orc
from workloads import nets
import local_check as LC
from parity_metrics import rel_l2


class OracleBackedState:
    """Looks like binding.TrainState to the checker, but every tensor comes from the oracle."""

    def __init__(self, net, wl):
        self.net = net
        out = orc.train_step(net, wl["x"], wl["labels"], wl["params"])
        self.out = out
        rnd = (lambda a: orc.round_bf16(a)) if net["dtype"] == "bf16" else (lambda a: a)
        ops, tensors, cot, self.stats = net["ops"], out["tensors"], {}, {}

        def contribute(t, g):
            if t != 0 and g is not None:
                cot[t] = rnd(cot[t] + g) if t in cot else rnd(g)

        hop = ops[-1]
        _, dx, _, _, _ = orc.head_fwd_vjp(tensors[hop["in"]], wl["params"][-1][0], wl["params"][-1][1], wl["labels"])
        contribute(hop["in"], dx)
        for i in range(len(ops) - 2, -1, -1):
            op, p = ops[i], wl["params"][i]
            kind, tin, dy, x, y = op["kind"], op["in"], cot[i + 1], tensors[op["in"]], tensors[i + 1]
            if kind == "conv":
                dz = dy
                if op["act"] != "none":
                    dz, _ = orc.bias_act_vjp(y, dy, op["act"], need_db=False)
                    cot[i + 1] = dz   # the library applies the activation pullback in place
                w = orc.round_bf16(p[0]) if net["dtype"] == "bf16" else p[0]
                contribute(tin, orc.conv2d_vjp(x, w, dz, op["stride"], op["pad"], op["groups"], need_dx=tin != 0)[0])
            elif kind == "bn":
                res = tensors[op["res"]] if op["res"] >= 0 else None
                _, mean, invstd = orc.bn_act_fwd(x, res, p[0], p[1], op["eps"], op["act"])
                self.stats[i] = (mean, invstd)
                dxi, dres, _, _ = orc.bn_act_vjp(x, y, p[0], mean, invstd, dy, op["act"], op["res"] >= 0)
                if op["res"] >= 0:
                    contribute(op["res"], dres)
                contribute(tin, dxi)
            elif kind == "avgpool2":
                contribute(tin, orc.avgpool2_vjp(dy, x.shape))
            elif kind == "maxpool3s2":
                contribute(tin, orc.maxpool3s2_vjp(x, dy))
            elif kind == "flatten":
                contribute(tin, dy.reshape(x.shape))
        self.cot = cot

    def tensor(self, t, cotangent=False):
        return np.array(self.cot[t] if cotangent else self.out["tensors"][t])

    def bn_stats(self, op):
        return self.stats[op]

    def results(self):
        o = self.out
        return {"loss": o["loss"], "grads": o["grads"], "params": o["params"], "velocity": o["velocity"]}


CASES = [("lenet5", dict(batch=4)), ("resnet56", dict(batch=4, blocks_per_stage=1, hw=16)),
         ("resnet50", dict(batch=2, hw=32, stages=(1, 1, 1, 1), classes=10)), ("mobilenetv2", dict(batch=2, hw=32, classes=8))]


@pytest.mark.parametrize("sampled", [False, True], ids=["full", "sampled"])
@pytest.mark.parametrize("name,kw", CASES, ids=[c[0] for c in CASES])
def test_checker_accepts_the_oracle_and_rejects_planted_mistakes(name, kw, sampled, monkeypatch):
    if sampled:
        monkeypatch.setattr(LC, "FULL_FLOPS", 2e5)
    net = nets.CONFIGS[name](**kw)
    wl = nets.make_workload(net, perturb=True)
    st = OracleBackedState(net, wl)
    ck = LC.LocalChecker(net, wl, st, samples=16)
    ck.run()
    assert len(ck.report) > 10
    rng = np.random.default_rng(1)
    ops = net["ops"]

    def expect_failure(mutate):
        bad = OracleBackedState.__new__(OracleBackedState)
        bad.__dict__ = dict(st.__dict__)
        bad.out = dict(st.out, tensors=[np.array(t) if t is not None else None for t in st.out["tensors"]],
                       grads=[[np.array(g) for g in p] for p in st.out["grads"]])
        bad.cot = {k: np.array(v) for k, v in st.cot.items()}
        mutate(bad)
        with pytest.raises(AssertionError):
            LC.LocalChecker(net, wl, bad, samples=16).run()

    conv_ops = [i for i, o in enumerate(ops) if o["kind"] == "conv"]
    i = conv_ops[len(conv_ops) // 2]

    def scale_activation(b):       # a wrong forward output
        b.out["tensors"][i + 1] = b.out["tensors"][i + 1] * 1.05
    expect_failure(scale_activation)

    def one_wrong_row(b):          # one pixel's channels of a forward output off by 2 %: invisible in the tensor's norm
        t = b.out["tensors"][i + 1]
        t[0, 0, 0, :] = t[0, 0, 0, :] * 1.02 + 0.02 * np.abs(t).max()
    expect_failure(one_wrong_row)

    def one_wrong_filter_entry(b):
        g = b.out["grads"][i][0]
        g.reshape(-1)[0] += 1e-2 * np.sqrt(np.mean(g * g))
    expect_failure(one_wrong_filter_entry)

    def wrong_wgrad(b):            # a transposed / dropped term shows up as a wrong filter gradient
        g = b.out["grads"][i][0]
        b.out["grads"][i][0] = g + 0.05 * np.abs(g).max() * rng.standard_normal(g.shape)
    expect_failure(wrong_wgrad)

    def wrong_cotangent(b):        # a missed fan-in contribution
        t = max(b.cot)
        b.cot[t] = b.cot[t] * 0.5
    expect_failure(wrong_cotangent)

    def wrong_update(b):
        b.out = dict(b.out, params=[[np.array(a) * (1 + 1e-3) for a in p] for p in b.out["params"]])
    expect_failure(wrong_update)


def _jittered_step(net, wl, jitter, monkeypatch_ctx):
    rng = np.random.default_rng(5)
    fwd0 = orc.conv2d_fwd

    def fwd(*a, **k):
        y = fwd0(*a, **k)
        return y * (1.0 + jitter * rng.standard_normal(y.shape))

    monkeypatch_ctx.setattr(orc, "conv2d_fwd", fwd)
    out = orc.train_step(net, wl["x"], wl["labels"], wl["params"])
    monkeypatch_ctx.undo()
    return out


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_whole_step_gradients_amplify_a_1e6_jitter(dtype, monkeypatch):
    """Documents the size of the effect; the bounds are deliberately loose (an order of magnitude)."""
    net = nets.resnet50(batch=8, hw=64, stages=(2, 2, 1, 1), classes=40, dtype=dtype)
    wl = nets.make_workload(net)
    a = orc.train_step(net, wl["x"], wl["labels"], wl["params"])
    b = _jittered_step(net, wl, 1e-6, monkeypatch)
    errs = sorted(rel_l2(x, y) for p, q in zip(b["grads"], a["grads"]) for x, y in zip(p, q))
    median, worst = errs[len(errs) // 2], errs[-1]
    loss_err = abs(a["loss"] - b["loss"]) / abs(a["loss"])
    print("%s: jitter 1e-6 -> loss %.2e, median gradient rel-L2 %.2e, worst %.2e" % (dtype, loss_err, median, worst))
    assert worst > 1e-4          # at least 100x amplification somewhere
    if dtype == "bf16":
        assert median > 2e-2     # beyond the bound a whole-step bf16 gradient comparison would use
        assert loss_err < 5e-3   # the loss itself stays comparable
