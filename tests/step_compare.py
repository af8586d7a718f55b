"""End-to-end comparison of a finished training step with the oracle's (loss, every gradient, velocity and
updated parameter).  Used by the GPU parity tests; `gpu` is any dict with loss / grads / params / velocity and
a `state` whose tensor(t) returns the step's activations.  Test infrastructure (CPU side)."""
import numpy as np

from parity_metrics import rel_l2, rel_inf


def count_mask_flips(net, gpu, ref):
    """Elements whose ReLU / ReLU6 decision differs between the GPU's and the oracle's forward pass (one
    side sits at a kink, the other a rounding error away from it).  A single such element changes the
    gradients downstream by about 1/sqrt(elements of its tensor)."""
    st, flips = gpu["state"], 0
    for i, op in enumerate(net["ops"][:-1]):
        act = op.get("act", "none")
        if op["kind"] in ("conv", "bn") and act != "none":
            a, b = st.tensor(i + 1), ref["tensors"][i + 1]
            flips += int(((a > 0) != (b > 0)).sum())
            if act == "relu6":
                flips += int(((a < 6) != (b < 6)).sum())
    return flips


def _is_channel_sum(net, i, j):
    """Gradient tensor j of op i is a per-channel sum of cotangent terms (dgamma, dbeta, a bias gradient)."""
    kind = net["ops"][i]["kind"]
    return kind == "bn" or (kind in ("conv", "head") and j == 1)


def _term_rss(net, ref, i, j):
    """Per channel, the root of the sum of squares of the terms a channel-sum gradient adds up, from the
    oracle's own tensors: dz for dbeta / bias gradients, dz * xhat for dgamma."""
    op = net["ops"][i]
    if op["kind"] == "head":
        n = ref["logits"].shape[0]
        return np.full(ref["logits"].shape[1], 1.0 / np.sqrt(n))   # |dz| <= 1/n per sample
    dy, y = ref["cotangents"][i + 1], ref["tensors"][i + 1]
    act = op.get("act", "none")
    dz = dy if act == "none" else dy * ((y > 0) & ((y < 6) if act == "relu6" else True))
    if op["kind"] == "bn" and j == 0:
        x = ref["tensors"][op["in"]]
        x2 = x.reshape(-1, x.shape[-1])
        dz = dz * ((x - x2.mean(axis=0)) / np.sqrt(x2.var(axis=0) + op["eps"]))
    return np.sqrt((dz.reshape(-1, dz.shape[-1]) ** 2).sum(axis=0))


def compare_step_strict(net, wl, gpu, ref, loss_tol=1e-4, grad_tol=1e-3, param_tol=1e-3, say=print):
    """End to end, no exception: the loss, every gradient tensor, every velocity and every updated
    parameter tensor within the stated relative-L2 bounds, and not one activation decision may differ.
    One refinement, not a loosening: a gradient that is a per-channel sum of terms (dgamma, dbeta, bias
    gradients) is held, per channel, to grad_tol times the root sum of squares of its terms when that is
    what the sum has cancelled down to (the beta of a BatchNorm that feeds a convolution followed by
    BatchNorm has gradient zero in exact arithmetic: its relative error means nothing)."""
    assert abs(gpu["loss"] - ref["loss"]) <= loss_tol * abs(ref["loss"]), (gpu["loss"], ref["loss"])
    flips = count_mask_flips(net, gpu, ref)
    assert flips == 0, "%d activation decisions differ on a kink-free workload" % flips
    worst = {"grad": (0.0, None), "param": (0.0, None)}
    cancelled = 0
    for i, (pg, pr) in enumerate(zip(gpu["grads"], ref["grads"])):
        for j, (a, b) in enumerate(zip(pg, pr)):
            assert np.isfinite(a).all(), (i, j)
            e = rel_l2(a, b)
            if e > grad_tol and _is_channel_sum(net, i, j):
                rss = _term_rss(net, ref, i, j)
                assert np.all(np.abs(a - b) <= grad_tol * rss), ("gradient (cancelling sum)", i, j, net["ops"][i]["kind"], e)
                cancelled += 1
            else:
                assert e <= grad_tol, ("gradient", i, j, net["ops"][i]["kind"], e, rel_inf(a, b))
                assert rel_l2(gpu["velocity"][i][j], ref["velocity"][i][j]) <= grad_tol, ("velocity", i, j)
                if e > worst["grad"][0]:
                    worst["grad"] = (e, (i, j, net["ops"][i]["kind"]))
            ep = rel_l2(gpu["params"][i][j], ref["params"][i][j])
            assert ep <= param_tol, ("param", i, j, ep)
            if ep > worst["param"][0]:
                worst["param"] = (ep, (i, j))
    say("%s (kink free): loss gpu %.7g oracle %.7g; worst rel-L2 gradient %.3g at %s, parameter %.3g; %d sums that cancel "
        "held to the scale of their terms" % (net["name"], gpu["loss"], ref["loss"], worst["grad"][0], worst["grad"][1],
                                              worst["param"][0], cancelled))


def compare_step_full_size(net, gpu, ref, loss_tol, median_tol, say=print):
    """End to end at full size.  Tens of millions of pre-activations: a few of them lie within rounding
    distance of a kink whatever the seed, their activation decisions differ between any two correct
    implementations, and each such element moves the gradients upstream of it by about 1/sqrt(elements of
    its tensor).  Held here: the loss to its stated bound, the number of differing decisions to
    max(3, 2e-6 of the activations), and the MEDIAN per-tensor relative-L2 error of the gradients and of the
    updated parameters to the stated gradient bound.  (Every tensor of the same step is held to the per-op
    bounds by the local checks.)"""
    assert abs(gpu["loss"] - ref["loss"]) <= loss_tol * abs(ref["loss"]), (gpu["loss"], ref["loss"])
    flips = count_mask_flips(net, gpu, ref)
    elems = sum(t.size for t in ref["tensors"][1:-1])
    ge = [rel_l2(a, b) for pg, pr in zip(gpu["grads"], ref["grads"]) for a, b in zip(pg, pr)]
    pe = [rel_l2(a, b) for pg, pr in zip(gpu["params"], ref["params"]) for a, b in zip(pg, pr)]
    for pg in gpu["grads"]:
        for a in pg:
            assert np.isfinite(a).all()
    say("%s (full size): loss gpu %.7g oracle %.7g (rel %.2g); %d of %d activation decisions differ; per-tensor "
        "gradient rel-L2 median %.3g, 90th percentile %.3g, max %.3g; parameter rel-L2 median %.3g, max %.3g"
        % (net["name"], gpu["loss"], ref["loss"], abs(gpu["loss"] - ref["loss"]) / abs(ref["loss"]), flips, elems,
           float(np.median(ge)), float(np.percentile(ge, 90)), max(ge), float(np.median(pe)), max(pe)))
    assert flips <= max(3, 2e-6 * elems), ("activation decisions differ in too many places", flips, elems)
    assert float(np.median(ge)) <= median_tol, ("median gradient error", float(np.median(ge)))
    assert float(np.median(pe)) <= median_tol, ("median parameter error", float(np.median(pe)))
