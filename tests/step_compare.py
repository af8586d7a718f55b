"""End-to-end comparison of a finished training step with the oracle's (loss, every gradient, velocity and
updated parameter).  Used by the GPU parity tests; `gpu` is any dict with loss / grads / params / velocity and
a `state` whose tensor(t) returns the step's activations.  Test infrastructure (CPU side)."""
import numpy as np

from parity_metrics import rel_l2, rel_inf


def mask_flips(net, gpu, ref):
    """Per activated tensor: (tensor id, elements, number of elements whose ReLU / ReLU6 decision differs between
    the GPU's and the oracle's forward pass).  One side sits at a kink, the other a rounding error away from it;
    a single such element changes the gradients upstream of it by about 1/sqrt(elements of its tensor)."""
    st, out = gpu["state"], []
    for i, op in enumerate(net["ops"][:-1]):
        act = op.get("act", "none")
        if op["kind"] in ("conv", "bn") and act != "none":
            a, b = st.tensor(i + 1), ref["tensors"][i + 1]
            n = int(((a > 0) != (b > 0)).sum())
            if act == "relu6":
                n += int(((a < 6) != (b < 6)).sum())
            out.append((i + 1, int(b.size), n))
    return out


def count_mask_flips(net, gpu, ref):
    return sum(n for _, _, n in mask_flips(net, gpu, ref))


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
    BatchNorm has gradient zero in exact arithmetic: its relative error means nothing), and the parameter
    it updates to lr times that."""
    assert abs(gpu["loss"] - ref["loss"]) <= loss_tol * abs(ref["loss"]), (gpu["loss"], ref["loss"])
    flips = count_mask_flips(net, gpu, ref)
    assert flips == 0, "%d activation decisions differ on a kink-free workload" % flips
    worst = {"grad": (0.0, None), "param": (0.0, None)}
    cancelled = 0
    for i, (pg, pr) in enumerate(zip(gpu["grads"], ref["grads"])):
        for j, (a, b) in enumerate(zip(pg, pr)):
            assert np.isfinite(a).all(), (i, j)
            e = rel_l2(a, b)
            pa, pb = gpu["params"][i][j], ref["params"][i][j]
            if e > grad_tol and _is_channel_sum(net, i, j):
                rss = _term_rss(net, ref, i, j)
                assert np.all(np.abs(a - b) <= grad_tol * rss), ("gradient (cancelling sum)", i, j, net["ops"][i]["kind"], e)
                assert np.all(np.abs(pa - pb) <= param_tol * np.abs(pb) + net["lr"] * grad_tol * rss), ("param (cancelling sum)", i, j)
                cancelled += 1
                continue
            assert e <= grad_tol, ("gradient", i, j, net["ops"][i]["kind"], e, rel_inf(a, b))
            assert rel_l2(gpu["velocity"][i][j], ref["velocity"][i][j]) <= grad_tol, ("velocity", i, j)
            if e > worst["grad"][0]:
                worst["grad"] = (e, (i, j, net["ops"][i]["kind"]))
            ep = rel_l2(pa, pb)
            assert ep <= param_tol, ("param", i, j, ep)
            if ep > worst["param"][0]:
                worst["param"] = (ep, (i, j))
    say("%s (kink free): loss gpu %.7g oracle %.7g; worst rel-L2 gradient %.3g at %s, parameter %.3g; %d sums that cancel "
        "held to the scale of their terms" % (net["name"], gpu["loss"], ref["loss"], worst["grad"][0], worst["grad"][1],
                                              worst["param"][0], cancelled))


def compare_step_full_size(net, gpu, ref, loss_tol, grad_tol, say=print, flip_frac=2e-6):
    """End to end at full size.  Tens of millions of pre-activations: a few of them lie within rounding
    distance of a kink whatever the seed, their activation decisions differ between any two correct
    implementations, and each such element adds or removes one term of its tensor's cotangent, which moves
    every gradient upstream of it by about 1/sqrt(elements of that tensor) in relative L2.  Held here:
      * the loss to its stated bound (it is continuous across a kink);
      * the number of differing decisions to max(3, flip_frac of the activations);
      * the MEDIAN per-tensor relative-L2 error of the gradients to grad_tol + 3 * sqrt(sum over the differing
        decisions of 1/elements of their tensor): the stated bound, plus what the counted flips account for
        (root sum of squares of independent contributions, with a factor 3 for their spread).  With no flip
        this is the stated bound itself;
      * the median error of the updated parameters likewise.
    A gradient that is a per-channel sum (dgamma, dbeta, bias gradients) is measured against the larger of its
    own norm and the root sum of squares of its terms when the oracle's cotangents are given (sums that cancel
    to zero have no meaningful relative error).  Every tensor of the same step is also held to the per-op bounds
    by the local checks, element by element."""
    assert abs(gpu["loss"] - ref["loss"]) <= loss_tol * abs(ref["loss"]), (gpu["loss"], ref["loss"])
    per_tensor = mask_flips(net, gpu, ref)
    flips = sum(n for _, _, n in per_tensor)
    elems = sum(e for _, e, _ in per_tensor)
    flip_term = float(np.sqrt(sum(n / e for _, e, n in per_tensor)))
    have_cot = bool(ref.get("cotangents"))
    ge, pe = [], []
    for i, (pg, pr) in enumerate(zip(gpu["grads"], ref["grads"])):
        for j, (a, b) in enumerate(zip(pg, pr)):
            assert np.isfinite(a).all(), (i, j)
            den = float(np.linalg.norm(b))
            if have_cot and _is_channel_sum(net, i, j):
                den = max(den, float(np.linalg.norm(_term_rss(net, ref, i, j))))
            ge.append(float(np.linalg.norm(a - b)) / den if den > 0 else 0.0)
            pb = ref["params"][i][j]
            pden = max(float(np.linalg.norm(pb)), net["lr"] * den)
            pe.append(float(np.linalg.norm(gpu["params"][i][j] - pb)) / pden if pden > 0 else 0.0)
    bound = grad_tol + 3.0 * flip_term
    say("%s (full size): loss gpu %.7g oracle %.7g (rel %.2g); %d of %d activation decisions differ (they account for %.3g "
        "of relative gradient error); per-tensor gradient rel-L2 median %.3g, 90th percentile %.3g, max %.3g (median bound "
        "%.3g); parameter rel-L2 median %.3g, max %.3g"
        % (net["name"], gpu["loss"], ref["loss"], abs(gpu["loss"] - ref["loss"]) / abs(ref["loss"]), flips, elems, flip_term,
           float(np.median(ge)), float(np.percentile(ge, 90)), max(ge), bound, float(np.median(pe)), max(pe)))
    assert flips <= max(3, flip_frac * elems), ("activation decisions differ in too many places", flips, elems)
    assert float(np.median(ge)) <= bound, ("median gradient error", float(np.median(ge)), bound)
    assert float(np.median(pe)) <= bound, ("median parameter error", float(np.median(pe)), bound)
    return flips, float(np.median(ge)), max(ge)
