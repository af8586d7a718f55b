"""Error measures of the parity tests: per tensor, norm-wise and element by element.

Norm-wise:  rel_l2 = ||a - b||_2 / ||b||_2 (the gate the workload's tolerances are stated in) and
            rel_inf = ||a - b||_inf / ||b||_inf (reported beside it).
Element by element (so that a wrong row inside a large tensor cannot hide in the norm):
  fp32 results   |a - b| <= atol + 1e-4 |b|  for every element
  bf16 results   a and round_bf16(b) are both on the bf16 grid; their distance in units of the spacing
                 of the grid at b (one "ulp" = 2^(exponent(b) - 7)), after taking atol off, is at most
                 1 on at least 99.9 % of the elements and at most 2 on every element.
atol covers the elements that cancellation leaves near zero, where the accumulation error of either
side (fp32: about 1e-7 sqrt(k) of the magnitude of the terms) is large against the element itself
and against the grid spacing there.  It is a fraction of the tensor's root mean square: 1e-4 rms for
fp32 results (thirty to a hundred times the measured accumulation error, ten thousand times below a
wrong value), 3e-5 rms for bf16 ones (a hundred times below the grid spacing of a typical element, 4e-3 rms).
"""
import numpy as np

F32_RTOL = 1e-4
F32_ATOL_RMS = 1e-4
BF16_ATOL_RMS = 3e-5
BF16_FRAC_WITHIN_1 = 0.999
BF16_MAX_ULPS = 2.0


def rel_l2(a, b):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    den = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / den) if den > 0 else float(np.linalg.norm(a - b))


def rel_inf(a, b):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    den = float(np.abs(b).max()) if b.size else 0.0
    num = float(np.abs(a - b).max()) if b.size else 0.0
    return num / den if den > 0 else num


def _rms(b):
    return float(np.sqrt(np.mean(np.square(b)))) if b.size else 0.0


def bf16_ulp(b):
    """Spacing of the bf16 grid at |b| (8 significant bits): 2^(e - 7) for 2^e <= |b| < 2^(e+1);
    the smallest normal spacing for zeros."""
    _, e = np.frexp(b)            # |b| = m 2^e with 0.5 <= m < 1
    e = np.maximum(e, -125)
    return np.ldexp(1.0, e - 8)


def elementwise_f32(a, b, rtol=F32_RTOL, atol=None, atol_rms=F32_ATOL_RMS, atol_extra=None):
    """Returns (ok, worst) where worst = max |a-b| / (atol + rtol |b|) (<= 1 passes).  atol defaults to
    atol_rms * rms(b); atol_extra (scalar or array that broadcasts against b) is added to it: the
    accumulation-error allowance of a contraction whose terms are large against its result."""
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    if b.size == 0:
        return True, 0.0
    if atol is None:
        atol = atol_rms * _rms(b)
    if atol_extra is not None:
        atol = atol + np.asarray(atol_extra, np.float64)
    if np.ndim(atol) == 0 and atol == 0.0 and not np.any(b):
        return bool(not np.any(a)), float(np.abs(a).max())
    d = np.abs(a - b)
    np.divide(d, atol + rtol * np.abs(b), out=d)
    worst = float(d.max())
    return bool(np.isfinite(worst) and worst <= 1.0), worst


def elementwise_bf16(a, b_rounded, atol=None, atol_rms=BF16_ATOL_RMS, operand_scale=None):
    """a: GPU values (on the bf16 grid), b_rounded: the oracle's values rounded to the bf16 grid.
    operand_scale (optional, same shape): for a value that is a rounded SUM of bf16 operands, the largest
    operand magnitude; the grid spacing is then taken at max(|b|, operand_scale), because one rounding
    flip of an operand moves the sum by the operand's spacing however far the operands cancel.
    Returns (ok, frac_within_1, max_ulps)."""
    a, b = np.asarray(a, np.float64), np.asarray(b_rounded, np.float64)
    if b.size == 0:
        return True, 1.0, 0.0
    if atol is None:
        atol = atol_rms * _rms(b)
    d = np.abs(a - b)
    d -= atol
    np.maximum(d, 0.0, out=d)
    d /= bf16_ulp(b if operand_scale is None else np.maximum(np.abs(b), operand_scale))
    mx = float(d.max())
    frac = float(np.count_nonzero(d <= 1.0)) / d.size
    ok = np.isfinite(mx) and mx <= BF16_MAX_ULPS and frac >= BF16_FRAC_WITHIN_1
    return bool(ok), frac, mx


def check_tensor(what, got, ref, bf16, l2_tol, atol=None, atol_extra=None, operand_scale=None):
    """Norm-wise and element-wise comparison of one tensor.  `ref` is the oracle's value, already rounded
    to the bf16 grid when bf16 is set.  Returns a record (what, rel_l2, l2_tol, rel_inf, detail) and
    raises AssertionError on a violation."""
    e2, ei = rel_l2(got, ref), rel_inf(got, ref)
    assert np.isfinite(e2), "%s: not finite" % what
    if atol_extra is not None and e2 > l2_tol:
        # a contraction whose terms are large against its result: the norm-wise gate gets the norm of the same
        # per-element accumulation allowance on top of the relative bound
        ref64 = np.asarray(ref, np.float64)
        extra = float(np.linalg.norm(np.broadcast_to(np.asarray(atol_extra, np.float64), ref64.shape)))
        den = float(np.linalg.norm(ref64))
        assert e2 * den <= l2_tol * den + extra, "%s: ||gpu - oracle|| %.3g > %.3g ||oracle|| + %.3g" % (what, e2 * den, l2_tol, extra)
    else:
        assert e2 <= l2_tol, "%s: rel-L2 %.3g > %.3g (rel-inf %.3g)" % (what, e2, l2_tol, ei)
    if bf16:
        ok, frac, mx = elementwise_bf16(got, ref, atol, operand_scale=operand_scale)
        detail = "within 1 ulp %.5f, max %.2f ulp" % (frac, mx)
    else:
        ok, worst = elementwise_f32(got, ref, atol=atol, atol_extra=atol_extra)
        detail = "worst element %.3g of its bound" % worst
    assert ok, "%s: element-wise check failed (%s; rel-L2 %.3g, rel-inf %.3g)" % (what, detail, e2, ei)
    return (what, e2, l2_tol, ei, detail)
