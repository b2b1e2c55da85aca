"""Validity checks for the strictly balanced gate (Appendix F) on the GPU.

The oracle evaluates Eq.(15) as the plain binary64 softmax rounded once to fp32; the kernel has
its own summation order, so its G_sigma may differ from the oracle's in the last bit.  Eq.(18)
and Eq.(19) compare those values (across tokens, against thresholds), so where two compared values
are closer than the rounding error either decision is a correct evaluation of the method.  The
checks therefore are:
  * G_sigma within one fp32 ulp of the oracle, element by element;
  * the GPU's masks and lists are exactly what the brute-force definitions give on the GPU's OWN
    G_sigma (so the selection itself has no slack at all);
  * the GPU's masks agree with the oracle's wherever the oracle's comparison is decided by more
    than the rounding error; the entries left undecided are counted and reported.
Everything downstream of the masks (denominators, loss, outputs, gradients) is then compared
with the oracle evaluated on its own G_sigma and the validated mask."""
import numpy as np

from oracle import moe_oracle as O

TINY = 1e-27          # the kernel clips logit differences at 64: values below e^-64 are not compared in ulps


def check_gsigma(got, X):
    got = np.asarray(got, np.float32)
    X = np.asarray(X, np.float32)
    assert got.shape == X.shape
    assert np.isfinite(got).all() and (got >= 0).all()
    diff = np.abs(got.astype(np.float64) - X.astype(np.float64))
    ulp = np.spacing(np.maximum(np.abs(X), np.float32(1e-37))).astype(np.float64)
    ok = (diff <= ulp) | ((X < TINY) & (got < TINY))
    assert ok.all(), "G_sigma off by more than one ulp in %d of %d values (worst %.2f ulp)" % (
        (~ok).sum(), X.size, (diff / ulp)[~ok].max())
    return float((got == X).mean())


def check_batchwise_mask(got_gsigma, got_mask, got_tokens, X, m):
    """got_mask [T,n] bool, got_tokens [n,m]; X the oracle's G_sigma.  Returns the number of
    entries whose membership the oracle's values leave undecided."""
    T, n = X.shape
    own_mask, own_toks = O.batchwise_mask(got_gsigma, m)     # Eq.(18) by sorting, on the GPU's own values
    assert np.array_equal(got_mask, own_mask), "mask is not the m largest per column of the kernel's own G_sigma"
    assert np.array_equal(np.asarray(got_tokens)[:, :m], own_toks)
    assert (got_mask.sum(axis=0) == m).all()
    if m == 0 or m == T:
        assert got_mask.all() if m == T else not got_mask.any()
        return 0
    X64 = X.astype(np.float64)
    srt = -np.sort(-X64, axis=0)
    v_m, v_next = srt[m - 1], srt[m]                          # m-th and (m+1)-th largest per column
    margin = 2.0 * np.spacing(v_m.astype(np.float32)).astype(np.float64)
    must_keep = X64 > (v_next + margin)[None, :]
    must_drop = X64 < (v_m - margin)[None, :]
    assert got_mask[must_keep].all(), "an entry clearly among the m largest of its column was dropped"
    assert not got_mask[must_drop].any(), "an entry clearly below the m largest of its column was kept"
    return int((~(must_keep | must_drop)).sum())


def check_threshold_mask(got_gsigma, got_mask, X, thresholds):
    thr = np.asarray(thresholds, np.float32)
    assert np.array_equal(got_mask, O.threshold_mask(got_gsigma, thr)), \
        "mask is not [G_sigma > T_i] on the kernel's own G_sigma"
    X64 = X.astype(np.float64)
    margin = np.spacing(np.maximum(np.abs(X), np.float32(1e-37))).astype(np.float64)
    t64 = thr.astype(np.float64)[None, :]
    above = X64 - margin > t64
    below = X64 + margin <= t64
    assert got_mask[above].all() and not got_mask[below].any()
    return int((~(above | below)).sum())
