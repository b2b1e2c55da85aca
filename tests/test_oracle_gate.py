"""Pins for the oracle's gating (CPU only): each test checks the oracle against something the
paper or the mathematics fixes, never against the oracle's own formula."""
import itertools
from fractions import Fraction

import numpy as np
import pytest
from scipy.special import ndtr, softmax

from oracle import moe_oracle as O


def _round_f32(fr: Fraction) -> np.float32:
    """Round an exact rational to binary32, nearest-even (normal range only)."""
    if fr == 0:
        return np.float32(0.0)
    sign = -1 if fr < 0 else 1
    fr = abs(fr)
    e = 0
    while fr >= 2:
        fr /= 2
        e += 1
    while fr < 1:
        fr *= 2
        e -= 1
    scaled = fr * (1 << 23)                      # in [2^23, 2^24)
    q, rem = divmod(scaled.numerator, scaled.denominator)
    twice = 2 * rem
    if twice > scaled.denominator or (twice == scaled.denominator and (q & 1)):
        q += 1
    return np.float32(sign * float(q) * 2.0 ** (e - 23))


def test_dot_chain_is_the_sequential_fused_chain():
    """R1: acc = fma(x_j, W_ji, acc), j ascending, emulated with exact rationals."""
    rng = np.random.default_rng(1)
    T, d, n = 3, 37, 5
    x = rng.standard_normal((T, d)).astype(np.float32)
    W = (0.3 * rng.standard_normal((d, n))).astype(np.float32)
    got = O.dot_chain_f32(x, W)
    for t in range(T):
        for i in range(n):
            acc = np.float32(0.0)
            for j in range(d):
                acc = _round_f32(Fraction(float(x[t, j])) * Fraction(float(W[j, i])) + Fraction(float(acc)))
            assert got[t, i] == acc, (t, i)


def test_dot_chain_rows_gather_and_close_to_fp64():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((50, 512)).astype(np.float32)
    W = (0.02 * rng.standard_normal((512, 33))).astype(np.float32)
    rows = np.array([7, 7, 0, 49, 13], dtype=np.int32)
    got = O.dot_chain_f32(x, W, rows)
    assert np.array_equal(got, O.dot_chain_f32(x, W)[rows])
    ref = x[rows].astype(np.float64) @ W.astype(np.float64)
    assert np.abs(got - ref).max() < 5e-6


def test_softplus_matches_binary64_library_within_one_ulp():
    """R2 vs log(1+exp(z)) from numpy in binary64, rounded to binary32."""
    rng = np.random.default_rng(3)
    z = np.concatenate([rng.standard_normal(200000) * 3, np.linspace(-70, 70, 20001),
                        np.array([0.0, -0.0, 1e-30, -1e-30, 64.0, -64.0, 88.0])]).astype(np.float32)
    got = O.softplus_f32(z)
    zc = np.clip(z.astype(np.float64), -64.0, None)          # documented clip at -64
    ref64 = np.logaddexp(0.0, zc)
    ref = ref64.astype(np.float32)
    assert np.all(got > 0) and np.all(np.isfinite(got))
    ulp = np.spacing(ref)
    assert np.abs(got.astype(np.float64) - ref.astype(np.float64)).max() <= ulp.max()
    assert np.all(np.abs(got - ref) <= ulp)
    assert (got == ref).mean() > 0.9999
    # and the binary64 value before rounding is far more accurate than an fp32 ulp
    assert np.abs(got.astype(np.float64) - ref64).max() <= 0.5000001 * ulp.max()
    assert got[z == 0][0] == np.float32(np.log(2.0))


def test_noise_term_is_one_fused_multiply_add():
    """R3: H = fma(eps, sp, clean + bias), checked with exact rationals."""
    rng = np.random.default_rng(4)
    x = rng.standard_normal((4, 16)).astype(np.float32)
    Wg = rng.standard_normal((16, 6)).astype(np.float32)
    Wn = rng.standard_normal((16, 6)).astype(np.float32)
    eps = rng.standard_normal((4, 6)).astype(np.float32)
    bias = rng.standard_normal(6).astype(np.float32)
    lg = O.noisy_logits_f32(x, Wg, Wn, eps, bias)
    clean = O.dot_chain_f32(x, Wg)
    assert np.array_equal(lg.cleanb, clean + bias[None, :])
    assert np.array_equal(lg.sp, O.softplus_f32(O.dot_chain_f32(x, Wn)))
    for t in range(4):
        for i in range(6):
            want = _round_f32(Fraction(float(eps[t, i])) * Fraction(float(lg.sp[t, i]))
                              + Fraction(float(lg.cleanb[t, i])))
            assert lg.H[t, i] == want
    nf = O.noisy_logits_f32(x, Wg, Wn, None, None)
    assert np.array_equal(nf.H, clean)


def test_topk_brute_force_with_ties():
    """Eq.(5) against Python's sort on every small row drawn from a 3-value alphabet (many ties)."""
    vals = [np.float32(-1.0), np.float32(0.0), np.float32(2.5)]
    for n in range(1, 6):
        rows = np.array(list(itertools.product(vals, repeat=n)), dtype=np.float32)
        for k in range(1, n + 1):
            got = O.keep_top_k(rows, k)
            for r, row in enumerate(rows):
                want = sorted(range(n), key=lambda i: (-float(row[i]), i))[:k]
                assert list(got[r]) == want
    z = np.array([[0.0, -0.0, 0.0, -0.0]], dtype=np.float32)      # signed zeros compare equal
    assert list(O.keep_top_k(z, 3)[0]) == [0, 1, 2]


def test_k_equals_n_without_noise_is_plain_softmax_gating():
    """Eq.(3)-(5) with k = n and no noise reduce to Eq.(2), Softmax(x W_g)."""
    rng = np.random.default_rng(5)
    T, d, n = 64, 32, 8
    x = rng.standard_normal((T, d)).astype(np.float32)
    Wg = (0.3 * rng.standard_normal((d, n))).astype(np.float32)
    Wn = (0.3 * rng.standard_normal((d, n))).astype(np.float32)
    lg = O.noisy_logits_f32(x, Wg, Wn, None)
    fw = O.gate_and_losses(lg, n)
    G = O.dense_gates(fw.idx, fw.gates, n)
    ref = softmax(x.astype(np.float64) @ Wg.astype(np.float64), axis=1)
    assert np.abs(G - ref).max() < 2e-6
    assert np.allclose(fw.load, T)                       # k = n: every expert always selected
    assert fw.loss_load == 0.0


def test_gate_invariants_and_selection_criterion():
    """Exactly k non-zero gates summing to 1; and Appendix A's criterion: G(x)_i != 0 iff H_i is
    greater than the k-th greatest element of H excluding itself (brute-forced with np.delete)."""
    rng = np.random.default_rng(6)
    T, d, n, k = 200, 24, 11, 4
    x = rng.standard_normal((T, d)).astype(np.float32)
    Wg = (0.4 * rng.standard_normal((d, n))).astype(np.float32)
    Wn = (0.4 * rng.standard_normal((d, n))).astype(np.float32)
    eps = rng.standard_normal((T, n)).astype(np.float32)
    lg = O.noisy_logits_f32(x, Wg, Wn, eps)
    fw = O.gate_and_losses(lg, k)
    G = O.dense_gates(fw.idx, fw.gates, n)
    assert np.all((G > 0).sum(axis=1) == k)
    assert np.allclose(G.sum(axis=1), 1.0, atol=1e-14)
    assert np.all(np.diff(np.take_along_axis(lg.H, fw.idx.astype(np.int64), 1), axis=1) <= 0)
    thr, in_top, j_in, j_out = O.kth_excluding(lg.H, k, fw.idx)
    for t in range(T):
        for i in range(n):
            rest = np.sort(np.delete(lg.H[t], i))[::-1]
            assert thr[t, i] == rest[k - 1]
            assert (G[t, i] > 0) == (lg.H[t, i] > rest[k - 1])
        assert lg.H[t, j_in[t]] == np.sort(lg.H[t])[::-1][k]
        assert lg.H[t, j_out[t]] == np.sort(lg.H[t])[::-1][k - 1]
    assert abs(fw.importance.sum() - T) < 1e-9


def test_zero_initialised_gate_gives_noise_only_selection():
    """Appendix A, 'Initial Load Imbalance': W_g = W_noise = 0 gives no signal and some noise:
    H = eps * ln2, selection = top-k of eps, gates = softmax(ln2 * eps_topk),
    P(x,i) = Phi(-kth_excluding(eps))."""
    rng = np.random.default_rng(7)
    T, d, n, k = 300, 16, 9, 3
    x = rng.standard_normal((T, d)).astype(np.float32)
    Z = np.zeros((d, n), dtype=np.float32)
    eps = rng.standard_normal((T, n)).astype(np.float32)
    lg = O.noisy_logits_f32(x, Z, Z, eps)
    ln2 = np.float32(np.log(2.0))
    assert np.all(lg.cleanb == 0) and np.all(lg.sp == ln2)
    assert np.array_equal(lg.H, eps * ln2)
    fw = O.gate_and_losses(lg, k)
    want_idx = np.argsort(-eps, axis=1, kind="stable")[:, :k]
    assert np.array_equal(fw.idx, want_idx)
    top = np.take_along_axis(eps.astype(np.float64), want_idx, 1)
    assert np.abs(fw.gates - softmax(np.log(2.0) * top, axis=1)).max() < 1e-6
    srt = -np.sort(-eps.astype(np.float64), axis=1)
    G = O.dense_gates(fw.idx, fw.gates, n)
    thr_eps = np.where(G > 0, srt[:, [k]], srt[:, [k - 1]])
    _, P = O.load(lg, k, fw.idx)
    assert np.abs(P - ndtr(-thr_eps)).max() < 1e-6


def test_importance_and_cv_closed_forms():
    n, T = 7, 50
    idx = np.full((T, 1), 3, dtype=np.int32)
    gates = np.ones((T, 1))
    imp = O.importance(idx, gates, n)
    assert imp[3] == T and imp.sum() == T
    assert abs(O.cv_squared(imp) - (n - 1)) < 1e-12          # everything on one expert
    assert O.cv_squared(np.full(n, 4.2)) == 0.0              # perfectly even
    v = np.array([1.0, 2.0, 3.0, 4.0])
    assert abs(O.cv_squared(v) - np.var(v) / np.mean(v) ** 2) < 1e-15
    assert abs(O.cv_squared(v) - 0.2) < 1e-15                # var 1.25, mean 2.5
    # gradient of CV^2 against central differences
    g = O.dcv_squared(v)
    for i in range(4):
        e = np.zeros(4)
        e[i] = 1e-6
        fd = (O.cv_squared(v + e) - O.cv_squared(v - e)) / 2e-6
        assert abs(fd - g[i]) < 1e-8


def test_load_two_experts_closed_form():
    """n = 2, k = 1: expert i is chosen iff its fresh noisy logit beats the other's H, so
    P(x,i) = Phi((clean_i - H_other) / sp_i) (Eq.(8)-(9))."""
    from scipy.stats import norm
    rng = np.random.default_rng(8)
    T, d = 400, 12
    x = rng.standard_normal((T, d)).astype(np.float32)
    Wg = (0.5 * rng.standard_normal((d, 2))).astype(np.float32)
    Wn = (0.5 * rng.standard_normal((d, 2))).astype(np.float32)
    eps = rng.standard_normal((T, 2)).astype(np.float32)
    lg = O.noisy_logits_f32(x, Wg, Wn, eps)
    idx = O.keep_top_k(lg.H, 1)
    L, P = O.load(lg, 1, idx)
    c, s, H = (a.astype(np.float64) for a in (lg.cleanb, lg.sp, lg.H))
    want = np.stack([norm.cdf((c[:, 0] - H[:, 1]) / s[:, 0]), norm.cdf((c[:, 1] - H[:, 0]) / s[:, 1])], 1)
    assert np.abs(P - want).max() < 1e-12
    assert np.allclose(L, want.sum(0))


def test_load_monte_carlo_of_the_operational_definition():
    """Appendix A: P(x,i) is the probability that G(x)_i is non-zero when the noise on element i
    alone is redrawn and the other elements keep their sampled noise."""
    rng = np.random.default_rng(9)
    T, d, n, k = 3, 8, 6, 2
    x = rng.standard_normal((T, d)).astype(np.float32)
    Wg = (0.5 * rng.standard_normal((d, n))).astype(np.float32)
    Wn = (0.5 * rng.standard_normal((d, n))).astype(np.float32)
    eps = rng.standard_normal((T, n)).astype(np.float32)
    lg = O.noisy_logits_f32(x, Wg, Wn, eps)
    idx = O.keep_top_k(lg.H, k)
    _, P = O.load(lg, k, idx)
    draws = 400000
    for t in range(T):
        for i in range(n):
            z = rng.standard_normal(draws)
            Hi = lg.cleanb[t, i].astype(np.float64) + z * lg.sp[t, i].astype(np.float64)
            others = np.delete(lg.H[t].astype(np.float64), i)
            kth = np.sort(others)[::-1][k - 1]
            freq = (Hi > kth).mean()
            assert abs(freq - P[t, i]) < 4e-3, (t, i, freq, P[t, i])


def test_fp32_selection_vs_fp64_selection_is_reported_not_failed():
    """The pinned fp32 arithmetic stays within a few 1e-6 of binary64 and rarely changes top-k."""
    rng = np.random.default_rng(10)
    T, d, n, k = 2048, 512, 64, 4
    x = rng.standard_normal((T, d)).astype(np.float32)
    Wg = (0.02 * rng.standard_normal((d, n))).astype(np.float32)
    Wn = (0.02 * rng.standard_normal((d, n))).astype(np.float32)
    eps = rng.standard_normal((T, n)).astype(np.float32)
    l32 = O.noisy_logits_f32(x, Wg, Wn, eps)
    l64 = O.noisy_logits_f64(x, Wg, Wn, eps)
    assert np.abs(l32.H - l64.H).max() < 1e-5
    differing = (O.keep_top_k(l32.H, k) != O.keep_top_k(l64.H, k)).any(axis=1).sum()
    assert differing <= 3
