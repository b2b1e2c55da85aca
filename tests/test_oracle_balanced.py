"""Pins for the oracle's strictly balanced gating (Appendix F, Eq.(15)-(20)): every function is
checked against something other than itself -- a library softmax, brute-force counting on tiny
inputs, closed forms, and the reductions to the dense softmax mixture the paper states."""
import itertools

import numpy as np
import pytest
from scipy.special import softmax

from oracle import moe_oracle as O


def _inputs(T, d, n, seed, scale=0.3):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((T, d)).astype(np.float32)
    W = (scale * rng.standard_normal((d, n))).astype(np.float32)
    return x, W


def test_softmax_gate_matches_library_softmax():
    x, W = _inputs(300, 64, 40, 1)
    clean, X = O.softmax_gate_f32(x, W)
    ref = softmax(x.astype(np.float64) @ W.astype(np.float64), axis=1)
    # fp32 logits (error ~1e-6 relative on exp) and one rounding of the result
    assert np.abs(X.astype(np.float64) - ref).max() <= 2e-6
    assert np.abs(X.astype(np.float64).sum(axis=1) - 1.0).max() <= 5e-7
    # on the SAME fp32 logits the library softmax in binary64 differs only by its summation order:
    # after the one rounding to fp32 the two agree except where the value sits on a rounding boundary
    ref2 = softmax(clean.astype(np.float64), axis=1)
    ulp = np.spacing(ref2.astype(np.float32)).astype(np.float64)
    assert (np.abs(X.astype(np.float64) - ref2) <= 0.5000001 * ulp).all()
    assert (X == ref2.astype(np.float32)).mean() > 0.9999
    # logits are the sequential fma chain the noisy gate selects on
    assert np.array_equal(clean, O.dot_chain_f32(x, W))


def test_softmax_gate_shift_invariance_and_two_expert_closed_form():
    """Softmax over two experts is the logistic function of the logit difference; adding a
    constant to every logit of a row (a bias equal for all experts) changes nothing beyond the
    rounding of the shifted logits."""
    rng = np.random.default_rng(7)
    x = rng.standard_normal((50, 8)).astype(np.float32)
    W = (0.5 * rng.standard_normal((8, 2))).astype(np.float32)
    clean, X = O.softmax_gate_f32(x, W)
    diff = clean[:, 0].astype(np.float64) - clean[:, 1].astype(np.float64)
    logistic = 1.0 / (1.0 + np.exp(-diff))
    assert np.abs(X[:, 0].astype(np.float64) - logistic).max() <= 6e-8
    assert np.abs(X[:, 1].astype(np.float64) - (1.0 - logistic)).max() <= 6e-8
    _, Xb = O.softmax_gate_f32(x, W, bias=np.full(2, 0.25, np.float32))   # 0.25: exact in fp32
    assert np.abs(Xb.astype(np.float64) - X.astype(np.float64)).max() <= 2e-7


def test_softmax_gate_large_spread_and_single_expert():
    x = np.array([[100.0, 0.0], [-100.0, 0.0]], np.float32)
    W = np.array([[1.0, 0.0, -1.0], [0.0, 0.0, 0.0]], np.float32)
    _, X = O.softmax_gate_f32(x, W)
    assert X[0, 0] == 1.0 and X[1, 2] == 1.0 and (X >= 0).all() and np.isfinite(X).all()
    assert X[0, 1] == np.float32(np.exp(-100.0))
    x1, W1 = _inputs(5, 8, 1, 2)
    _, X1 = O.softmax_gate_f32(x1, W1)
    assert (X1 == 1.0).all()


def _brute_mask(X, m):
    T, n = X.shape
    mask = np.zeros((T, n), bool)
    for i in range(n):
        for j in range(T):
            ahead = sum(1 for jj in range(T) if X[jj, i] > X[j, i] or (X[jj, i] == X[j, i] and jj < j))
            mask[j, i] = ahead < m
    return mask


@pytest.mark.parametrize("T,n,m", [(6, 3, 2), (5, 2, 5), (7, 4, 0), (8, 3, 3)])
def test_batchwise_mask_brute_force(T, n, m):
    rng = np.random.default_rng(T * 100 + n)
    X = rng.random((T, n)).astype(np.float32)
    X[rng.integers(0, T, 3), rng.integers(0, n, 3)] = X[0, 0]          # ties, also across rows of a column
    X[1, :] = X[0, :]
    mask, toks = O.batchwise_mask(X, m)
    assert np.array_equal(mask, _brute_mask(X, m))
    assert (mask.sum(axis=0) == m).all()                               # every expert gets exactly m
    assert toks.shape == (n, m)
    for i in range(n):
        assert np.array_equal(toks[i], np.nonzero(mask[:, i])[0])       # ascending token order


def test_all_equal_column_keeps_lowest_tokens():
    X = np.full((9, 2), 0.5, np.float32)
    mask, toks = O.batchwise_mask(X, 4)
    assert np.array_equal(toks, np.array([[0, 1, 2, 3], [0, 1, 2, 3]], np.int32))


def test_gates_normalised_and_unkept_tokens_zero():
    x, W = _inputs(64, 16, 8, 3)
    _, X = O.softmax_gate_f32(x, W)
    mask, _ = O.batchwise_mask(X, 8)          # m = k T / n with k = 1: some tokens get no expert
    G, denom = O.balanced_gates(X, mask)
    kept_any = mask.any(axis=1)
    assert (~kept_any).any() and kept_any.any()
    assert np.allclose(G[kept_any].sum(axis=1), 1.0, atol=1e-15)
    assert (G[~kept_any] == 0).all() and (denom[~kept_any] == 0).all()
    assert ((G > 0) == mask).all()
    # Eq.(16) written out for one kept entry
    j, i = np.argwhere(mask)[5]
    assert G[j, i] == pytest.approx(float(X[j, i]) / float(X[j][mask[j]].astype(np.float64).sum()), rel=1e-15)


def test_full_mask_is_the_dense_softmax_mixture():
    """m = |X| (k = n): every entry is kept, G = G_sigma (Eq.(16) normalises a row that already
    sums to one) and the layer is the dense mixture of Eq.(2), which the flat oracle also reaches
    with k = n and no noise."""
    T, d, n = 24, 16, 4
    x, W = _inputs(T, d, n, 4)
    clean, X = O.softmax_gate_f32(x, W)
    mask, toks = O.batchwise_mask(X, T)
    assert mask.all()
    G, _ = O.balanced_gates(X, mask)
    assert np.abs(G - X.astype(np.float64)).max() <= 2e-7
    lg = O.noisy_logits_f32(x, W, np.zeros_like(W), None, None)
    fw = O.gate_and_losses(lg, n, 0.0, 0.0)
    dense = O.dense_gates(fw.idx, fw.gates, n)
    assert np.abs(G - dense).max() <= 2e-7
    rng = np.random.default_rng(5)
    Ws = [(rng.standard_normal((d, 8)), rng.standard_normal((8, d))) for _ in range(n)]
    y = O.balanced_output(x, G, lambda e: Ws[e])
    y_flat = O.moe_output(x, fw.idx, fw.gates, lambda e: Ws[e], n)
    assert np.abs(y - y_flat).max() <= 1e-5 * np.abs(y_flat).max()


def test_threshold_mask_and_batchwise_loss_closed_forms():
    X = np.array([[0.9, 0.2], [0.6, 0.7], [0.3, 0.5], [0.1, 0.4]], np.float32)
    mask, _ = O.batchwise_mask(X, 2)           # column 0 keeps tokens 0,1; column 1 keeps 1,2
    assert np.array_equal(mask, np.array([[1, 0], [1, 1], [0, 1], [0, 0]], bool))
    # thresholds strictly between the m-th and (m+1)-th value of each column: masks agree, loss 0
    Tsep = np.array([0.45, 0.45])
    assert np.array_equal(O.threshold_mask(X, Tsep), mask)
    assert O.batchwise_loss(X, mask, Tsep) == 0.0
    # a too-low threshold lets extra entries through: each contributes (X - T) > 0
    Tlow = np.array([0.25, 0.45])
    extra = (float(X[2, 0]) - 0.25)
    assert O.batchwise_loss(X, mask, Tlow) == pytest.approx(extra, rel=1e-12)
    # a too-high threshold drops kept entries: each contributes (T - X) > 0
    Thigh = np.array([0.45, 0.65])
    assert O.batchwise_loss(X, mask, Thigh) == pytest.approx(0.65 - float(X[2, 1]), rel=1e-12)
    # the loss is never negative
    rng = np.random.default_rng(6)
    Xr = rng.random((50, 6)).astype(np.float32)
    mr, _ = O.batchwise_mask(Xr, 10)
    for _ in range(20):
        assert O.batchwise_loss(Xr, mr, rng.random(6)) >= 0.0


def test_threshold_gradient_by_central_differences():
    """L_batchwise is piecewise linear in the thresholds: away from the values of X a central
    difference is exact, and the gradient is (kept by the batchwise mask) - (above the threshold)."""
    rng = np.random.default_rng(41)
    T, n, m = 40, 6, 10
    X = rng.random((T, n)).astype(np.float32)
    mask, _ = O.batchwise_mask(X, m)
    thr = np.quantile(X, 1 - m / T, axis=0) * (1 + 0.2 * rng.standard_normal(n))
    g = O.batchwise_loss_dthresholds(X, mask, thr)
    step = 1e-7
    assert np.abs(X.astype(np.float64) - thr[None, :]).min() > 10 * step
    for i in range(n):
        p, q = thr.copy(), thr.copy()
        p[i] += step
        q[i] -= step
        num = (O.batchwise_loss(X, mask, p) - O.batchwise_loss(X, mask, q)) / (2 * step)
        assert abs(num - g[i]) < 1e-6, (i, num, g[i])
    counts_thr = (X.astype(np.float64) > thr[None, :]).sum(axis=0)
    assert np.array_equal(g, m - counts_thr)
    # at the batchwise optimum (threshold between the m-th and (m+1)-th largest) the gradient vanishes
    s = np.sort(X.astype(np.float64), axis=0)
    best = 0.5 * (s[T - m] + s[T - m - 1])
    assert not O.batchwise_loss_dthresholds(X, mask, best).any()


# ---- backward through Eq.(15), (16), (20) and the experts -----------------------------------------

def _tiny_balanced_problem(seed, T=12, n=4, k=2, d=6, h=5):
    rng = np.random.default_rng(seed)
    x = rng.normal(size=(T, d))
    W_g = rng.normal(size=(d, n)) * 0.5
    bias = rng.normal(size=n) * 0.1
    W1 = rng.normal(size=(n, d, h)) * 0.5
    W2 = rng.normal(size=(n, h, d)) * 0.5
    dy = rng.normal(size=(T, d))
    thr = np.full(n, 1.0 / n) + rng.normal(size=n) * 0.02
    return x, W_g, bias, W1, W2, dy, thr, k * T // n


@pytest.mark.parametrize("seed,w_b", [(0, 0.0), (1, 0.3), (2, 1.0)])
def test_balanced_backward_by_central_differences(seed, w_b):
    """Every gradient the oracle returns against central differences of the binary64 objective.
    The masks are recomputed at every perturbed point and must not change (the step is far below
    the gaps of these inputs), so the differences see the true piecewise-smooth function."""
    x, W_g, bias, W1, W2, dy, thr, m = _tiny_balanced_problem(seed)
    wf = lambda e, W1=W1, W2=W2: (W1[e], W2[e])
    J0, mb, mt, Gs = O.balanced_objective(x, W_g, bias, thr, m, wf, dy, w_b)
    g = O.balanced_backward(x, W_g, Gs, mb, thr, wf, dy, w_b)
    step = 1e-6

    def fd(arr, index, weight_fn=None):
        vals = []
        for sgn in (+1, -1):
            old = arr[index]
            arr[index] = old + sgn * step
            J, mb2, mt2, _ = O.balanced_objective(x, W_g, bias, thr, m, weight_fn or wf, dy, w_b)
            arr[index] = old
            assert (mb2 == mb).all() and (mt2 == mt).all(), "a mask flipped: pick another seed"
            vals.append(J)
        return (vals[0] - vals[1]) / (2 * step)

    rng = np.random.default_rng(100 + seed)
    for _ in range(10):
        i = (rng.integers(x.shape[0]), rng.integers(x.shape[1]))
        assert fd(x, i) == pytest.approx(g.dx[i], rel=2e-5, abs=2e-7)
        i = (rng.integers(W_g.shape[0]), rng.integers(W_g.shape[1]))
        assert fd(W_g, i) == pytest.approx(g.dW_g[i], rel=2e-5, abs=2e-7)
        i = (rng.integers(W1.shape[0]), rng.integers(W1.shape[1]), rng.integers(W1.shape[2]))
        assert fd(W1, i) == pytest.approx(g.dW1[i[0]][i[1:]], rel=2e-5, abs=2e-7)
        i = (rng.integers(W2.shape[0]), rng.integers(W2.shape[1]), rng.integers(W2.shape[2]))
        assert fd(W2, i) == pytest.approx(g.dW2[i[0]][i[1:]], rel=2e-5, abs=2e-7)
    for i in range(bias.shape[0]):
        assert fd(bias, i) == pytest.approx(g.dbias[i], rel=2e-5, abs=2e-7)


def test_balanced_backward_closed_forms():
    """(a) one expert: G = 1 whatever the logits, so nothing reaches W_g.  (b) m = T: every expert
    keeps every token, G = G_sigma, and the gate gradient is that of a dense softmax mixture,
    dlogit_i = G_i (c_i - sum_j G_j c_j) with c_i = <dy, E_i(x)>.  (c) the logit gradients of a
    token sum to zero (the softmax is shift invariant)."""
    x, W_g, bias, W1, W2, dy, thr, m = _tiny_balanced_problem(5, T=8, n=1, k=1)
    wf = lambda e: (W1[e], W2[e])
    _, mb, _, Gs = O.balanced_objective(x, W_g, bias, thr, m, wf, dy, 0.0)
    g = O.balanced_backward(x, W_g, Gs, mb, thr, wf, dy, 0.0)
    assert np.abs(g.dW_g).max() == 0.0
    z = x @ W1[0]
    assert np.allclose(g.dx, (dy @ W2[0].T * (z > 0)) @ W1[0].T, rtol=1e-12, atol=1e-12)

    x, W_g, bias, W1, W2, dy, thr, _ = _tiny_balanced_problem(6, T=8, n=4, k=4)
    wf = lambda e: (W1[e], W2[e])
    _, mb, _, Gs = O.balanced_objective(x, W_g, bias, thr, 8, wf, dy, 0.0)
    assert mb.all()
    g = O.balanced_backward(x, W_g, Gs, mb, thr, wf, dy, 0.0)
    c = np.stack([np.einsum("td,td->t", dy, np.maximum(x @ W1[e], 0) @ W2[e]) for e in range(4)], axis=1)
    ref = Gs * (c - (Gs * c).sum(axis=1, keepdims=True))
    assert np.allclose(g.dlogits, ref, rtol=1e-10, atol=1e-12)
    assert np.allclose(g.dW_g, x.T @ ref, rtol=1e-10, atol=1e-12)

    x, W_g, bias, W1, W2, dy, thr, m = _tiny_balanced_problem(7)
    wf = lambda e: (W1[e], W2[e])
    _, mb, _, Gs = O.balanced_objective(x, W_g, bias, thr, m, wf, dy, 0.7)
    g = O.balanced_backward(x, W_g, Gs, mb, thr, wf, dy, 0.7)
    assert np.abs(g.dlogits.sum(axis=1)).max() < 1e-12
