"""Pins for the oracle's experts, Eq.(1) output, routing, hierarchical form and backward pass."""
import numpy as np
import pytest
from scipy.special import softmax

from oracle import moe_oracle as O


def _weights(rng, n, d, h, scale=0.2):
    W1 = scale * rng.standard_normal((n, d, h))
    W2 = scale * rng.standard_normal((n, h, d))
    return W1, W2, (lambda e: (W1[e], W2[e]))


def test_expert_is_a_two_layer_relu_network_triple_loop():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((3, 5))
    W1 = rng.standard_normal((5, 7))
    W2 = rng.standard_normal((7, 4))
    got = O.expert_ffn(x, W1, W2)
    for t in range(3):
        hid = [max(0.0, sum(x[t, j] * W1[j, r] for j in range(5))) for r in range(7)]
        for c in range(4):
            assert abs(got[t, c] - sum(hid[r] * W2[r, c] for r in range(7))) < 1e-12


def test_single_expert_layer_is_the_plain_mlp():
    """n = 1 (the MoE-1-Wide analogue of Appendix C): the gate is 1 and y = E_1(x)."""
    rng = np.random.default_rng(1)
    T, d, h = 20, 8, 16
    x = rng.standard_normal((T, d)).astype(np.float32)
    W1, W2, wf = _weights(rng, 1, d, h)
    lg = O.noisy_logits_f32(x, rng.standard_normal((d, 1)), rng.standard_normal((d, 1)),
                            rng.standard_normal((T, 1)))
    fw = O.gate_and_losses(lg, 1)
    assert np.all(fw.gates == 1.0) and np.all(fw.idx == 0)
    y = O.moe_output(x, fw.idx, fw.gates, wf, 1)
    assert np.abs(y - np.maximum(x.astype(np.float64) @ W1[0], 0) @ W2[0]).max() < 1e-12


def test_dense_mixture_when_k_equals_n():
    """k = n, no noise: y is the dense softmax mixture sum_i Softmax(x W_g)_i E_i(x)."""
    rng = np.random.default_rng(2)
    T, d, h, n = 16, 8, 12, 4
    x = rng.standard_normal((T, d)).astype(np.float32)
    Wg = (0.5 * rng.standard_normal((d, n))).astype(np.float32)
    W1, W2, wf = _weights(rng, n, d, h)
    lg = O.noisy_logits_f32(x, Wg, Wg, None)
    fw = O.gate_and_losses(lg, n)
    y = O.moe_output(x, fw.idx, fw.gates, wf, n)
    G = softmax(x.astype(np.float64) @ Wg.astype(np.float64), axis=1)
    E = np.einsum("nth,nhd->ntd", np.maximum(np.einsum("td,ndh->nth", x.astype(np.float64), W1), 0), W2)
    want = np.einsum("tn,ntd->td", G, E)
    assert np.abs(y - want).max() < 1e-6


def test_identical_experts_make_gating_irrelevant():
    """Gates sum to one, so if every expert has the same weights y = E(x) whatever is chosen."""
    rng = np.random.default_rng(3)
    T, d, h, n, k = 40, 8, 12, 6, 3
    x = rng.standard_normal((T, d)).astype(np.float32)
    W1 = rng.standard_normal((d, h))
    W2 = rng.standard_normal((h, d))
    lg = O.noisy_logits_f32(x, rng.standard_normal((d, n)), rng.standard_normal((d, n)),
                            rng.standard_normal((T, n)))
    fw = O.gate_and_losses(lg, k)
    y = O.moe_output(x, fw.idx, fw.gates, lambda e: (W1, W2), n)
    assert np.abs(y - O.expert_ffn(x, W1, W2)).max() < 1e-12
    sub = np.array([5, 0, 39])
    assert np.abs(O.moe_output(x, fw.idx, fw.gates, lambda e: (W1, W2), n, sub) - y[sub]).max() < 1e-12


def test_routing_brute_force():
    rng = np.random.default_rng(4)
    T, k, n = 57, 3, 9
    idx = np.stack([rng.permutation(n)[:k] for _ in range(T)]).astype(np.int32)
    counts, offsets, perm, inv = O.routing(idx, n + 2)  # two experts that nobody picks
    flat = idx.reshape(-1)
    want_perm = []
    for e in range(n + 2):
        members = [a for a in range(T * k) if flat[a] == e]
        assert counts[e] == len(members)
        assert offsets[e] == len(want_perm)
        want_perm += members
    assert offsets[-1] == T * k and counts[-1] == 0 and counts[-2] == 0
    assert list(perm) == want_perm
    assert np.array_equal(inv[perm], np.arange(T * k))
    assert sorted(perm) == list(range(T * k))


def _hier_inputs(rng, T, d, a, b, k_p):
    x = rng.standard_normal((T, d)).astype(np.float32)
    g = lambda *s: (0.4 * rng.standard_normal(s)).astype(np.float32)
    return (x, g(d, a), g(d, a), rng.standard_normal((T, a)).astype(np.float32),
            g(a, d, b), g(a, d, b), rng.standard_normal((T, k_p, b)).astype(np.float32))


def test_hierarchical_reduces_to_flat_over_groups_when_b_is_1():
    rng = np.random.default_rng(5)
    T, d, a, k_p = 60, 10, 7, 3
    x, Wgp, Wnp, ep, Wgs, Wns, es = _hier_inputs(rng, T, d, a, 1, k_p)
    hf = O.hier_gate_and_losses(x, Wgp, Wnp, ep, Wgs, Wns, es, k_p, 1)
    flat = O.gate_and_losses(O.noisy_logits_f32(x, Wgp, Wnp, ep), k_p)
    assert np.array_equal(hf.idx, flat.idx)
    assert np.abs(hf.gates - flat.gates).max() < 1e-15
    assert np.abs(hf.importance - flat.importance).max() < 1e-12
    # Eq.(14) with b = 1 and k_s = n_s = 1: Load_i(X^(i)) = |X^(i)|, so Load_H = Load_primary
    assert np.abs(hf.load - flat.load).max() < 1e-9
    assert hf.group_counts.sum() == k_p * T


def test_hierarchical_reduces_to_flat_over_experts_when_a_is_1():
    rng = np.random.default_rng(6)
    T, d, b, k_s = 50, 10, 8, 2
    x, Wgp, Wnp, ep, Wgs, Wns, es = _hier_inputs(rng, T, d, 1, b, 1)
    hf = O.hier_gate_and_losses(x, Wgp, Wnp, ep, Wgs, Wns, es, 1, k_s)
    flat = O.gate_and_losses(O.noisy_logits_f32(x, Wgs[0], Wns[0], es[:, 0, :]), k_s)
    assert np.array_equal(hf.idx, flat.idx)
    assert np.abs(hf.gates - flat.gates).max() < 1e-15
    assert np.abs(hf.load - flat.load).max() < 1e-9       # Load_primary = T = |X^(0)|
    assert abs(hf.loss_load - flat.loss_load) < 1e-12


def test_hierarchical_invariants_and_eq12_by_nested_loops():
    rng = np.random.default_rng(7)
    T, d, h, a, b, k_p, k_s = 30, 8, 6, 4, 5, 2, 2
    x, Wgp, Wnp, ep, Wgs, Wns, es = _hier_inputs(rng, T, d, a, b, k_p)
    W1, W2, wf = _weights(rng, a * b, d, h)
    hf = O.hier_gate_and_losses(x, Wgp, Wnp, ep, Wgs, Wns, es, k_p, k_s)
    assert np.allclose(hf.gates.sum(axis=1), 1.0, atol=1e-14)
    assert hf.group_counts.sum() == k_p * T
    assert abs(hf.importance.sum() - T) < 1e-9
    y = O.moe_output(x, hf.idx, hf.gates, wf, a * b)
    # Eq.(12) written as the double sum over groups and experts with dense gate vectors
    Gp = O.dense_gates(hf.group_idx, hf.group_gates, a)
    for t in range(T):
        want = np.zeros(d)
        for i in range(a):
            if Gp[t, i] == 0:
                continue
            p = list(hf.group_idx[t]).index(i)
            li = O.noisy_logits_f32(x[t:t + 1], Wgs[i], Wns[i], es[t:t + 1, p, :])
            fi = O.gate_and_losses(li, k_s)
            Gi = O.dense_gates(fi.idx, fi.gates, b)[0]
            for j in range(b):
                if Gi[j] != 0:
                    want += Gp[t, i] * Gi[j] * O.expert_ffn(x[t:t + 1], W1[i * b + j], W2[i * b + j])[0]
        assert np.abs(y[t] - want).max() < 1e-12


def _fd_setup(seed, T=6, d=5, h=7, n=6, k=2):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((T, d))
    Wg = 0.7 * rng.standard_normal((d, n))
    Wn = 0.7 * rng.standard_normal((d, n))
    eps = rng.standard_normal((T, n))
    bias = 0.3 * rng.standard_normal(n)
    W1, W2, wf = _weights(rng, n, d, h, 0.5)
    dy = rng.standard_normal((T, d))
    return x, Wg, Wn, eps, bias, W1, W2, wf, dy, k


@pytest.mark.parametrize("w_imp,w_load", [(0.1, 0.1), (0.0, 0.0), (1.0, 0.0), (0.0, 1.0)])
def test_backward_against_central_finite_differences(w_imp, w_load):
    """Gradients of J = <dy,y> + L_importance + L_load vs central differences of the binary64
    forward, with the selection frozen (it is piecewise constant)."""
    x, Wg, Wn, eps, bias, W1, W2, wf, dy, k = _fd_setup(11)
    lg = O.noisy_logits_f64(x, Wg, Wn, eps, bias)
    fwd = O.gate_and_losses(lg, k, w_imp, w_load)
    gr = O.flat_backward(x, Wg, Wn, fwd, k, wf, dy, w_imp, w_load)
    gap = np.sort(lg.H, axis=1)
    assert np.min(np.diff(gap, axis=1)) > 1e-4            # away from ties

    def J(x_=x, Wg_=Wg, Wn_=Wn, bias_=bias, wf_=wf):
        return O.flat_objective(x_, Wg_, Wn_, eps, bias_, k, wf_, dy, w_imp, w_load, fixed_idx=fwd.idx)

    def fd(arr, analytic, make):
        rng = np.random.default_rng(0)
        for _ in range(12):
            pos = tuple(rng.integers(0, s) for s in arr.shape)
            step = 1e-6
            p = arr.copy(); p[pos] += step
            m = arr.copy(); m[pos] -= step
            num = (make(p) - make(m)) / (2 * step)
            assert abs(num - analytic[pos]) < 2e-6 * max(1.0, abs(num)), (pos, num, analytic[pos])

    fd(x, gr.dx, lambda v: J(x_=v))
    fd(Wg, gr.dW_g, lambda v: J(Wg_=v))
    fd(Wn, gr.dW_noise, lambda v: J(Wn_=v))
    fd(bias, gr.dbias, lambda v: J(bias_=v))
    for e in list(gr.dW1)[:3]:
        def with_w1(v, e=e):
            return J(wf_=lambda q: ((v if q == e else W1[q]), W2[q]))

        def with_w2(v, e=e):
            return J(wf_=lambda q: (W1[q], (v if q == e else W2[q])))
        fd(W1[e], gr.dW1[e], with_w1)
        fd(W2[e], gr.dW2[e], with_w2)


def test_without_losses_noise_matrix_only_sees_kept_experts():
    """With both loss weights zero, d J / d raw is non-zero only at the kept (t, i)."""
    x, Wg, Wn, eps, bias, W1, W2, wf, dy, k = _fd_setup(12)
    lg = O.noisy_logits_f64(x, Wg, Wn, eps, bias)
    fwd = O.gate_and_losses(lg, k, 0.0, 0.0)
    gr = O.flat_backward(x, Wg, Wn, fwd, k, wf, dy, 0.0, 0.0)
    # dW_noise = x^T draw with draw supported on kept entries: columns nobody kept get zero
    unused = [i for i in range(Wg.shape[1]) if not (fwd.idx == i).any()]
    for i in unused:
        assert np.all(gr.dW_noise[:, i] == 0) and np.all(gr.dW_g[:, i] == 0)


def test_paper_counts_fixture():
    vals = {}
    with open(__file__.rsplit("/", 1)[0] + "/golden/paper_counts.txt") as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                key, v = line.split()
                vals[key] = int(v)
    d, h, k = 512, 1024, 4
    assert d * h + h * d == vals["params_per_expert"]
    assert k * (d * h + h * d) == vals["macs_per_token_k4"]
    assert 4 * 8192 // 256 == vals["mean_rows_per_expert_n256_b8192"]


def test_bf16_rounding_helper_matches_torch():
    import torch
    rng = np.random.default_rng(3)
    a = np.concatenate([rng.standard_normal(100000).astype(np.float32) * 3,
                        np.array([1.0, 1.00390625, 1.001953125, 1.005859375, -2.5, 0.0], np.float32)])
    want = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(O.round_to_bf16(a), want)


def _hier_fd_setup(seed, T=7, d=5, h=6, a=3, b=4):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((T, d))
    Wgp, Wnp = 0.7 * rng.standard_normal((d, a)), 0.7 * rng.standard_normal((d, a))
    Wgs, Wns = 0.7 * rng.standard_normal((a, d, b)), 0.7 * rng.standard_normal((a, d, b))
    ep = rng.standard_normal((T, a))
    W1, W2, wf = _weights(rng, a * b, d, h, 0.5)
    dy = rng.standard_normal((T, d))
    return x, Wgp, Wnp, ep, Wgs, Wns, W1, W2, wf, dy, rng


@pytest.mark.parametrize("w_imp,w_load", [(0.1, 0.1), (0.0, 0.0), (1.0, 0.0), (0.0, 1.0)])
def test_hierarchical_backward_against_central_finite_differences(w_imp, w_load):
    """Gradients through Eq.(12)-(14) vs central differences of the binary64 forward with both
    levels' selections frozen."""
    k_p, k_s = 2, 2
    x, Wgp, Wnp, ep, Wgs, Wns, W1, W2, wf, dy, rng = _hier_fd_setup(21)
    es = rng.standard_normal((x.shape[0], k_p, Wgs.shape[2]))
    parts = O._hier_forward_parts(x, Wgp, Wnp, ep, Wgs, Wns, es, k_p, k_s, O.noisy_logits_f64)
    gidx, sidx = parts["gidx"], parts["sec_idx"]
    assert (parts["gcount"] > 0).all()
    gr = O.hier_backward(x, Wgp, Wnp, ep, Wgs, Wns, es, k_p, k_s, wf, dy, w_imp, w_load,
                         logits_fn=O.noisy_logits_f64)

    def J(x_=x, Wgp_=Wgp, Wnp_=Wnp, Wgs_=Wgs, Wns_=Wns, wf_=wf):
        return O.hier_objective(x_, Wgp_, Wnp_, ep, Wgs_, Wns_, es, k_p, k_s, wf_, dy, w_imp, w_load, gidx, sidx)

    def fd(arr, analytic, make, count=10):
        r = np.random.default_rng(1)
        for _ in range(count):
            pos = tuple(r.integers(0, s) for s in arr.shape)
            step = 1e-6
            p = arr.copy(); p[pos] += step
            m = arr.copy(); m[pos] -= step
            num = (make(p) - make(m)) / (2 * step)
            assert abs(num - analytic[pos]) < 3e-6 * max(1.0, abs(num)), (pos, num, analytic[pos])

    fd(x, gr.dx, lambda v: J(x_=v))
    fd(Wgp, gr.dWg_p, lambda v: J(Wgp_=v))
    fd(Wnp, gr.dWn_p, lambda v: J(Wnp_=v))
    fd(Wgs, gr.dWg_s, lambda v: J(Wgs_=v), 16)
    fd(Wns, gr.dWn_s, lambda v: J(Wns_=v), 16)
    for e in list(gr.dW1)[:2]:
        fd(W1[e], gr.dW1[e], lambda v, e=e: J(wf_=lambda q: ((v if q == e else W1[q]), W2[q])), 6)
        fd(W2[e], gr.dW2[e], lambda v, e=e: J(wf_=lambda q: (W1[q], (v if q == e else W2[q]))), 6)


def test_hierarchical_backward_with_one_group_is_the_flat_backward():
    """a = 1, k_primary = 1: the primary gate is the constant 1, Load_H = Load of the only
    secondary gate, so every gradient must equal the flat layer's over the b experts."""
    rng = np.random.default_rng(22)
    T, d, h, b, k = 9, 6, 5, 5, 2
    x = rng.standard_normal((T, d))
    Wg, Wn = 0.6 * rng.standard_normal((d, b)), 0.6 * rng.standard_normal((d, b))
    eps = rng.standard_normal((T, b))
    W1, W2, wf = _weights(rng, b, d, h, 0.5)
    dy = rng.standard_normal((T, d))
    Wgp, Wnp = rng.standard_normal((d, 1)), rng.standard_normal((d, 1))
    gr = O.hier_backward(x, Wgp, Wnp, rng.standard_normal((T, 1)), Wg[None], Wn[None], eps[:, None, :], 1, k, wf, dy,
                         0.3, 0.7, logits_fn=O.noisy_logits_f64)
    lg = O.noisy_logits_f64(x, Wg, Wn, eps)
    fwd = O.gate_and_losses(lg, k, 0.3, 0.7)
    fl = O.flat_backward(x, Wg, Wn, fwd, k, wf, dy, 0.3, 0.7)
    assert np.allclose(gr.dx, fl.dx, rtol=1e-10, atol=1e-12)
    assert np.allclose(gr.dWg_s[0], fl.dW_g, rtol=1e-10, atol=1e-12)
    assert np.allclose(gr.dWn_s[0], fl.dW_noise, rtol=1e-10, atol=1e-12)
    assert np.abs(gr.dWg_p).max() < 1e-12 and np.abs(gr.dWn_p).max() < 1e-12     # a constant gate learns nothing
    for e in fl.dW1:
        assert np.allclose(gr.dW1[e], fl.dW1[e], rtol=1e-10, atol=1e-12)
        assert np.allclose(gr.dW2[e], fl.dW2[e], rtol=1e-10, atol=1e-12)


def test_layer_epilogue_closed_forms():
    """Appendix C: sigmoid, inverted dropout, residual.  Checked against scipy's logistic function,
    the p = 0 and all-dropped special cases, and the 1/(1-p) scaling that keeps the expectation."""
    from scipy.special import expit
    rng = np.random.default_rng(31)
    y = 4.0 * rng.standard_normal((50, 8))
    x = rng.standard_normal((50, 8))
    assert np.allclose(O.layer_epilogue(y, x, None, 0.0), x + expit(y), rtol=1e-14)
    keep_all = np.ones_like(y, bool)
    assert np.allclose(O.layer_epilogue(y, x, keep_all, 0.25), x + expit(y) / 0.75, rtol=1e-14)
    assert np.array_equal(O.layer_epilogue(y, x, ~keep_all, 0.25), x)
    # averaged over every mask with exactly half the units kept, dropout with p = 1/2 is the identity
    import itertools
    yy, xx = y[:1, :4], x[:1, :4]
    acc = np.zeros_like(yy)
    masks = [m for m in itertools.product([False, True], repeat=4) if sum(m) == 2]
    for m in masks:
        acc += O.layer_epilogue(yy, xx, np.array(m)[None, :], 0.5)
    assert np.allclose(acc / len(masks), xx + expit(yy), rtol=1e-13)
    # symmetry of the logistic function: sigmoid(-y) = 1 - sigmoid(y)
    assert np.allclose(O.layer_epilogue(-y, 0 * x, None, 0.0), 1.0 - O.layer_epilogue(y, 0 * x, None, 0.0), atol=1e-15)


def test_expert_input_grad_by_central_differences_and_mask_override():
    """expert_input_grad is the derivative of <dout, relu(x W1) W2> in x (checked numerically away
    from the kink); with an explicit mask it is linear in the mask: switching one hidden unit on
    adds exactly that unit's path dout.W2[u,:] * W1[:,u]."""
    rng = np.random.default_rng(21)
    d, h, rows = 6, 9, 4
    W1, W2 = rng.standard_normal((d, h)), rng.standard_normal((h, d))
    xe, dout = rng.standard_normal((rows, d)), rng.standard_normal((rows, d))
    assert np.abs(xe @ W1).min() > 1e-3
    g = O.expert_input_grad(xe, dout, W1, W2)
    f = lambda xx: float((dout * O.expert_ffn(xx, W1, W2)).sum())
    step = 1e-6
    for r in range(rows):
        for j in range(d):
            e = np.zeros_like(xe)
            e[r, j] = step
            assert g[r, j] == pytest.approx((f(xe + e) - f(xe - e)) / (2 * step), rel=1e-6, abs=1e-8)
    mask = (xe @ W1) > 0
    r, u = np.argwhere(~mask)[0]
    flipped = mask.copy()
    flipped[r, u] = True
    delta = O.expert_input_grad(xe, dout, W1, W2, relu_mask=flipped) - g
    expect = np.zeros_like(g)
    expect[r] = (dout[r] @ W2[u, :]) * W1[:, u]
    assert np.abs(delta - expect).max() <= 1e-12
    # and it is what experts_backward accumulates into dx for a batch that uses one expert
    idx = np.zeros((rows, 1), np.int64)
    gates = rng.random((rows, 1)) + 0.5
    dy = rng.standard_normal((rows, d))
    dx, _, _, _ = O.experts_backward(xe, idx, gates, lambda e: (W1, W2), dy)
    assert np.abs(dx - O.expert_input_grad(xe, gates * dy, W1, W2)).max() <= 1e-12
