"""Pins for the oracle's factored-second-moment Adam step (Appendix D): closed forms and the
properties the paper states, each computed independently of the function under test."""
import numpy as np

from oracle import moe_oracle as O


def _rng(seed):
    return np.random.default_rng(seed)


def test_constant_magnitude_gradient_gives_sign_update():
    """|G| = g everywhere: every second-moment estimate is g^2 after bias correction, so at every
    step W moves by lr * sign(G) * g / (g + eps), as plain Adam with beta1 = 0 does."""
    rng = _rng(1)
    R, C, g, lr, eps, b2 = 7, 5, 0.03, 1e-2, 1e-8, 0.9
    W = rng.standard_normal((R, C))
    vr, vc = np.zeros(R), np.zeros(C)
    for step in range(1, 6):
        S = np.where(rng.random((R, C)) < 0.5, -1.0, 1.0)
        Wn, vr, vc = O.factored_adam_step(W, g * S, vr, vc, lr, b2, eps, step)
        assert np.allclose(Wn, W - lr * S * g / (g + eps), rtol=1e-12, atol=0)
        W = Wn


def test_rank_one_squared_gradient_equals_full_adam():
    """G*G = u v^T is exactly representable by the two vectors: the factored step must equal Adam
    (beta1 = 0) with the full matrix of second moments, written out here from its definition."""
    rng = _rng(2)
    R, C, lr, eps, b2 = 6, 9, 3e-3, 1e-6, 0.99
    u, v = rng.random(R) + 0.1, rng.random(C) + 0.1
    S = np.where(rng.random((R, C)) < 0.5, -1.0, 1.0)
    G = S * np.sqrt(np.outer(u, v))
    W = rng.standard_normal((R, C))
    Wn, vr, vc = O.factored_adam_step(W, G, np.zeros(R), np.zeros(C), lr, b2, eps, 1)
    V = (1 - b2) * G * G                      # full estimator after one step from zero
    ref = W - lr * G / (np.sqrt(V / (1 - b2)) + eps)
    assert np.allclose(Wn, ref, rtol=1e-12, atol=0)


def test_vectors_are_the_row_and_column_averages_of_the_full_estimator():
    """Run the FULL matrix recursion next to the factored one for several random steps: the kept
    vectors must be its row-wise and column-wise averages, their means must agree, and the
    factored estimator must have the same row and column averages as the full one."""
    rng = _rng(3)
    R, C, b2 = 8, 12, 0.95
    V = np.zeros((R, C))
    vr, vc = np.zeros(R), np.zeros(C)
    W = rng.standard_normal((R, C))
    for step in range(1, 8):
        G = rng.standard_normal((R, C)) * rng.random((R, 1)) * rng.random((1, C))
        V = b2 * V + (1 - b2) * G * G
        W, vr, vc = O.factored_adam_step(W, G, vr, vc, 1e-3, b2, 1e-8, step)
        assert np.allclose(vr, V.mean(axis=1), rtol=1e-12)
        assert np.allclose(vc, V.mean(axis=0), rtol=1e-12)
        assert np.isclose(vr.mean(), vc.mean(), rtol=1e-12)
        Vhat = np.outer(vr, vc) / vr.mean()
        assert np.allclose(Vhat.mean(axis=1), V.mean(axis=1), rtol=1e-12)
        assert np.allclose(Vhat.mean(axis=0), V.mean(axis=0), rtol=1e-12)


def test_update_matches_formula_on_a_tiny_case():
    """2 x 2 worked by hand: G = [[1, 2], [3, 4]], zero state, beta2 = 0.5, step 1."""
    G = np.array([[1.0, 2.0], [3.0, 4.0]])
    W = np.zeros((2, 2))
    Wn, vr, vc = O.factored_adam_step(W, G, np.zeros(2), np.zeros(2), 1.0, 0.5, 0.0, 1)
    # row means of G^2: 2.5, 12.5; column means: 5, 10; all halved by (1 - beta2); mean 3.75
    assert np.allclose(vr, [1.25, 6.25]) and np.allclose(vc, [2.5, 5.0])
    vhat = np.array([[1.25 * 2.5, 1.25 * 5.0], [6.25 * 2.5, 6.25 * 5.0]]) / 3.75 / 0.5
    assert np.allclose(Wn, -G / np.sqrt(vhat), rtol=1e-14)


def test_zero_gradient_history_leaves_weights():
    W = np.arange(6.0).reshape(2, 3)
    Wn, vr, vc = O.factored_adam_step(W, np.zeros((2, 3)), np.zeros(2), np.zeros(3), 0.1, 0.9, 1e-8, 1)
    assert np.array_equal(Wn, W) and not vr.any() and not vc.any()


def test_state_memory_is_rows_plus_columns():
    """The point of the factoring: R + C numbers of state instead of R * C."""
    _, vr, vc = O.factored_adam_step(np.zeros((512, 1024)), np.ones((512, 1024)), np.zeros(512), np.zeros(1024),
                                     1e-3, 0.999, 1e-8, 1)
    assert vr.size + vc.size == 512 + 1024
