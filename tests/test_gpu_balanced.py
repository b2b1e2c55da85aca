"""GPU parity of strictly balanced gating (Appendix F, Eq.(15)-(20)) against the oracle: the softmax
gate within one fp32 ulp of the plain binary64 definition; the batchwise mask and the per-expert
token lists exactly the brute-force definition of Eq.(18) on the kernel's own gate values and equal
to the oracle's wherever the oracle's comparison is decided beyond rounding (tests/balanced_checks.py);
the denominators and L_batchwise within 1e-5, the layer output within the bf16 tolerance."""
import sys

import numpy as np
import pytest
import torch

import moe_workloads as W
from oracle import moe_oracle as O
from tests import balanced_checks as BC
from tests import gpu_harness as G

pytestmark = pytest.mark.gpu
TOL_F32 = 1e-5
TOL_BF16 = 2e-2


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def api():
    assert torch.cuda.is_available()
    from paper_1701_06538_amd import api as _api
    return _api


def make_thresholds(X, m, seed):
    """Per-expert thresholds near the m-th largest value of the column, so that the two masks of
    Eq.(20) differ on a few percent of the entries."""
    T = X.shape[0]
    rng = np.random.default_rng(seed)
    q = np.sort(X.astype(np.float64), axis=0)[max(T - m, 0) if m > 0 else T - 1]
    return (q * (1.0 + 0.05 * rng.standard_normal(q.shape))).astype(np.float32)


def check_gate(run, x, W_g, bias, thresholds):
    """Returns (oracle G_sigma, validated batchwise mask, Eq.(16) gates of the oracle on that mask)."""
    c = run.cfg
    T, n = c.T, c.n
    _, X = O.softmax_gate_f32(x, W_g, bias)
    got = run.gsigma.cpu().numpy()[:T]
    same = BC.check_gsigma(got, X)
    mask = run.kept_mask()
    undecided = BC.check_batchwise_mask(got, mask, run.tokens.cpu().numpy(), X, run.m)
    ref_mask, _ = O.batchwise_mask(X, run.m)
    say("  G_sigma: %.4f of the values equal to the oracle's in bits, rest within 1 ulp; mask entries the "
        "oracle leaves undecided: %d; entries that differ from the oracle's mask: %d"
        % (same, undecided, (mask != ref_mask).sum()))
    Gm, denom = O.balanced_gates(X, mask)
    d_got = run.denom.cpu().numpy()[:T].astype(np.float64)
    assert np.abs(d_got - denom).max() <= TOL_F32 * max(denom.max(), 1e-30)
    assert ((denom == 0) == (d_got == 0)).all()
    if thresholds is not None:
        thr_mask = O.threshold_mask(got, thresholds)            # checked against the oracle's below
        BC.check_threshold_mask(got, thr_mask, X, thresholds)
        diff = thr_mask.astype(np.float64) - mask
        ref = float((diff * (X.astype(np.float64) - np.asarray(thresholds, np.float64)[None, :])).sum())
        ref_plain = O.batchwise_loss(X, ref_mask, thresholds)   # Eq.(20) entirely on the oracle's side
        assert abs(ref - ref_plain) <= 1e-6 * abs(ref_plain) + 1e-9
        gl = float(run.loss.cpu().numpy()[0])
        assert abs(gl - ref_plain) <= TOL_F32 * abs(ref_plain) + 1e-9, (gl, ref_plain)
        dthr = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
        run.api.moe_batchwise_loss_grad(c, run.gsigma, run.thr, dthr)
        torch.cuda.synchronize()
        assert np.array_equal(dthr.cpu().numpy().astype(np.float64), O.batchwise_loss_dthresholds(got, mask, thresholds))
    return X, mask, Gm


GATE_CASES = {
    # name: (T, n, k, d, with_bias, gate_std)
    "small": (256, 8, 2, 512, False, 0.02),
    "ragged_n40": (1000, 40, 4, 512, True, 0.05),
    "one_expert": (130, 1, 1, 512, False, 0.02),
    "m_equals_T": (96, 4, 4, 512, False, 0.02),
    "n320_d256": (640, 320, 4, 256, False, 0.05),
    "cfg1_shape": (8192, 256, 4, 512, True, 0.02),
    "n2048": (4096, 2048, 4, 512, False, 0.05),
}


@pytest.mark.parametrize("name", list(GATE_CASES))
def test_gate_balanced(api, name):
    T, n, k, d, with_bias, std = GATE_CASES[name]
    say("gate_balanced", name)
    shape = W.scaled_config(W.CONFIGS[1], T=T, n=n, k=k, d=d)
    x, W_g, _, _, bias = G.flat_inputs(shape, with_bias=with_bias, gate_std=std)
    _, X = O.softmax_gate_f32(x, W_g, bias)
    thr = make_thresholds(X, T * k // n, 5)
    run = G.BalancedRun(api, shape, x, W_g, bias, thr)
    run.gate()
    check_gate(run, x, W_g, bias, thr)


def test_gate_balanced_ties(api):
    """Duplicated tokens give equal values within every column: the lower token index is kept."""
    say("gate_balanced ties")
    shape = W.scaled_config(W.CONFIGS[1], T=512, n=16, k=2)
    x, W_g, _, _, _ = G.flat_inputs(shape)
    x[100:120] = x[5]
    x[256:] = x[:256]                       # token t and t+256 are the same row
    run = G.BalancedRun(api, shape, x, W_g, None, None)
    run.gate()
    X, mask, _ = check_gate(run, x, W_g, None, None)
    assert (X[256:] == X[:256]).all()
    assert not (mask[256:] & ~mask[:256]).any()      # the later copy is never kept without the earlier


def test_gate_balanced_no_thresholds_leaves_loss(api):
    say("gate_balanced no thresholds")
    shape = W.scaled_config(W.CONFIGS[1], T=128, n=8, k=2)
    x, W_g, _, _, _ = G.flat_inputs(shape)
    run = G.BalancedRun(api, shape, x, W_g, None, None)
    run.gate()
    assert np.isnan(run.loss.cpu().numpy()[0])
    check_gate(run, x, W_g, None, None)


def test_balanced_rejects_unbalanced_batch(api):
    shape = W.scaled_config(W.CONFIGS[1], T=100, n=8, k=3)      # 300 rows over 8 experts
    cfg = api.make_config(shape)
    assert api.moe_balanced_rows_per_expert(cfg) == -1
    assert api.moe_balanced_workspace_bytes(cfg) == 0
    t = torch.zeros(16, device="cuda")
    with pytest.raises(api.MoeError) as e:
        api.moe_gate_balanced(cfg, t, t, None, None, t, t, t, t, t, torch.zeros(256, dtype=torch.uint8, device="cuda"))
    assert e.value.status == api.MOE_EINVAL


def test_balanced_empty_batch(api):
    shape = W.scaled_config(W.CONFIGS[1], T=0, n=8, k=2)
    x = np.zeros((0, shape.d), np.float32)
    W_g = np.zeros((shape.d, shape.n), np.float32)
    run = G.BalancedRun(api, shape, x, W_g, None, None)
    run.gate()
    assert run.m == 0


LAYER_CASES = {
    # name: (T, n, k, d, h, dtype, sampled tokens or None)
    "small_bf16": (256, 8, 2, 512, 1024, "bf16", None),
    "ragged_bf16": (1000, 40, 4, 512, 1024, "bf16", None),
    "small_f32": (192, 8, 2, 512, 1024, "f32", None),
    "d256_h512": (640, 16, 2, 256, 512, "bf16", None),
    "cfg1_shape": (8192, 256, 4, 512, 1024, "bf16", 192),
}


@pytest.mark.parametrize("name", list(LAYER_CASES))
def test_layer_balanced(api, name):
    T, n, k, d, h, dtype, sample = LAYER_CASES[name]
    say("layer_balanced", name)
    shape = W.scaled_config(W.CONFIGS[1], T=T, n=n, k=k, d=d, h=h, expert_dtype=dtype)
    x, W_g, _, _, bias = G.flat_inputs(shape, with_bias=True, gate_std=0.05)
    W1, W2 = G.device_weights(shape)
    if dtype == "bf16":
        W1, W2 = W1.to(torch.bfloat16), W2.to(torch.bfloat16)
    _, X = O.softmax_gate_f32(x, W_g, bias)
    thr = make_thresholds(X, T * k // n, 9)
    run = G.BalancedRun(api, shape, x, W_g, bias, thr, W1, W2)
    run.layer()
    _, mask, Gm = check_gate(run, x, W_g, bias, thr)
    toks = None
    if sample:
        rng = np.random.default_rng(3)
        unkept = np.nonzero(~mask.any(axis=1))[0][:8]
        toks = np.unique(np.concatenate([rng.choice(T, sample, replace=False), unkept, [0, T - 1]]))
    y_ref = O.balanced_output(x, Gm, G.oracle_weight_fn(shape), toks)
    y = run.y.cpu().numpy()[:T]
    y = y if toks is None else y[toks]
    row, mx = G.rel_errors(y, y_ref)
    say("  y row-rel %.2e max-rel %.2e, tokens without an expert: %d" % (row, mx, (~mask.any(axis=1)).sum()))
    tol = TOL_BF16 if dtype == "bf16" else TOL_F32
    assert row <= tol and mx <= tol
    zero_rows = ~(Gm > 0).any(axis=1) if toks is None else ~(Gm[toks] > 0).any(axis=1)
    assert (y[zero_rows] == 0).all()


THRESHOLD_CASES = {
    # name: (T, n, k, d, h, dtype, capacity factor, sampled tokens or None)
    "small_bf16": (256, 8, 2, 512, 1024, "bf16", 2.0, None),
    "ragged_bf16": (1001, 40, 4, 512, 1024, "bf16", 2.0, None),
    "small_f32": (192, 8, 2, 512, 1024, "f32", 2.0, None),
    "d256_h512": (640, 16, 2, 256, 512, "bf16", 1.5, None),
    "n320": (900, 320, 4, 512, 1024, "bf16", 2.0, 128),
    "cfg1_shape": (8192, 256, 4, 512, 1024, "bf16", 1.25, 192),
}


def run_threshold(api, shape, x, W_g, bias, thr, W1, W2, capacity):
    cfg = api.make_config(shape)
    T, n, d = cfg.T, cfg.n, cfg.d
    f32 = dict(dtype=torch.float32, device="cuda")
    i32 = dict(dtype=torch.int32, device="cuda")
    out = dict(y=torch.full((T, d), float("nan"), **f32), gsigma=torch.full((T, n), float("nan"), **f32),
               counts=torch.full((n,), -7, **i32), tokens=torch.full((max(capacity, 1),), -7, **i32),
               kept=torch.full((T, (n + 31) // 32), 0x5a5a5a5a, **i32), denom=torch.full((T,), float("nan"), **f32),
               rows_total=torch.full((4,), -7, **i32))
    ws = torch.empty(max(256, api.moe_threshold_workspace_bytes(cfg, capacity)), dtype=torch.uint8, device="cuda")
    api.moe_layer_forward_threshold(cfg, G.dev(x), G.dev(W_g), None if bias is None else G.dev(bias), G.dev(thr),
                                    W1, W2, capacity, out["y"], out["gsigma"], out["counts"], out["tokens"],
                                    out["kept"], out["denom"], out["rows_total"], ws)
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in out.items()}


def unpack_kept(words, n):
    words = words.view(np.uint32)
    bits = (words[:, :, None] >> np.arange(32, dtype=np.uint32)[None, None, :]) & 1
    return bits.reshape(words.shape[0], -1)[:, :n].astype(bool)


@pytest.mark.parametrize("name", list(THRESHOLD_CASES))
def test_layer_threshold(api, name):
    T, n, k, d, h, dtype, cap, sample = THRESHOLD_CASES[name]
    say("layer_threshold", name)
    shape = W.scaled_config(W.CONFIGS[1], T=T, n=n, k=k, d=d, h=h, expert_dtype=dtype)
    x, W_g, _, _, bias = G.flat_inputs(shape, with_bias=True, gate_std=0.05)
    W1, W2 = G.device_weights(shape)
    _, X = O.softmax_gate_f32(x, W_g, bias)
    thr = make_thresholds(X, max(1, T * k // n), 11)
    thr[0] = 0.0 if n > 1 else thr[0]          # an expert that keeps every token
    if n > 2:
        thr[2] = 2.0                            # and one that keeps none
    mask = O.threshold_mask(X, thr)
    capacity = int(cap * mask.sum()) + 7
    got = run_threshold(api, shape, x, W_g, bias, thr, W1, W2, capacity)
    BC.check_gsigma(got["gsigma"], X)
    mask = unpack_kept(got["kept"], n)                  # Eq.(19) on the kernel's own values, validated:
    undecided = BC.check_threshold_mask(got["gsigma"], mask, X, thr)
    say("  threshold-mask entries the oracle leaves undecided: %d, differing: %d"
        % (undecided, (mask != O.threshold_mask(X, thr)).sum()))
    assert np.array_equal(got["counts"], mask.sum(axis=0))
    assert got["rows_total"][0] == mask.sum()
    ref_list = np.concatenate([np.nonzero(mask[:, e])[0] for e in range(n)]).astype(np.int32)
    assert np.array_equal(got["tokens"][:ref_list.size], ref_list)
    Gm, denom = O.balanced_gates(X, mask)
    assert np.abs(got["denom"].astype(np.float64) - denom).max() <= TOL_F32 * max(denom.max(), 1e-30)
    toks = None
    if sample:
        rng = np.random.default_rng(4)
        unkept = np.nonzero(~mask.any(axis=1))[0][:8]
        toks = np.unique(np.concatenate([rng.choice(T, sample, replace=False), unkept, [0, T - 1]]))
    y_ref = O.balanced_output(x, Gm, G.oracle_weight_fn(shape), toks)
    y = got["y"] if toks is None else got["y"][toks]
    row, mx = G.rel_errors(y, y_ref)
    say("  rows %d (capacity %d), y row-rel %.2e max-rel %.2e" % (mask.sum(), capacity, row, mx))
    tol = TOL_BF16 if dtype == "bf16" else TOL_F32
    assert row <= tol and mx <= tol


def test_layer_threshold_capacity_exceeded(api):
    """More kept rows than the caller made room for: the total is reported, no expert runs, y = 0."""
    say("layer_threshold capacity exceeded")
    shape = W.scaled_config(W.CONFIGS[1], T=512, n=16, k=2)
    x, W_g, _, _, _ = G.flat_inputs(shape, gate_std=0.05)
    W1, W2 = G.device_weights(shape)
    _, X = O.softmax_gate_f32(x, W_g)
    thr = make_thresholds(X, 64, 12)
    mask = O.threshold_mask(X, thr)
    capacity = int(mask.sum()) // 2
    got = run_threshold(api, shape, x, W_g, None, thr, W1, W2, capacity)
    BC.check_gsigma(got["gsigma"], X)
    mask = unpack_kept(got["kept"], shape.n)
    BC.check_threshold_mask(got["gsigma"], mask, X, thr)
    assert got["rows_total"][0] == mask.sum() > capacity
    assert np.array_equal(got["counts"], mask.sum(axis=0))
    assert not got["y"].any()
