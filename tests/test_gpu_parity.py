"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Bars: top-k indices, counts, offsets, permutations bit-exact; the fp32 logits the selection is
taken on bit-exact (same pinned arithmetic on both sides); gate values, fp32 outputs and losses
within 1e-5 relative; bf16-expert outputs within 2e-2 relative."""
import sys

import numpy as np
import pytest
import torch

import moe_workloads as W
from oracle import moe_oracle as O
from tests import gpu_harness as G

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-5
TOL_BF16 = 2e-2


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def api():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_1701_06538_amd import api as _api
    return _api


def _shape(base, **kw):
    return W.scaled_config(W.CONFIGS[base], **kw)


def check_gate(run, fw, shape):
    k, n = shape.k, shape.n
    assert np.array_equal(run.cleanb.cpu().numpy(), fw.logits.cleanb), "clean logits differ in bits"
    assert np.array_equal(run.sp.cpu().numpy(), fw.logits.sp), "softplus differs in bits"
    assert np.array_equal(run.topk_idx.cpu().numpy(), fw.idx), "top-k indices differ"
    g = run.topk_gate.cpu().numpy().astype(np.float64)
    assert np.abs(g - fw.gates).max() <= TOL_F32 * 1.0
    if k < n:
        order = np.argsort(-fw.logits.H, axis=1, kind="stable")
        assert np.array_equal(run.next_idx.cpu().numpy(), order[:, k].astype(np.int32))
    else:
        assert np.all(run.next_idx.cpu().numpy() == -1)


def check_losses(run, fw):
    imp = run.importance.cpu().numpy().astype(np.float64)
    ld = run.load.cpu().numpy().astype(np.float64)
    assert np.abs(imp - fw.importance).max() <= TOL_F32 * np.abs(fw.importance).max()
    assert np.abs(ld - fw.load).max() <= TOL_F32 * np.abs(fw.load).max()
    L = run.losses.cpu().numpy().astype(np.float64)
    for got, ref in ((L[0], fw.loss_importance), (L[1], fw.loss_load)):
        assert abs(got - ref) <= TOL_F32 * abs(ref) + 1e-8, (got, ref)
    w_i, w_l = run.cfg.w_importance, run.cfg.w_load
    assert abs(L[2] * w_i - L[0]) <= 1e-6 * abs(L[0]) + 1e-9
    assert abs(L[3] * w_l - L[1]) <= 1e-6 * abs(L[1]) + 1e-9


def check_route(run, idx, n):
    counts, offsets, perm, inv = O.routing(idx, n)
    assert np.array_equal(run.counts.cpu().numpy(), counts)
    assert np.array_equal(run.offsets.cpu().numpy(), offsets)
    A = idx.size
    assert np.array_equal(run.perm.cpu().numpy()[:A], perm)
    assert np.array_equal(run.inv_perm.cpu().numpy()[:A], inv)
    # tile table: covers every non-empty expert's rows exactly once, in order
    TM = run.api.moe_tile_rows(run.cfg)
    nt = int(run.num_tiles.cpu().numpy()[0])
    te = run.tile_expert.cpu().numpy()[:nt]
    tr = run.tile_row0.cpu().numpy()[:nt]
    want_e, want_r = [], []
    for e in range(n):
        for j in range(0, counts[e], TM):
            want_e.append(e)
            want_r.append(offsets[e] + j)
    assert list(te) == want_e and list(tr) == want_r
    assert nt <= run.api.moe_max_tiles(run.cfg)


GATE_CASES = [
    # name, base, overrides, with_bias, noise
    ("cfg0", 0, dict(), False, True),
    ("ragged_T_n", 1, dict(T=1000, n=200, k=4), False, True),
    ("odd_n_k3", 1, dict(T=333, n=37, k=3), True, True),
    ("k_equals_n", 1, dict(T=130, n=8, k=8), False, True),
    ("noise_free_k1", 1, dict(T=257, n=64, k=1), False, False),
    ("n2048_k4", 2, dict(T=192), False, True),
    ("k2_n64", 1, dict(T=500, n=64, k=2), False, True),
]


@pytest.mark.parametrize("name,base,ov,with_bias,noise", GATE_CASES, ids=[c[0] for c in GATE_CASES])
def test_gate_route_losses_parity(api, name, base, ov, with_bias, noise):
    shape = _shape(base, **ov)
    if with_bias:
        shape = W.scaled_config(shape, zipf_beta=0.5)
    say("case", name, shape)
    x, W_g, W_noise, eps, bias = G.flat_inputs(shape, with_bias)
    if not noise:
        eps = None
    fw = G.oracle_flat(shape, x, W_g, W_noise, eps, bias)
    run = G.FlatRun(api, shape, x, W_g, W_noise, eps, bias, None, None)
    run.gate(); run.route(); run.losses_()
    torch.cuda.synchronize()
    check_gate(run, fw, shape)
    check_route(run, fw.idx, shape.n)
    check_losses(run, fw)


def test_gate_route_losses_random_shapes(api):
    """A seeded sweep of odd shapes (T, n, k, d drawn at random, some with a bias, some noise-free,
    some with duplicated token rows so that whole rows of logits tie): logits, top-k indices, the
    next-best expert, counts, offsets, permutation and tile table bit for bit, gate values and
    losses within the fp32 tolerance."""
    rng = np.random.default_rng(20240607)
    for case in range(16):
        n = int(rng.choice([4, 6, 12, 20, 33, 64, 100, 128, 257, 300, 512, 640]))
        k = int(rng.integers(1, min(n, 8) + 1))
        T = int(rng.integers(1, 1500))
        d = int(rng.choice([32, 64, 96, 256, 512]))
        with_bias, noise = bool(rng.integers(2)), bool(rng.integers(4))
        shape = _shape(1, T=T, n=n, k=k, d=d, h=64)
        if with_bias:
            shape = W.scaled_config(shape, zipf_beta=0.5)
        say("random case", case, dict(T=T, n=n, k=k, d=d, bias=with_bias, noise=noise))
        x, W_g, W_noise, eps, bias = G.flat_inputs(shape, with_bias)
        if T > 8 and case % 3 == 0:       # tokens with identical rows (and identical noise): identical decisions
            x[T // 2:T // 2 + 4] = x[0]
            eps[T // 2:T // 2 + 4] = eps[0]
        if not noise:
            eps = None
        fw = G.oracle_flat(shape, x, W_g, W_noise, eps, bias)
        run = G.FlatRun(api, shape, x, W_g, W_noise, eps, bias, None, None)
        run.gate(); run.route(); run.losses_()
        torch.cuda.synchronize()
        check_gate(run, fw, shape)
        check_route(run, fw.idx, shape.n)
        check_losses(run, fw)


WIDE_CASES = [
    # the four-waves-per-row top-k kernel (1024 < n <= 2048): widths off every tile size, k from 1 to
    # 8 (both list-length instantiations), with a bias, noise-free, and with tied rows
    # name, n, k, T, with_bias, noise
    ("n1025_k1", 1025, 1, 130, False, True),
    ("n1025_k8", 1025, 8, 97, True, True),
    ("n1500_k3", 1500, 3, 200, False, True),
    ("n1500_k8_noise_free", 1500, 8, 64, False, False),
    ("n2047_k1_noise_free", 2047, 1, 75, True, False),
    ("n2047_k3", 2047, 3, 140, True, True),
    ("n2047_k8", 2047, 8, 50, False, True),
    # more than 2048 experts in one gating level: rows walked as chunks of 2048 columns (2, 4 and 8
    # chunks, the last one partly or wholly past the end of the row)
    ("n4096_k4", 4096, 4, 70, False, True),
    ("n5000_k8", 5000, 8, 40, True, True),
    ("n8192_k2_noise_free", 8192, 2, 33, False, False),
    ("n12345_k4", 12345, 4, 24, True, True),
    ("n16384_k8", 16384, 8, 20, False, True),
]


@pytest.mark.parametrize("name,n,k,T,with_bias,noise", WIDE_CASES, ids=[c[0] for c in WIDE_CASES])
def test_gate_wide_rows(api, name, n, k, T, with_bias, noise):
    shape = _shape(1, T=T, n=n, k=k, d=128, h=64)
    if with_bias:
        shape = W.scaled_config(shape, zipf_beta=0.5)
    say("case wide", name, shape)
    x, W_g, W_noise, eps, bias = G.flat_inputs(shape, with_bias)
    # in-row ties: duplicated gate columns (same clean and raw logit) with the same noise draw give
    # equal H at different experts, some of them across the quarters the four waves own
    for src, dst in ((3, 700), (3, n - 1), (510, 511), (1023, 1024), (2047, 2048), (5, n // 2 + 1)):
        if max(src, dst) >= n:
            continue
        W_g[:, dst], W_noise[:, dst], eps[:, dst] = W_g[:, src], W_noise[:, src], eps[:, src]
        if bias is not None:
            bias[dst] = bias[src]
    x[T // 2:T // 2 + 3] = x[1]            # and whole rows that tie with each other
    eps[T // 2:T // 2 + 3] = eps[1]
    if not noise:
        eps = None
    fw = G.oracle_flat(shape, x, W_g, W_noise, eps, bias)
    assert (fw.logits.H[:, 3] == fw.logits.H[:, 700]).all()
    run = G.FlatRun(api, shape, x, W_g, W_noise, eps, bias, None, None)
    run.gate(); run.route(); run.losses_()
    torch.cuda.synchronize()
    check_gate(run, fw, shape)
    check_route(run, fw.idx, shape.n)
    check_losses(run, fw)


def test_gate_zero_initialised_matrices(api):
    """W_g = W_noise = 0 (the paper's initialisation): selection = top-k of the noise."""
    shape = _shape(1, T=512, n=256)
    say("case zero-init", shape)
    x, _, _, eps, _ = G.flat_inputs(shape)
    Z = np.zeros((shape.d, shape.n), np.float32)
    run = G.FlatRun(api, shape, x, Z, Z, eps, None, None, None)
    run.gate()
    torch.cuda.synchronize()
    fw = G.oracle_flat(shape, x, Z, Z, eps, None)
    assert np.array_equal(run.topk_idx.cpu().numpy(), fw.idx)
    assert np.all(run.sp.cpu().numpy() == np.float32(np.log(2.0)))


def test_route_extreme_imbalance_and_empty_experts(api):
    shape = _shape(1, T=777, n=300, k=4)
    say("case route-extremes", shape)
    rng = np.random.default_rng(5)
    x, W_g, W_noise, eps, _ = G.flat_inputs(shape)
    run = G.FlatRun(api, shape, x, W_g, W_noise, eps, None, None, None)
    # (a) every token picks experts 0..3 ; (b) zipf-skewed random picks with many empty experts
    idx_a = np.tile(np.arange(4, dtype=np.int32), (shape.T, 1))
    p = 1.0 / np.arange(1, 101) ** 1.5
    idx_b = np.stack([rng.choice(100, size=4, replace=False, p=p / p.sum()) for _ in range(shape.T)]).astype(np.int32) * 3
    for idx in (idx_a, idx_b):
        run.route(G.dev(idx))
        torch.cuda.synchronize()
        check_route(run, idx, shape.n)


def _ffn_case(api, shape, tol, name):
    say("case", name, shape)
    x, W_g, W_noise, eps, bias = G.flat_inputs(shape)
    fw = G.oracle_flat(shape, x, W_g, W_noise, eps, bias)
    W1, W2 = G.device_weights(shape)
    run = G.FlatRun(api, shape, x, W_g, W_noise, eps, bias, W1, W2)
    run.stages()
    check_gate(run, fw, shape)
    check_route(run, fw.idx, shape.n)
    wf = G.oracle_weight_fn(shape)
    y_ref = O.moe_output(x, fw.idx, fw.gates, wf, shape.n)
    # per-assignment expert outputs
    out = run.out_sorted.cpu().numpy()
    inv = run.inv_perm.cpu().numpy()
    for t in (0, shape.T // 2, shape.T - 1):
        for s in range(shape.k):
            e = int(fw.idx[t, s])
            ref = O.expert_ffn(x[t:t + 1], *wf(e))[0]
            row, mx = G.rel_errors(out[inv[t * shape.k + s]], ref)
            assert row <= tol, (t, s, row)
    row, mx = G.rel_errors(run.y.cpu().numpy(), y_ref)
    say("  y errors: row-rel %.3e  max-abs-rel %.3e" % (row, mx))
    assert row <= tol and mx <= tol
    check_losses(run, fw)
    # fused entry point gives the same bits as the stage-by-stage calls
    y_stage = run.y.clone()
    run.y.fill_(float("nan"))
    run.fused()
    assert torch.equal(run.y, y_stage)
    return run


def test_layer_cfg0_fp32(api):
    _ffn_case(api, W.CONFIGS[0], TOL_F32, "cfg0 full")


def test_layer_fp32_ragged_small_dims(api):
    _ffn_case(api, _shape(0, T=150, d=64, h=96, n=5, k=2), TOL_F32, "fp32 ragged small")


def test_layer_fp32_expert_shapes_off_the_tiles(api):
    """fp32 experts whose sizes do not divide the matrix-core kernel's 64 x 64 tile or its 32-deep
    slab: hidden sizes 20, 36 and 100 (tail columns, tail of k in the second product), d = 32, 96, 160."""
    _ffn_case(api, _shape(0, T=90, d=32, h=36, n=6, k=2), TOL_F32, "fp32 d=32 h=36")
    _ffn_case(api, _shape(0, T=201, d=96, h=100, n=9, k=3), TOL_F32, "fp32 d=96 h=100")
    _ffn_case(api, _shape(0, T=70, d=160, h=20, n=4, k=1), TOL_F32, "fp32 h=20")


def test_layer_bf16_small(api):
    _ffn_case(api, _shape(1, T=300, n=8, k=2), TOL_BF16, "bf16 T=300 n=8")


def test_layer_bf16_other_expert_shapes(api):
    """bf16 experts that are not 512 x 1024 take the plain path (gather, two grouped GEMMs)."""
    _ffn_case(api, _shape(1, T=400, d=256, h=512, n=12, k=2), TOL_BF16, "bf16 d=256 h=512")
    _ffn_case(api, _shape(1, T=300, d=512, h=2048, n=6, k=3), TOL_BF16, "bf16 d=512 h=2048")


def test_layer_bf16_one_token_per_expert_tail(api):
    _ffn_case(api, _shape(1, T=65, n=70, k=1), TOL_BF16, "bf16 tiny tiles")


def test_layer_bf16_sparse_skewed_batch(api):
    """A sparse batch (12 rows per expert on average) under a skewed gate: empty experts, single-row
    tiles, full tiles and experts with many tiles in one launch of the one-tile-per-expert kernel;
    every output row of every expert and y are compared."""
    shape = W.scaled_config(_shape(1, T=1500, n=512, k=4), zipf_beta=0.6)
    say("case bf16 sparse skewed batch", shape)
    x, W_g, W_noise, eps, bias = G.flat_inputs(shape, with_bias=True)
    fw = G.oracle_flat(shape, x, W_g, W_noise, eps, bias)
    W1, W2 = G.device_weights(shape)
    run = G.FlatRun(api, shape, x, W_g, W_noise, eps, bias, W1, W2)
    TM = api.moe_tile_rows(run.cfg)
    run.stages()
    check_gate(run, fw, shape)
    check_route(run, fw.idx, shape.n)
    counts, offsets, perm, _ = O.routing(fw.idx, shape.n)
    say("  rows per expert: max %d, empty %d, single-row %d, more than one tile %d"
        % (counts.max(), (counts == 0).sum(), (counts == 1).sum(), (counts > TM).sum()))
    assert (counts == 0).any() and (counts > TM).any() and (counts == 1).any() and (counts >= TM).any()
    wf = G.device_weight_fn(shape, W1, W2)
    out = run.out_sorted.cpu().numpy()
    worst = 0.0
    for e in np.nonzero(counts)[0]:
        r0, r1 = int(offsets[e]), int(offsets[e + 1])
        ref = O.expert_ffn(x[perm[r0:r1] // shape.k], *wf(e))
        worst = max(worst, G.rel_errors(out[r0:r1], ref)[0])
    say("  out_sorted, every row of every expert: worst row-rel %.3e" % worst)
    assert worst <= TOL_BF16
    y_ref = O.moe_output(x, fw.idx, fw.gates, wf, shape.n)
    row, mx = G.rel_errors(run.y.cpu().numpy(), y_ref)
    assert row <= TOL_BF16 and mx <= TOL_BF16
    y1 = run.y.clone()
    run.fused()
    assert torch.equal(run.y, y1)


def test_layer_cfg1_full(api):
    run = _ffn_case(api, W.CONFIGS[1], TOL_BF16, "cfg1 full")
    # determinism: a second fused run reproduces every bit
    y1 = run.y.clone()
    imp1 = run.importance.clone()
    run.fused()
    assert torch.equal(run.y, y1) and torch.equal(run.importance, imp1)


def test_error_paths(api):
    c = api.make_config(W.CONFIGS[0])
    t = torch.zeros(16, device="cuda")
    with pytest.raises(api.MoeError) as ei:
        api.moe_combine(c, None, t, t, t)
    assert ei.value.status == api.MOE_EINVAL
    bad = api.make_config(W.CONFIGS[0], k=17)
    with pytest.raises(api.MoeError):
        api.moe_combine(bad, t, t, t, t)


def test_degenerate_shapes(api):
    """n = 1, k = 1 (the layer is one MLP) and every token on the same experts (one expert with
    many row tiles, all others empty)."""
    _ffn_case(api, _shape(1, T=200, n=1, k=1), TOL_BF16, "bf16 single expert")
    shape = _shape(1, T=700, n=16, k=2)
    x, W_g, W_noise, eps, bias = G.flat_inputs(shape)
    W_g = np.zeros_like(W_g)
    W_g[:, 3] = 0.0
    big = np.zeros(shape.n, np.float32)
    big[3], big[11] = 50.0, 40.0                       # bias makes experts 3 and 11 win everywhere
    fw = G.oracle_flat(shape, x, W_g, W_noise, eps, big)
    assert set(np.unique(fw.idx)) == {3, 11}
    W1, W2 = G.device_weights(shape)
    run = G.FlatRun(api, shape, x, W_g, W_noise, eps, big, W1, W2)
    run.fused()
    assert np.array_equal(run.topk_idx.cpu().numpy(), fw.idx)
    y_ref = O.moe_output(x, fw.idx, fw.gates, G.oracle_weight_fn(shape), shape.n)
    row, mx = G.rel_errors(run.y.cpu().numpy(), y_ref)
    assert row <= TOL_BF16 and mx <= TOL_BF16
    check_losses(run, fw)


def test_empty_batch(api):
    """T = 0: every entry point accepts it and launches nothing that could fault."""
    shape = _shape(1, T=0, n=8, k=2)
    x = np.zeros((0, shape.d), np.float32)
    Wg = np.zeros((shape.d, shape.n), np.float32)
    eps = np.zeros((0, shape.n), np.float32)
    W1, W2 = G.device_weights(shape)
    run = G.FlatRun(api, shape, x, Wg, Wg, eps, None, W1, W2)
    run.fused()
    L = api.moe_get_workspace_layout(run.cfg)
    counts = run.workspace[L.counts:L.counts + 4 * shape.n].view(torch.int32).cpu().numpy()
    assert not counts.any()
    assert not run.losses.cpu().numpy().any() and not run.importance.cpu().numpy().any()


@pytest.mark.parametrize("which", ["cfg0_f32", "bf16_ragged"])
def test_combine_epilogue(api, which):
    """Appendix C: sigmoid, dropout and the residual connection fused into the combine."""
    say("combine epilogue", which)
    shape = W.CONFIGS[0] if which == "cfg0_f32" else _shape(1, T=300, n=8, k=2)
    tol = TOL_F32 if which == "cfg0_f32" else TOL_BF16
    x, W_g, W_noise, eps, bias = G.flat_inputs(shape)
    fw = G.oracle_flat(shape, x, W_g, W_noise, eps, bias)
    W1, W2 = G.device_weights(shape)
    run = G.FlatRun(api, shape, x, W_g, W_noise, eps, bias, W1, W2)
    run.stages()
    y_ref = O.moe_output(x, fw.idx, fw.gates, G.oracle_weight_fn(shape), shape.n)
    out = torch.full_like(run.y, float("nan"))
    for p, with_x in ((0.4, True), (0.1, False)):
        keep = W.dropout_keep(shape, p)
        assert 0 < keep.mean() < 1
        api.moe_combine_epilogue(run.cfg, run.out_sorted, run.topk_gate, run.inv_perm, run.x if with_x else None,
                                 G.dev(keep), p, out)
        torch.cuda.synchronize()
        ref = O.layer_epilogue(y_ref, x if with_x else np.zeros_like(x), keep.astype(bool), p)
        row, mx = G.rel_errors(out.cpu().numpy(), ref)
        say("  p=%.1f residual=%s: row-rel %.2e max-rel %.2e" % (p, with_x, row, mx))
        assert mx <= tol
        if with_x:
            assert row <= tol
        assert (out.cpu().numpy()[keep == 0] == (x[keep == 0] if with_x else 0)).all()   # dropped: only the residual
    api.moe_combine_epilogue(run.cfg, run.out_sorted, run.topk_gate, run.inv_perm, run.x, None, 0.0, out)
    torch.cuda.synchronize()
    row, mx = G.rel_errors(out.cpu().numpy(), O.layer_epilogue(y_ref, x, None, 0.0))
    assert row <= tol and mx <= tol
    with pytest.raises(api.MoeError):
        api.moe_combine_epilogue(run.cfg, run.out_sorted, run.topk_gate, run.inv_perm, run.x, None, 0.3, out)


def test_layer_forward_in_a_hip_graph(api):
    """The layer call allocates nothing, clears nothing with memset nodes and never synchronises, so
    it can be captured: three replays with fresh inputs copied into the captured buffers, with eager
    work in between, each equal to the eager call on the same inputs bit for bit."""
    shape = _shape(1, T=1024, n=64, k=4)
    say("hip graph", shape)
    x, W_g, W_noise, eps, bias = G.flat_inputs(shape, True)
    W1, W2 = G.device_weights(shape)
    cap = G.FlatRun(api, shape, x, W_g, W_noise, eps, bias, W1, W2)
    cap.fused()                                   # warm-up outside the capture (one-time function attributes)
    eager = G.FlatRun(api, shape, x, W_g, W_noise, eps, bias, W1, W2)
    ws = cap.workspace
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        api.moe_layer_forward(cap.cfg, cap.x, cap.W_g, cap.W_noise, cap.bias, cap.eps, cap.W1, cap.W2, cap.y,
                              cap.topk_idx, cap.topk_gate, cap.importance, cap.load, cap.losses, ws)
    rng = np.random.default_rng(5)
    for rep in range(3):
        xi = (x * np.float32(1.0 + 0.25 * rep) + rng.standard_normal(x.shape).astype(np.float32) * np.float32(0.1 * rep))
        cap.x.copy_(G.dev(xi))
        cap.y.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        eager.x.copy_(G.dev(xi))
        eager.fused()                             # the program's own eager work between replays
        assert torch.equal(cap.topk_idx, eager.topk_idx), rep
        assert torch.equal(cap.y, eager.y), rep
        assert torch.equal(cap.losses[:2], eager.losses[:2]), rep
        assert torch.equal(cap.importance, eager.importance) and torch.equal(cap.load, eager.load)
