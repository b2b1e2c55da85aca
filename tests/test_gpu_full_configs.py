"""Full-size runs of the workloads the oracle cannot finish whole: gating, routing and losses are
compared for every token (the oracle's gate is cheap); the expert outputs y are compared on a
sample of tokens the oracle evaluates one expert at a time."""
import sys
import time

import numpy as np
import pytest
import torch

import moe_workloads as W
from oracle import moe_oracle as O
from tests import gpu_harness as G

pytestmark = pytest.mark.gpu
TOL_F32, TOL_BF16 = 1e-5, 2e-2


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def api():
    assert torch.cuda.is_available()
    from paper_1701_06538_amd import api as _api
    return _api


def sample_tokens(T, count, seed):
    rng = np.random.default_rng(seed)
    s = rng.choice(T, size=count, replace=False)
    s[:3] = [0, T // 2, T - 1]
    return np.unique(s)


def timed(fn, reps=5):
    fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / reps * 1e3


def check_flat_full(api, shape, with_bias, nsample):
    say("full config", shape)
    x, W_g, W_noise, eps, bias = G.flat_inputs(shape, with_bias)
    t0 = time.perf_counter()
    fw = G.oracle_flat(shape, x, W_g, W_noise, eps, bias)
    say("  oracle gate+losses %.1f s" % (time.perf_counter() - t0))
    W1, W2 = G.device_weights(shape)
    run = G.FlatRun(api, shape, x, W_g, W_noise, eps, bias, W1, W2)
    run.fused()
    assert np.array_equal(run.topk_idx.cpu().numpy(), fw.idx), "top-k differs"
    assert np.abs(run.topk_gate.cpu().numpy().astype(np.float64) - fw.gates).max() <= TOL_F32
    counts, offsets, perm, inv = O.routing(fw.idx, shape.n)
    L = run.api.moe_get_workspace_layout(run.cfg)
    ws = run.workspace
    A = shape.T * shape.k
    view = lambda off, cnt: ws[off:off + 4 * cnt].view(torch.int32).cpu().numpy()
    assert np.array_equal(view(L.counts, shape.n), counts)
    assert np.array_equal(view(L.offsets, shape.n + 1), offsets)
    assert np.array_equal(view(L.perm, A), perm)
    assert np.array_equal(view(L.inv_perm, A), inv)
    say("  load max/mean %.2f, empty experts %d" % (counts.max() / counts.mean(), int((counts == 0).sum())))
    imp = run.importance.cpu().numpy().astype(np.float64)
    ld = run.load.cpu().numpy().astype(np.float64)
    assert np.abs(imp - fw.importance).max() <= TOL_F32 * np.abs(fw.importance).max()
    assert np.abs(ld - fw.load).max() <= TOL_F32 * np.abs(fw.load).max()
    Ls = run.losses.cpu().numpy().astype(np.float64)
    assert abs(Ls[0] - fw.loss_importance) <= TOL_F32 * abs(fw.loss_importance) + 1e-8
    assert abs(Ls[1] - fw.loss_load) <= TOL_F32 * abs(fw.loss_load) + 1e-8
    sub = sample_tokens(shape.T, nsample, shape.seed)
    t0 = time.perf_counter()
    y_ref = O.moe_output(x, fw.idx, fw.gates, G.oracle_weight_fn(shape), shape.n, token_subset=sub)
    say("  oracle y on %d sampled tokens %.1f s" % (len(sub), time.perf_counter() - t0))
    row, mx = G.rel_errors(run.y.cpu().numpy()[sub], y_ref)
    say("  y errors on the sample: row-rel %.3e max-abs-rel %.3e" % (row, mx))
    assert row <= TOL_BF16 and mx <= TOL_BF16
    assert torch.isfinite(run.y).all()
    ms = timed(run.fused)
    say("  moe_layer_forward %.3f ms -> %.2f M tokens/s" % (ms, shape.T / ms / 1e3))


def test_cfg2_full_flat_n2048(api):
    check_flat_full(api, W.CONFIGS[2], False, 24)


def test_cfg4_forward_full_skewed(api):
    check_flat_full(api, W.CONFIGS[4], True, 24)


def test_cfg3_full_hierarchical(api):
    shape = W.CONFIGS[3]
    say("full config", shape)
    inputs = W.hier_gate_inputs(shape)
    t0 = time.perf_counter()
    x, Wg_p, Wn_p, eps_p, Wg_s, Wn_s, eps_s = inputs
    hf = O.hier_gate_and_losses(x, Wg_p, Wn_p, eps_p, Wg_s, Wn_s, eps_s, shape.k_primary, shape.k_secondary,
                                shape.w_importance, shape.w_load)
    say("  oracle gates+losses %.1f s" % (time.perf_counter() - t0))
    t0 = time.perf_counter()
    W1, W2 = G.device_weights(shape, chunk=256)
    torch.cuda.synchronize()
    say("  34 GB of expert weights generated on the GPU in %.1f s" % (time.perf_counter() - t0))
    run = G.HierRun(api, shape, inputs, W1, W2)
    run.forward()
    assert np.array_equal(run.topk_idx.cpu().numpy(), hf.idx), "global expert ids differ"
    assert np.abs(run.topk_gate.cpu().numpy().astype(np.float64) - hf.gates).max() <= TOL_F32
    counts, offsets, perm, inv = O.routing(hf.idx, shape.n)
    A = shape.T * shape.k
    assert np.array_equal(run.ws_view("counts", shape.n, torch.int32).cpu().numpy(), counts)
    assert np.array_equal(run.ws_view("perm", A, torch.int32).cpu().numpy(), perm)
    say("  rows/expert mean %.1f max %d, empty experts %d" % (counts.mean(), counts.max(), int((counts == 0).sum())))
    imp = run.importance.cpu().numpy().astype(np.float64)
    ld = run.load.cpu().numpy().astype(np.float64)
    assert np.abs(imp - hf.importance).max() <= TOL_F32 * np.abs(hf.importance).max()
    assert np.abs(ld - hf.load).max() <= TOL_F32 * np.abs(hf.load).max()
    Ls = run.losses.cpu().numpy().astype(np.float64)
    assert abs(Ls[0] - hf.loss_importance) <= TOL_F32 * abs(hf.loss_importance) + 1e-8
    assert abs(Ls[1] - hf.loss_load) <= TOL_F32 * abs(hf.loss_load) + 1e-8
    sub = sample_tokens(shape.T, 24, shape.seed)
    y_ref = O.moe_output(x, hf.idx, hf.gates, G.oracle_weight_fn(shape), shape.n, token_subset=sub)
    row, mx = G.rel_errors(run.y.cpu().numpy()[sub], y_ref)
    say("  y errors on the sample: row-rel %.3e max-abs-rel %.3e" % (row, mx))
    assert row <= TOL_BF16 and mx <= TOL_BF16
    assert torch.isfinite(run.y).all()
    ms = timed(run.forward, reps=3)
    say("  moe_layer_forward_hier %.3f ms -> %.2f M tokens/s" % (ms, shape.T / ms / 1e3))
