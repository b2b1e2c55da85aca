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
    run = G.HierRun(api, shape, inputs, W1, W2, flags=api.MOE_FLAG_SAVE_HIDDEN)
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

    # backward at full size (69 GB of fp32 weight gradients): the weight gradients of sampled
    # experts against the oracle, properties for everything else (the whole backward is compared
    # with the oracle at smaller sizes in test_gpu_hier_backward.py)
    dy = W.upstream_grad(shape)
    f32 = dict(dtype=torch.float32, device="cuda")
    T, d, h, n, a, b = shape.T, shape.d, shape.h, shape.n, shape.a, shape.b
    out = dict(dx=torch.empty((T, d), **f32), dWg_p=torch.empty((d, a), **f32), dWn_p=torch.empty((d, a), **f32),
               dWg_s=torch.empty((a, d, b), **f32), dWn_s=torch.empty((a, d, b), **f32),
               dW1=torch.empty((n, d, h), **f32), dW2=torch.empty((n, h, d), **f32))
    bws = torch.empty(api.moe_backward_hier_workspace_bytes(run.cfg), dtype=torch.uint8, device="cuda")
    dyd = G.dev(dy)

    def backward():
        api.moe_layer_backward_hier(run.cfg, run.x, run.Wg_p, run.Wn_p, run.eps_p, run.Wg_s, run.Wn_s, run.eps_s,
                                    run.W1, run.W2, dyd, run.topk_idx, run.topk_gate, run.workspace, out["dx"],
                                    out["dWg_p"], out["dWn_p"], out["dWg_s"], out["dWn_s"], out["dW1"],
                                    out["dW2"], bws)
    backward()
    torch.cuda.synchronize()
    sample = [int(np.argmax(counts)), 0, 1, b - 1, b, n // 2 + 3, n - 1] + [int(e) for e in np.nonzero(counts == 0)[0][:2]]
    _, _, dW1s, dW2s = O.experts_backward(O.round_to_bf16(x), hf.idx, hf.gates, G.oracle_weight_fn(shape), dy,
                                          only=sample)
    worst = 0.0
    for e in sorted(set(sample)):
        g1, g2 = out["dW1"][e].cpu().numpy(), out["dW2"][e].cpu().numpy()
        if e in dW1s:
            for got, ref in ((g1, dW1s[e]), (g2, dW2s[e])):
                rel = float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300))
                worst = max(worst, rel)
        else:
            assert counts[e] == 0 and not g1.any() and not g2.any()
    say("  backward: worst relative error of the sampled experts' dW1/dW2 %.2e" % worst)
    assert worst <= TOL_BF16
    used = torch.from_numpy(counts > 0).cuda()
    assert not out["dW1"][~used].any() and not out["dW2"][~used].any(), "experts without tokens must get zero gradients"
    for k_, v in out.items():
        assert torch.isfinite(v).all(), k_
    groups_used = torch.from_numpy(hf.group_counts > 0).cuda()
    assert not out["dWg_s"][~groups_used].any()
    assert out["dx"].abs().max() > 0 and out["dWg_p"].abs().max() > 0
    ms_b = timed(backward, reps=2)
    say("  moe_layer_backward_hier %.3f ms" % ms_b)
