"""Full-size runs of configs 2, 3 and 4 in the launch configuration the benchmark times: gating,
routing, losses AND the outputs y are compared with the oracle for every token, so every expert,
every row tile (first, last, longest, single-row) and every weight offset is covered.  The oracle
reads the expert matrices from the device tensors the input generator filled (tests/gpu_harness.py:
device_weight_fn; checked bit for bit against the host generator on a sample), which is what makes
a whole-batch binary64 evaluation of up to 16384 experts affordable.  Config 3's backward pass is
compared whole as well (dx row by row, both gate levels' gradients, 64 experts' dW1/dW2)."""
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


def timed(fn, reps=5):
    fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / reps * 1e3


def progress_every(step, what):
    def cb(e0):
        if e0 % step == 0:
            say("    %s: expert %d" % (what, e0))
    return cb


def sampled_experts(counts, count, seed):
    """Expert ids covering the special tile shapes: longest, shortest non-empty, first and last
    non-empty, some whose row count is a multiple of the 64-row tile or one off it, the rest random."""
    nz = np.nonzero(counts > 0)[0]
    picks = [int(np.argmax(counts)), int(nz[np.argmin(counts[nz])]), int(nz[0]), int(nz[-1])]
    for r in (1, 63, 64, 65, 127, 128, 129):
        hit = np.nonzero(counts == r)[0]
        picks += [int(e) for e in hit[:2]]
    rng = np.random.default_rng(seed)
    picks += [int(e) for e in rng.choice(nz, size=min(count, nz.size), replace=False)]
    out = []
    for e in picks:
        if e not in out:
            out.append(e)
    return out[:count]


def check_y_whole(y_gpu, y_ref, tol):
    row, mx = G.rel_errors(y_gpu, y_ref)
    say("  y, all %d tokens: worst row-rel %.3e, max-abs-rel %.3e" % (y_ref.shape[0], row, mx))
    assert row <= tol and mx <= tol


def check_flat_full(api, shape, with_bias):
    say("full config", shape)
    x, W_g, W_noise, eps, bias = G.flat_inputs(shape, with_bias)
    t0 = time.perf_counter()
    fw = G.oracle_flat(shape, x, W_g, W_noise, eps, bias)
    say("  oracle gate+losses %.1f s" % (time.perf_counter() - t0))
    W1, W2 = G.device_weights(shape)
    G.check_device_weights(shape, W1, W2, [0, shape.n // 2 + 1, shape.n - 1])
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
    t0 = time.perf_counter()
    wf = G.device_weight_fn(shape, W1, W2, block=32, progress=progress_every(512, "oracle y"))
    y_ref = O.moe_output(x, fw.idx, fw.gates, wf, shape.n)
    say("  oracle y on all %d tokens %.1f s" % (shape.T, time.perf_counter() - t0))
    check_y_whole(run.y.cpu().numpy(), y_ref, TOL_BF16)
    # the expert kernel's own output, whole experts: first/last/longest/single-row tiles
    out_sorted = ws[L.out_sorted:L.out_sorted + 4 * A * shape.d].view(torch.float32).view(A, shape.d)
    worst = 0.0
    picks = sampled_experts(counts, 64, shape.seed)
    for e in picks:
        r0, r1 = int(offsets[e]), int(offsets[e + 1])
        toks = perm[r0:r1] // shape.k
        ref = O.expert_ffn(x[toks], *wf(e))
        worst = max(worst, G.rel_errors(out_sorted[r0:r1].cpu().numpy(), ref)[0])
    say("  out_sorted, all rows of %d experts (rows %d..%d): worst row-rel %.3e"
        % (len(picks), counts[picks].min(), counts[picks].max(), worst))
    assert worst <= TOL_BF16
    ms = timed(run.fused)
    say("  moe_layer_forward %.3f ms -> %.2f M tokens/s" % (ms, shape.T / ms / 1e3))


def test_cfg2_full_flat_n2048(api):
    check_flat_full(api, W.CONFIGS[2], False)


def test_cfg4_forward_full_skewed(api):
    check_flat_full(api, W.CONFIGS[4], True)


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
    G.check_device_weights(shape, W1, W2, [0, 257, shape.n // 2 + 1, shape.n - 1])
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
    t0 = time.perf_counter()
    wf = G.device_weight_fn(shape, W1, W2, block=64, progress=progress_every(2048, "oracle y"))
    y_ref = O.moe_output(x, hf.idx, hf.gates, wf, shape.n)
    say("  oracle y on all %d tokens %.1f s" % (shape.T, time.perf_counter() - t0))
    check_y_whole(run.y.cpu().numpy(), y_ref, TOL_BF16)
    del y_ref
    ms = timed(run.forward, reps=3)
    say("  moe_layer_forward_hier %.3f ms -> %.2f M tokens/s" % (ms, shape.T / ms / 1e3))

    # backward at full size (69 GB of fp32 weight gradients), compared whole: dx row by row, both
    # gate levels' gradients, the weight gradients of 64 sampled experts; experts and groups nobody
    # reached must get zeros
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
    sample = sampled_experts(counts, 62, shape.seed) + [int(e) for e in np.nonzero(counts == 0)[0][:2]]
    t0 = time.perf_counter()
    xb = O.round_to_bf16(x)
    wf = G.device_weight_fn(shape, W1, W2, block=64, progress=progress_every(2048, "oracle backward"))
    gr = O.hier_backward(x, Wg_p, Wn_p, eps_p, Wg_s, Wn_s, eps_s, shape.k_primary, shape.k_secondary, wf, dy,
                         shape.w_importance, shape.w_load, experts_for_dW=sample, expert_input=xb)
    say("  oracle backward on all %d tokens %.1f s" % (T, time.perf_counter() - t0))
    hidden = run.ws_view("hidden", A * h, torch.bfloat16).view(A, h)
    wf1 = G.device_weight_fn(shape, W1, W2)
    dx_fro, dx_explained, worst_z = G.check_dx_rows(
        out["dx"].cpu().numpy(), gr.dx, xb, dy, hf.idx, hf.gates, wf1,
        lambda t, s: hidden[int(inv[t * shape.k + s])].float().cpu().numpy(), TOL_BF16)
    say("  dx: Frobenius rel %.2e; rows over %.0e explained by hidden units on the ReLU kink: %d of %d "
        "(largest |z| of such a unit %.1e)" % (dx_fro, TOL_BF16, dx_explained, T, worst_z))
    assert dx_explained <= 1e-3 * T
    errs = dict(dx=dx_fro)
    for q in ("dWg_p", "dWn_p"):
        errs[q] = G.fro_rel(out[q].cpu().numpy(), getattr(gr, q))
    for q in ("dWg_s", "dWn_s"):
        got = out[q].cpu().numpy()
        ref = getattr(gr, q)
        errs[q] = max(G.fro_rel(got[i], ref[i]) for i in range(a) if hf.group_counts[i] > 0)
        for i in range(a):
            if hf.group_counts[i] == 0:
                assert not got[i].any(), "a group no token chose must get zero gradients"
    worst = 0.0
    for e in sorted(set(sample)):
        g1, g2 = out["dW1"][e].cpu().numpy(), out["dW2"][e].cpu().numpy()
        if e in gr.dW1:
            worst = max(worst, G.fro_rel(g1, gr.dW1[e]), G.fro_rel(g2, gr.dW2[e]))
        else:
            assert counts[e] == 0 and not g1.any() and not g2.any()
    errs["dW1/dW2 of %d experts" % len(set(sample))] = worst
    say("  backward relative errors:", {k_: "%.2e" % v for k_, v in errs.items()})
    for k_, v in errs.items():
        assert v <= TOL_BF16, (k_, v)
    used = torch.from_numpy(counts > 0).cuda()
    assert not out["dW1"][~used].any() and not out["dW2"][~used].any(), "experts without tokens must get zero gradients"
    for k_, v in out.items():
        assert torch.isfinite(v).all(), k_
    ms_b = timed(backward, reps=2)
    say("  moe_layer_backward_hier %.3f ms" % ms_b)
