"""GPU parity of the backward pass (flat layer, bf16 experts) against the oracle's gradients, which
are themselves pinned by finite differences on the CPU."""
import sys
import time

import numpy as np
import pytest
import torch

import moe_workloads as W
from oracle import moe_oracle as O
from tests import gpu_harness as G

pytestmark = pytest.mark.gpu
TOL_BF16 = 2e-2


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def api():
    assert torch.cuda.is_available()
    from paper_1701_06538_amd import api as _api
    return _api


def fro_rel(got, ref):
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    return float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300))


def run_backward(api, shape, with_bias, dy, w_override=None, flags=0, inputs=None):
    if w_override is not None:
        shape = W.scaled_config(shape, w_importance=w_override[0], w_load=w_override[1])
    x, W_g, W_noise, eps, bias = G.flat_inputs(shape, with_bias) if inputs is None else inputs
    W1, W2 = G.device_weights(shape)
    run = G.FlatRun(api, shape, x, W_g, W_noise, eps, bias, W1, W2, flags=flags)
    run.fused()
    f32 = dict(dtype=torch.float32, device="cuda")
    T, d, h, n = shape.T, shape.d, shape.h, shape.n
    out = dict(dx=torch.full((T, d), float("nan"), **f32), dW_g=torch.full((d, n), float("nan"), **f32),
               dW_noise=torch.full((d, n), float("nan"), **f32), dW1=torch.full((n, d, h), float("nan"), **f32),
               dW2=torch.full((n, h, d), float("nan"), **f32))
    bws = torch.empty(max(256, api.moe_backward_workspace_bytes(run.cfg)), dtype=torch.uint8, device="cuda")
    dyd = G.dev(dy)

    def call():
        api.moe_layer_backward(run.cfg, run.x, run.W_g, run.W_noise, run.eps, run.W1, run.W2, dyd,
                               run.topk_idx, run.topk_gate, run.workspace, out["dx"], out["dW_g"],
                               out["dW_noise"], out["dW1"], out["dW2"], bws)
        torch.cuda.synchronize()
    call()
    return shape, (x, W_g, W_noise, eps, bias), run, out, call


def oracle_backward(shape, inputs, dy, experts_for_dW=None, weight_fn=None):
    x, W_g, W_noise, eps, bias = inputs
    fw = G.oracle_flat(shape, x, W_g, W_noise, eps, bias)
    # bf16 workloads: the experts' input activations are bf16(x) (the ReLU mask is decided on them)
    gr = O.flat_backward(x, W_g, W_noise, fw, shape.k, weight_fn or G.oracle_weight_fn(shape), dy, shape.w_importance,
                         shape.w_load, experts_for_dW=experts_for_dW,
                         expert_input=O.round_to_bf16(x) if shape.expert_dtype == "bf16" else None)
    return fw, gr


CASES = [
    ("small", dict(T=512, n=32), False, 0),
    ("ragged_bias", dict(T=777, n=64, k=3), True, 0),
    ("k1", dict(T=300, n=32, k=1), False, 0),
    ("saved_hidden", dict(T=777, n=64, k=3), True, 1),      # MOE_FLAG_SAVE_HIDDEN: no recomputation
    ("cfg1_shape", dict(T=2048, n=256), False, 0),           # the other flat workloads' expert counts
    ("cfg2_shape", dict(T=800, n=2048), False, 1),          # (few rows per expert, many empty experts)
    ("d256_h512", dict(T=600, n=32, d=256, h=512), False, 0),  # experts off the fused kernel's shape
    ("d256_h512_saved", dict(T=600, n=32, d=256, h=512), False, 1),  # kept hidden and input rows on the unfused path
    ("n20_bf16", dict(T=400, n=20, k=3), False, 0),            # expert count off the tile sizes
    ("n640_small_experts", dict(T=900, n=640, k=2, d=256, h=256), True, 0),   # 512 < n <= 1024: four column groups per lane in the gate kernel
    # fp32 experts: every GEMM on the fp32 matrix cores
    ("cfg0_f32", dict(T=256, n=16, k=4, expert_dtype="f32"), False, 0),
    ("f32_ragged", dict(T=150, d=64, h=96, n=8, k=2, expert_dtype="f32"), True, 0),
    ("n4096_f32", dict(T=96, d=64, h=64, n=4096, k=2, expert_dtype="f32"), False, 0),   # a flat gate wider than 2048 experts
]
TOL_F32_EXPERTS = 1e-5


@pytest.mark.parametrize("name,ov,with_bias,flags", CASES, ids=[c[0] for c in CASES])
def test_backward_parity(api, name, ov, with_bias, flags):
    shape = W.scaled_config(W.CONFIGS[4], **ov)
    if with_bias:
        shape = W.scaled_config(shape, zipf_beta=0.5)
    say("case backward", name, shape)
    dy = W.upstream_grad(shape)
    shape, inputs, run, out, call = run_backward(api, shape, with_bias, dy, flags=flags)
    fw, gr = oracle_backward(shape, inputs, dy, weight_fn=G.weight_fn_for(shape, run.W1, run.W2))
    assert np.array_equal(run.topk_idx.cpu().numpy(), fw.idx)
    errs = dict(dx=G.rel_errors(out["dx"].cpu().numpy(), gr.dx)[0],
                dW_g=fro_rel(out["dW_g"].cpu().numpy(), gr.dW_g),
                dW_noise=fro_rel(out["dW_noise"].cpu().numpy(), gr.dW_noise))
    dW1 = out["dW1"].cpu().numpy()
    dW2 = out["dW2"].cpu().numpy()
    worst1 = worst2 = 0.0
    for e in range(shape.n):
        if e in gr.dW1:
            worst1 = max(worst1, fro_rel(dW1[e], gr.dW1[e]))
            worst2 = max(worst2, fro_rel(dW2[e], gr.dW2[e]))
        else:
            assert not dW1[e].any() and not dW2[e].any(), "expert without tokens must get zero gradients"
    errs["dW1"], errs["dW2"] = worst1, worst2
    say("  relative errors:", {k: "%.2e" % v for k, v in errs.items()})
    tol = TOL_BF16 if shape.expert_dtype == "bf16" else TOL_F32_EXPERTS
    for k, v in errs.items():
        assert v <= tol, (k, v)
    # bit-reproducible
    keep = {k: v.clone() for k, v in out.items()}
    call()
    for k in keep:
        assert torch.equal(keep[k], out[k]), k


def test_gate_gradients_alone_are_fp32_accurate(api):
    """dy = 0 leaves J = L_importance + L_load: every gradient then comes from the fp32 gate path."""
    shape = W.scaled_config(W.CONFIGS[4], T=1024, n=64)
    say("case backward losses-only", shape)
    dy = np.zeros((shape.T, shape.d), np.float32)
    shape, inputs, run, out, call = run_backward(api, shape, False, dy)
    fw, gr = oracle_backward(shape, inputs, dy)
    e = dict(dx=fro_rel(out["dx"].cpu().numpy(), gr.dx), dW_g=fro_rel(out["dW_g"].cpu().numpy(), gr.dW_g),
             dW_noise=fro_rel(out["dW_noise"].cpu().numpy(), gr.dW_noise))
    say("  relative errors:", {k: "%.2e" % v for k, v in e.items()})
    for k, v in e.items():
        assert v <= 1e-5, (k, v)
    assert not out["dW1"].any() and not out["dW2"].any()


def test_backward_with_tiny_noise_scale(api):
    """Experts whose noise logit sits near -12 or -20: Softplus(raw) ~ e^raw is 6e-6 or 2e-9 and its
    derivative, the sigmoid, is as small.  Every expert's column of dW_noise is compared on its own,
    so the columns whose values are tiny are not hidden behind the ordinary ones."""
    shape = W.scaled_config(W.CONFIGS[4], T=384, n=16, k=2, d=64, h=96, expert_dtype="f32")
    say("case backward tiny noise scale", shape)
    x, W_g, W_noise, eps, bias = G.flat_inputs(shape, False)
    x[:, 0] = 10.0
    shift = np.zeros(shape.n, np.float32)
    shift[1::3], shift[2::3] = -1.2, -2.0            # raw = 10 * shift + N(0, ~0.16)
    W_noise[0, :] = shift
    dy = W.upstream_grad(shape)
    shape, inputs, run, out, call = run_backward(api, shape, False, dy, inputs=(x, W_g, W_noise, eps, bias))
    fw, gr = oracle_backward(shape, inputs, dy)
    assert np.array_equal(run.topk_idx.cpu().numpy(), fw.idx)
    sp = fw.logits.sp
    say("  Softplus range per class: %.1e .. %.1e" % (sp.min(), sp.max()))
    assert sp.min() < 1e-8 and sp.max() > 0.3
    got = out["dW_noise"].cpu().numpy().astype(np.float64)
    col = np.linalg.norm(got - gr.dW_noise, axis=0) / np.maximum(np.linalg.norm(gr.dW_noise, axis=0), 1e-300)
    say("  per-expert relative error of dW_noise: max %.2e (tiny-scale experts %.2e)" % (col.max(), col[shift < 0].max()))
    assert (np.linalg.norm(gr.dW_noise, axis=0) > 0).all()
    assert col.max() <= 1e-5
    assert fro_rel(out["dW_g"].cpu().numpy(), gr.dW_g) <= 1e-5
    assert G.rel_errors(out["dx"].cpu().numpy(), gr.dx)[0] <= 1e-5


def test_backward_empty_batch(api):
    """T = 0: no token reaches any expert, so every gradient is written as zero."""
    shape = W.scaled_config(W.CONFIGS[4], T=0, n=8, k=2, d=256, h=256)
    say("case backward empty batch")
    dy = np.zeros((0, shape.d), np.float32)
    shape, inputs, run, out, call = run_backward(api, shape, False, dy)
    for q in ("dW_g", "dW_noise", "dW1", "dW2"):
        assert not out[q].any() and torch.isfinite(out[q]).all(), q


def test_backward_without_losses(api):
    shape = W.scaled_config(W.CONFIGS[4], T=512, n=32)
    dy = W.upstream_grad(shape)
    shape, inputs, run, out, call = run_backward(api, shape, False, dy, w_override=(0.0, 0.0))
    fw, gr = oracle_backward(shape, inputs, dy)
    for name, ref in (("dx", gr.dx), ("dW_g", gr.dW_g), ("dW_noise", gr.dW_noise)):
        assert fro_rel(out[name].cpu().numpy(), ref) <= TOL_BF16, name


def test_cfg4_full_training_step(api):
    """Config 4 at full size: T=65536, n=512, Zipf-skewed loads, forward + backward, every gradient
    compared whole: dx row by row, dW_g and dW_noise, dW1 and dW2 of all 512 experts."""
    shape = W.CONFIGS[4]
    say("full config", shape)
    dy = W.upstream_grad(shape)
    shape, inputs, run, out, call = run_backward(api, shape, True, dy, flags=api.MOE_FLAG_SAVE_HIDDEN)
    G.check_device_weights(shape, run.W1, run.W2, [0, 255, shape.n - 1])
    t0 = time.perf_counter()
    counts = np.bincount(run.topk_idx.cpu().numpy().reshape(-1), minlength=shape.n)
    wf = G.device_weight_fn(shape, run.W1, run.W2, block=16)
    fw, gr = oracle_backward(shape, inputs, dy, weight_fn=wf)
    say("  oracle forward+backward %.1f s; load max/mean %.1f" % (time.perf_counter() - t0, counts.max() / counts.mean()))
    assert np.array_equal(run.topk_idx.cpu().numpy(), fw.idx)
    L = api.moe_get_workspace_layout(run.cfg)
    A, h = shape.T * shape.k, shape.h
    hidden = run.workspace[L.hidden:L.hidden + 2 * A * h].view(torch.bfloat16).view(A, h)
    inv = run.workspace[L.inv_perm:L.inv_perm + 4 * A].view(torch.int32).cpu().numpy()
    dx_fro, dx_explained, worst_z = G.check_dx_rows(
        out["dx"].cpu().numpy(), gr.dx, O.round_to_bf16(inputs[0]), dy, fw.idx, fw.gates,
        G.device_weight_fn(shape, run.W1, run.W2),
        lambda t, s: hidden[int(inv[t * shape.k + s])].float().cpu().numpy(), TOL_BF16)
    say("  dx: Frobenius rel %.2e; rows over %.0e explained by hidden units on the ReLU kink: %d of %d "
        "(largest |z| of such a unit %.1e)" % (dx_fro, TOL_BF16, dx_explained, shape.T, worst_z))
    assert dx_explained <= 1e-3 * shape.T
    errs = dict(dx=dx_fro,
                dW_g=fro_rel(out["dW_g"].cpu().numpy(), gr.dW_g),
                dW_noise=fro_rel(out["dW_noise"].cpu().numpy(), gr.dW_noise))
    w1 = w2 = 0.0
    for e in range(shape.n):
        g1, g2 = out["dW1"][e].cpu().numpy(), out["dW2"][e].cpu().numpy()
        if e in gr.dW1:
            w1, w2 = max(w1, fro_rel(g1, gr.dW1[e])), max(w2, fro_rel(g2, gr.dW2[e]))
        else:
            assert not g1.any() and not g2.any()
    errs["dW1 (worst of %d experts)" % len(gr.dW1)], errs["dW2 (worst)"] = w1, w2
    say("  relative errors:", {k: "%.2e" % v for k, v in errs.items()})
    for k, v in errs.items():
        assert v <= TOL_BF16, (k, v)
    assert torch.isfinite(out["dW1"]).all() and torch.isfinite(out["dW2"]).all()

    def step():
        run.api.moe_layer_forward(run.cfg, run.x, run.W_g, run.W_noise, run.bias, run.eps, run.W1, run.W2,
                                  run.y, run.topk_idx, run.topk_gate, run.importance, run.load, run.losses,
                                  run.workspace)
        call()
    step()
    t0 = time.perf_counter()
    for _ in range(3):
        step()
    ms = (time.perf_counter() - t0) / 3 * 1e3
    say("  forward+backward step %.3f ms -> %.2f M tokens/s" % (ms, shape.T / ms / 1e3))


def test_side_streams_give_the_same_results(api):
    """Every kernel goes to the caller's stream: forward + backward issued on two non-blocking side
    streams at once (own buffers and workspaces each, no synchronisation in between) reproduce the
    default-stream results bit for bit."""
    shape = W.scaled_config(W.CONFIGS[4], T=1024, n=64, k=3, zipf_beta=0.5)
    say("side streams", shape)
    dy = W.upstream_grad(shape)
    _, inputs, run0, out0, _ = run_backward(api, shape, True, dy, flags=api.MOE_FLAG_SAVE_HIDDEN)
    x, W_g, W_noise, eps, bias = inputs
    f32 = dict(dtype=torch.float32, device="cuda")
    T, d, h, n = shape.T, shape.d, shape.h, shape.n
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    held = []
    for s in streams:
        with torch.cuda.stream(s):
            W1, W2 = G.device_weights(shape)
            run = G.FlatRun(api, shape, x, W_g, W_noise, eps, bias, W1, W2, flags=api.MOE_FLAG_SAVE_HIDDEN)
            ws = torch.empty(api.moe_workspace_bytes(run.cfg), dtype=torch.uint8, device="cuda")
            out = dict(dx=torch.empty((T, d), **f32), dW_g=torch.empty((d, n), **f32), dW_noise=torch.empty((d, n), **f32),
                       dW1=torch.empty((n, d, h), **f32), dW2=torch.empty((n, h, d), **f32))
            bws = torch.empty(api.moe_backward_workspace_bytes(run.cfg), dtype=torch.uint8, device="cuda")
            dyd = G.dev(dy)
            api.moe_layer_forward(run.cfg, run.x, run.W_g, run.W_noise, run.bias, run.eps, run.W1, run.W2, run.y,
                                  run.topk_idx, run.topk_gate, run.importance, run.load, run.losses, ws)
            api.moe_layer_backward(run.cfg, run.x, run.W_g, run.W_noise, run.eps, run.W1, run.W2, dyd, run.topk_idx,
                                   run.topk_gate, ws, out["dx"], out["dW_g"], out["dW_noise"], out["dW1"],
                                   out["dW2"], bws)
            held.append((run, out, ws, bws, dyd, W1, W2))
    for s in streams:
        s.synchronize()
    torch.cuda.synchronize()
    for run, out, *_ in held:
        assert torch.equal(run.y, run0.y) and torch.equal(run.topk_idx, run0.topk_idx)
        assert torch.equal(run.losses[:2], run0.losses[:2])
        for q in out0:
            assert torch.equal(out[q], out0[q]), q
