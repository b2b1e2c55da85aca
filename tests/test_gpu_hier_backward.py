"""GPU parity of the hierarchical layer's backward pass (Appendix B, Eq.(12)-(14)) against the
oracle's gradients, which are pinned by finite differences on the CPU."""
import sys

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


def run_hier_backward(api, shape, dy, gate_std=0.02, flags=0):
    inputs = W.hier_gate_inputs(shape, gate_std)
    W1, W2 = G.device_weights(shape, chunk=256)
    run = G.HierRun(api, shape, inputs, W1, W2, flags=flags)
    run.forward()
    T, d, h, n, a, b = shape.T, shape.d, shape.h, shape.n, shape.a, shape.b
    f32 = dict(dtype=torch.float32, device="cuda")
    nan = float("nan")
    out = dict(dx=torch.full((T, d), nan, **f32), dWg_p=torch.full((d, a), nan, **f32),
               dWn_p=torch.full((d, a), nan, **f32), dWg_s=torch.full((a, d, b), nan, **f32),
               dWn_s=torch.full((a, d, b), nan, **f32), dW1=torch.full((n, d, h), nan, **f32),
               dW2=torch.full((n, h, d), nan, **f32))
    bws = torch.empty(api.moe_backward_hier_workspace_bytes(run.cfg), dtype=torch.uint8, device="cuda")
    dyd = G.dev(dy)

    def call():
        api.moe_layer_backward_hier(run.cfg, run.x, run.Wg_p, run.Wn_p, run.eps_p, run.Wg_s, run.Wn_s, run.eps_s,
                                    run.W1, run.W2, dyd, run.topk_idx, run.topk_gate, run.workspace, out["dx"],
                                    out["dWg_p"], out["dWn_p"], out["dWg_s"], out["dWn_s"], out["dW1"],
                                    out["dW2"], bws)
        torch.cuda.synchronize()
    call()
    return inputs, run, out, call


def oracle_hier_backward(shape, inputs, dy, experts_for_dW=None, weight_fn=None):
    x, Wg_p, Wn_p, eps_p, Wg_s, Wn_s, eps_s = inputs
    return O.hier_backward(x, Wg_p, Wn_p, eps_p, Wg_s, Wn_s, eps_s, shape.k_primary, shape.k_secondary,
                           weight_fn or G.oracle_weight_fn(shape), dy, shape.w_importance, shape.w_load,
                           experts_for_dW=experts_for_dW, expert_input=O.round_to_bf16(x))


CASES = [
    # name, overrides, gate std, loss weights or None.  Most cases use 256 x 256 experts: the oracle
    # generates every used expert's weights, and both gating levels need at least 32 x 32 = 1024 experts.
    ("small", dict(T=512, a=32, b=32, d=256, h=256), 0.02, None),
    ("saved_hidden", dict(T=512, a=32, b=32, d=256, h=256, flags=1), 0.02, None),   # MOE_FLAG_SAVE_HIDDEN
    ("ragged_empty_groups", dict(T=333, a=64, b=32, k_primary=1, k_secondary=3, d=256, h=512), 0.05, None),
    ("losses_off", dict(T=400, a=32, b=32, d=256, h=256), 0.02, (0.0, 0.0)),
    ("paper_expert", dict(T=96, a=32, b=32), 0.02, None),
    ("medium", dict(T=4096, a=32, b=64, d=256, h=256), 0.02, None),
]


@pytest.mark.parametrize("name,ov,std,wl", CASES, ids=[c[0] for c in CASES])
def test_hier_backward_parity(api, name, ov, std, wl):
    ov = dict(ov)
    flags = ov.pop("flags", 0)
    ov["n"] = ov["a"] * ov["b"]
    kp, ks = ov.get("k_primary", 2), ov.get("k_secondary", 2)
    ov["k"] = kp * ks
    if wl is not None:
        ov["w_importance"], ov["w_load"] = wl
    shape = W.scaled_config(W.CONFIGS[3], **ov)
    say("case hier backward", name, shape)
    dy = W.upstream_grad(shape)
    inputs, run, out, call = run_hier_backward(api, shape, dy, std, flags)
    hf = O.hier_gate_and_losses(*inputs, shape.k_primary, shape.k_secondary, shape.w_importance, shape.w_load)
    assert np.array_equal(run.topk_idx.cpu().numpy(), hf.idx)
    gr = oracle_hier_backward(shape, inputs, dy, weight_fn=G.weight_fn_for(shape, run.W1, run.W2, many=2048))
    errs = dict(dx=G.rel_errors(out["dx"].cpu().numpy(), gr.dx)[0],
                dWg_p=fro_rel(out["dWg_p"].cpu().numpy(), gr.dWg_p),
                dWn_p=fro_rel(out["dWn_p"].cpu().numpy(), gr.dWn_p),
                dWg_s=fro_rel(out["dWg_s"].cpu().numpy(), gr.dWg_s),
                dWn_s=fro_rel(out["dWn_s"].cpu().numpy(), gr.dWn_s))
    dWg_s = out["dWg_s"].cpu().numpy()
    for i in range(shape.a):
        if hf.group_counts[i] == 0:
            assert not dWg_s[i].any(), "a group no token chose must get zero gradients"
    # experts nobody reached: checked on the device; the others are fetched one by one
    used = torch.zeros(shape.n, dtype=torch.bool, device="cuda")
    used[torch.tensor(sorted(gr.dW1), device="cuda")] = True
    assert not out["dW1"][~used].any() and not out["dW2"][~used].any()
    worst1 = worst2 = 0.0
    for e in gr.dW1:
        worst1 = max(worst1, fro_rel(out["dW1"][e].cpu().numpy(), gr.dW1[e]))
        worst2 = max(worst2, fro_rel(out["dW2"][e].cpu().numpy(), gr.dW2[e]))
    errs["dW1"], errs["dW2"] = worst1, worst2
    say("  relative errors:", {k: "%.2e" % v for k, v in errs.items()})
    for k, v in errs.items():
        assert v <= TOL_BF16, (k, v)
    keep = {k: v.clone() for k, v in out.items() if k not in ("dW1", "dW2")}
    sums = (out["dW1"].sum(dtype=torch.float64).item(), out["dW2"].sum(dtype=torch.float64).item())
    call()
    for k in keep:
        assert torch.equal(keep[k], out[k]), k
    assert sums == (out["dW1"].sum(dtype=torch.float64).item(), out["dW2"].sum(dtype=torch.float64).item())


def test_hier_gate_gradients_alone_are_fp32_accurate(api):
    """dy = 0 leaves J = L_importance + L_load: every gradient then comes from the fp32 gate path
    through Eq.(13) and Eq.(14)."""
    shape = W.scaled_config(W.CONFIGS[3], T=1024, a=32, b=32, n=1024, d=256, h=256)
    say("case hier backward losses-only", shape)
    dy = np.zeros((shape.T, shape.d), np.float32)
    inputs, run, out, call = run_hier_backward(api, shape, dy)
    gr = oracle_hier_backward(shape, inputs, dy)
    e = {k: fro_rel(out[k].cpu().numpy(), getattr(gr, k)) for k in ("dx", "dWg_p", "dWn_p", "dWg_s", "dWn_s")}
    say("  relative errors:", {k: "%.2e" % v for k, v in e.items()})
    for k, v in e.items():
        assert v <= 1e-5, (k, v)
    assert not out["dW1"].any() and not out["dW2"].any()
