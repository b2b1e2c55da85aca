"""GPU parity of the factored-second-moment Adam step for the expert matrices (Appendix D) against
the oracle: parameters, both state vectors and the refreshed bf16 copy over several steps."""
import sys

import numpy as np
import pytest
import torch

import moe_workloads as W
from oracle import moe_oracle as O

pytestmark = pytest.mark.gpu
TOL = 1e-5


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def api():
    assert torch.cuda.is_available()
    from paper_1701_06538_amd import api as _api
    return _api


CASES = {
    # name: (n, d, h, dtype, steps)
    "tiny_f32": (3, 64, 96, "f32", 3),
    "ragged_f32": (2, 96, 132, "f32", 2),
    "paper_expert_bf16": (4, 512, 1024, "bf16", 3),
    "wide_rows_bf16": (2, 128, 2048, "bf16", 2),
    "very_wide_rows_f32": (1, 32, 4160, "f32", 2),
}


def rel(got, ref):
    return float(np.abs(np.asarray(got, np.float64) - ref).max() / max(np.abs(ref).max(), 1e-300))


@pytest.mark.parametrize("name", list(CASES))
def test_adam_step(api, name):
    n, d, h, dtype, steps = CASES[name]
    say("adam", name)
    shape = W.scaled_config(W.CONFIGS[1], T=64, n=n, k=1, d=d, h=h, expert_dtype=dtype)
    cfg = api.make_config(shape)
    rng = np.random.default_rng(11)
    lr, beta2, eps = 1e-2, 0.95, 1e-8
    Wm = [rng.standard_normal((n, d, h)).astype(np.float32) * 0.05, rng.standard_normal((n, h, d)).astype(np.float32) * 0.05]
    ref_W = [w.astype(np.float64) for w in Wm]
    ref_vr = [np.zeros((n, d)), np.zeros((n, h))]
    ref_vc = [np.zeros((n, h)), np.zeros((n, d))]
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    g_W = [dev(w) for w in Wm]
    g_vr = [torch.zeros((n, d), device="cuda"), torch.zeros((n, h), device="cuda")]
    g_vc = [torch.zeros((n, h), device="cuda"), torch.zeros((n, d), device="cuda")]
    copies = [None, None]
    if dtype == "bf16":
        copies = [torch.zeros((n, d, h), dtype=torch.bfloat16, device="cuda"),
                  torch.zeros((n, h, d), dtype=torch.bfloat16, device="cuda")]
    ws = torch.empty(max(256, api.moe_adam_workspace_bytes(cfg)), dtype=torch.uint8, device="cuda")
    for step in range(1, steps + 1):
        # gradients with a row and column structure, one expert without any gradient at step 1
        G = [rng.standard_normal(w.shape).astype(np.float32) * rng.random((n, w.shape[1], 1)).astype(np.float32)
             * rng.random((n, 1, w.shape[2])).astype(np.float32) for w in Wm]
        if step == 1:
            G[0][n - 1] = 0.0
        api.moe_expert_adam_step(cfg, lr, beta2, eps, step, dev(G[0]), dev(G[1]), g_W[0], g_W[1], copies[0],
                                 copies[1], g_vr[0], g_vc[0], g_vr[1], g_vc[1], ws)
        torch.cuda.synchronize()
        for w in range(2):
            for e in range(n):
                ref_W[w][e], ref_vr[w][e], ref_vc[w][e] = O.factored_adam_step(
                    ref_W[w][e], G[w][e], ref_vr[w][e], ref_vc[w][e], lr, beta2, eps, step)
            got = g_W[w].cpu().numpy()
            assert rel(got, ref_W[w]) <= TOL, (step, w, rel(got, ref_W[w]))
            assert rel(g_vr[w].cpu().numpy(), ref_vr[w]) <= TOL
            assert rel(g_vc[w].cpu().numpy(), ref_vc[w]) <= TOL
            # the step itself, not hidden behind the size of W
            upd_ref = ref_W[w] - (Wm[w].astype(np.float64) if step == 1 else prev[w])
            upd_got = got.astype(np.float64) - (Wm[w].astype(np.float64) if step == 1 else prev[w])
            assert np.abs(upd_got - upd_ref).max() <= 1e-4 * np.abs(upd_ref).max() + 1e-9
            if copies[w] is not None:
                bits = copies[w].view(torch.int16).cpu().numpy().view(np.uint16)
                want = (O.round_to_bf16(got).view(np.uint32) >> 16).astype(np.uint16)
                assert np.array_equal(bits, want)
        if step == 1:
            assert np.array_equal(g_W[0].cpu().numpy()[n - 1], Wm[0][n - 1])      # no history: unchanged
        prev = [w.copy() for w in ref_W]


def test_adam_rejects_bad_arguments(api):
    shape = W.scaled_config(W.CONFIGS[1], T=8, n=2, k=1, d=64, h=64)
    cfg = api.make_config(shape)
    t = torch.zeros(2 * 64 * 64, device="cuda")
    ws = torch.empty(max(256, api.moe_adam_workspace_bytes(cfg)), dtype=torch.uint8, device="cuda")
    with pytest.raises(api.MoeError) as e:
        api.moe_expert_adam_step(cfg, 1e-3, 0.9, 1e-8, 0, t, t, t, t, None, None, t, t, t, t, ws)   # step 0
    assert e.value.status == api.MOE_EINVAL
    with pytest.raises(api.MoeError) as e:
        api.moe_expert_adam_step(cfg, 1e-3, 0.9, 1e-8, 1, t, t, t, t, None, None, t, t, t, t, ws[:16])
    assert e.value.status == api.MOE_EWORKSPACE


def test_adam_step_with_sums_from_the_backward_pass(api):
    """MOE_FLAG_ADAM_MOMENTS: the weight-gradient kernels leave per-block sums of squares in the
    backward workspace; the step that uses them must agree with the step that makes its own pass
    over the gradients, and with the oracle."""
    from tests import gpu_harness as G
    say("adam fused moments")
    shape = W.scaled_config(W.CONFIGS[4], T=700, n=32, k=3, d=256, h=512)
    x, W_g, W_noise, eps, bias = G.flat_inputs(shape)
    W1, W2 = G.device_weights(shape)
    run = G.FlatRun(api, shape, x, W_g, W_noise, eps, bias, W1, W2, flags=api.MOE_FLAG_ADAM_MOMENTS)
    run.fused()
    T, d, h, n = shape.T, shape.d, shape.h, shape.n
    f32 = dict(dtype=torch.float32, device="cuda")
    grads = [torch.empty((T, d), **f32), torch.empty((d, n), **f32), torch.empty((d, n), **f32),
             torch.empty((n, d, h), **f32), torch.empty((n, h, d), **f32)]
    bws = torch.empty(api.moe_backward_workspace_bytes(run.cfg), dtype=torch.uint8, device="cuda")
    dy = G.dev(W.upstream_grad(shape))
    api.moe_layer_backward(run.cfg, run.x, run.W_g, run.W_noise, run.eps, run.W1, run.W2, dy, run.topk_idx,
                           run.topk_gate, run.workspace, grads[0], grads[1], grads[2], grads[3], grads[4], bws)
    torch.cuda.synchronize()
    ows = torch.empty(max(256, api.moe_adam_workspace_bytes(run.cfg)), dtype=torch.uint8, device="cuda")
    results = []
    for fused in (False, True):
        masters = [run.W1.to(torch.float32), run.W2.to(torch.float32)]
        copies = [torch.zeros_like(run.W1), torch.zeros_like(run.W2)]
        st = [torch.zeros((n, d), **f32), torch.zeros((n, h), **f32), torch.zeros((n, h), **f32), torch.zeros((n, d), **f32)]
        api.moe_expert_adam_step(run.cfg, 1e-2, 0.9, 1e-8, 1, grads[3], grads[4], masters[0], masters[1], copies[0],
                                 copies[1], st[0], st[1], st[2], st[3], ows, backward_workspace=bws if fused else None)
        torch.cuda.synchronize()
        results.append((masters, st, copies))
    (m0, s0, c0), (m1, s1, c1) = results
    for a, b in zip(s0, s1):
        assert rel(b.cpu().numpy(), a.cpu().numpy().astype(np.float64)) <= TOL
    for a, b in zip(m0, m1):
        assert rel(b.cpu().numpy(), a.cpu().numpy().astype(np.float64)) <= TOL
    # and against the oracle, expert by expert, from the gradients the backward pass wrote
    g1 = grads[3].cpu().numpy()
    w1 = run.W1.to(torch.float32).cpu().numpy()
    for e in (0, 7, n - 1):
        ref_W, ref_vr, ref_vc = O.factored_adam_step(w1[e], g1[e], np.zeros(d), np.zeros(h), 1e-2, 0.9, 1e-8, 1)
        assert rel(m1[0][e].cpu().numpy(), ref_W) <= TOL
        assert rel(s1[0][e].cpu().numpy(), ref_vr) <= TOL and rel(s1[1][e].cpu().numpy(), ref_vc) <= TOL
    with pytest.raises(api.MoeError):      # the flag is what sizes and fills those sums
        plain = api.make_config(shape)
        api.moe_expert_adam_step(plain, 1e-2, 0.9, 1e-8, 1, grads[3], grads[4], m0[0], m0[1], c0[0], c0[1],
                                 s0[0], s0[1], s0[2], s0[3], ows, backward_workspace=bws)


def test_adam_step_with_sums_from_the_hierarchical_backward_pass(api):
    """The same sums of squares left by moe_layer_backward_hier: the step that takes them from the
    backward workspace must agree with the step that makes its own pass over the gradients."""
    from tests import gpu_harness as G
    say("adam fused moments, hierarchical")
    shape = W.scaled_config(W.CONFIGS[3], T=600, a=32, b=32, n=1024, k_primary=2, k_secondary=2, k=4,
                            d=256, h=256)
    inputs = W.hier_gate_inputs(shape, 0.02)
    W1, W2 = G.device_weights(shape, chunk=256)
    run = G.HierRun(api, shape, inputs, W1, W2, flags=api.MOE_FLAG_ADAM_MOMENTS)
    run.forward()
    T, d, h, n, a, b = shape.T, shape.d, shape.h, shape.n, shape.a, shape.b
    f32 = dict(dtype=torch.float32, device="cuda")
    out = [torch.empty((T, d), **f32), torch.empty((d, a), **f32), torch.empty((d, a), **f32),
           torch.empty((a, d, b), **f32), torch.empty((a, d, b), **f32), torch.empty((n, d, h), **f32),
           torch.empty((n, h, d), **f32)]
    plain_cfg = api.make_config(shape)
    assert api.moe_backward_hier_workspace_bytes(run.cfg) > api.moe_backward_hier_workspace_bytes(plain_cfg)
    bws = torch.empty(api.moe_backward_hier_workspace_bytes(run.cfg), dtype=torch.uint8, device="cuda")
    dy = G.dev(W.upstream_grad(shape))
    api.moe_layer_backward_hier(run.cfg, run.x, run.Wg_p, run.Wn_p, run.eps_p, run.Wg_s, run.Wn_s, run.eps_s,
                                run.W1, run.W2, dy, run.topk_idx, run.topk_gate, run.workspace, *out, bws)
    torch.cuda.synchronize()
    ows = torch.empty(max(256, api.moe_adam_workspace_bytes(run.cfg)), dtype=torch.uint8, device="cuda")
    results = []
    for fused in (False, True):
        masters = [run.W1.to(torch.float32), run.W2.to(torch.float32)]
        copies = [torch.zeros_like(run.W1), torch.zeros_like(run.W2)]
        st = [torch.zeros((n, d), **f32), torch.zeros((n, h), **f32), torch.zeros((n, h), **f32), torch.zeros((n, d), **f32)]
        api.moe_expert_adam_step(run.cfg, 1e-2, 0.9, 1e-8, 1, out[5], out[6], masters[0], masters[1], copies[0],
                                 copies[1], st[0], st[1], st[2], st[3], ows, backward_workspace=bws if fused else None)
        torch.cuda.synchronize()
        results.append((masters, st, copies))
    (m0, s0, c0), (m1, s1, c1) = results
    used = (out[5].abs().amax(dim=(1, 2)) > 0).sum().item()
    assert used > n // 4          # most experts got rows, so the comparison is not of zeros
    for x0, x1 in zip(s0 + m0, s1 + m1):
        assert rel(x1.cpu().numpy(), x0.cpu().numpy().astype(np.float64)) <= TOL
    g2 = out[6].cpu().numpy()
    w2 = run.W2.to(torch.float32).cpu().numpy()
    e = int(torch.argmax(out[6].abs().amax(dim=(1, 2))).item())
    ref_W, ref_vr, ref_vc = O.factored_adam_step(w2[e], g2[e], np.zeros(h), np.zeros(d), 1e-2, 0.9, 1e-8, 1)
    assert rel(m1[1][e].cpu().numpy(), ref_W) <= TOL
    assert rel(s1[2][e].cpu().numpy(), ref_vr) <= TOL and rel(s1[3][e].cpu().numpy(), ref_vc) <= TOL


def test_training_step_with_adam_at_full_size(api):
    """The training workload at full size (T = 65536, 512 experts, skewed loads): forward, backward
    with the sums of squares taken in the weight-gradient kernels, then the Adam step of all 1024
    matrices; sampled experts against the oracle's step applied to the gradients the GPU produced
    (the gradients themselves are checked at this size by the backward tests)."""
    from tests import gpu_harness as G
    shape = W.CONFIGS[4]
    say("adam at full size", shape.name)
    x, W_g, W_noise, eps, bias = G.flat_inputs(shape, True)
    W1, W2 = G.device_weights(shape)
    run = G.FlatRun(api, shape, x, W_g, W_noise, eps, bias, W1, W2,
                    flags=api.MOE_FLAG_SAVE_HIDDEN | api.MOE_FLAG_ADAM_MOMENTS)
    run.fused()
    T, d, h, n = shape.T, shape.d, shape.h, shape.n
    f32 = dict(dtype=torch.float32, device="cuda")
    grads = [torch.empty((T, d), **f32), torch.empty((d, n), **f32), torch.empty((d, n), **f32),
             torch.empty((n, d, h), **f32), torch.empty((n, h, d), **f32)]
    bws = torch.empty(api.moe_backward_workspace_bytes(run.cfg), dtype=torch.uint8, device="cuda")
    dy = G.dev(W.upstream_grad(shape))
    api.moe_layer_backward(run.cfg, run.x, run.W_g, run.W_noise, run.eps, run.W1, run.W2, dy, run.topk_idx,
                           run.topk_gate, run.workspace, grads[0], grads[1], grads[2], grads[3], grads[4], bws)
    masters = [run.W1.to(torch.float32), run.W2.to(torch.float32)]
    before = [m.clone() for m in masters]
    copies = [torch.zeros_like(run.W1), torch.zeros_like(run.W2)]
    st = [torch.zeros((n, d), **f32), torch.zeros((n, h), **f32), torch.zeros((n, h), **f32), torch.zeros((n, d), **f32)]
    ows = torch.empty(max(256, api.moe_adam_workspace_bytes(run.cfg)), dtype=torch.uint8, device="cuda")
    # the hyper-parameters cross the C ABI as fp32: the oracle gets the same (rounded) values, or
    # 1 - beta2 would differ by 1.3e-5 of itself
    lr, beta2, eps_adam = (float(np.float32(v)) for v in (1e-3, 0.999, 1e-8))
    api.moe_expert_adam_step(run.cfg, lr, beta2, eps_adam, 1, grads[3], grads[4], masters[0], masters[1], copies[0],
                             copies[1], st[0], st[1], st[2], st[3], ows, backward_workspace=bws)
    torch.cuda.synchronize()
    counts = np.bincount(run.topk_idx.cpu().numpy().reshape(-1), minlength=n)
    sample = sorted({0, 17, 300, 511, int(np.argmax(counts)), int(np.argmin(counts))})
    for w, (R, C) in enumerate(((d, h), (h, d))):
        for e in sample:
            g = grads[3 + w][e].cpu().numpy()
            ref_W, ref_vr, ref_vc = O.factored_adam_step(before[w][e].cpu().numpy(), g, np.zeros(R), np.zeros(C),
                                                         lr, beta2, eps_adam, 1)
            got = masters[w][e].cpu().numpy()
            assert rel(got, ref_W) <= TOL, (w, e)
            assert rel(st[2 * w][e].cpu().numpy(), ref_vr) <= TOL and rel(st[2 * w + 1][e].cpu().numpy(), ref_vc) <= TOL
            upd_ref = ref_W - before[w][e].cpu().numpy().astype(np.float64)
            upd_got = got.astype(np.float64) - before[w][e].cpu().numpy().astype(np.float64)
            assert np.abs(upd_got - upd_ref).max() <= 1e-4 * np.abs(upd_ref).max() + 1e-9
            bits = copies[w][e].view(torch.int16).cpu().numpy().view(np.uint16)
            assert np.array_equal(bits, (O.round_to_bf16(got).view(np.uint32) >> 16).astype(np.uint16))
    assert all(torch.isfinite(m).all() for m in masters)
