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
