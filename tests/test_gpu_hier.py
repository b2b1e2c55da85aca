"""GPU parity of the hierarchical layer (Appendix B, Eq.(12)-(14)) against the CPU oracle."""
import sys

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


def oracle_hier(shape, inputs):
    x, Wg_p, Wn_p, eps_p, Wg_s, Wn_s, eps_s = inputs
    return O.hier_gate_and_losses(x, Wg_p, Wn_p, eps_p, Wg_s, Wn_s, eps_s, shape.k_primary,
                                  shape.k_secondary, shape.w_importance, shape.w_load)


def check_hier_gate(run, hf, shape):
    T, kp, ks = shape.T, shape.k_primary, shape.k_secondary
    assert np.array_equal(run.ws_view("p_idx", T * kp, torch.int32).cpu().numpy().reshape(T, kp), hf.group_idx)
    assert np.array_equal(run.ws_view("s_idx", T * kp * ks, torch.int32).cpu().numpy().reshape(T, kp, ks), hf.sec_idx)
    assert np.array_equal(run.topk_idx.cpu().numpy(), hf.idx), "global expert ids differ"
    g = run.topk_gate.cpu().numpy().astype(np.float64)
    assert np.abs(g - hf.gates).max() <= TOL_F32
    assert np.array_equal(run.ws_view("p_counts", shape.a, torch.int32).cpu().numpy(), hf.group_counts.astype(np.int32))


def check_hier_losses(run, hf):
    imp = run.importance.cpu().numpy().astype(np.float64)
    ld = run.load.cpu().numpy().astype(np.float64)
    assert np.abs(imp - hf.importance).max() <= TOL_F32 * np.abs(hf.importance).max()
    assert np.abs(ld - hf.load).max() <= TOL_F32 * np.abs(hf.load).max()
    L = run.losses.cpu().numpy().astype(np.float64)
    assert abs(L[0] - hf.loss_importance) <= TOL_F32 * abs(hf.loss_importance) + 1e-8
    assert abs(L[1] - hf.loss_load) <= TOL_F32 * abs(hf.loss_load) + 1e-8


CASES = [
    ("small", dict(T=300, a=4, b=8)),
    ("empty_groups", dict(T=3, a=8, b=16)),
    ("ragged", dict(T=1111, a=5, b=40)),
    ("k_p1_k_s3", dict(T=257, a=6, b=12, k_primary=1, k_secondary=3)),
    ("medium", dict(T=4096, a=16, b=64)),
    ("wide_secondary_b1280", dict(T=600, a=2, b=1280, d=128, h=128)),   # secondary rows on the four-waves-per-row top-k
]


@pytest.mark.parametrize("name,ov", CASES, ids=[c[0] for c in CASES])
def test_hier_layer_parity(api, name, ov):
    shape = W.scaled_config(W.CONFIGS[3], **ov)
    say("case hier", name, shape)
    inputs = W.hier_gate_inputs(shape)
    hf = oracle_hier(shape, inputs)
    W1, W2 = G.device_weights(shape)
    run = G.HierRun(api, shape, inputs, W1, W2)
    run.forward()
    check_hier_gate(run, hf, shape)
    y_ref = O.moe_output(inputs[0], hf.idx, hf.gates, G.weight_fn_for(shape, W1, W2), shape.n)
    row, mx = G.rel_errors(run.y.cpu().numpy(), y_ref)
    say("  y errors: row-rel %.3e max-abs-rel %.3e" % (row, mx))
    assert row <= TOL_BF16 and mx <= TOL_BF16
    check_hier_losses(run, hf)
    # routing over all a*b experts is the same brute-force permutation
    counts, offsets, perm, inv = O.routing(hf.idx, shape.n)
    A = shape.T * shape.k
    assert np.array_equal(run.ws_view("counts", shape.n, torch.int32).cpu().numpy(), counts)
    assert np.array_equal(run.ws_view("perm", A, torch.int32).cpu().numpy(), perm)
    # bit-reproducible
    y1 = run.y.clone()
    run.forward()
    assert torch.equal(run.y, y1)
