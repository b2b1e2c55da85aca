"""The routing entry point that allocates nothing (moe_route_static: chunk histograms in a device
array inside the library) against moe_route on the same inputs, bit for bit, on two calls in a row,
the second with a smaller input that leaves stale histogram cells of the first call behind."""
import sys

import numpy as np
import pytest
import torch

import moe_workloads as W

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def api():
    assert torch.cuda.is_available()
    from paper_1701_06538_amd import api as _api
    return _api


def route_outputs(api, cfg, n, A):
    i32 = dict(dtype=torch.int32, device="cuda")
    mt = api.moe_max_tiles(cfg) + 8
    return dict(counts=torch.full((n,), -7, **i32), offsets=torch.full((n + 1,), -7, **i32),
                perm=torch.full((max(A, 1),), -7, **i32), inv_perm=torch.full((max(A, 1),), -7, **i32),
                tile_expert=torch.full((mt,), -7, **i32), tile_row0=torch.full((mt,), -7, **i32),
                num_tiles=torch.full((4,), -7, **i32))


def run_pair(api, T, n, k, seed):
    shape = W.scaled_config(W.CONFIGS[2], T=T, n=n, k=k)
    cfg = api.make_config(shape)
    rng = np.random.default_rng(seed)
    # k distinct experts per token, skewed so that some experts are empty and some long
    p = 1.0 / np.arange(1, n + 1) ** 0.7
    p /= p.sum()
    idx = np.stack([rng.choice(n, size=k, replace=False, p=p) for _ in range(T)]).astype(np.int32)
    idx_d = torch.from_numpy(idx).cuda()
    A = T * k
    ref = route_outputs(api, cfg, n, A)
    ws = torch.empty(max(16, api.moe_route_workspace_bytes(cfg)), dtype=torch.uint8, device="cuda")
    api.moe_route(cfg, idx_d, ref["counts"], ref["offsets"], ref["perm"], ref["inv_perm"], ref["tile_expert"],
                  ref["tile_row0"], ref["num_tiles"], ws)
    got = route_outputs(api, cfg, n, A)
    api.moe_route_static(cfg, idx_d, got["counts"], got["offsets"], got["perm"], got["inv_perm"],
                         got["tile_expert"], got["tile_row0"], got["num_tiles"])
    torch.cuda.synchronize()
    nt = int(ref["num_tiles"][0])
    assert int(got["num_tiles"][0]) == nt
    for q in ("counts", "offsets", "perm", "inv_perm"):
        assert torch.equal(got[q], ref[q]), q
    for q in ("tile_expert", "tile_row0"):
        assert torch.equal(got[q][:nt], ref[q][:nt]), q
    assert int(ref["counts"].sum()) == A
    return api.moe_route_workspace_bytes(cfg)


def test_route_static_matches_route_twice_in_a_row(api):
    say("route_static: T=8192 n=2048 k=4, then T=1000 n=1500 k=3")
    big = run_pair(api, 8192, 2048, 4, 1)       # the general path: histograms of 128 chunks x 2048 experts
    small = run_pair(api, 1000, 1500, 3, 2)     # smaller: most of the first call's cells stay behind
    assert 0 < small < big <= api.MOE_ROUTE_STATIC_MAX_WORKSPACE_BYTES


def test_route_static_rejects_what_does_not_fit(api):
    shape = W.CONFIGS[3]                         # 16384 experts: 32 MiB of histograms
    cfg = api.make_config(shape)
    assert api.moe_route_workspace_bytes(cfg) > api.MOE_ROUTE_STATIC_MAX_WORKSPACE_BYTES
    t = torch.zeros(16, dtype=torch.int32, device="cuda")
    with pytest.raises(api.MoeError) as e:
        api.moe_route_static(cfg, t, t, t, t, t, t, t, t)
    assert e.value.status == api.MOE_EWORKSPACE
