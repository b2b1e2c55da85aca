"""The seeded input generators: deterministic, right shapes/distributions, no method arithmetic."""
import numpy as np
import torch

import moe_workloads as W


def test_configs_match_the_five_workloads():
    c = W.CONFIGS
    assert [(s.T, s.n, s.k) for s in c] == [(256, 16, 4), (8192, 256, 4), (32768, 2048, 4),
                                            (65536, 16384, 4), (65536, 512, 4)]
    assert all(s.d == 512 and s.h == 1024 for s in c)
    assert c[3].a == 64 and c[3].b == 256 and c[3].k_primary == 2 and c[3].k_secondary == 2
    assert c[0].expert_dtype == "f32" and c[1].expert_dtype == "bf16"
    assert c[4].backward and c[4].zipf_beta > 0


def test_dense_inputs_are_seeded_and_distributed_as_stated():
    cfg = W.scaled_config(W.CONFIGS[1], T=512, n=64)
    x, Wg, Wn, eps = W.gate_inputs(cfg)
    x2, Wg2, _, _ = W.gate_inputs(cfg)
    assert np.array_equal(x, x2) and np.array_equal(Wg, Wg2)
    assert x.dtype == np.float32 and x.shape == (512, 512) and eps.shape == (512, 64)
    assert abs(x.std() - 1.0) < 0.01 and abs(Wg.std() - 0.02) < 0.001 and abs(Wn.std() - 0.02) < 0.001
    assert not np.array_equal(Wg, Wn)
    other = W.gate_inputs(W.scaled_config(cfg, seed=cfg.seed + 1))[0]
    assert not np.array_equal(x, other)


def test_expert_weights_are_glorot_uniform_and_reproducible():
    cfg = W.CONFIGS[1]
    w1 = W.expert_weights(cfg, 0, 7)
    w2 = W.expert_weights(cfg, 1, 7)
    assert w1.shape == (512, 1024) and w2.shape == (1024, 512) and w1.dtype == torch.bfloat16
    again = W.expert_weights_all(cfg, 0, [3, 7])[1]
    assert torch.equal(w1, again)
    f = W.expert_weights(cfg, 0, 7, dtype=torch.float32)
    lim = 0.0625                                      # sqrt(6 / (512 + 1024))
    assert float(f.min()) >= -lim and float(f.max()) < lim
    assert abs(float(f.mean())) < 2e-4
    assert abs(float(f.std()) - lim / np.sqrt(3.0)) < 2e-4
    assert not torch.equal(W.expert_weights(cfg, 0, 8), w1)
    assert not torch.equal(W.expert_weights(cfg, 1, 7).T.contiguous(), w1)
    # neighbouring elements are uncorrelated
    a = f.flatten()[:-1].double()
    b = f.flatten()[1:].double()
    assert abs(float((a * b).mean()) / float(f.double().var())) < 5e-3


def test_zipf_bias_is_centred_and_skewed():
    cfg = W.CONFIGS[4]
    b = W.zipf_gate_bias(cfg)
    assert b.shape == (512,) and abs(b.mean()) < 1e-6
    assert b.max() - b.min() > 1.0
