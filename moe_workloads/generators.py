"""Seeded generators for every input tensor of the MoE layer workloads.

* Dense fp32 inputs (tokens x, gate matrices, gate noise, upstream gradient) are drawn
  on the host with numpy's counter-based Philox generator, one sub-stream per tensor.
* Expert weights are *procedural*: element (expert, matrix, flat index) is a pure integer
  hash of its coordinates, mapped to Glorot-uniform U(-a, a).  Because only integer and
  exactly representable float operations are used, the same function evaluated with torch
  on the CPU (for the oracle, one expert at a time) and on the GPU (for the HIP path, all
  experts, never crossing PCIe) yields identical bits.

Nothing here performs any step of the MoE method itself.
"""
import math

import numpy as np
import torch

# Philox sub-stream ids, one per tensor kind.
STREAMS = {
    "x": 1, "W_g": 2, "W_noise": 3, "eps": 4, "dy": 5,
    "W_g_primary": 6, "W_noise_primary": 7, "eps_primary": 8,
    "W_g_secondary": 9, "W_noise_secondary": 10, "eps_secondary": 11,
    "zipf_perm": 12, "dropout": 13,
}

_M32 = 0xFFFFFFFF
_M64 = 0xFFFFFFFFFFFFFFFF


def normal_f32(seed: int, stream: str, shape, std: float = 1.0) -> np.ndarray:
    """N(0, std^2) float32 array from Philox keyed by (seed, stream)."""
    gen = np.random.Generator(np.random.Philox(key=[seed & _M64, STREAMS[stream]]))
    out = gen.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        out *= np.float32(std)
    return out


def gate_inputs(cfg, gate_std: float = 0.02):
    """x ~ N(0,1) [T,d]; W_g, W_noise ~ N(0, gate_std^2) [d,n]; eps ~ N(0,1) [T,n]."""
    x = normal_f32(cfg.seed, "x", (cfg.T, cfg.d))
    W_g = normal_f32(cfg.seed, "W_g", (cfg.d, cfg.n), gate_std)
    W_noise = normal_f32(cfg.seed, "W_noise", (cfg.d, cfg.n), gate_std)
    eps = normal_f32(cfg.seed, "eps", (cfg.T, cfg.n))
    return x, W_g, W_noise, eps


def hier_gate_inputs(cfg, gate_std: float = 0.02):
    """Hierarchical gate inputs: primary matrices [d,a], noise [T,a]; one secondary pair of
    matrices per group [a,d,b]; secondary noise per primary slot [T,k_primary,b]."""
    x = normal_f32(cfg.seed, "x", (cfg.T, cfg.d))
    Wg_p = normal_f32(cfg.seed, "W_g_primary", (cfg.d, cfg.a), gate_std)
    Wn_p = normal_f32(cfg.seed, "W_noise_primary", (cfg.d, cfg.a), gate_std)
    eps_p = normal_f32(cfg.seed, "eps_primary", (cfg.T, cfg.a))
    Wg_s = normal_f32(cfg.seed, "W_g_secondary", (cfg.a, cfg.d, cfg.b), gate_std)
    Wn_s = normal_f32(cfg.seed, "W_noise_secondary", (cfg.a, cfg.d, cfg.b), gate_std)
    eps_s = normal_f32(cfg.seed, "eps_secondary", (cfg.T, cfg.k_primary, cfg.b))
    return x, Wg_p, Wn_p, eps_p, Wg_s, Wn_s, eps_s


def upstream_grad(cfg) -> np.ndarray:
    return normal_f32(cfg.seed, "dy", (cfg.T, cfg.d))


def dropout_keep(cfg, drop_prob: float) -> np.ndarray:
    """The dropout draw for the layer output [T,d] as bytes: 1 = the activation survives (uniform
    numbers from Philox keyed by (seed, "dropout"), kept where u >= drop_prob)."""
    gen = np.random.Generator(np.random.Philox(key=[cfg.seed & _M64, STREAMS["dropout"]]))
    return (gen.random(size=(cfg.T, cfg.d), dtype=np.float32) >= drop_prob).astype(np.uint8)


def zipf_gate_bias(cfg, s: float = 1.1) -> np.ndarray:
    """Per-expert additive logit bias beta * (-s * ln(rank) - mean), ranks a seeded permutation.

    Not part of the paper's gate; it is an *input* that skews expert popularity the way an
    unbalanced trained gate does (Table 6, first row: max/mean load 17.8)."""
    gen = np.random.Generator(np.random.Philox(key=[cfg.seed & _M64, STREAMS["zipf_perm"]]))
    ranks = gen.permutation(cfg.n).astype(np.float64) + 1.0
    raw = -s * np.log(ranks)
    return (cfg.zipf_beta * (raw - raw.mean())).astype(np.float32)


def _splitmix64(z: int) -> int:
    z = (z + 0x9E3779B97F4A7C15) & _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


def _matrix_keys(seed: int, expert: int, which: int):
    """Two 32-bit keys for (seed, expert, matrix) from host-side integer mixing."""
    z = _splitmix64((seed & _M64) ^ _splitmix64((expert << 2) | which))
    return z & _M32, (z >> 32) & _M32


def _hash_u24(flat_idx: torch.Tensor, key_lo: torch.Tensor, key_hi: torch.Tensor) -> torch.Tensor:
    """Per-element 32-bit avalanche hash carried in int64 lanes; returns its top 24 bits."""
    v = (flat_idx + key_lo) & _M32
    v = v ^ (v >> 16)
    v = (v * 0x85EBCA6B) & _M32
    v = v ^ (v >> 13)
    v = (v * 0xC2B2AE35) & _M32
    v = v ^ (v >> 16)
    v = v ^ key_hi
    v = (v * 0x9E3779B1) & _M32
    v = v ^ (v >> 15)
    v = (v * 0x85EBCA77) & _M32
    v = v ^ (v >> 13)
    return v >> 8


def glorot_limit(fan_in: int, fan_out: int) -> float:
    return math.sqrt(6.0 / (fan_in + fan_out))


def expert_weights_all(cfg, which: int, experts, device="cpu", dtype=None) -> torch.Tensor:
    """Weights of matrix `which` (0: W1 [d,h] input->hidden, 1: W2 [h,d] hidden->output) for the
    given expert ids, stacked as [len(experts), rows, cols] in the paper's plain row-major
    layout.  Glorot-uniform: w = (2u - 1) * limit with u a 24-bit hash fraction; for
    d=512, h=1024 the limit is exactly 2^-4, so w is exact in fp32 before any bf16 rounding."""
    if dtype is None:
        dtype = torch.float32 if cfg.expert_dtype == "f32" else torch.bfloat16
    rows, cols = (cfg.d, cfg.h) if which == 0 else (cfg.h, cfg.d)
    limit = glorot_limit(cfg.d, cfg.h)
    experts = [int(e) for e in experts]
    keys = [_matrix_keys(cfg.seed, e, which) for e in experts]
    klo = torch.tensor([k[0] for k in keys], dtype=torch.int64, device=device).view(-1, 1)
    khi = torch.tensor([k[1] for k in keys], dtype=torch.int64, device=device).view(-1, 1)
    flat = torch.arange(rows * cols, dtype=torch.int64, device=device).view(1, -1)
    u24 = _hash_u24(flat, klo, khi)
    w = (u24.to(torch.float32) * (2.0 ** -23) - 1.0) * limit
    return w.to(dtype).view(len(experts), rows, cols)


def expert_weights(cfg, which: int, expert: int, device="cpu", dtype=None) -> torch.Tensor:
    return expert_weights_all(cfg, which, [expert], device=device, dtype=dtype)[0]
