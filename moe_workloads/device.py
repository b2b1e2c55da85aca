"""Inputs of a workload as the GPU path wants them: the host-drawn gate tensors of one shape, and the
procedural expert weights evaluated with torch on the device (same integer hash as on the CPU, so
the bits are identical and 34 GB never cross PCIe).  Input generation only."""
import torch

from . import generators as W


def flat_inputs(shape, with_bias=False, gate_std=0.02):
    x, W_g, W_noise, eps = W.gate_inputs(shape, gate_std)
    bias = W.zipf_gate_bias(shape) if with_bias else None
    return x, W_g, W_noise, eps, bias


def device_weights(shape, chunk=64):
    """Expert weights generated on the GPU in the paper's plain layout."""
    outs = []
    for which in (0, 1):
        parts = [W.expert_weights_all(shape, which, range(e0, min(shape.n, e0 + chunk)), device="cuda")
                 for e0 in range(0, shape.n, chunk)]
        outs.append(torch.cat(parts, dim=0).contiguous())
    return outs
