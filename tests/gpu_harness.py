"""Helpers for the GPU parity tests: the oracle side of a comparison on the same seeded inputs
the HIP path gets (the GPU-side buffer plumbing lives in paper_1701_06538_amd/runner.py, the device
input generation in moe_workloads/device.py; both are re-exported here for the tests)."""
import numpy as np
import torch

import moe_workloads as W
from moe_workloads.device import device_weights, flat_inputs  # noqa: F401
from paper_1701_06538_amd.runner import BalancedRun, FlatRun, HierRun, dev  # noqa: F401


def oracle_weight_fn(shape):
    def fn(e):
        w1 = W.expert_weights(shape, 0, e).to(torch.float64).numpy()
        w2 = W.expert_weights(shape, 1, e).to(torch.float64).numpy()
        return w1, w2
    return fn


def device_weight_fn(shape, W1, W2, block=1, progress=None):
    """weight_fn for the oracle that reads the expert matrices from the device tensors the input
    generator filled (moe_workloads.device.device_weights: the same integer hash as
    moe_workloads.expert_weights on the CPU, evaluated by torch on the GPU -- inputs, not results of
    the HIP path), widened to binary64 on the device and copied `block` experts at a time.
    Regenerating a matrix on the host costs ~30 ms; a full-size check visits up to 16384 experts.
    check_device_weights() ties the two generators together bit for bit."""
    cache = {"b0": -1}

    def fn(e):
        e = int(e)
        b0 = e // block * block
        if cache["b0"] != b0:
            cache["b0"] = b0
            cache["w1"] = W1[b0:b0 + block].to(torch.float64).cpu().numpy()
            cache["w2"] = W2[b0:b0 + block].to(torch.float64).cpu().numpy()
            if progress is not None:
                progress(b0)
        return cache["w1"][e - b0], cache["w2"][e - b0]
    return fn


def check_device_weights(shape, W1, W2, experts):
    """The device tensors hold exactly what the host generator gives for these experts."""
    for e in experts:
        assert torch.equal(W1[e].cpu(), W.expert_weights(shape, 0, int(e))), e
        assert torch.equal(W2[e].cpu(), W.expert_weights(shape, 1, int(e))), e


def weight_fn_for(shape, W1, W2, many=512):
    """The oracle's expert matrices: from the host generator for layers of fewer than `many`
    experts, else from the generator's device tensors (checked against the host generator on three
    experts): regenerating a thousand 512 x 1024 pairs on the host takes half a minute."""
    if shape.n < many:
        return oracle_weight_fn(shape)
    check_device_weights(shape, W1, W2, [0, shape.n // 2 + 1, shape.n - 1])
    return device_weight_fn(shape, W1, W2, block=16)


def oracle_flat(shape, x, W_g, W_noise, eps, bias):
    from oracle import moe_oracle as O
    lg = O.noisy_logits_f32(x, W_g, W_noise, eps, bias)
    return O.gate_and_losses(lg, shape.k, shape.w_importance, shape.w_load)


def rel_errors(got, ref):
    """(max per-row relative L2 error, max-abs error / max-abs ref)."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    num = np.linalg.norm(got - ref, axis=-1)
    den = np.linalg.norm(ref, axis=-1)
    row = float(np.max(num / np.maximum(den, 1e-300))) if ref.size else 0.0
    mx = float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-300)) if ref.size else 0.0
    return row, mx


def fro_rel(got, ref):
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    return float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300))


def check_dx_rows(got_dx, ref_dx, x_experts, dy, idx, gates, weight_fn, gpu_hidden_row, tol, tau=2e-5):
    """Row-by-row comparison of dx at sizes where single hidden units sit on the ReLU kink.

    Every row must be within `tol` (relative L2) of the oracle's.  A row that is not is accepted only
    if it is explained: some hidden unit of one of its experts has a pre-activation of magnitude
    <= tau in the oracle's binary64 (the kernel's fp32 accumulation can land on the other side of
    zero, and relu' is a binary decision: either side is a correct evaluation), and the oracle's
    row re-evaluated with the kernel's decision AT THOSE UNITS ONLY (O.expert_input_grad with an
    explicit mask) is within `tol`.  gpu_hidden_row(t, s) -> the kernel's hidden activations [h] of
    assignment (t, s).  Returns (Frobenius relative error, number of explained rows, largest |z| of
    a unit whose decision differed)."""
    from oracle import moe_oracle as O
    got = np.asarray(got_dx, np.float64)
    ref = np.asarray(ref_dx, np.float64)
    dy = np.asarray(dy, np.float64)
    xe = np.asarray(x_experts, np.float64)
    rel = np.linalg.norm(got - ref, axis=1) / np.maximum(np.linalg.norm(ref, axis=1), 1e-300)
    bad = np.nonzero(rel > tol)[0]
    worst_z = 0.0
    for t in bad:
        alt = ref[t].copy()
        flips = 0
        for s in range(idx.shape[1]):
            W1, W2 = weight_fn(int(idx[t, s]))
            z = xe[t] @ np.asarray(W1, np.float64)
            ambiguous = np.abs(z) <= tau
            mask_alt = np.where(ambiguous, np.asarray(gpu_hidden_row(int(t), s)) > 0, z > 0)
            differ = mask_alt != (z > 0)
            if differ.any():
                flips += int(differ.sum())
                worst_z = max(worst_z, float(np.abs(z[differ]).max()))
                dout = (gates[t, s] * dy[t])[None, :]
                alt += (O.expert_input_grad(xe[t:t + 1], dout, W1, W2, relu_mask=mask_alt[None, :])
                        - O.expert_input_grad(xe[t:t + 1], dout, W1, W2))[0]
        rel_alt = float(np.linalg.norm(got[t] - alt) / max(np.linalg.norm(alt), 1e-300))
        assert flips > 0, "dx row %d is off by %.2e and no hidden unit of its experts sits on the ReLU kink" % (t, rel[t])
        assert rel_alt <= tol, "dx row %d: %.2e even with the kernel's decisions at %d kink units" % (t, rel_alt, flips)
    return fro_rel(got, ref), int(bad.size), worst_z
