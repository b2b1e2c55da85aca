"""Benchmark of the Sparsely-Gated MoE layer on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config N] [--no-cpu-baseline] ...

A step is one pass of the whole hot path (gate -> route -> expert FFN -> combine -> losses; the
training workload adds the backward pass) over one batch of seeded synthetic input that is already
resident in HBM.  With no --config the headline is the largest single-GPU workload (config 3:
hierarchical, 16384 experts, 34 GB of expert weights) and the other four workloads are timed in the
same run and reported under "per_config".  Every workload is timed the same way: W warm-up steps,
then K steps each bracketed by a HIP event pair on the launch stream; ms_per_step is the MEDIAN of
the K event times (the wall-clock mean over the same K steps is reported beside it).  One more event
pair inside every timed step brackets the dominant kernel (the expert FFN) for the roofline figure;
a separate, untimed pass brackets every stage.  Prints ONE JSON line.
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
BF16_MFMA_PEAK_TFLOPS = 2500.0  # dense bf16 MFMA, published
FP32_MFMA_PEAK_TFLOPS = 157.3   # fp32 matrix/vector, published
STAGES = ["gate", "route", "expert_ffn", "combine", "aux_losses"]
HEADLINE_CONFIG = 3


class HipEvents:
    """hipEvent_t handles made with the HIP runtime that torch already loaded."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]

    def create(self):
        ev = ctypes.c_void_p()
        err = self.hip.hipEventCreate(ctypes.byref(ev))
        assert err == 0, "hipEventCreate failed: %d" % err
        return ev.value

    def record(self, ev):
        import torch
        err = self.hip.hipEventRecord(ev, torch.cuda.current_stream().cuda_stream)
        assert err == 0, "hipEventRecord failed: %d" % err

    def elapsed_ms(self, a, b):
        out = ctypes.c_float()
        err = self.hip.hipEventElapsedTime(ctypes.byref(out), a, b)
        assert err == 0, "hipEventElapsedTime failed: %d" % err
        return out.value

    def destroy(self, ev):
        self.hip.hipEventDestroy(ev)


def read_traffic(name):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary
    (profiles/<name>), or None when no summary has been recorded."""
    path = os.path.join(ROOT, "profiles", name)
    if not os.path.exists(path):
        return None
    for line in open(path):
        if line.startswith("traffic_bytes_per_launch:"):
            return float(line.split(":")[1])
    return None


def _threads():
    try:
        import threadpoolctl
        return int(max([p["num_threads"] for p in threadpoolctl.threadpool_info()] + [1]))
    except Exception:
        return int(os.cpu_count())


def _host_weights(W1, W2, experts):
    """The expert matrices the oracle needs, copied from the device tensors the input generator
    filled (inputs: fetched before the clock starts, as fp32 arrays holding the bf16 or fp32 values
    exactly).  Returns weight_fn(e); the oracle widens what it gets to binary64 itself."""
    import torch
    held = {int(e): (W1[int(e)].to(torch.float32).cpu().numpy(), W2[int(e)].to(torch.float32).cpu().numpy())
            for e in experts}
    return lambda e: held[int(e)]


def cpu_baseline_flat(shape, inputs, W1, W2, dy, sample_tokens):
    """The oracle as it stands, timed on the host on the first `sample_tokens` tokens of the same
    seeded workload: forward (gate, routing, experts in binary64, combine, losses) and, for the
    training workload, the backward pass on the same tokens."""
    import numpy as np

    from oracle import moe_oracle as O
    x, W_g, W_noise, eps, bias = inputs
    S = min(sample_tokens, shape.T)
    x, eps = x[:S], eps[:S]
    lg = O.noisy_logits_f32(x, W_g, W_noise, eps, bias)      # untimed: finds which experts to copy
    used = np.unique(O.keep_top_k(lg.H, shape.k))
    wf = _host_weights(W1, W2, used)
    t0 = time.perf_counter()
    lg = O.noisy_logits_f32(x, W_g, W_noise, eps, bias)
    fw = O.gate_and_losses(lg, shape.k, shape.w_importance, shape.w_load)
    O.routing(fw.idx, shape.n)
    y = O.moe_output(x, fw.idx, fw.gates, wf, shape.n)
    what = "full forward (gate, routing, experts in fp64, combine, losses)"
    if shape.backward:
        gr = O.flat_backward(x, W_g, W_noise, fw, shape.k, wf, dy[:S], shape.w_importance, shape.w_load,
                             expert_input=O.round_to_bf16(x))
        assert np.isfinite(gr.dx).all()
        what = "forward + backward (all gradients)"
    dt = time.perf_counter() - t0
    assert np.isfinite(y).all()
    return {"value": S / dt, "unit": "tokens/s", "cores": _threads(), "kind": "oracle",
            "sample": "first %d of %d tokens of the same seeded workload, %s, %.1f s" % (S, shape.T, what, dt)}


def cpu_baseline_hier(shape, inputs, W1, W2, dy, sample_tokens, backward):
    import numpy as np

    from oracle import moe_oracle as O
    x, Wg_p, Wn_p, eps_p, Wg_s, Wn_s, eps_s = inputs
    S = min(sample_tokens, shape.T)
    x, eps_p, eps_s = x[:S], eps_p[:S], eps_s[:S]
    hf = O.hier_gate_and_losses(x, Wg_p, Wn_p, eps_p, Wg_s, Wn_s, eps_s, shape.k_primary, shape.k_secondary,
                                shape.w_importance, shape.w_load)     # untimed: which experts to copy
    wf = _host_weights(W1, W2, np.unique(hf.idx))
    t0 = time.perf_counter()
    hf = O.hier_gate_and_losses(x, Wg_p, Wn_p, eps_p, Wg_s, Wn_s, eps_s, shape.k_primary, shape.k_secondary,
                                shape.w_importance, shape.w_load)
    O.routing(hf.idx, shape.n)
    y = O.moe_output(x, hf.idx, hf.gates, wf, shape.n)
    what = "full forward (both gate levels, routing, experts in fp64, combine, losses of Eq.(13)-(14))"
    if backward:
        gr = O.hier_backward(x, Wg_p, Wn_p, eps_p, Wg_s, Wn_s, eps_s, shape.k_primary, shape.k_secondary, wf,
                             dy[:S], shape.w_importance, shape.w_load, expert_input=O.round_to_bf16(x))
        assert np.isfinite(gr.dx).all()
        what = "forward + backward"
    dt = time.perf_counter() - t0
    assert np.isfinite(y).all()
    return {"value": S / dt, "unit": "tokens/s", "cores": _threads(), "kind": "oracle",
            "sample": "first %d of %d tokens of the same seeded workload, %s, %.1f s" % (S, shape.T, what, dt)}


def cpu_baseline_balanced(shape, inputs, W1, W2, sample_tokens):
    """The oracle's strictly balanced layer (Appendix F) on the first `sample_tokens` tokens taken as
    a batch of their own (every expert keeps sample_tokens*k/n of them)."""
    import numpy as np

    from oracle import moe_oracle as O
    x, W_g = inputs[0], inputs[1]
    S = min(sample_tokens, shape.T)
    x = x[:S]
    wf = _host_weights(W1, W2, range(shape.n))
    t0 = time.perf_counter()
    _, X = O.softmax_gate_f32(x, W_g)
    mask, _ = O.batchwise_mask(X, S * shape.k // shape.n)
    Gm, _ = O.balanced_gates(X, mask)
    y = O.balanced_output(x, Gm, wf)
    dt = time.perf_counter() - t0
    assert np.isfinite(y).all()
    return {"value": S / dt, "unit": "tokens/s", "cores": _threads(), "kind": "oracle",
            "sample": "first %d of %d tokens of the same seeded workload as one balanced batch, full forward "
                      "(softmax gate, batchwise mask, experts in fp64, combine), %.1f s" % (S, shape.T, dt)}


def run_workload(cfg_index, args, hip, K, warmup):
    """Times one workload; returns its result dict (the fields of a bench line)."""
    import numpy as np
    import torch

    import moe_workloads as W
    import moe_workloads.device as D
    from paper_1701_06538_amd import api     # raises if the HIP library is missing: no fallback
    from paper_1701_06538_amd import runner as G

    shape = W.CONFIGS[cfg_index]
    balanced = args.gating == "balanced"
    f32 = dict(dtype=torch.float32, device="cuda")
    backward = shape.backward or args.backward
    dy = W.upstream_grad(shape) if backward else None
    dyd = G.dev(dy) if backward else None
    bws = None
    if balanced:
        if shape.hierarchical or shape.backward:
            sys.exit("bench.py: --gating balanced runs the flat forward configs only")
        inputs = D.flat_inputs(shape, with_bias=shape.zipf_beta > 0)
        x, W_g, _, _, bias = inputs
        W1, W2 = D.device_weights(shape, chunk=256)
        thr = np.full((shape.n,), 1.0 / shape.n, np.float32)
        run = G.BalancedRun(api, shape, x, W_g, bias, thr, W1, W2,
                            flags=api.MOE_FLAG_SAVE_HIDDEN if backward else 0)
        ws = run.ws
        if backward:
            bg = [torch.empty((shape.T, shape.d), **f32), torch.empty((shape.d, shape.n), **f32),
                  torch.empty((shape.n, shape.d, shape.h), **f32), torch.empty((shape.n, shape.h, shape.d), **f32)]
            bws = torch.empty(api.moe_backward_balanced_workspace_bytes(run.cfg), dtype=torch.uint8, device="cuda")

        def step(events=None):
            ev = None if events is None else [0, 0, events[4], events[5], 0]
            api.moe_layer_forward_balanced_profiled(run.cfg, run.x, run.W_g, run.bias, run.thr, run.W1, run.W2,
                                                    run.y, run.gsigma, run.tokens, run.kept, run.denom,
                                                    run.loss, ws, ev)
            if backward:
                api.moe_layer_backward_balanced(run.cfg, run.x, run.W_g, run.thr, run.W1, run.W2, dyd, run.gsigma,
                                                run.tokens, run.kept, run.denom, ws, 0.1, bg[0], bg[1], bg[2],
                                                bg[3], bws)
    elif shape.hierarchical:
        inputs = W.hier_gate_inputs(shape)
        W1, W2 = D.device_weights(shape, chunk=256)
        run = G.HierRun(api, shape, inputs, W1, W2, flags=api.MOE_FLAG_SAVE_HIDDEN if backward else 0)
        ws = run.workspace
        if backward:
            hg = [torch.empty((shape.T, shape.d), **f32), torch.empty((shape.d, shape.a), **f32),
                  torch.empty((shape.d, shape.a), **f32), torch.empty((shape.a, shape.d, shape.b), **f32),
                  torch.empty((shape.a, shape.d, shape.b), **f32), torch.empty((shape.n, shape.d, shape.h), **f32),
                  torch.empty((shape.n, shape.h, shape.d), **f32)]
            bws = torch.empty(api.moe_backward_hier_workspace_bytes(run.cfg), dtype=torch.uint8, device="cuda")

        def step(events=None):
            api.moe_layer_forward_hier_profiled(run.cfg, run.x, run.Wg_p, run.Wn_p, run.eps_p, run.Wg_s, run.Wn_s,
                                                run.eps_s, run.W1, run.W2, run.y, run.topk_idx, run.topk_gate,
                                                run.importance, run.load, run.losses, ws, events)
            if backward:
                api.moe_layer_backward_hier(run.cfg, run.x, run.Wg_p, run.Wn_p, run.eps_p, run.Wg_s, run.Wn_s,
                                            run.eps_s, run.W1, run.W2, dyd, run.topk_idx, run.topk_gate, ws, hg[0],
                                            hg[1], hg[2], hg[3], hg[4], hg[5], hg[6], bws)
    else:
        inputs = D.flat_inputs(shape, with_bias=shape.zipf_beta > 0)
        x, W_g, W_noise, eps, bias = inputs
        W1, W2 = D.device_weights(shape)
        run = G.FlatRun(api, shape, x, W_g, W_noise, eps, bias, W1, W2,
                        flags=(api.MOE_FLAG_SAVE_HIDDEN if backward else 0)
                        | (api.MOE_FLAG_ADAM_MOMENTS if (backward and args.optimizer) else 0))
        ws = torch.empty(api.moe_workspace_bytes(run.cfg), dtype=torch.uint8, device="cuda")
        if backward:
            grads = [torch.empty((shape.T, shape.d), **f32), torch.empty((shape.d, shape.n), **f32),
                     torch.empty((shape.d, shape.n), **f32), torch.empty((shape.n, shape.d, shape.h), **f32),
                     torch.empty((shape.n, shape.h, shape.d), **f32)]
            bws = torch.empty(api.moe_backward_workspace_bytes(run.cfg), dtype=torch.uint8, device="cuda")

        def step(events=None):
            api.moe_layer_forward_profiled(run.cfg, run.x, run.W_g, run.W_noise, run.bias, run.eps, run.W1,
                                           run.W2, run.y, run.topk_idx, run.topk_gate, run.importance,
                                           run.load, run.losses, ws, events)
            if backward:
                api.moe_layer_backward(run.cfg, run.x, run.W_g, run.W_noise, run.eps, run.W1, run.W2, dyd,
                                       run.topk_idx, run.topk_gate, ws, grads[0], grads[1], grads[2],
                                       grads[3], grads[4], bws)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()

    # timed region: K steps, each inside its own event pair, plus one pair around the expert kernel
    step_ev = [(hip.create(), hip.create()) for _ in range(K)]
    ffn_ev = [(hip.create(), hip.create()) for _ in range(K)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        hip.record(step_ev[i][0])
        step([0, 0, 0, 0, ffn_ev[i][0], ffn_ev[i][1], 0, 0, 0, 0])
        hip.record(step_ev[i][1])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    step_ms = [hip.elapsed_ms(a, b) for a, b in step_ev]
    ms_per_step = float(np.median(step_ms))
    ffn_ms = float(np.mean([hip.elapsed_ms(a, b) for a, b in ffn_ev]))

    # second, untimed pass with every stage bracketed (diagnostics only)
    reps = min(K, 30)
    if balanced:
        bal_ev = [[hip.create() for _ in range(5)] for _ in range(reps)]
        for evs in bal_ev:
            api.moe_layer_forward_balanced_profiled(run.cfg, run.x, run.W_g, run.bias, run.thr, run.W1, run.W2,
                                                    run.y, run.gsigma, run.tokens, run.kept, run.denom,
                                                    run.loss, ws, evs)
        torch.cuda.synchronize()
        pairs = {"gate": (0, 1), "tiles": (1, 2), "expert_ffn": (2, 3), "combine": (3, 4)}
        stage_ms = {name: float(np.median([hip.elapsed_ms(evs[a], evs[b]) for evs in bal_ev]))
                    for name, (a, b) in pairs.items()}
        used = shape.n
    else:
        all_ev = [[hip.create() for _ in range(10)] for _ in range(reps)]
        for evs in all_ev:
            step(evs)
        torch.cuda.synchronize()
        stage_ms = {name: float(np.median([hip.elapsed_ms(evs[2 * i], evs[2 * i + 1]) for evs in all_ev]))
                    for i, name in enumerate(STAGES)}
        lay = api.moe_get_workspace_layout(run.cfg)
        cnt = ws[lay.counts:lay.counts + 4 * shape.n].view(torch.int32).cpu().numpy()
        used = int((cnt > 0).sum())

    A = shape.T * shape.k
    wbytes = 2 if shape.expert_dtype == "bf16" else 4
    # algorithmic bytes of one expert-kernel launch: every used expert's two matrices once, the
    # gathered fp32 token rows once, the fp32 expert outputs once
    ffn_bytes = used * 2 * shape.d * shape.h * wbytes + A * shape.d * 4 + A * shape.d * 4
    ffn_flops = 4.0 * shape.d * shape.h * A
    ffn_gbs = ffn_bytes / (ffn_ms * 1e-3) / 1e9
    ffn_tflops = ffn_flops / (ffn_ms * 1e-3) / 1e12
    kernel = "ffn_bf16_kernel" if wbytes == 2 else "ffn_f32_mfma_kernel (two launches)"
    tag = shape.name.split("_")[0]
    traffic = read_traffic("ffn_bf16_%s%s_pmc.txt" % (tag, "_balanced" if balanced else ""))
    # which bound binds the expert stage: weight streaming below ~315 rows per expert, the matrix cores above
    mfma_peak = BF16_MFMA_PEAK_TFLOPS if wbytes == 2 else FP32_MFMA_PEAK_TFLOPS
    t_hbm, t_mfma = ffn_bytes / (HBM_PEAK_GBS * 1e9), ffn_flops / (mfma_peak * 1e12)
    if t_mfma > t_hbm:
        roofline = {"kernel": kernel, "bound": "mfma", "achieved": ffn_tflops, "peak": mfma_peak,
                    "unit": "TFLOP/s", "frac": ffn_tflops / mfma_peak, "traffic": traffic,
                    "kernel_ms": ffn_ms, "algorithmic_flops": ffn_flops, "hbm_gbs": ffn_gbs}
    else:
        roofline = {"kernel": kernel, "bound": "hbm", "achieved": ffn_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": ffn_gbs / HBM_PEAK_GBS, "traffic": traffic, "kernel_ms": ffn_ms,
                    "algorithmic_bytes": ffn_bytes, "mfma_tflops": ffn_tflops}

    # every stage against the bound that binds it at the published peaks (diagnostic pass times)
    if shape.hierarchical:
        gate_flops = 4.0 * shape.d * (shape.a * shape.T + shape.b * shape.T * shape.k_primary)
    else:
        gate_flops = 4.0 * shape.d * shape.n * shape.T * (0.5 if balanced else 1.0)
    comb_bytes = A * shape.d * 4 + shape.T * shape.d * 4
    bound_ms = {"gate": gate_flops / (FP32_MFMA_PEAK_TFLOPS * 1e12) * 1e3,
                "expert_ffn": max(t_hbm, t_mfma) * 1e3, "combine": comb_bytes / (HBM_PEAK_GBS * 1e9) * 1e3}
    stage_frac = {s: bound_ms[s] / stage_ms[s] for s in bound_ms if stage_ms.get(s)}

    fwd_bwd = shape.backward or ((shape.hierarchical or balanced) and args.backward)
    out = {
        "metric": "MoE-layer tokens/sec (%s) at d=512,h=1024" % ("fwd+bwd" if fwd_bwd else "fwd"),
        "value": shape.T / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "warmup": warmup, "ms_per_step": ms_per_step,
        "wall_ms_per_step": wall / K * 1e3,
        "step_ms_min_max": [float(min(step_ms)), float(max(step_ms))],
        "timing": "median of %d per-step HIP event pairs after %d warm-up steps" % (K, warmup),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if shape.expert_dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": shape.name, "T": shape.T, "d": shape.d, "h": shape.h, "n": shape.n,
                   "k": shape.k, "experts_used": used,
                   "gating": ("strictly balanced (softmax, batchwise mask)" if balanced else
                              "fp32 noisy top-k, two levels %d x %d" % (shape.a, shape.b) if shape.hierarchical
                              else "fp32 noisy top-k"),
                   "expert_math": "bf16 MFMA, fp32 accumulate" if wbytes == 2 else "fp32"},
        "roofline": roofline,
        "stage_ms": stage_ms,
        "stage_bound_ms": bound_ms,
        "stage_frac_of_bound": stage_frac,
    }
    if args.optimizer and shape.backward and not balanced:
        masters = [run.W1.to(torch.float32), run.W2.to(torch.float32)]
        state = [torch.zeros((shape.n, shape.d), **f32), torch.zeros((shape.n, shape.h), **f32),
                 torch.zeros((shape.n, shape.h), **f32), torch.zeros((shape.n, shape.d), **f32)]
        ows = torch.empty(api.moe_adam_workspace_bytes(run.cfg), dtype=torch.uint8, device="cuda")
        opt_ev = [(hip.create(), hip.create()) for _ in range(6)]
        for i, (e0, e1) in enumerate(opt_ev):
            hip.record(e0)
            api.moe_expert_adam_step(run.cfg, 1e-3, 0.999, 1e-8, i + 1, grads[3], grads[4], masters[0], masters[1],
                                     run.W1, run.W2, state[0], state[1], state[2], state[3], ows,
                                     backward_workspace=bws)
            hip.record(e1)
        torch.cuda.synchronize()
        opt_ms = float(np.mean([hip.elapsed_ms(a, b) for a, b in opt_ev[1:]]))
        elems = 2 * shape.n * shape.d * shape.h
        # gradients read once (their sums of squares come from the weight-gradient kernels), fp32
        # parameters read and written, bf16 copy written
        opt_bytes = elems * (4 + 4 + 4 + 2)
        out["optimizer"] = {"kernel": "moe_expert_adam_step (2 kernels per matrix family, sums of squares "
                                      "taken in the backward pass)", "ms": opt_ms,
                            "algorithmic_bytes": opt_bytes, "bound": "hbm",
                            "achieved": opt_bytes / (opt_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                            "frac": opt_bytes / (opt_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
    if args.epilogue and not balanced:
        # the combine with the layer's tail fused in (sigmoid, dropout, residual), on the rows and
        # gate values the last step left in the workspace; own event pairs, outside the timed region
        drop = 0.4
        keep = G.dev(W.dropout_keep(shape, drop))
        view = lambda off, count, dt: ws[off:off + count * 4].view(dt)
        rows = view(lay.out_sorted, A * shape.d, torch.float32)
        inv = view(lay.inv_perm, A, torch.int32)
        y2 = torch.empty((shape.T, shape.d), **f32)
        epi_ev = [(hip.create(), hip.create()) for _ in range(reps + 2)]
        for e0, e1 in epi_ev:
            hip.record(e0)
            api.moe_combine_epilogue(run.cfg, rows, run.topk_gate, inv, run.x, keep, drop, y2)
            hip.record(e1)
        torch.cuda.synchronize()
        epi_ms = float(np.median([hip.elapsed_ms(a, b) for a, b in epi_ev[2:]]))
        # expert rows and y as in the combine, plus the residual input (fp32) and the dropout draw (bytes)
        epi_bytes = comb_bytes + shape.T * shape.d * 4 + shape.T * shape.d
        out["combine_epilogue"] = {"kernel": "moe_combine_epilogue (sigmoid, dropout %.1f, residual)" % drop,
                                   "ms": epi_ms, "algorithmic_bytes": epi_bytes, "bound": "hbm",
                                   "achieved": epi_bytes / (epi_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                                   "unit": "GB/s", "frac": epi_bytes / (epi_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
    if not args.no_cpu_baseline:
        sample = args.cpu_sample
        if balanced:
            out["cpu_baseline"] = cpu_baseline_balanced(shape, inputs, W1, W2, sample or 8192)
        elif shape.hierarchical:
            out["cpu_baseline"] = cpu_baseline_hier(shape, inputs, W1, W2, dy, sample or 1024, backward)
        else:
            default = {0: 256, 1: 8192, 2: 8192, 4: 16384}.get(cfg_index, 1024)
            out["cpu_baseline"] = cpu_baseline_flat(shape, inputs, W1, W2, dy, sample or default)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=None,
                    help="time only this workload (index into the five); default: config 3 as the headline "
                         "and the other four under \"per_config\"")
    ap.add_argument("--gating", choices=["noisy_topk", "balanced"], default="noisy_topk",
                    help="balanced: the strictly balanced gate of Appendix F on the same workload "
                         "(flat forward configs only; needs --config)")
    ap.add_argument("--backward", action="store_true",
                    help="hierarchical config, or --gating balanced: time forward + backward per step")
    ap.add_argument("--epilogue", action="store_true",
                    help="also time moe_combine_epilogue (combine + sigmoid, dropout, residual) on the step's rows")
    ap.add_argument("--optimizer", action="store_true",
                    help="training config: also time the factored-second-moment Adam step of the expert "
                         "matrices (outside the timed region; reported under \"optimizer\")")
    ap.add_argument("--cpu-sample", type=int, default=None,
                    help="tokens of the workload the oracle is timed on (default per workload: 256 / 8192 / "
                         "8192 / 1024 / 16384 for configs 0 ... 4, up to ten seconds of host time each)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy kernel, so that rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE readings can be scaled by a kernel of known traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs the MoE layer on ONE GPU (one GPU's share of the batch at its "
                 "real shape); --gpus %d is not available: nothing here spans GPUs." % args.gpus)
    if args.gating == "balanced" and args.config is None:
        args.config = 1
    if args.steps < 1 or args.warmup < 0:
        sys.exit("bench.py: --steps must be >= 1 and --warmup >= 0")

    import torch

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    torch.cuda.set_device(0)
    hip = HipEvents()

    if args.pmc_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")     # 1 GiB
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                                                      # one elementwise copy kernel
        torch.cuda.synchronize()
        del src, dst

    if args.config is not None:
        out = run_workload(args.config, args, hip, args.steps, args.warmup)
    else:
        out = run_workload(HEADLINE_CONFIG, args, hip, args.steps, args.warmup)
        torch.cuda.empty_cache()
        per = {}
        for c in (0, 1, 2, 4):
            r = run_workload(c, args, hip, args.steps, args.warmup)
            per[r["config"]["workload"]] = {q: r[q] for q in (
                "metric", "value", "unit", "ms_per_step", "wall_ms_per_step", "steps", "warmup", "dtype", "config",
                "roofline", "stage_ms", "stage_frac_of_bound", "cpu_baseline") if q in r}
            torch.cuda.empty_cache()
        out["per_config"] = per
    print(json.dumps(out))


if __name__ == "__main__":
    main()
