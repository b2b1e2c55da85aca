"""Benchmark of the MoE-layer forward pass on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1] [--no-cpu-baseline]

A step is one pass of the whole hot path (gate -> route -> expert FFN -> combine -> losses,
i.e. moe_layer_forward) over one batch of seeded synthetic input that is already resident in
HBM.  Prints ONE JSON line: tokens/s, the roofline of the dominant kernel (the expert FFN,
timed live with HIP events recorded on the launch stream inside the timed region) and the CPU
oracle's throughput on a bounded sample of the same workload.
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
STAGES = ["gate", "route", "expert_ffn", "combine", "aux_losses"]


class HipEvents:
    """hipEvent_t handles made with the HIP runtime that torch already loaded."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]

    def create(self):
        ev = ctypes.c_void_p()
        err = self.hip.hipEventCreate(ctypes.byref(ev))
        assert err == 0, "hipEventCreate failed: %d" % err
        return ev.value

    def record(self, ev):
        import torch
        self.hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
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


def cpu_baseline(shape, sample_tokens):
    """The oracle as it stands, timed on the host on the first `sample_tokens` tokens of the same
    seeded workload (same gate matrices, noise and expert weights).  Expert weights are inputs:
    they are generated before the clock starts."""
    import numpy as np
    import torch

    import moe_workloads as W
    from oracle import moe_oracle as O

    x, W_g, W_noise, eps = W.gate_inputs(shape)
    x, eps = x[:sample_tokens], eps[:sample_tokens]
    w1 = W.expert_weights_all(shape, 0, range(shape.n))
    w2 = W.expert_weights_all(shape, 1, range(shape.n))

    def wf(e):
        return w1[e].to(torch.float64).numpy(), w2[e].to(torch.float64).numpy()

    t0 = time.perf_counter()
    lg = O.noisy_logits_f32(x, W_g, W_noise, eps)
    fw = O.gate_and_losses(lg, shape.k, shape.w_importance, shape.w_load)
    O.routing(fw.idx, shape.n)
    y = O.moe_output(x, fw.idx, fw.gates, wf, shape.n)
    dt = time.perf_counter() - t0
    assert np.isfinite(y).all()
    try:
        import threadpoolctl
        threads = max([p["num_threads"] for p in threadpoolctl.threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count()
    return {"value": sample_tokens / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": "first %d of %d tokens of the same seeded workload, full forward "
                      "(gate, routing, experts in fp64, combine, losses), %.1f s" % (sample_tokens, shape.T, dt)}


def cpu_baseline_balanced(shape, sample_tokens):
    """The oracle's strictly balanced layer (Appendix F) on the first `sample_tokens` tokens taken as
    a batch of their own (every expert keeps sample_tokens*k/n of them)."""
    import numpy as np
    import torch

    import moe_workloads as W
    from oracle import moe_oracle as O

    x, W_g, _, _ = W.gate_inputs(shape)
    x = x[:sample_tokens]
    w1 = W.expert_weights_all(shape, 0, range(shape.n))
    w2 = W.expert_weights_all(shape, 1, range(shape.n))

    def wf(e):
        return w1[e].to(torch.float64).numpy(), w2[e].to(torch.float64).numpy()

    t0 = time.perf_counter()
    _, X = O.softmax_gate_f32(x, W_g)
    mask, _ = O.batchwise_mask(X, sample_tokens * shape.k // shape.n)
    Gm, _ = O.balanced_gates(X, mask)
    y = O.balanced_output(x, Gm, wf)
    dt = time.perf_counter() - t0
    assert np.isfinite(y).all()
    try:
        import threadpoolctl
        threads = max([p["num_threads"] for p in threadpoolctl.threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count()
    return {"value": sample_tokens / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": "first %d of %d tokens of the same seeded workload as one balanced batch, full forward "
                      "(softmax gate, batchwise mask, experts in fp64, combine), %.1f s" % (sample_tokens, shape.T, dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=1, help="index into the five workloads (default 1)")
    ap.add_argument("--gating", choices=["noisy_topk", "balanced"], default="noisy_topk",
                    help="balanced: the strictly balanced gate of Appendix F on the same workload "
                         "(flat forward configs only)")
    ap.add_argument("--backward", action="store_true",
                    help="hierarchical config, or --gating balanced: time forward + backward per step")
    ap.add_argument("--optimizer", action="store_true",
                    help="training configs: also time the factored-second-moment Adam step of the expert "
                         "matrices (outside the timed region; reported under \"optimizer\")")
    ap.add_argument("--cpu-sample", type=int, default=None,
                    help="tokens of the workload the oracle is timed on (default: all 8192 of the metric's "
                         "workload, a few seconds of host time; 2048 for the other configs)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy kernel, so that rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE readings can be scaled by a kernel of known traffic")
    args = ap.parse_args()
    if args.cpu_sample is None:
        args.cpu_sample = 8192 if args.config == 1 else 2048
    if args.steps is None:
        args.steps = 200 if args.config <= 1 else 20
    if args.gpus != 1:
        sys.exit("bench.py: this build runs the MoE layer on ONE GPU (one GPU's share of the batch at its "
                 "real shape); --gpus %d is not available: nothing here spans GPUs." % args.gpus)

    import numpy as np
    import torch

    import moe_workloads as W
    from paper_1701_06538_amd import api     # raises if the HIP library is missing: no fallback
    from tests import gpu_harness as G

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    torch.cuda.set_device(0)
    shape = W.CONFIGS[args.config]
    hip = HipEvents()
    balanced = args.gating == "balanced"
    if balanced:
        if shape.hierarchical or shape.backward:
            sys.exit("bench.py: --gating balanced runs the flat forward configs only")
        x, W_g, _, _, bias = G.flat_inputs(shape, with_bias=shape.zipf_beta > 0)
        W1, W2 = G.device_weights(shape, chunk=256)
        thr = np.full((shape.n,), 1.0 / shape.n, np.float32)
        run = G.BalancedRun(api, shape, x, W_g, bias, thr, W1, W2,
                            flags=api.MOE_FLAG_SAVE_HIDDEN if args.backward else 0)
        ws = run.ws

        if args.backward:
            dy = G.dev(W.upstream_grad(shape))
            f32 = dict(dtype=torch.float32, device="cuda")
            bg = [torch.empty((shape.T, shape.d), **f32), torch.empty((shape.d, shape.n), **f32),
                  torch.empty((shape.n, shape.d, shape.h), **f32), torch.empty((shape.n, shape.h, shape.d), **f32)]
            bbws = torch.empty(api.moe_backward_balanced_workspace_bytes(run.cfg), dtype=torch.uint8, device="cuda")

        def step(events=None):
            ev = None if events is None else [0, 0, events[4], events[5], 0]
            api.moe_layer_forward_balanced_profiled(run.cfg, run.x, run.W_g, run.bias, run.thr, run.W1, run.W2,
                                                    run.y, run.gsigma, run.tokens, run.kept, run.denom,
                                                    run.loss, ws, ev)
            if args.backward:
                api.moe_layer_backward_balanced(run.cfg, run.x, run.W_g, run.thr, run.W1, run.W2, dy, run.gsigma,
                                                run.tokens, run.kept, run.denom, ws, 0.1, bg[0], bg[1], bg[2],
                                                bg[3], bbws)
    elif shape.hierarchical:
        inputs = W.hier_gate_inputs(shape)
        W1, W2 = G.device_weights(shape, chunk=256)
        run = G.HierRun(api, shape, inputs, W1, W2, flags=api.MOE_FLAG_SAVE_HIDDEN if args.backward else 0)
        ws = run.workspace
        if args.backward:
            dy = G.dev(W.upstream_grad(shape))
            f32 = dict(dtype=torch.float32, device="cuda")
            hg = [torch.empty((shape.T, shape.d), **f32), torch.empty((shape.d, shape.a), **f32),
                  torch.empty((shape.d, shape.a), **f32), torch.empty((shape.a, shape.d, shape.b), **f32),
                  torch.empty((shape.a, shape.d, shape.b), **f32), torch.empty((shape.n, shape.d, shape.h), **f32),
                  torch.empty((shape.n, shape.h, shape.d), **f32)]
            hbws = torch.empty(api.moe_backward_hier_workspace_bytes(run.cfg), dtype=torch.uint8, device="cuda")

        def step(events=None):
            if events is not None and events[4]:
                hip.record(events[4])
            api.moe_layer_forward_hier(run.cfg, run.x, run.Wg_p, run.Wn_p, run.eps_p, run.Wg_s, run.Wn_s,
                                       run.eps_s, run.W1, run.W2, run.y, run.topk_idx, run.topk_gate,
                                       run.importance, run.load, run.losses, ws)
            if events is not None and events[5]:
                hip.record(events[5])
            if args.backward:
                api.moe_layer_backward_hier(run.cfg, run.x, run.Wg_p, run.Wn_p, run.eps_p, run.Wg_s, run.Wn_s,
                                            run.eps_s, run.W1, run.W2, dy, run.topk_idx, run.topk_gate, ws, hg[0],
                                            hg[1], hg[2], hg[3], hg[4], hg[5], hg[6], hbws)
    else:
        x, W_g, W_noise, eps, bias = G.flat_inputs(shape, with_bias=shape.zipf_beta > 0)
        W1, W2 = G.device_weights(shape)
        run = G.FlatRun(api, shape, x, W_g, W_noise, eps, bias, W1, W2,
                        flags=(api.MOE_FLAG_SAVE_HIDDEN if shape.backward else 0)
                        | (api.MOE_FLAG_ADAM_MOMENTS if (shape.backward and args.optimizer) else 0))
        ws = torch.empty(api.moe_workspace_bytes(run.cfg), dtype=torch.uint8, device="cuda")
        if shape.backward:
            dy = G.dev(W.upstream_grad(shape))
            f32 = dict(dtype=torch.float32, device="cuda")
            grads = [torch.empty((shape.T, shape.d), **f32), torch.empty((shape.d, shape.n), **f32),
                     torch.empty((shape.d, shape.n), **f32), torch.empty((shape.n, shape.d, shape.h), **f32),
                     torch.empty((shape.n, shape.h, shape.d), **f32)]
            bws = torch.empty(api.moe_backward_workspace_bytes(run.cfg), dtype=torch.uint8, device="cuda")

        def step(events=None):
            api.moe_layer_forward_profiled(run.cfg, run.x, run.W_g, run.W_noise, run.bias, run.eps, run.W1,
                                           run.W2, run.y, run.topk_idx, run.topk_gate, run.importance,
                                           run.load, run.losses, ws, events)
            if shape.backward:
                api.moe_layer_backward(run.cfg, run.x, run.W_g, run.W_noise, run.eps, run.W1, run.W2, dy,
                                       run.topk_idx, run.topk_gate, ws, grads[0], grads[1], grads[2],
                                       grads[3], grads[4], bws)

    if args.pmc_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")     # 1 GiB
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                                                      # one elementwise copy kernel
        torch.cuda.synchronize()
        del src, dst

    if args.config > 1:
        args.warmup = min(args.warmup, 3)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # timed region: K steps, each with one event pair around the expert kernel
    K = args.steps
    ffn_ev = [(hip.create(), hip.create()) for _ in range(K)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        step([0, 0, 0, 0, ffn_ev[i][0], ffn_ev[i][1], 0, 0, 0, 0])   # hierarchical: brackets the whole call
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ffn_ms = float(np.mean([hip.elapsed_ms(a, b) for a, b in ffn_ev]))

    # second, untimed pass with every stage bracketed (diagnostics only)
    stage_ms = None
    if not shape.hierarchical and not balanced:
        all_ev = [[hip.create() for _ in range(10)] for _ in range(min(K, 50))]
        for evs in all_ev:
            step(evs)
        torch.cuda.synchronize()
        stage_ms = {name: float(np.mean([hip.elapsed_ms(evs[2 * i], evs[2 * i + 1]) for evs in all_ev]))
                    for i, name in enumerate(STAGES)}

    if balanced:
        used = shape.n
        bal_ev = [[hip.create() for _ in range(5)] for _ in range(min(K, 50))]
        for evs in bal_ev:
            api.moe_layer_forward_balanced_profiled(run.cfg, run.x, run.W_g, run.bias, run.thr, run.W1, run.W2,
                                                    run.y, run.gsigma, run.tokens, run.kept, run.denom,
                                                    run.loss, ws, evs)
        torch.cuda.synchronize()
        pairs = {"gate": (0, 1), "tiles": (1, 2), "experts": (2, 3), "combine": (3, 4)}
        stage_ms = {name: float(np.mean([hip.elapsed_ms(evs[a], evs[b]) for evs in bal_ev]))
                    for name, (a, b) in pairs.items()}
    else:
        lay = run.api.moe_get_workspace_layout(run.cfg)
        cnt = ws[lay.counts:lay.counts + 4 * shape.n].view(torch.int32).cpu().numpy()
        used = int((cnt > 0).sum())
    A = shape.T * shape.k
    wbytes = 2 if shape.expert_dtype == "bf16" else 4
    # algorithmic bytes of one expert-kernel launch: every used expert's two matrices once, the
    # gathered fp32 token rows once, the fp32 expert outputs once
    ffn_bytes = used * 2 * shape.d * shape.h * wbytes + A * shape.d * 4 + A * shape.d * 4
    ffn_flops = 4.0 * shape.d * shape.h * A
    achieved = ffn_bytes / (ffn_ms * 1e-3) / 1e9
    ms_per_step = elapsed / K * 1e3

    out = {
        "metric": "MoE-layer tokens/sec (%s) at d=512,h=1024" % (
            "fwd+bwd" if (shape.backward or ((shape.hierarchical or balanced) and args.backward)) else "fwd"),
        "value": shape.T / (elapsed / K),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if shape.expert_dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": shape.name, "T": shape.T, "d": shape.d, "h": shape.h, "n": shape.n,
                   "k": shape.k, "experts_used": used,
                   "gating": "strictly balanced (softmax, batchwise mask)" if balanced else "fp32 noisy top-k",
                   "expert_math": "bf16 MFMA, fp32 accumulate" if wbytes == 2 else "fp32"},
        "roofline": {"kernel": "ffn_bf16_kernel" if wbytes == 2 else "ffn_f32_mfma_kernel (two launches)",
                     "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": read_traffic("ffn_bf16_%s_pmc.txt" % shape.name.split("_")[0]),
                     "kernel_ms": ffn_ms, "algorithmic_bytes": ffn_bytes,
                     "mfma_tflops": ffn_flops / (ffn_ms * 1e-3) / 1e12},
        "stage_ms": stage_ms,
    }
    if shape.hierarchical:
        out["roofline"].update({"kernel": "moe_layer_forward_hier (whole call)", "note": "event pair brackets the whole layer"})
    if args.optimizer and shape.backward:
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
    if balanced:
        out["roofline"]["traffic"] = read_traffic("ffn_bf16_%s_balanced_pmc.txt" % shape.name.split("_")[0])
    if not args.no_cpu_baseline and balanced:
        out["cpu_baseline"] = cpu_baseline_balanced(shape, min(args.cpu_sample, shape.T))
    elif not args.no_cpu_baseline and not shape.hierarchical and not shape.backward:
        out["cpu_baseline"] = cpu_baseline(shape, min(args.cpu_sample, shape.T))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
