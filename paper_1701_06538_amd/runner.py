"""Buffer plumbing around the C ABI binding: one object per layer variant that allocates the device
tensors a call needs (torch provides the memory) and issues the calls stage by stage or fused.
No arithmetic of the method happens here; every step runs in the HIP library."""
import numpy as np
import torch


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


class FlatRun:
    """One forward pass of the flat layer on the GPU, stage by stage or fused."""

    def __init__(self, api, shape, x, W_g, W_noise, eps, bias, W1, W2, flags=0):
        self.api = api
        self.shape = shape
        self.cfg = api.make_config(shape, flags=flags)
        c = self.cfg
        self.x, self.W_g, self.W_noise = dev(x), dev(W_g), dev(W_noise)
        self.eps = None if eps is None else dev(eps)
        self.bias = None if bias is None else dev(bias)
        self.W1, self.W2 = W1, W2                     # device tensors [n,d,h], [n,h,d]
        T, n, k, d = c.T, c.n, c.k, c.d
        A = T * k
        i32 = dict(dtype=torch.int32, device="cuda")
        f32 = dict(dtype=torch.float32, device="cuda")
        self.topk_idx = torch.full((T, k), -7, **i32)
        self.topk_gate = torch.full((T, k), float("nan"), **f32)
        self.cleanb = torch.full((T, n), float("nan"), **f32)
        self.sp = torch.full((T, n), float("nan"), **f32)
        self.next_idx = torch.full((T,), -7, **i32)
        self.partials = torch.full((max(1, api.moe_gate_partial_rows(c)), 2, n), float("nan"), **f32)
        self.counts = torch.full((n,), -7, **i32)
        self.offsets = torch.full((n + 1,), -7, **i32)
        self.perm = torch.full((max(A, 1),), -7, **i32)
        self.inv_perm = torch.full((max(A, 1),), -7, **i32)
        mt = api.moe_max_tiles(c) + 8
        self.tile_expert = torch.full((mt,), -7, **i32)
        self.tile_row0 = torch.full((mt,), -7, **i32)
        self.num_tiles = torch.full((4,), -7, **i32)
        self.route_ws = torch.empty(max(16, api.moe_route_workspace_bytes(c)), dtype=torch.uint8, device="cuda")
        self.out_sorted = torch.full((max(A, 1), d), float("nan"), **f32)
        self.ffn_ws = torch.empty(max(16, api.moe_ffn_workspace_bytes(c)), dtype=torch.uint8, device="cuda")
        self.aux_ws = torch.empty(max(16, api.moe_aux_workspace_bytes(c)), dtype=torch.uint8, device="cuda")
        self.y = torch.full((max(T, 1), d), float("nan"), **f32)
        self.importance = torch.full((n,), float("nan"), **f32)
        self.load = torch.full((n,), float("nan"), **f32)
        self.losses = torch.full((4,), float("nan"), **f32)

    def gate(self):
        self.api.moe_gate(self.cfg, self.x, self.W_g, self.W_noise, self.bias, self.eps, self.topk_idx,
                          self.topk_gate, self.cleanb, self.sp, self.next_idx, self.partials)

    def route(self, idx=None):
        self.api.moe_route(self.cfg, self.topk_idx if idx is None else idx, self.counts, self.offsets,
                           self.perm, self.inv_perm, self.tile_expert, self.tile_row0, self.num_tiles,
                           self.route_ws)

    def ffn(self):
        self.api.moe_expert_ffn(self.cfg, self.x, self.perm, self.offsets, self.tile_expert, self.tile_row0,
                                self.num_tiles, self.W1, self.W2, self.out_sorted, self.ffn_ws)

    def combine(self):
        self.api.moe_combine(self.cfg, self.out_sorted, self.topk_gate, self.inv_perm, self.y)

    def losses_(self):
        self.api.moe_aux_losses(self.cfg, self.partials, self.importance, self.load, self.losses, self.aux_ws)

    def stages(self):
        self.gate(); self.route(); self.ffn(); self.combine(); self.losses_()
        torch.cuda.synchronize()

    def fused(self):
        ws = torch.empty(self.api.moe_workspace_bytes(self.cfg), dtype=torch.uint8, device="cuda")
        self.workspace = ws
        self.api.moe_layer_forward(self.cfg, self.x, self.W_g, self.W_noise, self.bias, self.eps, self.W1,
                                   self.W2, self.y, self.topk_idx, self.topk_gate, self.importance,
                                   self.load, self.losses, ws)
        torch.cuda.synchronize()


class BalancedRun:
    """One forward pass with strictly balanced gating (Appendix F) on the GPU."""

    def __init__(self, api, shape, x, W_g, bias, thresholds, W1=None, W2=None, flags=0):
        self.api = api
        self.cfg = c = api.make_config(shape, flags=flags)
        T, n, d = c.T, c.n, c.d
        self.m = api.moe_balanced_rows_per_expert(c)
        assert self.m == T * c.k // n
        self.x, self.W_g = dev(x), dev(W_g)
        self.bias = None if bias is None else dev(bias)
        self.thr = None if thresholds is None else dev(thresholds)
        self.W1, self.W2 = W1, W2
        f32 = dict(dtype=torch.float32, device="cuda")
        self.gsigma = torch.full((max(T, 1), n), float("nan"), **f32)
        self.tokens = torch.full((n, max(self.m, 1)), -7, dtype=torch.int32, device="cuda")
        self.kw = (n + 31) // 32
        self.kept = torch.full((max(T, 1), self.kw), 0x5a5a5a5a, dtype=torch.int32, device="cuda")
        self.denom = torch.full((max(T, 1),), float("nan"), **f32)
        self.loss = torch.full((4,), float("nan"), **f32)
        self.y = torch.full((max(T, 1), d), float("nan"), **f32)
        self.ws = torch.empty(max(256, api.moe_balanced_workspace_bytes(c)), dtype=torch.uint8, device="cuda")

    def gate(self):
        self.api.moe_gate_balanced(self.cfg, self.x, self.W_g, self.bias, self.thr, self.gsigma, self.tokens,
                                   self.kept, self.denom, self.loss, self.ws)
        torch.cuda.synchronize()

    def layer(self):
        self.api.moe_layer_forward_balanced(self.cfg, self.x, self.W_g, self.bias, self.thr, self.W1, self.W2,
                                            self.y, self.gsigma, self.tokens, self.kept, self.denom,
                                            self.loss, self.ws)
        torch.cuda.synchronize()

    def kept_mask(self):
        words = self.kept.cpu().numpy().view(np.uint32)
        T, n = self.cfg.T, self.cfg.n
        bits = (words[:, :, None] >> np.arange(32, dtype=np.uint32)[None, None, :]) & 1
        return bits.reshape(words.shape[0], -1)[:T, :n].astype(bool)


class HierRun:
    """One forward pass of the hierarchical layer on the GPU through the C ABI."""

    def __init__(self, api, shape, inputs, W1, W2, flags=0):
        self.api, self.shape = api, shape
        self.cfg = api.make_config(shape, flags=flags)
        x, Wg_p, Wn_p, eps_p, Wg_s, Wn_s, eps_s = inputs
        self.x = dev(x)
        self.Wg_p, self.Wn_p, self.eps_p = dev(Wg_p), dev(Wn_p), dev(eps_p)
        self.Wg_s, self.Wn_s, self.eps_s = dev(Wg_s), dev(Wn_s), dev(eps_s)
        self.W1, self.W2 = W1, W2
        T, n, k, d = shape.T, shape.n, shape.k, shape.d
        i32 = dict(dtype=torch.int32, device="cuda")
        f32 = dict(dtype=torch.float32, device="cuda")
        self.topk_idx = torch.full((T, k), -7, **i32)
        self.topk_gate = torch.full((T, k), float("nan"), **f32)
        self.y = torch.full((T, d), float("nan"), **f32)
        self.importance = torch.full((n,), float("nan"), **f32)
        self.load = torch.full((n,), float("nan"), **f32)
        self.losses = torch.full((4,), float("nan"), **f32)
        self.workspace = torch.empty(api.moe_workspace_bytes(self.cfg), dtype=torch.uint8, device="cuda")
        self.layout = api.moe_get_workspace_layout(self.cfg)

    def ws_view(self, field, count, dtype):
        off = getattr(self.layout, field)
        nbytes = count * torch.tensor([], dtype=dtype).element_size()
        return self.workspace[off:off + nbytes].view(dtype)

    def gate(self):
        self.api.moe_gate_hier(self.cfg, self.x, self.Wg_p, self.Wn_p, self.eps_p, self.Wg_s, self.Wn_s,
                               self.eps_s, self.topk_idx, self.topk_gate, self.workspace)
        torch.cuda.synchronize()

    def forward(self):
        self.api.moe_layer_forward_hier(self.cfg, self.x, self.Wg_p, self.Wn_p, self.eps_p, self.Wg_s,
                                        self.Wn_s, self.eps_s, self.W1, self.W2, self.y, self.topk_idx,
                                        self.topk_gate, self.importance, self.load, self.losses,
                                        self.workspace)
        torch.cuda.synchronize()
