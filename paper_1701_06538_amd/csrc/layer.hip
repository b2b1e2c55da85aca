// moe_layer_forward: a1..a5 enqueued back to back on one stream.  Nothing returns to the host
// between stages: per-expert counts, offsets and the row-tile table are produced and consumed
// on the device, and the expert kernel is launched over an upper bound of tiles.
#include "stages.h"

namespace moe {

static size_t align_up(size_t v) { return (v + 255) & ~(size_t)255; }

int workspace_layout(const moe_config *cfg, moe_workspace_layout *L) {
    int st = check_config(cfg);
    if (st != MOE_OK) return st;
    *L = moe_workspace_layout{};
    const bool hier = cfg->a > 0;
    const size_t T = (size_t)cfg->T, n = (size_t)cfg->n, A = T * (size_t)cfg->k;
    const size_t MT = (size_t)moe_max_tiles(cfg) + 8;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off = align_up(off + (bytes ? bytes : 1));
        return at;
    };
    // the gate whose [rows, cols] logits feed the final top-k: the flat gate, or the secondary one
    const size_t gate_n = hier ? (size_t)cfg->b : n;
    const size_t gate_rows = hier ? T * (size_t)cfg->k_primary : T;
    const size_t MTp = hier ? (size_t)ceil_div((int64_t)gate_rows, kGateBM) + cfg->a + 8 : 0;
    size_t part_rows;
    if (hier) part_rows = MTp * (size_t)(kGateBM / gate_rows_per_block((int64_t)gate_rows, (int)gate_n));
    else part_rows = (size_t)moe_gate_partial_rows(cfg);
    L->cleanb = take(gate_rows * gate_n * 4);
    L->sp = take(gate_rows * gate_n * 4);
    L->next_idx = take(gate_rows * 4);
    L->partials = take(part_rows * 2 * gate_n * 4);
    L->counts = take(n * 4);
    L->offsets = take((n + 1) * 4);
    L->perm = take(A * 4);
    L->inv_perm = take(A * 4);
    L->tile_expert = take(MT * 4);
    L->tile_row0 = take(MT * 4);
    L->num_tiles = take(16);
    L->route_ws = take(route_ws_bytes((int64_t)A, cfg->n));
    L->out_sorted = take(A * (size_t)cfg->d * 4);
    L->ffn_ws = take(moe_ffn_workspace_bytes(cfg));
    L->aux_ws = take(hier ? 2 * n * 8 : aux_ws_bytes(moe_gate_partial_rows(cfg), cfg->n));
    L->hidden = L->xs = (size_t)-1;
    if ((cfg->flags & MOE_FLAG_SAVE_HIDDEN) && cfg->expert_dtype == MOE_DTYPE_BF16) {
        L->hidden = take(A * (size_t)cfg->h * 2);
        if (!hier) L->xs = take(A * (size_t)cfg->d * 2);   // the routed input rows as the experts saw them
    }
    if (hier) {
        const size_t a = (size_t)cfg->a, kp = (size_t)cfg->k_primary, ks = (size_t)cfg->k_secondary;
        const size_t Ap = T * kp;
        const int64_t prow = ceil_div((int64_t)T, gate_rows_per_block((int64_t)T, cfg->a));
        L->p_cleanb = take(T * a * 4);
        L->p_sp = take(T * a * 4);
        L->p_next_idx = take(T * 4);
        L->p_partials = take((size_t)prow * 2 * a * 4);
        L->p_idx = take(Ap * 4);
        L->p_gate = take(Ap * 4);
        L->p_counts = take(a * 4);
        L->p_offsets = take((a + 1) * 4);
        L->p_perm = take(Ap * 4);
        L->p_inv_perm = take(Ap * 4);
        L->p_tile_group = take(MTp * 4);
        L->p_tile_row0 = take(MTp * 4);
        L->p_num_tiles = take(16);
        L->p_tile_offsets = take((a + 1) * 4);
        L->p_route_ws = take(route_ws_bytes((int64_t)Ap, cfg->a));
        L->p_aux_ws = take(aux_ws_bytes(prow, cfg->a));
        L->s_idx = take(Ap * ks * 4);
        L->s_gate = take(Ap * ks * 4);
    }
    L->total = off;
    return MOE_OK;
}

}  // namespace moe

using namespace moe;

extern "C" size_t moe_aux_workspace_bytes(const moe_config *cfg) {
    if (check_config(cfg) != MOE_OK) return 0;
    return aux_ws_bytes(moe_gate_partial_rows(cfg), cfg->n);
}

extern "C" int moe_aux_losses(const moe_config *cfg, const float *partials, float *importance,
                              float *load, float *losses, void *workspace, void *stream) {
    int st = check_config(cfg);
    if (st != MOE_OK) return st;
    if (cfg->a != 0) return MOE_EINVAL;
    if (!partials || !importance || !load || !losses || !workspace) return MOE_EINVAL;
    return launch_aux_losses(partials, moe_gate_partial_rows(cfg), cfg->n, cfg->w_importance,
                             cfg->w_load, importance, load, losses, (double *)workspace,
                             (hipStream_t)stream);
}

extern "C" int moe_get_workspace_layout(const moe_config *cfg, moe_workspace_layout *out) {
    if (!out) return MOE_EINVAL;
    return workspace_layout(cfg, out);
}

extern "C" size_t moe_workspace_bytes(const moe_config *cfg) {
    moe_workspace_layout L;
    if (workspace_layout(cfg, &L) != MOE_OK) return 0;
    return L.total;
}

__global__ void fill_zero_kernel(float *p, int64_t count) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < count) p[i] = 0.f;
}

// T = 0: nothing to gate or route.  Counts, offsets and the tile table are zeroed (so the
// workspace is consistent), Importance = Load = 0 and the losses are reported as 0.
static int forward_empty(const moe_config *cfg, const moe_workspace_layout &L, char *ws,
                         float *importance, float *load, float *losses, void *stream) {
    RouteArgs ra{};
    ra.A = 0; ra.n = cfg->n; ra.tile_rows = moe_tile_rows(cfg);
    ra.counts = (int32_t *)(ws + L.counts); ra.offsets = (int32_t *)(ws + L.offsets);
    ra.perm = (int32_t *)(ws + L.perm); ra.inv_perm = (int32_t *)(ws + L.inv_perm);
    ra.tile_expert = (int32_t *)(ws + L.tile_expert); ra.tile_row0 = (int32_t *)(ws + L.tile_row0);
    ra.num_tiles = (int32_t *)(ws + L.num_tiles);
    ra.hist = (int32_t *)(ws + L.route_ws);
    int st = launch_route(ra, (hipStream_t)stream);
    if (st != MOE_OK) return st;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)ceil_div(cfg->n, 256)), dim3(256), 0,
                       (hipStream_t)stream, importance, (int64_t)cfg->n);
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)ceil_div(cfg->n, 256)), dim3(256), 0,
                       (hipStream_t)stream, load, (int64_t)cfg->n);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(1), dim3(256), 0, (hipStream_t)stream, losses, (int64_t)4);
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}

static int record(void *const *ev, int i, void *stream) {
    if (!ev || !ev[i]) return MOE_OK;
    MOE_HIP_TRY(hipEventRecord((hipEvent_t)ev[i], (hipStream_t)stream));
    return MOE_OK;
}

extern "C" int moe_layer_forward_profiled(const moe_config *cfg, const float *x, const float *W_g,
                                          const float *W_noise, const float *gate_bias,
                                          const float *eps, const void *W1, const void *W2,
                                          float *y, int32_t *topk_idx, float *topk_gate,
                                          float *importance, float *load, float *losses,
                                          void *workspace, size_t workspace_bytes,
                                          void *const *stage_events, void *stream) {
    moe_workspace_layout L;
    int st = workspace_layout(cfg, &L);
    if (st != MOE_OK) return st;
    if (cfg->a != 0) return MOE_EINVAL;
    if (!importance || !load || !losses || !workspace || !aligned16(workspace)) return MOE_EINVAL;
    if (workspace_bytes < L.total) return MOE_EWORKSPACE;
    char *ws = (char *)workspace;
    if (cfg->T == 0) return forward_empty(cfg, L, ws, importance, load, losses, stream);
    if (!x || !W_g || !W_noise || !W1 || !W2 || !y || !topk_idx || !topk_gate) return MOE_EINVAL;
    if (!aligned16(x) || !aligned16(y) || !aligned16(W1) || !aligned16(W2)) return MOE_EINVAL;
    float *cleanb = (float *)(ws + L.cleanb), *sp = (float *)(ws + L.sp);
    int32_t *next_idx = (int32_t *)(ws + L.next_idx);
    float *partials = (float *)(ws + L.partials);
    int32_t *counts = (int32_t *)(ws + L.counts), *offsets = (int32_t *)(ws + L.offsets);
    int32_t *perm = (int32_t *)(ws + L.perm), *inv_perm = (int32_t *)(ws + L.inv_perm);
    int32_t *tile_expert = (int32_t *)(ws + L.tile_expert), *tile_row0 = (int32_t *)(ws + L.tile_row0);
    int32_t *num_tiles = (int32_t *)(ws + L.num_tiles);
    float *out_sorted = (float *)(ws + L.out_sorted);
    void *const *ev = stage_events;

#define MOE_STAGE(i, call)                                        \
    if ((st = record(ev, 2 * (i), stream)) != MOE_OK) return st;  \
    if ((st = (call)) != MOE_OK) return st;                       \
    if ((st = record(ev, 2 * (i) + 1, stream)) != MOE_OK) return st;

    MOE_STAGE(0, moe_gate(cfg, x, W_g, W_noise, gate_bias, eps, topk_idx, topk_gate, cleanb, sp,
                          next_idx, partials, stream))
    // Few experts and a short assignment list: the stages between the big kernels are launch
    // bound, so the loss sums share a launch with routing and their last step shares one with
    // the combine (stage 4 is then empty).
    const bool fuse = route_is_small((int64_t)cfg->T * cfg->k, cfg->n) && aligned16(out_sorted);
    const int64_t prow = moe_gate_partial_rows(cfg);
    if (fuse) {
        RouteArgs ra{};
        ra.idx = topk_idx; ra.A = (int64_t)cfg->T * cfg->k; ra.n = cfg->n;
        ra.tile_rows = moe_tile_rows(cfg);
        ra.counts = counts; ra.offsets = offsets; ra.perm = perm; ra.inv_perm = inv_perm;
        ra.tile_expert = tile_expert; ra.tile_row0 = tile_row0; ra.num_tiles = num_tiles;
        ra.tile_offsets = nullptr;
        ra.hist = (int32_t *)(ws + L.route_ws);
        MOE_STAGE(1, launch_route_small_sums(ra, partials, prow, (double *)(ws + L.aux_ws),
                                             (hipStream_t)stream))
    } else {
        MOE_STAGE(1, moe_route(cfg, topk_idx, counts, offsets, perm, inv_perm, tile_expert, tile_row0,
                               num_tiles, ws + L.route_ws, stream))
    }
    MOE_STAGE(2, expert_ffn_with_hidden(cfg, x, perm, offsets, tile_expert, tile_row0, num_tiles, W1, W2,
                                        out_sorted, ws + L.ffn_ws,
                                        L.hidden == (size_t)-1 ? nullptr : (uint16_t *)(ws + L.hidden),
                                        (hipStream_t)stream,
                                        L.xs == (size_t)-1 ? nullptr : (uint16_t *)(ws + L.xs)))
    if (fuse) {
        MOE_STAGE(3, launch_combine_losses(out_sorted, topk_gate, inv_perm, y, cfg->T, cfg->d, cfg->k,
                                           prow, cfg->n, (double *)(ws + L.aux_ws), cfg->w_importance,
                                           cfg->w_load, importance, load, losses, (hipStream_t)stream))
        MOE_STAGE(4, MOE_OK)
    } else {
        MOE_STAGE(3, moe_combine(cfg, out_sorted, topk_gate, inv_perm, y, stream))
        MOE_STAGE(4, moe_aux_losses(cfg, partials, importance, load, losses, ws + L.aux_ws, stream))
    }
#undef MOE_STAGE
    return MOE_OK;
}

extern "C" int moe_layer_forward(const moe_config *cfg, const float *x, const float *W_g,
                                 const float *W_noise, const float *gate_bias, const float *eps,
                                 const void *W1, const void *W2, float *y, int32_t *topk_idx,
                                 float *topk_gate, float *importance, float *load, float *losses,
                                 void *workspace, size_t workspace_bytes, void *stream) {
    return moe_layer_forward_profiled(cfg, x, W_g, W_noise, gate_bias, eps, W1, W2, y, topk_idx,
                                      topk_gate, importance, load, losses, workspace,
                                      workspace_bytes, nullptr, stream);
}

// ---------------------------------------------------------------------------------------
// hierarchical layer (Appendix B)
// ---------------------------------------------------------------------------------------
extern "C" int moe_gate_hier(const moe_config *cfg, const float *x, const float *Wg_p,
                             const float *Wn_p, const float *eps_p, const float *Wg_s,
                             const float *Wn_s, const float *eps_s, int32_t *topk_idx,
                             float *topk_gate, void *workspace, size_t workspace_bytes,
                             void *stream) {
    moe_workspace_layout L;
    int st = workspace_layout(cfg, &L);
    if (st != MOE_OK) return st;
    if (cfg->a <= 0) return MOE_EINVAL;
    if (!x || !Wg_p || !Wn_p || !Wg_s || !Wn_s || !topk_idx || !topk_gate || !workspace)
        return MOE_EINVAL;
    if (!aligned16(x) || !aligned16(Wg_p) || !aligned16(Wn_p) || !aligned16(Wg_s) ||
        !aligned16(Wn_s) || !aligned16(workspace) || (eps_p && !aligned16(eps_p)) ||
        (eps_s && !aligned16(eps_s)))
        return MOE_EINVAL;
    if (workspace_bytes < L.total) return MOE_EWORKSPACE;
    if ((st = check_gate_level(cfg->T, cfg->d, cfg->a, cfg->k_primary)) != MOE_OK) return st;
    if ((st = check_gate_level((int64_t)cfg->T * cfg->k_primary, cfg->d, cfg->b, cfg->k_secondary)) != MOE_OK)
        return st;
    hipStream_t s = (hipStream_t)stream;
    char *ws = (char *)workspace;
    const int64_t T = cfg->T, Ap = T * cfg->k_primary;
    float *p_cleanb = (float *)(ws + L.p_cleanb), *p_sp = (float *)(ws + L.p_sp);
    int32_t *p_idx = (int32_t *)(ws + L.p_idx);
    float *p_gate = (float *)(ws + L.p_gate);
    int32_t *p_offsets = (int32_t *)(ws + L.p_offsets), *p_perm = (int32_t *)(ws + L.p_perm);
    int32_t *p_tile_group = (int32_t *)(ws + L.p_tile_group), *p_tile_row0 = (int32_t *)(ws + L.p_tile_row0);
    int32_t *p_num_tiles = (int32_t *)(ws + L.p_num_tiles);

    // primary gate over the a groups
    LogitsArgs la{};
    la.x = x; la.Wg = Wg_p; la.Wn = Wn_p; la.cleanb = p_cleanb; la.sp = p_sp;
    la.R = T; la.d = cfg->d; la.n = cfg->a;
    if ((st = launch_gate_logits(la, ceil_div(T, kGateBM), s)) != MOE_OK) return st;
    TopkArgs ta{};
    ta.cleanb = p_cleanb; ta.sp = p_sp; ta.eps = eps_p; ta.R = T; ta.n = cfg->a; ta.k = cfg->k_primary;
    ta.idx = p_idx; ta.gate = p_gate; ta.next_idx = (int32_t *)(ws + L.p_next_idx);
    ta.partials = (float *)(ws + L.p_partials);
    ta.rows_per_block = gate_rows_per_block(T, cfg->a);
    if ((st = launch_gate_topk(ta, ceil_div(T, ta.rows_per_block), s)) != MOE_OK) return st;

    // X^(i): rows grouped by primary group, in 128-row tiles that never straddle groups
    RouteArgs ra{};
    ra.idx = p_idx; ra.A = Ap; ra.n = cfg->a; ra.tile_rows = kGateBM;
    ra.counts = (int32_t *)(ws + L.p_counts); ra.offsets = p_offsets; ra.perm = p_perm;
    ra.inv_perm = (int32_t *)(ws + L.p_inv_perm);
    ra.tile_expert = p_tile_group; ra.tile_row0 = p_tile_row0; ra.num_tiles = p_num_tiles;
    ra.tile_offsets = (int32_t *)(ws + L.p_tile_offsets);
    ra.hist = (int32_t *)(ws + L.p_route_ws);
    if ((st = launch_route(ra, s)) != MOE_OK) return st;

    // secondary gates, each on its own rows and with its own matrices
    const int64_t max_tiles_p = ceil_div(Ap, kGateBM) + cfg->a;
    float *s_cleanb = (float *)(ws + L.cleanb), *s_sp = (float *)(ws + L.sp);
    LogitsArgs lb{};
    lb.x = x; lb.Wg = Wg_s; lb.Wn = Wn_s; lb.cleanb = s_cleanb; lb.sp = s_sp;
    lb.R = Ap; lb.d = cfg->d; lb.n = cfg->b;
    lb.row_src = p_perm; lb.row_div = cfg->k_primary;
    lb.tile_group = p_tile_group; lb.tile_row0 = p_tile_row0; lb.num_tiles = p_num_tiles;
    lb.group_offsets = p_offsets;
    if ((st = launch_gate_logits(lb, max_tiles_p, s)) != MOE_OK) return st;
    TopkArgs tb{};
    tb.cleanb = s_cleanb; tb.sp = s_sp; tb.eps = eps_s; tb.R = Ap; tb.n = cfg->b; tb.k = cfg->k_secondary;
    tb.row_map = p_perm;
    tb.tile_row0 = p_tile_row0; tb.num_tiles = p_num_tiles; tb.tile_group = p_tile_group;
    tb.group_offsets = p_offsets;
    tb.idx = (int32_t *)(ws + L.s_idx); tb.gate = (float *)(ws + L.s_gate);
    tb.next_idx = (int32_t *)(ws + L.next_idx); tb.partials = (float *)(ws + L.partials);
    tb.rows_per_block = gate_rows_per_block(Ap, cfg->b);
    if ((st = launch_gate_topk(tb, max_tiles_p * (kGateBM / tb.rows_per_block), s)) != MOE_OK) return st;

    return launch_hier_compose(p_idx, p_gate, tb.idx, tb.gate, T, cfg->k_primary, cfg->k_secondary,
                               cfg->b, topk_idx, topk_gate, s);
}

extern "C" int moe_aux_losses_hier(const moe_config *cfg, const float *topk_gate, const int32_t *perm,
                                   const int32_t *offsets, void *workspace, size_t workspace_bytes,
                                   float *importance, float *load, float *losses, void *stream) {
    moe_workspace_layout L;
    int st = workspace_layout(cfg, &L);
    if (st != MOE_OK) return st;
    if (cfg->a <= 0) return MOE_EINVAL;
    if (!topk_gate || !perm || !offsets || !workspace || !importance || !load || !losses)
        return MOE_EINVAL;
    if (workspace_bytes < L.total) return MOE_EWORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    char *ws = (char *)workspace;
    const int64_t T = cfg->T, Ap = T * cfg->k_primary;
    const int64_t prow = ceil_div(T, gate_rows_per_block(T, cfg->a));
    double *p_sums = (double *)(ws + L.p_aux_ws);
    st = launch_partial_sums((const float *)(ws + L.p_partials), prow, cfg->a, p_sums, s);
    if (st != MOE_OK) return st;
    HierLossArgs ha{};
    ha.gate = topk_gate; ha.perm = perm; ha.offsets = offsets;
    ha.p_sums = p_sums; ha.s_partials = (const float *)(ws + L.partials);
    ha.p_counts = (const int32_t *)(ws + L.p_counts);
    ha.p_tile_offsets = (const int32_t *)(ws + L.p_tile_offsets);
    ha.a = cfg->a; ha.b = cfg->b; ha.sub = kGateBM / gate_rows_per_block(Ap, cfg->b);
    ha.sums64 = (double *)(ws + L.aux_ws);
    ha.importance = importance; ha.load = load;
    return launch_hier_losses(ha, cfg->w_importance, cfg->w_load, losses, s);
}

extern "C" int moe_layer_forward_hier_profiled(const moe_config *cfg, const float *x, const float *Wg_p,
                                               const float *Wn_p, const float *eps_p, const float *Wg_s,
                                               const float *Wn_s, const float *eps_s, const void *W1,
                                               const void *W2, float *y, int32_t *topk_idx,
                                               float *topk_gate, float *importance, float *load,
                                               float *losses, void *workspace, size_t workspace_bytes,
                                               void *const *stage_events, void *stream) {
    moe_workspace_layout L;
    int st = workspace_layout(cfg, &L);
    if (st != MOE_OK) return st;
    if (cfg->a <= 0) return MOE_EINVAL;
    if (!W1 || !W2 || !y || !importance || !load || !losses || !workspace) return MOE_EINVAL;
    if (!aligned16(y) || !aligned16(W1) || !aligned16(W2)) return MOE_EINVAL;
    if (workspace_bytes < L.total) return MOE_EWORKSPACE;
    char *ws = (char *)workspace;
    void *const *ev = stage_events;
    int32_t *counts = (int32_t *)(ws + L.counts), *offsets = (int32_t *)(ws + L.offsets);
    int32_t *perm = (int32_t *)(ws + L.perm), *inv_perm = (int32_t *)(ws + L.inv_perm);
    int32_t *tile_expert = (int32_t *)(ws + L.tile_expert), *tile_row0 = (int32_t *)(ws + L.tile_row0);
    int32_t *num_tiles = (int32_t *)(ws + L.num_tiles);
    float *out_sorted = (float *)(ws + L.out_sorted);
#define MOE_STAGE(i, call)                                        \
    if ((st = record(ev, 2 * (i), stream)) != MOE_OK) return st;  \
    if ((st = (call)) != MOE_OK) return st;                       \
    if ((st = record(ev, 2 * (i) + 1, stream)) != MOE_OK) return st;
    MOE_STAGE(0, moe_gate_hier(cfg, x, Wg_p, Wn_p, eps_p, Wg_s, Wn_s, eps_s, topk_idx, topk_gate, workspace,
                               workspace_bytes, stream))
    MOE_STAGE(1, moe_route(cfg, topk_idx, counts, offsets, perm, inv_perm, tile_expert, tile_row0, num_tiles,
                           ws + L.route_ws, stream))
    MOE_STAGE(2, expert_ffn_with_hidden(cfg, x, perm, offsets, tile_expert, tile_row0, num_tiles, W1, W2,
                                        out_sorted, ws + L.ffn_ws,
                                        L.hidden == (size_t)-1 ? nullptr : (uint16_t *)(ws + L.hidden),
                                        (hipStream_t)stream))
    MOE_STAGE(3, moe_combine(cfg, out_sorted, topk_gate, inv_perm, y, stream))
    MOE_STAGE(4, moe_aux_losses_hier(cfg, topk_gate, perm, offsets, workspace, workspace_bytes, importance,
                                     load, losses, stream))
#undef MOE_STAGE
    return MOE_OK;
}

extern "C" int moe_layer_forward_hier(const moe_config *cfg, const float *x, const float *Wg_p,
                                      const float *Wn_p, const float *eps_p, const float *Wg_s,
                                      const float *Wn_s, const float *eps_s, const void *W1,
                                      const void *W2, float *y, int32_t *topk_idx, float *topk_gate,
                                      float *importance, float *load, float *losses, void *workspace,
                                      size_t workspace_bytes, void *stream) {
    return moe_layer_forward_hier_profiled(cfg, x, Wg_p, Wn_p, eps_p, Wg_s, Wn_s, eps_s, W1, W2, y, topk_idx,
                                           topk_gate, importance, load, losses, workspace, workspace_bytes,
                                           nullptr, stream);
}
