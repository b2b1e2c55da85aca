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
    const size_t T = (size_t)cfg->T, n = (size_t)cfg->n, A = T * (size_t)cfg->k;
    const size_t MT = (size_t)moe_max_tiles(cfg) + 8;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off = align_up(off + (bytes ? bytes : 1));
        return at;
    };
    const size_t gate_n = cfg->a > 0 ? (size_t)cfg->b : n;   // columns of the (secondary) gate
    const size_t gate_rows = cfg->a > 0 ? T * (size_t)cfg->k_primary : T;
    L->cleanb = take(gate_rows * gate_n * 4);
    L->sp = take(gate_rows * gate_n * 4);
    L->next_idx = take(gate_rows * 4);
    L->partials = take((size_t)(ceil_div((int64_t)gate_rows, gate_rows_per_block((int64_t)gate_rows, (int)gate_n)) + 16 * (cfg->a > 0 ? cfg->a : 0)) * 2 * gate_n * 4);
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
    L->aux_ws = take(aux_ws_bytes(cfg->a > 0 ? (int64_t)T * cfg->k_primary : moe_gate_partial_rows(cfg), cfg->n));
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
    if (!x || !W_g || !W_noise || !W1 || !W2 || !y || !topk_idx || !topk_gate || !importance ||
        !load || !losses || !workspace)
        return MOE_EINVAL;
    if (!aligned16(workspace) || !aligned16(x) || !aligned16(y) || !aligned16(W1) || !aligned16(W2))
        return MOE_EINVAL;
    if (workspace_bytes < L.total) return MOE_EWORKSPACE;
    char *ws = (char *)workspace;
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
    MOE_STAGE(1, moe_route(cfg, topk_idx, counts, offsets, perm, inv_perm, tile_expert, tile_row0,
                           num_tiles, ws + L.route_ws, stream))
    MOE_STAGE(2, moe_expert_ffn(cfg, x, perm, offsets, tile_expert, tile_row0, num_tiles, W1, W2,
                                out_sorted, ws + L.ffn_ws, stream))
    MOE_STAGE(3, moe_combine(cfg, out_sorted, topk_gate, inv_perm, y, stream))
    MOE_STAGE(4, moe_aux_losses(cfg, partials, importance, load, losses, ws + L.aux_ws, stream))
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
