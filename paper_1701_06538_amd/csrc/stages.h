// Argument blocks and launchers of the individual stages (internal; shared by the stage
// files and by the layer composition).
#pragma once
#include "common.h"

namespace moe {

struct LogitsArgs {
    const float *x;            // [*, d]
    const float *Wg, *Wn;      // [groups][d][n]; Wn null: clean logits only (sp is not written)
    const float *bias;         // [n] or null
    float *cleanb, *sp;        // [R][n]
    int64_t R;                 // rows
    int d, n;
    // row gather (hierarchical secondary gate): token = row_src[r] / row_div; null = identity
    const int32_t *row_src;
    int row_div;
    // row tiles that never straddle a group; null = one group, tile t covers rows 128t..
    const int32_t *tile_group, *tile_row0, *num_tiles, *group_offsets;
};

struct TopkArgs {
    const float *cleanb, *sp;  // [R][n]
    const float *eps;          // [*][n] or null
    int64_t R;
    int n, k;
    // row r reads eps row / writes output row row_map[r] (null: r)
    const int32_t *row_map;
    const int32_t *tile_row0, *num_tiles, *tile_group, *group_offsets;  // null = flat
    int32_t *idx;              // [*][k]
    float *gate;               // [*][k]
    int32_t *next_idx;         // [*] or null
    float *partials;           // [gridDim.x][2][n]
    int rows_per_block;        // 8 or 32 (divides the 128-row logits tile)
};

struct RouteArgs {
    const int32_t *idx;  // [A]
    int64_t A;
    int n;
    int tile_rows;
    int chunk;           // assignments per chunk (multiple of 64)
    int num_chunks;
    int32_t *counts, *offsets, *perm, *inv_perm;
    int32_t *tile_expert, *tile_row0, *num_tiles;
    int32_t *tile_offsets;  // [n+1] or null: exclusive scan of tiles per expert
    int32_t *hist;          // workspace [num_chunks][n]
};

struct FfnArgs {
    const float *x;           // [T,d]
    const int32_t *perm;      // [A]
    const int32_t *offsets;   // [n+1]
    const int32_t *tile_expert, *tile_row0, *num_tiles;
    const void *W1, *W2;
    float *out;               // [A,d]
    float *hidden;            // fp32 path workspace [A,h]
    uint16_t *hid_out;        // bf16 path: optional copy of the hidden activations [A,h], or null
    uint16_t *xs_out;         // bf16 path: optional copy of the routed input rows, rounded to bf16 [A,d], or null
    int d, h, k;
    int k_shift;              // log2(k) when k is a power of two, else -1
};

int launch_gate_logits(const LogitsArgs &a, int64_t row_tiles, hipStream_t st);
int launch_gate_topk(const TopkArgs &a, int64_t blocks, hipStream_t st);
int gate_rows_per_block(int64_t rows, int n);
size_t route_ws_bytes(int64_t A, int n);
// grouped row GEMMs of the expert backward pass
enum { EPI_RELU_BF16 = 0, EPI_MASK_BF16 = 1, EPI_F32 = 2 };

struct GGRows {
    const uint16_t *A;     // [A_rows, K] sorted rows, k contiguous
    const uint16_t *B;     // per expert: B_KN ? [K, N] : [N, K]
    void *C;               // [A_rows, N] bf16 or fp32
    const uint16_t *mask;  // [A_rows, N] (EPI_MASK_BF16)
    int K, N;
    const int32_t *offsets, *tile_expert, *tile_row0, *num_tiles;
    int tile_rows;         // rows per tile of the table if smaller than the kernel's own tile (0: not)
};

// 128-row-tile kernel (K % 32 == 0, N % 128 == 0; B stored [K,N] if b_kn, else [N,K])
int launch_gg_rows128(const GGRows &p, bool b_kn, int epi, int64_t max_tiles, hipStream_t st);
int launch_gg_rows256(const GGRows &p, int epi, int64_t max_tiles, hipStream_t st);

// per-expert weight gradient C_e[M, N] = sum over the expert's rows of A[r, :]^T B[r, :]  (M, N % 256 == 0)
struct GGWgrad {
    const uint16_t *A;   // [A_rows, M] sorted rows
    const uint16_t *B;   // [A_rows, N] sorted rows
    float *C;            // [n, M, N]
    int M, N;
    const int32_t *offsets;
    const int32_t *order;   // experts by decreasing row count (launch_expert_order)
    // optional: per-block sums of squares for the optimiser, rowpart [n][N/256][M], colpart [n][M/256][N]
    float *rowpart, *colpart;
};
int launch_gg_wgrad(const GGWgrad &p, int n, hipStream_t st);
// byte offsets, inside the backward workspace, of the sums of squares that moe_layer_backward leaves
// with MOE_FLAG_ADAM_MOMENTS: {rowpart(dW1), colpart(dW1), rowpart(dW2), colpart(dW2)}
int backward_moments_offsets(const moe_config *cfg, size_t off[4]);
// order[r] = the expert with the r-th most rows (equal counts: lower index first)
int launch_expert_order(const int32_t *offsets, int n, int32_t *order, hipStream_t st);

// strictly balanced gating (Appendix F): what its backward pass needs from the forward code.
// Byte offsets, inside the forward workspace of moe_layer_forward_balanced, of pos [T,n] (a kept
// token's place in its expert's list), offsets [n+1], the expert outputs [k*T, d] and the expert
// kernels' own workspace; hidden: the bf16 hidden activations [k*T, h] kept under
// MOE_FLAG_SAVE_HIDDEN, or (size_t)-1.
struct BalancedFwdView {
    size_t pos, offsets, out_rows, ffn_ws, hidden, total;
};
int balanced_forward_view(const moe_config *cfg, BalancedFwdView *v);
int launch_balanced_row_gates(const float *gsigma, const float *denom, const int32_t *tokens,
                              const int32_t *offsets, int n, int64_t rows, float *row_gate, hipStream_t st);
int launch_balanced_gate_bwd(const moe_config *cfg, const float *gsigma, const uint32_t *kept, const int32_t *pos,
                             const float *denom, const int32_t *offsets, const float *drow,
                             const float *thresholds, float w_batchwise, float *dlogit, hipStream_t st);
// dx[t] += sum of the rows of rows_mat [k*T, d] that belong to token t
int launch_add_kept_rows(const moe_config *cfg, const float *rows_mat, const uint32_t *kept, const int32_t *pos,
                         const int32_t *offsets, float *dx, hipStream_t st);

int launch_route(RouteArgs a, hipStream_t st);
bool route_is_small(int64_t A, int n);   // one-launch path (few experts, short assignment list)
// fused launches of the layer forward (small path only; aux_ws as in aux_ws_bytes)
int launch_route_small_sums(RouteArgs a, const float *partials, int64_t prow, double *aux_ws,
                            hipStream_t st);
int launch_combine_losses(const float *out_sorted, const float *gate, const int32_t *inv_perm, float *y,
                          int64_t T, int d, int k, int64_t prow, int n, double *aux_ws, float w_imp,
                          float w_load, float *importance, float *load, float *losses, hipStream_t st);
int launch_expert_ffn(const moe_config *cfg, const FfnArgs &a, int64_t max_tiles, hipStream_t st);
// Backward through both layers of the fused experts for routed rows, one launch (experts with about
// one 64-row tile of rows, 512 x 1024 bf16 experts): dz = (dout W2^T) * [hid > 0], dxs = dz W1^T.
struct FfnBwdRows {
    const uint16_t *dout;   // [A, d] bf16, sorted rows
    const uint16_t *hid;    // [A, h] bf16 hidden activations (the ReLU's output)
    const void *W1, *W2;    // [n, d, h], [n, h, d] bf16
    uint16_t *dz;           // out [A, h] bf16
    float *dxs;             // out [A, d] fp32
    const int32_t *offsets, *tile_expert, *tile_row0, *num_tiles;   // 64-row tile table
};
constexpr int kFfnBwdTileRows = 64;
bool ffn_bwd_rows_applies(const moe_config *cfg);
int launch_ffn_bwd_rows(const FfnBwdRows &a, int64_t max_tiles, hipStream_t st);
int expert_ffn_with_hidden(const moe_config *cfg, const float *x, const int32_t *perm,
                           const int32_t *offsets, const int32_t *tile_expert,
                           const int32_t *tile_row0, const int32_t *num_tiles, const void *W1,
                           const void *W2, float *out_sorted, void *workspace, uint16_t *hid_out,
                           hipStream_t st, uint16_t *xs_out = nullptr);
int launch_combine(const float *out_sorted, const float *gate, const int32_t *inv_perm, float *y,
                   int64_t T, int d, int k, hipStream_t st);
int launch_aux_losses(const float *partials, int64_t rows, int n, float w_imp, float w_load,
                      float *importance, float *load, float *losses, double *ws,
                      hipStream_t st);
size_t aux_ws_bytes(int64_t rows, int n);
int launch_hier_compose(const int32_t *p_idx, const float *p_gate, const int32_t *s_idx,
                        const float *s_gate, int64_t T, int k_p, int k_s, int b, int32_t *idx,
                        float *gate, hipStream_t st);
// fixed-order fp64 column sums of float partials [rows][2][n] -> sums64 [2n] (ws as in aux_ws_bytes)
int launch_partial_sums(const float *partials, int64_t rows, int n, double *ws, hipStream_t st);
struct HierLossArgs {
    const float *gate;          // [T*k] gate products
    const int32_t *perm, *offsets;  // route over all a*b experts
    const double *p_sums;       // [2a]: primary importance | load
    const float *s_partials;    // [blocks][2][b] secondary partial sums, blocks grouped by tile
    const int32_t *p_counts, *p_tile_offsets;
    int a, b, sub;              // sub = top-k blocks per 128-row tile
    double *sums64;             // out [2n]: importance | load
    float *importance, *load;   // out [n]
};
int launch_hier_losses(const HierLossArgs &a, float w_imp, float w_load, float *losses, hipStream_t st);

}  // namespace moe
