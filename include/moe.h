/*
 * moe.h -- C ABI of the MI355X (gfx950) Sparsely-Gated Mixture-of-Experts layer library.
 *
 * The layer (Section 2 of "Outrageously Large Neural Networks: The Sparsely-Gated
 * Mixture-of-Experts Layer"):
 *     y = sum_i G(x)_i E_i(x)                                   Eq.(1)
 *     G(x) = Softmax(KeepTopK(H(x), k))                         Eq.(3),(5)
 *     H(x)_i = (x W_g)_i + eps_i * Softplus((x W_noise)_i)      Eq.(4), eps ~ N(0,1) passed in
 *     E_i(x) = relu(x W1_i) W2_i                                Appendix C (no biases)
 *     L_importance = w_importance * CV(sum_x G(x))^2            Eq.(6),(7)
 *     L_load = w_load * CV(sum_x P(x,.))^2,                     Eq.(8)-(11), Appendix A
 *         P(x,i) = Phi((clean_i - kth_excluding(H,k,i)) / Softplus(raw_i))
 *
 * Conventions for every entry point
 *  - extern "C"; returns 0 (MOE_OK) or a negative moe_status; no exception crosses the ABI.
 *  - Every tensor pointer is a DEVICE pointer owned by the caller, dense row-major, 16-byte
 *    aligned, non-overlapping unless stated.  Outputs are fully overwritten.
 *  - The library allocates nothing and never synchronises with the host: all work is
 *    enqueued on `stream` (a hipStream_t passed as void*; NULL = the default stream).
 *  - Arguments are validated on the host before anything is launched; on error nothing runs.
 *  - Index tensors are int32.  "bf16" tensors are uint16 bit patterns of bfloat16.
 *  - Calls that share a workspace or an output on different streams race; distinct buffers
 *    on distinct streams are safe.
 */
#ifndef MOE_H_
#define MOE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum moe_status {
    MOE_OK = 0,
    MOE_EINVAL = -1,        /* null pointer, bad shape, k out of range, misaligned pointer */
    MOE_EUNSUPPORTED = -2,  /* valid request outside what the kernels were built for */
    MOE_EWORKSPACE = -3,    /* workspace smaller than moe_workspace_bytes() */
    MOE_EHIP = -4           /* a HIP runtime call failed; see moe_last_hip_error() */
} moe_status;

enum { MOE_DTYPE_F32 = 0, MOE_DTYPE_BF16 = 1 };

/* Shape of one layer call.  Flat MoE: a = b = k_primary = k_secondary = 0.
 * Hierarchical MoE (Appendix B): a groups of b experts, n = a*b, k = k_primary*k_secondary.
 * Supported: d % 32 == 0; bf16 experts: d and h multiples of 128 (the paper's 512 x 1024 expert
 * runs on a fused kernel that keeps the hidden layer on chip, other shapes on a plain two-GEMM
 * path with the hidden layer in the workspace); fp32 experts: d and h multiples of 4;
 * 1 <= k <= min(n, 8) (per level when hierarchical); n <= 16384 (flat, or a*b with either level up
 * to 16384); T*k < 2^31.  moe_layer_backward: n a multiple of 4; bf16 experts with d and h
 * multiples of 256, or fp32 experts. */
typedef struct moe_config {
    int32_t T;             /* tokens in the batch */
    int32_t d;             /* model width: expert input and output size */
    int32_t h;             /* expert hidden size */
    int32_t n;             /* number of experts */
    int32_t k;             /* experts per token */
    int32_t a, b;          /* hierarchical: groups, experts per group */
    int32_t k_primary, k_secondary;
    int32_t expert_dtype;  /* MOE_DTYPE_F32 or MOE_DTYPE_BF16: storage type of W1, W2 */
    float w_importance;    /* Eq.(7) */
    float w_load;          /* Eq.(11) */
    int32_t flags;         /* MOE_FLAG_* */
} moe_config;

/* With MOE_FLAG_SAVE_HIDDEN moe_layer_forward, moe_layer_forward_hier and moe_layer_forward_balanced
 * also keep the experts' hidden activations (bf16 [T*k, h], routed-row order) in the workspace, and
 * moe_layer_backward / _hier / _balanced read them instead of recomputing them (the flat layer also
 * keeps the routed input rows as the experts saw them, bf16 [T*k, d], which its backward pass would
 * otherwise gather and round again).  The paper
 * recomputes (Appendix D) to fit 12 GB devices; with 288 GB of HBM the 2*h bytes per routed row
 * are the cheaper side of the trade.  Without the flag the backward pass recomputes. */
/* With MOE_FLAG_ADAM_MOMENTS moe_layer_backward, moe_layer_backward_balanced and moe_layer_backward_hier
 * (bf16 experts) also leave, in the backward workspace, the
 * per-block sums of squares of dW1 and dW2 that the weight-gradient kernels have in registers
 * anyway; moe_expert_adam_step then skips its own pass over the gradients when it is handed that
 * workspace. */
enum { MOE_FLAG_SAVE_HIDDEN = 1, MOE_FLAG_ADAM_MOMENTS = 2 };

int moe_version(void);
const char *moe_strerror(int status);
/* hipError_t (as int) of the most recent failing HIP call on this thread, 0 if none. */
int moe_last_hip_error(void);

/* ---- sizes the caller needs to allocate buffers ------------------------------------ */

/* Rows of the per-block partial sums moe_gate writes: partials is float [rows][2][n]. */
int64_t moe_gate_partial_rows(const moe_config *cfg);
/* Bytes of scratch moe_route needs (chunk histograms). */
size_t moe_route_workspace_bytes(const moe_config *cfg);
/* Row-tile height of the expert kernel and the capacity of the tile table moe_route fills:
 * tile_expert and tile_row0 must hold moe_max_tiles() int32 each. */
int32_t moe_tile_rows(const moe_config *cfg);
int64_t moe_max_tiles(const moe_config *cfg);
/* Bytes of scratch moe_expert_ffn needs: the hidden layer of fp32 experts; the bf16 rows of x and
 * the hidden layer of bf16 experts off the fused kernel's shape; 0 for 512 x 1024 bf16 experts. */
size_t moe_ffn_workspace_bytes(const moe_config *cfg);
/* Bytes of scratch moe_aux_losses needs. */
size_t moe_aux_workspace_bytes(const moe_config *cfg);
/* Bytes of the single workspace of moe_layer_forward / moe_layer_forward_hier. */
size_t moe_workspace_bytes(const moe_config *cfg);

/* Where moe_layer_forward keeps its intermediates inside the workspace (byte offsets), so a
 * caller can inspect them or hand them to moe_layer_backward. */
typedef struct moe_workspace_layout {
    size_t cleanb, sp, next_idx, partials, counts, offsets, perm, inv_perm, tile_expert,
        tile_row0, num_tiles, route_ws, out_sorted, ffn_ws, aux_ws, hidden /* (size_t)-1 if absent */,
        total;
    /* hierarchical only */
    size_t p_cleanb, p_sp, p_next_idx, p_partials, p_idx, p_gate, p_counts, p_offsets, p_perm,
        p_inv_perm, p_tile_group, p_tile_row0, p_num_tiles, p_tile_offsets, p_route_ws, p_aux_ws,
        s_idx, s_gate;
    /* flat layer with MOE_FLAG_SAVE_HIDDEN and bf16 experts: the routed input rows rounded to bf16
     * [T*k, d], kept for moe_layer_backward; (size_t)-1 if absent */
    size_t xs;
} moe_workspace_layout;
int moe_get_workspace_layout(const moe_config *cfg, moe_workspace_layout *out);

/* ---- a1: noisy top-k gating, Eq.(3)-(5) -------------------------------------------- */
/*
 * x [T,d] f32; W_g, W_noise [d,n] f32; gate_bias [n] f32 or NULL (added to the clean logits;
 * the paper's gate has none); eps [T,n] f32 standard-normal draws, or NULL for the noise-free
 * gate H = x W_g.
 * Outputs: topk_idx [T,k] i32 (descending H; equal H: lower index first), topk_gate [T,k] f32
 * (softmax over the kept logits); cleanb [T,n] f32 = x W_g (+ bias); sp [T,n] f32 =
 * Softplus(x W_noise); next_idx [T] i32 = index of the (k+1)-th largest H (-1 when k = n);
 * partials f32 [moe_gate_partial_rows][2][n] = per-block sums of G(x) and of P(x,.) that
 * moe_aux_losses finishes.
 * Arithmetic of H (what makes top-k reproducible): each logit is one fp32 accumulator,
 * acc = fma(x[t][j], W[j][i], acc) for j ascending from +0; Softplus is evaluated in
 * binary64 from a fixed sequence of fused operations and rounded once to fp32;
 * H = fma(eps, sp, clean + bias).  Inputs must be finite.
 */
int moe_gate(const moe_config *cfg, const float *x, const float *W_g, const float *W_noise,
             const float *gate_bias, const float *eps, int32_t *topk_idx, float *topk_gate,
             float *cleanb, float *sp, int32_t *next_idx, float *partials, void *stream);

/* ---- a2: dispatch bookkeeping (Section 2: skip experts with G = 0; Section 3.1: one
 *      combined batch per expert) ------------------------------------------------------ */
/*
 * topk_idx [T,k] -> counts [n] (assignments per expert), offsets [n+1] (exclusive prefix
 * sum), perm [T*k] (sorted row -> assignment id a = t*k+s; stable: rows of one expert in
 * ascending a), inv_perm [T*k] (assignment id -> sorted row), and the row-tile table for the
 * expert kernel: tile_expert/tile_row0 [moe_max_tiles] and num_tiles [1] (tiles never straddle
 * experts; experts without tokens get no tile).  Deterministic: no position atomics.
 * workspace: moe_route_workspace_bytes() bytes.
 */
int moe_route(const moe_config *cfg, const int32_t *topk_idx, int32_t *counts, int32_t *offsets,
              int32_t *perm, int32_t *inv_perm, int32_t *tile_expert, int32_t *tile_row0,
              int32_t *num_tiles, void *workspace, void *stream);

/*
 * moe_route for callers that cannot allocate device memory or hand over a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same inputs, outputs
 * and results as moe_route; the chunk histograms live in a 4 MiB device array inside the library
 * image instead of a caller workspace (each GPU the library runs on holds that array until the
 * process ends).  The call allocates nothing.  Shapes whose moe_route_workspace_bytes() exceeds
 * MOE_ROUTE_STATIC_MAX_WORKSPACE_BYTES are rejected with MOE_EWORKSPACE before anything is
 * launched (the limit admits e.g. T*k = 131072 assignments over 2048 experts; few experts and a
 * short assignment list, n <= 512 and T*k <= 65536, need no scratch at all).  All calls on one GPU
 * share the one array: calls that overlap in time on the same GPU (different streams or host
 * threads) race; calls on one stream, or ordered by events, are safe.  Nothing has to be cleared
 * between calls: every cell read is written earlier in the same call.
 */
#define MOE_ROUTE_STATIC_MAX_WORKSPACE_BYTES ((size_t)4 << 20)
int moe_route_static(const moe_config *cfg, const int32_t *topk_idx, int32_t *counts,
                     int32_t *offsets, int32_t *perm, int32_t *inv_perm, int32_t *tile_expert,
                     int32_t *tile_row0, int32_t *num_tiles, void *stream);

/* ---- a3: the experts, E_i(x) = relu(x W1_i) W2_i (Appendix C) ------------------------ */
/*
 * x [T,d] f32; W1 [n,d,h] and W2 [n,h,d] in the paper's plain layout (input x hidden,
 * hidden x output), fp32 or bf16 per cfg->expert_dtype.  Rows are gathered through perm
 * (token = perm[row] / k).  out_sorted [T*k, d] f32, row r = E_{expert of r}(x_{token of r}).
 * bf16 experts: x and the hidden activations are rounded to bf16 (nearest-even), products
 * accumulate in fp32 on the matrix cores; the hidden layer never leaves the chip.
 * Experts with no rows are never read.
 */
int moe_expert_ffn(const moe_config *cfg, const float *x, const int32_t *perm,
                   const int32_t *offsets, const int32_t *tile_expert, const int32_t *tile_row0,
                   const int32_t *num_tiles, const void *W1, const void *W2, float *out_sorted,
                   void *workspace, void *stream);

/* ---- a4: y = sum_s gate[t,s] * E_{idx[t,s]}(x_t), Eq.(1) (Eq.(12) when the gates are the
 *      products of primary and secondary gates) ----------------------------------------- */
/* out_sorted [T*k,d] f32, topk_gate [T,k] f32, inv_perm [T*k] -> y [T,d] f32; slots are
 * accumulated in ascending s with fused multiply-adds. */
int moe_combine(const moe_config *cfg, const float *out_sorted, const float *topk_gate,
                const int32_t *inv_perm, float *y, void *stream);

/*
 * moe_combine fused with what the paper's language models put behind the MoE layer (Appendix C,
 * "Model Architecture"): sigmoid of the layer output, dropout (each activation dropped with
 * probability drop_prob, survivors divided by 1 - drop_prob), then the residual connection:
 *     y = x + keep * sigmoid(sum_s gate[t,s] out_sorted[row(t,s)]) / (1 - drop_prob).
 * keep [T,d] u8 is the dropout draw (non-zero = the activation survives; 4-byte aligned), an input
 * like every random number of the method, or NULL for no dropout (drop_prob must then be 0);
 * x [T,d] is the layer's input, or NULL for no residual connection.  0 <= drop_prob < 1.
 */
int moe_combine_epilogue(const moe_config *cfg, const float *out_sorted, const float *topk_gate,
                         const int32_t *inv_perm, const float *x, const uint8_t *keep,
                         float drop_prob, float *y, void *stream);

/* ---- a5: balancing losses, Eq.(6),(7),(10),(11) ---------------------------------------- */
/* partials from moe_gate -> importance [n] f32, load [n] f32, losses [4] f32 =
 * {w_importance*CV^2(importance), w_load*CV^2(load), CV^2(importance), CV^2(load)}; CV^2 uses
 * the population variance and is evaluated in fp64.  workspace: moe_aux_workspace_bytes()
 * bytes (the fp64 sums). */
int moe_aux_losses(const moe_config *cfg, const float *partials, float *importance, float *load,
                   float *losses, void *workspace, void *stream);

/* ---- the whole forward pass of the flat layer: a1..a5 on one stream ------------------- */
/* T = 0 is accepted (pointers to [T,...] tensors may then be NULL): counts, offsets and the tile
 * table in the workspace are zeroed, importance = load = 0 and the losses are reported as 0. */
int moe_layer_forward(const moe_config *cfg, const float *x, const float *W_g,
                      const float *W_noise, const float *gate_bias, const float *eps,
                      const void *W1, const void *W2, float *y, int32_t *topk_idx,
                      float *topk_gate, float *importance, float *load, float *losses,
                      void *workspace, size_t workspace_bytes, void *stream);

/* ---- hierarchical MoE (Appendix B, Eq.(12)-(14)) ---------------------------------------- */
/*
 * Two-level noisy top-k gating: a primary gate over the a groups (k_primary kept), then for every
 * kept group i the secondary gate G_i over its b experts (k_secondary kept), evaluated only on
 * X^(i) = {x : G_primary(x)_i > 0}.
 * x [T,d]; Wg_p, Wn_p [d,a]; eps_p [T,a]; Wg_s, Wn_s [a,d,b]; eps_s [T,k_primary,b] (noise of the
 * secondary gate reached through primary slot p); any eps may be NULL (noise-free level).
 * Outputs: topk_idx [T,k] = global expert id i*b + j, slot-major (primary slot, then secondary
 * slot, each in descending logit order); topk_gate [T,k] = G_primary(x)_i * G_i(x)_j.
 * workspace: moe_workspace_bytes(); it keeps every intermediate (primary and secondary logits,
 * per-level indices and gates, the grouping of rows by primary group) at the offsets
 * moe_get_workspace_layout reports, for moe_aux_losses_hier.
 * Same logit arithmetic as moe_gate at both levels.
 */
int moe_gate_hier(const moe_config *cfg, const float *x, const float *Wg_p, const float *Wn_p,
                  const float *eps_p, const float *Wg_s, const float *Wn_s, const float *eps_s,
                  int32_t *topk_idx, float *topk_gate, void *workspace, size_t workspace_bytes,
                  void *stream);

/* Importance_H (Eq.(13)) = sum of the gate products per expert; Load_H (Eq.(14)) =
 * Load_primary_i * Load_i(X^(i))_j / |X^(i)| (0 for an empty X^(i)); losses as in moe_aux_losses
 * with CV^2 taken over all a*b experts.  Needs the workspace moe_gate_hier filled and the
 * permutation moe_route built from topk_idx (perm, offsets). */
int moe_aux_losses_hier(const moe_config *cfg, const float *topk_gate, const int32_t *perm,
                        const int32_t *offsets, void *workspace, size_t workspace_bytes,
                        float *importance, float *load, float *losses, void *stream);

/* Whole forward pass of the hierarchical layer, Eq.(12): moe_gate_hier, moe_route,
 * moe_expert_ffn, moe_combine, moe_aux_losses_hier on one stream. */
int moe_layer_forward_hier(const moe_config *cfg, const float *x, const float *Wg_p,
                           const float *Wn_p, const float *eps_p, const float *Wg_s,
                           const float *Wn_s, const float *eps_s, const void *W1, const void *W2,
                           float *y, int32_t *topk_idx, float *topk_gate, float *importance,
                           float *load, float *losses, void *workspace, size_t workspace_bytes,
                           void *stream);

/* ---- a6: backward pass of the flat layer (Section 2.1, "Training the Gating Network";
 *      Appendix D: hidden activations are recomputed) ------------------------------------ */
/*
 * Gradients of J = <dy, y> + w_importance*CV^2(Importance) + w_load*CV^2(Load) with respect to
 * x, W_g, W_noise and every expert's W1, W2.  The top-k selection is piecewise constant: gradient
 * flows through the kept softmax values, through P(x,i) of Eq.(9) -- including the element
 * kth_excluding picks as threshold -- and through the experts; relu'(0) = 0.
 * Inputs: the forward call's inputs, dy [T,d] f32, its outputs topk_idx/topk_gate and its
 * workspace exactly as moe_layer_forward left it (logits, permutation, expert outputs, loss sums).
 * Outputs (overwritten): dx [T,d], dW_g, dW_noise [d,n], dW1 [n,d,h], dW2 [n,h,d], all f32
 * (fp32 master gradients; experts that received no token get zeros).
 * n a multiple of 4.  bf16 experts: d and h multiples of 256, expert math in bf16 MFMA with fp32
 * accumulation.  fp32 experts: d and h multiples of 4, n <= 65535, every GEMM on the fp32 matrix
 * cores; the hidden activations are the ones the forward pass left in its expert workspace.
 * Gate math in fp32.  workspace: moe_backward_workspace_bytes().
 * T = 0 is accepted (the [T, .] tensors may then be NULL): every weight gradient is written as zero.
 * The same holds for moe_layer_backward_hier and moe_layer_backward_balanced.
 */
size_t moe_backward_workspace_bytes(const moe_config *cfg);
int moe_layer_backward(const moe_config *cfg, const float *x, const float *W_g,
                       const float *W_noise, const float *eps, const void *W1, const void *W2,
                       const float *dy, const int32_t *topk_idx, const float *topk_gate,
                       const void *fwd_workspace, float *dx, float *dW_g, float *dW_noise,
                       float *dW1, float *dW2, void *workspace, size_t workspace_bytes,
                       void *stream);

/* ---- strictly balanced gating (Appendix F, Eq.(15)-(20)) ---------------------------------- */
/*
 * The gate that replaces noisy top-k where every expert must receive the same number of rows:
 *   G_sigma = Softmax(x W_g [+ gate_bias])                                   Eq.(15)
 *   M_batchwise keeps, for every expert, the m = k*T/n largest values of its column of G_sigma
 *   (equal values: the lower token index first)                             Eq.(17),(18)
 *   G(x)_i = G_sigma_i M_i / sum_j G_sigma_j M_j                             Eq.(16)
 * and, given per-expert thresholds, the loss that fits the inference-time mask
 * M_threshold = [G_sigma > T_i] to the batchwise one                        Eq.(19),(20)
 *   L_batchwise = sum_{t,i} (M_threshold - M_batchwise)(G_sigma - T_i).
 * cfg: flat (a == 0); k*T must be a multiple of n (else MOE_EINVAL); n <= 2048.
 * The softmax is computed in a pinned arithmetic (fp32 logits by the sequential fma chain of
 * moe_gate; exponentials, the sum and the division in binary64 by a fixed operation sequence;
 * one rounding to fp32), since the mask compares its values across tokens.
 * Device inputs: x [T,d], W_g [d,n], gate_bias [n] or NULL, thresholds [n] or NULL.
 * Device outputs (overwritten):
 *   gsigma [T,n] f32; tokens [n,m] i32, expert e's kept tokens in ascending order (its rows of the
 *   dispatch, which needs no further sort); kept [T, ceil(n/32)] u32, bit (e & 31) of word e >> 5
 *   set iff M_batchwise(t,e) = 1; denom [T] f32, the denominator of Eq.(16) (0 for a token no
 *   expert kept: its output row is zero); loss_batchwise [1] f32, written only if thresholds != NULL.
 * workspace: moe_balanced_workspace_bytes(), 16-byte aligned.  Asynchronous on `stream`.
 */
int64_t moe_balanced_rows_per_expert(const moe_config *cfg);   /* m, or -1 if cfg is not valid */
size_t moe_balanced_workspace_bytes(const moe_config *cfg);
int moe_gate_balanced(const moe_config *cfg, const float *x, const float *W_g,
                      const float *gate_bias, const float *thresholds, float *gsigma,
                      int32_t *tokens, uint32_t *kept, float *denom, float *loss_batchwise,
                      void *workspace, size_t workspace_bytes, void *stream);
/* What trains the thresholds: d L_batchwise / d T_i = m - #{t : G_sigma(t,i) > T_i} (both masks of
 * Eq.(20) are piecewise constant in T).  gsigma [T,n] as moe_gate_balanced wrote it, thresholds [n]
 * -> dthresholds [n] f32.  cfg as for moe_gate_balanced. */
int moe_batchwise_loss_grad(const moe_config *cfg, const float *gsigma, const float *thresholds,
                            float *dthresholds, void *stream);
/*
 * Backward pass of moe_layer_forward_balanced: gradients of
 *   J = <dy, y> + w_batchwise * L_batchwise
 * with respect to x, W_g and the expert matrices.  Both masks are piecewise constant, so the gate
 * is reached only through the values G_sigma: through the quotient of Eq.(16),
 *   dG_sigma_i = M_i (dG_i - sum_j G_j dG_j) / denom,   dG_i = <dy, E_i(x)>        (Eq.(1), Eq.(16))
 * through the factor (G_sigma - T_i) of Eq.(20) as printed, + w_batchwise (M_threshold - M_batchwise),
 * and from there through the softmax of Eq.(15) over all n experts; the experts as in
 * moe_layer_backward (for bf16 experts the hidden activations are recomputed, Appendix D, unless the
 * forward call ran with MOE_FLAG_SAVE_HIDDEN in the same cfg; relu'(0) = 0).
 * The thresholds' own gradient is moe_batchwise_loss_grad's.
 * cfg as for moe_layer_forward_balanced, with moe_layer_backward's shape restrictions
 * (n % 4 == 0; bf16 experts: d, h multiples of 256; fp32 experts: d, h multiples of 4, n <= 65535);
 * MOE_FLAG_ADAM_MOMENTS is honoured as there.
 * Device inputs: x, W_g, W1, W2 as in the forward call; thresholds [n] (may be NULL if
 * w_batchwise == 0); dy [T,d] f32; gsigma, tokens, kept, denom and fwd_workspace as the forward
 * call left them (read-only).
 * Device outputs (overwritten): dx [T,d], dW_g [d,n], dW1 [n,d,h], dW2 [n,h,d], all f32 (matrices of
 * an expert without rows are zero).  workspace: moe_backward_balanced_workspace_bytes().
 */
size_t moe_backward_balanced_workspace_bytes(const moe_config *cfg);
int moe_layer_backward_balanced(const moe_config *cfg, const float *x, const float *W_g,
                                const float *thresholds, const void *W1, const void *W2,
                                const float *dy, const float *gsigma, const int32_t *tokens,
                                const uint32_t *kept, const float *denom, const void *fwd_workspace,
                                float w_batchwise, float *dx, float *dW_g, float *dW1, float *dW2,
                                void *workspace, size_t workspace_bytes, void *stream);
/*
 * The whole layer with that gate: moe_gate_balanced, the experts of Section 3.2 / Appendix C on
 * their m rows each (W1 [n,d,h], W2 [n,h,d] as in moe_expert_ffn), and Eq.(1) with the gates of
 * Eq.(16) -> y [T,d] f32, each token adding its kept experts in ascending expert order.
 */
int moe_layer_forward_balanced(const moe_config *cfg, const float *x, const float *W_g,
                               const float *gate_bias, const float *thresholds, const void *W1,
                               const void *W2, float *y, float *gsigma, int32_t *tokens,
                               uint32_t *kept, float *denom, float *loss_batchwise,
                               void *workspace, size_t workspace_bytes, void *stream);
/* The same call with optional timing hooks: stage_events is a HOST array of 5 hipEvent_t (as
 * void*), or NULL, recorded on `stream` before the gate [0], after it [1], before the expert
 * kernels [2], after them [3] and after the combine [4].  NULL entries are skipped; the events
 * belong to the caller. */
int moe_layer_forward_balanced_profiled(const moe_config *cfg, const float *x, const float *W_g,
                                        const float *gate_bias, const float *thresholds,
                                        const void *W1, const void *W2, float *y, float *gsigma,
                                        int32_t *tokens, uint32_t *kept, float *denom,
                                        float *loss_batchwise, void *workspace,
                                        size_t workspace_bytes, void *const *stage_events,
                                        void *stream);

/*
 * Inference with the threshold mask (Appendix F, Eq.(19)): the layer with
 * G(x)_i = G_sigma_i M_i / sum_j G_sigma_j M_j,  M_i = [G_sigma(x)_i > T_i],
 * in place of the batchwise mask, so a token's experts no longer depend on the rest of the batch.
 * The number of rows per expert is then data dependent: the caller sizes the dispatch with
 * row_capacity (rows of expert input the workspace and `tokens` can hold, < 2^31; T*n < 2^31).
 * cfg as for moe_gate_balanced, except that k only has to be valid (it sizes nothing).
 * Device inputs as for moe_layer_forward_balanced; thresholds [n] f32 is required.
 * Device outputs (overwritten): y [T,d]; gsigma [T,n]; counts [n] i32 = rows per expert;
 * tokens [row_capacity] i32 = expert e's tokens in ascending order from the exclusive prefix sum of
 * counts on; kept [T, ceil(n/32)] u32 = the mask as bits; denom [T] f32; rows_total [1] i32 = sum of
 * counts.  If rows_total > row_capacity no expert runs and y is all zeros: the caller reads
 * rows_total after the stream has finished and calls again with a larger capacity.
 * workspace: moe_threshold_workspace_bytes(cfg, row_capacity).
 */
size_t moe_threshold_workspace_bytes(const moe_config *cfg, int64_t row_capacity);
int moe_layer_forward_threshold(const moe_config *cfg, const float *x, const float *W_g,
                                const float *gate_bias, const float *thresholds, const void *W1,
                                const void *W2, int64_t row_capacity, float *y, float *gsigma,
                                int32_t *counts, int32_t *tokens, uint32_t *kept, float *denom,
                                int32_t *rows_total, void *workspace, size_t workspace_bytes,
                                void *stream);

/* ---- optimiser step for the expert matrices (Appendix D, "Optimizer") --------------------- */
/*
 * Adam without a first-moment estimator (beta1 = 0) and with a FACTORED second-moment estimator:
 * for a parameter matrix [R, C] only the row-wise and column-wise averages v_row [R], v_col [C] of
 * the second-moment matrix are kept; both follow v <- beta2 v + (1 - beta2) avg(G*G), and the
 * step uses  Vhat[r,c] = v_row[r] v_col[c] / mean(v_row)  (the two means are equal):
 *     W <- W - lr * G / (sqrt(Vhat / (1 - beta2^step)) + eps)      (step counts from 1)
 * -- Adam's bias correction and epsilon placement, which the paper does not restate.  A matrix
 * whose gradient history is all zero is left unchanged.
 * Every expert's W1 [d,h] (R = d, C = h) and W2 [h,d] (R = h, C = d) is one such matrix.
 * Device inputs: dW1 [n,d,h], dW2 [n,h,d] f32 (as moe_layer_backward writes them).
 * Device in/out: W1_master, W2_master f32 parameters in the weights' layout; v_row1 [n,d],
 * v_col1 [n,h], v_row2 [n,h], v_col2 [n,d] f32 (zero before the first step).
 * Device outputs: W1_copy, W2_copy: the bf16 weights the layer reads (nearest-even rounding of the
 * updated parameters), or both NULL for fp32 experts, whose parameters are the weights themselves.
 * d and h multiples of 4; workspace: moe_adam_workspace_bytes().
 * backward_workspace: NULL, or the workspace moe_layer_backward (or _hier) has just filled under a cfg with
 * MOE_FLAG_ADAM_MOMENTS (the same cfg is passed here): the sums of squares of the gradients are
 * then taken from it instead of from a pass over dW1 and dW2.  Without it cfg->T and cfg->k are
 * not used.
 */
/* The hyper-parameters are fp32 as passed: 1 - beta2 and 1 - beta2^step are formed from the fp32
 * value of beta2 (0.999f is 0.99900001287...: a reference fed the decimal 0.999 differs by 1.3e-5
 * in 1 - beta2). */
typedef struct moe_adam_params {
    float lr, beta2, eps;
    int32_t step;          /* 1 for the first update */
} moe_adam_params;
size_t moe_adam_workspace_bytes(const moe_config *cfg);
int moe_expert_adam_step(const moe_config *cfg, const moe_adam_params *hp, const float *dW1,
                         const float *dW2, float *W1_master, float *W2_master, void *W1_copy,
                         void *W2_copy, float *v_row1, float *v_col1, float *v_row2, float *v_col2,
                         const void *backward_workspace, void *workspace, size_t workspace_bytes,
                         void *stream);

/* ---- backward pass of the hierarchical layer (Appendix B, Eq.(12)-(14)) ------------------- */
/*
 * Gradients of J = <dy, y> + w_importance*CV^2(Importance_H) + w_load*CV^2(Load_H) with respect
 * to x, both gating levels' matrices and every expert's W1, W2.  The chain rule runs through
 * gate(t,i,j) = G_primary(x_t)_i * G_i(x_t)_j (Eq.(12)), Importance_H (Eq.(13)) and
 * Load_H(i,j) = Load_primary(i) * Load_i(X^(i))_j / |X^(i)| (Eq.(14); |X^(i)| is a count, hence
 * constant), then through each level as through the flat gate (moe_layer_backward).
 * Inputs: the forward call's inputs, dy [T,d], its outputs topk_idx/topk_gate and its workspace as
 * moe_layer_forward_hier left it.  Outputs (overwritten): dx [T,d]; dWg_p, dWn_p [d,a];
 * dWg_s, dWn_s [a,d,b] (zeros for a group no token chose); dW1 [n,d,h], dW2 [n,h,d]; all f32.
 * bf16 experts, d and h multiples of 256, a and b multiples of 32; the hidden activations are
 * recomputed (Appendix D) unless the forward call kept them (MOE_FLAG_SAVE_HIDDEN).
 * workspace: moe_backward_hier_workspace_bytes().
 */
size_t moe_backward_hier_workspace_bytes(const moe_config *cfg);
int moe_layer_backward_hier(const moe_config *cfg, const float *x, const float *Wg_p,
                            const float *Wn_p, const float *eps_p, const float *Wg_s,
                            const float *Wn_s, const float *eps_s, const void *W1, const void *W2,
                            const float *dy, const int32_t *topk_idx, const float *topk_gate,
                            const void *fwd_workspace, float *dx, float *dWg_p, float *dWn_p,
                            float *dWg_s, float *dWn_s, float *dW1, float *dW2, void *workspace,
                            size_t workspace_bytes, void *stream);

/* Same as moe_layer_forward, with optional timing hooks: stage_events is a HOST array of 10
 * hipEvent_t (as void*), or NULL; entry 2i is recorded on `stream` just before stage i and entry
 * 2i+1 just after it, for i = 0 gate, 1 route, 2 experts, 3 combine, 4 losses.  NULL entries
 * are skipped.  The events belong to the caller. */
int moe_layer_forward_profiled(const moe_config *cfg, const float *x, const float *W_g,
                               const float *W_noise, const float *gate_bias, const float *eps,
                               const void *W1, const void *W2, float *y, int32_t *topk_idx,
                               float *topk_gate, float *importance, float *load, float *losses,
                               void *workspace, size_t workspace_bytes, void *const *stage_events,
                               void *stream);

/* moe_layer_forward_hier with the same timing hooks (10 events: gate = both levels, route,
 * experts, combine, losses). */
int moe_layer_forward_hier_profiled(const moe_config *cfg, const float *x, const float *Wg_p,
                                    const float *Wn_p, const float *eps_p, const float *Wg_s,
                                    const float *Wn_s, const float *eps_s, const void *W1,
                                    const void *W2, float *y, int32_t *topk_idx, float *topk_gate,
                                    float *importance, float *load, float *losses, void *workspace,
                                    size_t workspace_bytes, void *const *stage_events, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MOE_H_ */
