// Strictly balanced gating (Appendix F, Eq.(15)-(20)): G_sigma = Softmax(x W_g) over all experts,
// the batchwise mask that keeps the m = k|X|/n largest values of every expert's column, the gates
// renormalised over the kept experts of a token, the threshold mask used at inference and the
// loss that trains the thresholds.  Every expert receives exactly m rows, so dispatch is the
// per-expert token list itself.
//
//   softmax_rows_kernel     one wavefront per token: the softmax in a pinned arithmetic (binary64
//                           exponentials by a fixed operation sequence, a fixed summation tree, one
//                           division, one rounding to fp32), because the mask compares these values
//                           across tokens and must be reproducible bit for bit
//   transpose_kernel        G_sigma [T,n] -> [n,T], so that an expert's column is contiguous
//   select_columns_kernel   one workgroup per expert: the m-th largest value by a four-pass radix
//                           select (integer LDS histograms), then the kept tokens in ascending
//                           order (equal values: lower token first) with ballot-ranked positions
//   balanced_rows_kernel    one wavefront per token: denominator of Eq.(16) over the kept experts
//                           and the token's share of L_batchwise (Eq.(20))
//   combine_balanced_kernel Eq.(1) with the gates of Eq.(16): a token walks its kept experts in
//                           ascending order and finds its row in each expert's sorted list
#include "stages.h"

namespace moe {

// exp(-a) for a >= 0 in binary64: a clipped at 64, q = rint(a*log2e), r = fma(-q, ln2, a),
// degree-13 Taylor polynomial of exp(-r) in Horner form, exact scaling by 2^-q
__device__ __forceinline__ double exp_neg_spec(double a) {
    a = a > 64.0 ? 64.0 : a;
    const double q = rint(a * 1.4426950408889634);
    const double m = -__fma_rn(-q, 0.6931471805599453, a);
    double p = 1.0 / 6227020800.0;
    p = __fma_rn(p, m, 1.0 / 479001600.0);
    p = __fma_rn(p, m, 1.0 / 39916800.0);
    p = __fma_rn(p, m, 1.0 / 3628800.0);
    p = __fma_rn(p, m, 1.0 / 362880.0);
    p = __fma_rn(p, m, 1.0 / 40320.0);
    p = __fma_rn(p, m, 1.0 / 5040.0);
    p = __fma_rn(p, m, 1.0 / 720.0);
    p = __fma_rn(p, m, 1.0 / 120.0);
    p = __fma_rn(p, m, 1.0 / 24.0);
    p = __fma_rn(p, m, 1.0 / 6.0);
    p = __fma_rn(p, m, 0.5);
    p = __fma_rn(p, m, 1.0);
    p = __fma_rn(p, m, 1.0);
    return ldexp(p, -(int)q);
}

// Eq.(15).  Lane l sums its elements l, l+64, ... in ascending order, the 64 partial sums are
// added by the tree p_l += p_{l+off}, off = 32 .. 1, and lane 0's total divides every element.
template <int NCH>
__global__ __launch_bounds__(256) void softmax_rows_kernel(const float *__restrict__ logits, int64_t T,
                                                           int n, float *__restrict__ out) {
    const int lane = threadIdx.x & 63;
    const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    const float *row = logits + t * n;
    float l[NCH];
    float mx = -INFINITY;
#pragma unroll
    for (int q = 0; q < NCH; ++q) {
        const int i = lane + 64 * q;
        l[q] = row[min(i, n - 1)];
        mx = i < n ? fmaxf(mx, l[q]) : mx;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    double e[NCH];
    double p = 0.0;
#pragma unroll
    for (int q = 0; q < NCH; ++q) {
        e[q] = exp_neg_spec((double)mx - (double)l[q]);
        if (lane + 64 * q < n) p = __dadd_rn(p, e[q]);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) p = __dadd_rn(p, __shfl_down(p, off));
    const double s = __shfl(p, 0);
#pragma unroll
    for (int q = 0; q < NCH; ++q) {
        const int i = lane + 64 * q;
        if (i < n) out[t * n + i] = (float)__ddiv_rn(e[q], s);
    }
}

// out[c][r] = in[r][c], 64 x 64 tiles through LDS
__global__ __launch_bounds__(256) void transpose_kernel(const float *__restrict__ in, int64_t R, int C,
                                                        float *__restrict__ out) {
    __shared__ float tile[64][65];
    const int64_t r0 = (int64_t)blockIdx.x * 64;
    const int c0 = blockIdx.y * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int i = ty; i < 64; i += 4)
        if (r0 + i < R && c0 + tx < C) tile[i][tx] = in[(r0 + i) * C + c0 + tx];
    __syncthreads();
    for (int i = ty; i < 64; i += 4)
        if (c0 + i < C && r0 + tx < R) out[(int64_t)(c0 + i) * R + r0 + tx] = tile[tx][i];
}

__global__ void fill_u32_kernel(uint32_t *p, int64_t count, uint32_t v) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < count) p[i] = v;
}

// Eq.(18) for one expert: column = Gt[e][0..T), all values positive, so the fp32 bit patterns
// order like the values.  tokens[e][0..m) ascending; kept bit (t, e) set.
__global__ __launch_bounds__(256) void select_columns_kernel(const float *__restrict__ Gt, int64_t T,
                                                             int n, int m, int32_t *__restrict__ tokens,
                                                             uint32_t *__restrict__ kept, int kept_words) {
    __shared__ int hist[256];
    __shared__ uint32_t sh_prefix;
    __shared__ int sh_remaining;
    __shared__ int wave_eq[4], wave_take[4], carry_eq, carry_take;
    const int e = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t *col = reinterpret_cast<const uint32_t *>(Gt) + (int64_t)e * T;
    if (m <= 0) return;
    if (tid == 0) {
        sh_prefix = 0u;
        sh_remaining = m;
    }
    // the m-th largest key, one byte per pass from the top
    for (int pass = 3; pass >= 0; --pass) {
        hist[tid] = 0;
        __syncthreads();
        const uint32_t prefix = sh_prefix;
        const uint32_t hi_mask = pass == 3 ? 0u : (0xffffffffu << (8 * (pass + 1)));
        for (int64_t t = tid; t < T; t += 256) {
            const uint32_t key = col[t];
            if ((key & hi_mask) == prefix) atomicAdd(&hist[(key >> (8 * pass)) & 255u], 1);
        }
        __syncthreads();
        if (tid == 0) {
            int remaining = sh_remaining, b = 255;
            while (b > 0 && hist[b] < remaining) {
                remaining -= hist[b];
                --b;
            }
            sh_prefix = prefix | ((uint32_t)b << (8 * pass));
            sh_remaining = remaining;
        }
        __syncthreads();
    }
    const uint32_t vstar = sh_prefix;   // the m-th largest key
    const int ties = sh_remaining;      // how many tokens with that key are kept (lowest first)
    if (tid == 0) {
        carry_eq = 0;
        carry_take = 0;
    }
    __syncthreads();
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    for (int64_t base = 0; base < T; base += 256) {
        const int64_t t = base + tid;
        const uint32_t key = t < T ? col[t] : 0u;
        const bool gt = t < T && key > vstar;
        const bool eq = t < T && key == vstar;
        const unsigned long long beq = __ballot(eq);
        if (lane == 0) wave_eq[wave] = __popcll(beq);
        __syncthreads();
        int eq_before = carry_eq + __popcll(beq & lt_mask);
        for (int w = 0; w < wave; ++w) eq_before += wave_eq[w];
        const bool take = gt || (eq && eq_before < ties);
        const unsigned long long btk = __ballot(take);
        if (lane == 0) wave_take[wave] = __popcll(btk);
        __syncthreads();
        int pos = carry_take + __popcll(btk & lt_mask);
        for (int w = 0; w < wave; ++w) pos += wave_take[w];
        if (take) {
            tokens[(int64_t)e * m + pos] = (int32_t)t;
            atomicOr(&kept[t * kept_words + (e >> 5)], 1u << (e & 31));   // bitwise: order-independent
        }
        __syncthreads();
        if (tid == 0) {
            carry_eq += wave_eq[0] + wave_eq[1] + wave_eq[2] + wave_eq[3];
            carry_take += wave_take[0] + wave_take[1] + wave_take[2] + wave_take[3];
        }
        __syncthreads();
    }
}

// per token: denom_t = sum over kept experts of G_sigma (Eq.(16)); with thresholds also the token's
// term of Eq.(20), sum_i (M_threshold - M_batchwise)(X - T_i), written per block of four tokens
__global__ __launch_bounds__(256) void balanced_rows_kernel(const float *__restrict__ G,
                                                            const uint32_t *__restrict__ kept,
                                                            const float *__restrict__ thresholds,
                                                            int64_t T, int n, int kept_words,
                                                            float *__restrict__ denom,
                                                            double *__restrict__ loss_part) {
    __shared__ double wl[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t t = (int64_t)blockIdx.x * 4 + wave;
    double dsum = 0.0, lsum = 0.0;
    if (t < T) {
        for (int i = lane; i < n; i += 64) {
            const bool k = (kept[t * kept_words + (i >> 5)] >> (i & 31)) & 1u;
            const double x = (double)G[t * n + i];
            if (k) dsum += x;
            if (thresholds) {
                const double th = (double)thresholds[i];
                const double diff = (x > th ? 1.0 : 0.0) - (k ? 1.0 : 0.0);
                lsum += diff * (x - th);
            }
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        dsum += __shfl_xor(dsum, off);
        lsum += __shfl_xor(lsum, off);
    }
    if (lane == 0) {
        if (t < T) denom[t] = (float)dsum;
        wl[wave] = lsum;
    }
    __syncthreads();
    if (threadIdx.x == 0 && loss_part) loss_part[blockIdx.x] = ((wl[0] + wl[1]) + wl[2]) + wl[3];
}

// one workgroup: the partial sums in ascending order
__global__ __launch_bounds__(256) void sum_partials_kernel(const double *__restrict__ part, int64_t count,
                                                           float *__restrict__ out) {
    __shared__ double sh[256];
    double s = 0.0;
    const int64_t per = (count + 255) / 256;
    const int64_t b = (int64_t)threadIdx.x * per, e = min(count, b + per);
    for (int64_t i = b; i < e; ++i) s += part[i];
    sh[threadIdx.x] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        double tot = 0.0;
        for (int i = 0; i < 256; ++i) tot += sh[i];
        out[0] = (float)tot;
    }
}

// offsets, counts and the row-tile table of n experts with exactly m rows each
__global__ __launch_bounds__(256) void balanced_tiles_kernel(int n, int m, int TM, int32_t *counts,
                                                             int32_t *offsets, int32_t *tile_expert,
                                                             int32_t *tile_row0, int32_t *num_tiles) {
    const int tpe = (m + TM - 1) / TM;
    for (int e = blockIdx.x * 256 + threadIdx.x; e <= n; e += gridDim.x * 256) {
        offsets[e] = e * m;
        if (e < n) {
            counts[e] = m;
            for (int j = 0; j < tpe; ++j) {
                tile_expert[e * tpe + j] = e;
                tile_row0[e * tpe + j] = e * m + j * TM;
            }
        }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) num_tiles[0] = n * tpe;
}

// Eq.(1) with Eq.(16): one wavefront per token, kept experts in ascending order; the token's row
// in expert e's list (sorted by token) by binary search.
__global__ __launch_bounds__(256) void combine_balanced_kernel(const float4 *__restrict__ out_rows,
                                                               const float *__restrict__ G,
                                                               const uint32_t *__restrict__ kept,
                                                               const float *__restrict__ denom,
                                                               const int32_t *__restrict__ tokens,
                                                               int64_t T, int n, int m, int kept_words,
                                                               int d4, float4 *__restrict__ y) {
    const int lane = threadIdx.x & 63;
    const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    const float dn = denom[t];
    for (int c0 = 0; c0 < d4; c0 += 64) {
        const int c = c0 + lane;
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int w = 0; w < kept_words; ++w) {
            uint32_t bits = kept[t * kept_words + w];
            while (bits) {
                const int e = 32 * w + __ffs(bits) - 1;
                bits &= bits - 1;
                const int32_t *list = tokens + (int64_t)e * m;
                int lo = 0, hi = m;                       // first position with list[pos] >= t
                while (lo < hi) {
                    const int mid = (lo + hi) >> 1;
                    if (list[mid] < (int32_t)t) lo = mid + 1;
                    else hi = mid;
                }
                const float g = G[t * n + e] / dn;
                if (c < d4) {
                    const float4 v = out_rows[((int64_t)e * m + lo) * d4 + c];
                    acc.x = fmaf(g, v.x, acc.x);
                    acc.y = fmaf(g, v.y, acc.y);
                    acc.z = fmaf(g, v.z, acc.z);
                    acc.w = fmaf(g, v.w, acc.w);
                }
            }
        }
        if (c < d4) y[t * d4 + c] = acc;
    }
}

static size_t b_up256(size_t v) { return (v + 255) & ~(size_t)255; }

struct BalancedLayout {
    size_t clean, Gt, loss_part, counts, offsets, tile_expert, tile_row0, num_tiles, out_rows, ffn_ws, total;
};

static int balanced_layout(const moe_config *cfg, BalancedLayout *L) {
    const size_t T = cfg->T, n = cfg->n, A = T * (size_t)cfg->k;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off += b_up256(bytes ? bytes : 1);
        return at;
    };
    L->clean = take(T * n * 4);
    L->Gt = take(T * n * 4);
    L->loss_part = take(((T + 3) / 4) * 8);
    L->counts = take(n * 4);
    L->offsets = take((n + 1) * 4);
    const size_t mt = (size_t)moe_max_tiles(cfg) + 8;
    L->tile_expert = take(mt * 4);
    L->tile_row0 = take(mt * 4);
    L->num_tiles = take(16);
    L->out_rows = take(A * cfg->d * 4);
    moe_config f = *cfg;
    f.T = (int32_t)A;
    f.k = 1;
    L->ffn_ws = take(moe_ffn_workspace_bytes(&f));
    L->total = off;
    return MOE_OK;
}

static int balanced_check(const moe_config *cfg) {
    int st = check_config(cfg);
    if (st != MOE_OK) return st;
    if (cfg->a != 0) return MOE_EINVAL;
    if (cfg->n > kMaxGateExperts) return MOE_EUNSUPPORTED;
    if (((int64_t)cfg->T * cfg->k) % cfg->n != 0) return MOE_EINVAL;   // m = k|X|/n must be whole
    return MOE_OK;
}

}  // namespace moe

using namespace moe;

extern "C" int64_t moe_balanced_rows_per_expert(const moe_config *cfg) {
    if (balanced_check(cfg) != MOE_OK) return -1;
    return (int64_t)cfg->T * cfg->k / cfg->n;
}

extern "C" size_t moe_balanced_workspace_bytes(const moe_config *cfg) {
    if (balanced_check(cfg) != MOE_OK) return 0;
    BalancedLayout L;
    balanced_layout(cfg, &L);
    return L.total;
}

extern "C" int moe_gate_balanced(const moe_config *cfg, const float *x, const float *W_g,
                                 const float *gate_bias, const float *thresholds, float *gsigma,
                                 int32_t *tokens, uint32_t *kept, float *denom, float *loss_batchwise,
                                 void *workspace, size_t workspace_bytes, void *stream) {
    int st = balanced_check(cfg);
    if (st != MOE_OK) return st;
    if (!gsigma || !tokens || !kept || !denom || !workspace) return MOE_EINVAL;
    if (thresholds && !loss_batchwise) return MOE_EINVAL;
    BalancedLayout L;
    balanced_layout(cfg, &L);
    if (workspace_bytes < L.total) return MOE_EWORKSPACE;
    if (cfg->T == 0) return MOE_OK;
    if (!x || !W_g) return MOE_EINVAL;
    if (!aligned16(x) || !aligned16(W_g) || !aligned16(gsigma) || !aligned16(workspace)) return MOE_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    char *ws = (char *)workspace;
    const int64_t T = cfg->T;
    const int n = cfg->n, m = (int)(T * cfg->k / n), kw = (n + 31) / 32;
    float *clean = (float *)(ws + L.clean), *Gt = (float *)(ws + L.Gt);

    LogitsArgs la{};
    la.x = x; la.Wg = W_g; la.Wn = nullptr; la.bias = gate_bias; la.cleanb = clean; la.sp = nullptr;
    la.R = T; la.d = cfg->d; la.n = n;
    if ((st = launch_gate_logits(la, ceil_div(T, kGateBM), s)) != MOE_OK) return st;
    const unsigned rb = (unsigned)ceil_div(T, 4);
    if (n <= 256) hipLaunchKernelGGL(softmax_rows_kernel<4>, dim3(rb), dim3(256), 0, s, clean, T, n, gsigma);
    else if (n <= 512) hipLaunchKernelGGL(softmax_rows_kernel<8>, dim3(rb), dim3(256), 0, s, clean, T, n, gsigma);
    else if (n <= 1024) hipLaunchKernelGGL(softmax_rows_kernel<16>, dim3(rb), dim3(256), 0, s, clean, T, n, gsigma);
    else hipLaunchKernelGGL(softmax_rows_kernel<32>, dim3(rb), dim3(256), 0, s, clean, T, n, gsigma);
    MOE_LAUNCH_CHECK();
    hipLaunchKernelGGL(transpose_kernel, dim3((unsigned)ceil_div(T, 64), (unsigned)ceil_div(n, 64)), dim3(256), 0,
                       s, gsigma, T, n, Gt);
    hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)ceil_div(T * kw, 256)), dim3(256), 0, s, kept, T * kw, 0u);
    MOE_LAUNCH_CHECK();
    hipLaunchKernelGGL(select_columns_kernel, dim3(n), dim3(256), 0, s, Gt, T, n, m, tokens, kept, kw);
    MOE_LAUNCH_CHECK();
    double *lp = thresholds ? (double *)(ws + L.loss_part) : nullptr;
    hipLaunchKernelGGL(balanced_rows_kernel, dim3(rb), dim3(256), 0, s, gsigma, kept, thresholds, T, n, kw, denom, lp);
    MOE_LAUNCH_CHECK();
    if (thresholds) {
        hipLaunchKernelGGL(sum_partials_kernel, dim3(1), dim3(256), 0, s, lp, (int64_t)rb, loss_batchwise);
        MOE_LAUNCH_CHECK();
    }
    return MOE_OK;
}

extern "C" int moe_layer_forward_balanced(const moe_config *cfg, const float *x, const float *W_g,
                                          const float *gate_bias, const float *thresholds,
                                          const void *W1, const void *W2, float *y, float *gsigma,
                                          int32_t *tokens, uint32_t *kept, float *denom,
                                          float *loss_batchwise, void *workspace,
                                          size_t workspace_bytes, void *stream) {
    int st = moe_gate_balanced(cfg, x, W_g, gate_bias, thresholds, gsigma, tokens, kept, denom,
                               loss_batchwise, workspace, workspace_bytes, stream);
    if (st != MOE_OK) return st;
    if (cfg->T == 0) return MOE_OK;
    if (!W1 || !W2 || !y || !aligned16(y) || !aligned16(W1) || !aligned16(W2)) return MOE_EINVAL;
    BalancedLayout L;
    balanced_layout(cfg, &L);
    hipStream_t s = (hipStream_t)stream;
    char *ws = (char *)workspace;
    const int64_t T = cfg->T;
    const int n = cfg->n, m = (int)(T * cfg->k / n), kw = (n + 31) / 32;
    int32_t *counts = (int32_t *)(ws + L.counts), *offsets = (int32_t *)(ws + L.offsets);
    int32_t *tile_expert = (int32_t *)(ws + L.tile_expert), *tile_row0 = (int32_t *)(ws + L.tile_row0);
    int32_t *num_tiles = (int32_t *)(ws + L.num_tiles);
    float *out_rows = (float *)(ws + L.out_rows);
    hipLaunchKernelGGL(balanced_tiles_kernel, dim3((unsigned)ceil_div(n + 1, 256)), dim3(256), 0, s, n, m,
                       moe_tile_rows(cfg), counts, offsets, tile_expert, tile_row0, num_tiles);
    MOE_LAUNCH_CHECK();
    // the experts see n*m rows, each row one token: the routed-row list IS the per-expert token list
    moe_config f = *cfg;
    f.T = (int32_t)((int64_t)n * m);
    f.k = 1;
    st = expert_ffn_with_hidden(&f, x, tokens, offsets, tile_expert, tile_row0, num_tiles, W1, W2, out_rows,
                                ws + L.ffn_ws, nullptr, s);
    if (st != MOE_OK) return st;
    hipLaunchKernelGGL(combine_balanced_kernel, dim3((unsigned)ceil_div(T, 4)), dim3(256), 0, s,
                       (const float4 *)out_rows, gsigma, kept, denom, tokens, T, n, m, kw, cfg->d / 4, (float4 *)y);
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}
