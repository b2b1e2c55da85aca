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
                                                           int n, float *__restrict__ out,
                                                           uint32_t *__restrict__ kept, int kept_words) {
    const int lane = threadIdx.x & 63;
    const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    if (lane < kept_words) kept[t * kept_words + lane] = 0u;   // the selection ORs its bits into zeros
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

typedef uint32_t v4u __attribute__((ext_vector_type(4)));

// Eq.(18) for one expert: column = Gt[e][0..T), all values positive, so the fp32 bit patterns
// order like the values.  Writes tokens[e][0..m) ascending, pos[t][e] = the token's place in that
// list, and sets the kept bit (t, e); also the expert's share of the dispatch tables (m rows at
// offset e*m, ceil(m/TM) row tiles).
// A thread owns KPT consecutive tokens of a span of 256*KPT; a column that fits one span stays in
// registers for all passes.
// MODE: SEL_BATCHWISE as above.  The threshold mask of Eq.(19) runs the same column walk twice:
// SEL_THR_COUNT writes counts[e] = #{t : G_sigma(t,e) > T_e}; after the offsets are known,
// SEL_THR_COMPACT writes the list at offsets[e] (rows at or past `capacity` are dropped; the caller
// is told through the total row count).
enum { SEL_BATCHWISE = 0, SEL_THR_COUNT = 1, SEL_THR_COMPACT = 2 };

// key of a threshold: values are positive, so every threshold <= 0 keeps all of them
__device__ __forceinline__ uint32_t threshold_key(float th) { return th > 0.f ? __float_as_uint(th) : 0u; }

template <int KPT, bool VEC, int MODE>
__global__ __launch_bounds__(256) void select_columns_kernel(
    const float *__restrict__ Gt, int64_t T, int n, int m, int TM, int32_t *__restrict__ tokens,
    uint32_t *__restrict__ kept, int kept_words, int32_t *__restrict__ pos, int32_t *__restrict__ counts,
    int32_t *__restrict__ offsets, int32_t *__restrict__ tile_expert, int32_t *__restrict__ tile_row0,
    int32_t *__restrict__ num_tiles, const float *__restrict__ thresholds, int64_t capacity) {
    __shared__ int hist[256];
    __shared__ int wave_a[4], wave_b[4];
    __shared__ uint32_t sh_prefix;
    __shared__ int sh_remaining, carry_eq, carry_take;
    const int e = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) {
        sh_prefix = 0u;
        sh_remaining = m;
        carry_eq = 0;
        carry_take = 0;
    }
    if (MODE == SEL_BATCHWISE) {
        const int tpe = (m + TM - 1) / TM;
        if (tid == 0) {
            offsets[e] = e * m;
            counts[e] = m;
            if (e == n - 1) {
                offsets[n] = n * m;
                num_tiles[0] = n * tpe;
            }
        }
        for (int j = tid; j < tpe; j += 256) {
            tile_expert[e * tpe + j] = e;
            tile_row0[e * tpe + j] = e * m + j * TM;
        }
        if (m <= 0) return;
    }
    const uint32_t *col = reinterpret_cast<const uint32_t *>(Gt) + (int64_t)e * T;
    constexpr int64_t SPAN = 256 * KPT;
    const bool single = T <= SPAN;
    uint32_t kk[KPT];
    auto load = [&](int64_t base) {
        const int64_t t0 = base + (int64_t)tid * KPT;
        if (VEC) {
#pragma unroll
            for (int q = 0; q < KPT / 4; ++q) {
                const int64_t at = min(t0 + 4 * q, T - 4);    // clamped: tokens past T are masked below
                const v4u v = *reinterpret_cast<const v4u *>(col + at);
                kk[4 * q] = v.x; kk[4 * q + 1] = v.y; kk[4 * q + 2] = v.z; kk[4 * q + 3] = v.w;
            }
        } else {
#pragma unroll
            for (int j = 0; j < KPT; ++j) kk[j] = col[min(t0 + j, T - 1)];
        }
    };

    if (MODE == SEL_THR_COUNT) {
        const uint32_t tk = threshold_key(thresholds[e]);
        int c = 0;
        for (int64_t base = 0; base < T; base += SPAN) {
            load(base);
            const int64_t t0 = base + (int64_t)tid * KPT;
#pragma unroll
            for (int j = 0; j < KPT; ++j) c += t0 + j < T && kk[j] > tk;
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) c += __shfl_xor(c, off);
        if (lane == 0) wave_a[wave] = c;
        __syncthreads();
        if (tid == 0) counts[e] = wave_a[0] + wave_a[1] + wave_a[2] + wave_a[3];
        return;
    }

    // the m-th largest key, one byte per pass from the top
    for (int pass = 3; MODE == SEL_BATCHWISE && pass >= 0; --pass) {
        hist[tid] = 0;
        __syncthreads();
        const uint32_t prefix = sh_prefix;
        const int remaining = sh_remaining;
        const uint32_t hi_mask = pass == 3 ? 0u : (0xffffffffu << (8 * (pass + 1)));
        for (int64_t base = 0; base < T; base += SPAN) {
            if (!single || pass == 3) load(base);
            const int64_t t0 = base + (int64_t)tid * KPT;
            int run_bin = -1, run = 0;                       // equal neighbours share one LDS atomic
#pragma unroll
            for (int j = 0; j < KPT; ++j) {
                const bool in = t0 + j < T && (kk[j] & hi_mask) == prefix;
                const int bin = (int)((kk[j] >> (8 * pass)) & 255u);
                if (in) {
                    if (bin == run_bin) {
                        ++run;
                    } else {
                        if (run) atomicAdd(&hist[run_bin], run);
                        run_bin = bin;
                        run = 1;
                    }
                }
            }
            if (run) atomicAdd(&hist[run_bin], run);
        }
        __syncthreads();
        // bin b with  #(bins above b) < remaining <= #(bins above b) + hist[b]
        const int hcount = hist[tid];
        int sfx = hcount;                                    // sum over lanes >= lane of this wave
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int v = __shfl_down(sfx, off);
            if (lane + off < 64) sfx += v;
        }
        if (lane == 0) wave_a[wave] = sfx;
        __syncthreads();
        int above = sfx - hcount;
        for (int w = wave + 1; w < 4; ++w) above += wave_a[w];
        if (hcount > 0 && above < remaining && remaining <= above + hcount) {
            sh_prefix = prefix | ((uint32_t)tid << (8 * pass));
            sh_remaining = remaining - above;
        }
        __syncthreads();
    }
    if (MODE == SEL_THR_COMPACT) __syncthreads();    // the carries written above
    // batchwise: the m-th largest key and how many tokens with that key are kept (lowest first)
    const uint32_t vstar = MODE == SEL_BATCHWISE ? sh_prefix : threshold_key(thresholds[e]);
    const int ties = MODE == SEL_BATCHWISE ? sh_remaining : 0;
    const int64_t row_base = MODE == SEL_BATCHWISE ? (int64_t)e * m : (int64_t)offsets[e];

    for (int64_t base = 0; base < T; base += SPAN) {
        if (!single || MODE == SEL_THR_COMPACT) load(base);
        const int64_t t0 = base + (int64_t)tid * KPT;
        int gt_cnt = 0, eq_cnt = 0;
#pragma unroll
        for (int j = 0; j < KPT; ++j) {
            const bool valid = t0 + j < T;
            gt_cnt += valid && kk[j] > vstar;
            eq_cnt += valid && kk[j] == vstar;
        }
        // exclusive block scan of the equal counts, then of the kept counts they imply
        int inc = eq_cnt;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int v = __shfl_up(inc, off);
            if (lane >= off) inc += v;
        }
        if (lane == 63) wave_a[wave] = inc;
        __syncthreads();
        int eq_before = carry_eq + inc - eq_cnt;
        for (int w = 0; w < wave; ++w) eq_before += wave_a[w];
        const int take_cnt = gt_cnt + min(eq_cnt, max(ties - eq_before, 0));
        int inc2 = take_cnt;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int v = __shfl_up(inc2, off);
            if (lane >= off) inc2 += v;
        }
        if (lane == 63) wave_b[wave] = inc2;
        __syncthreads();
        int at = carry_take + inc2 - take_cnt;
        for (int w = 0; w < wave; ++w) at += wave_b[w];
#pragma unroll
        for (int j = 0; j < KPT; ++j) {
            const int64_t t = t0 + j;
            const bool valid = t < T;
            const bool eq = valid && kk[j] == vstar;
            const bool take = (valid && kk[j] > vstar) || (eq && eq_before < ties);
            eq_before += eq;
            if (take) {
                if (MODE == SEL_BATCHWISE || row_base + at < capacity) tokens[row_base + at] = (int32_t)t;
                pos[t * n + e] = at;
                atomicOr(&kept[t * kept_words + (e >> 5)], 1u << (e & 31));   // bitwise: order-independent
                ++at;
            }
        }
        __syncthreads();
        if (tid == 0) {
            carry_eq += wave_a[0] + wave_a[1] + wave_a[2] + wave_a[3];
            carry_take += wave_b[0] + wave_b[1] + wave_b[2] + wave_b[3];
        }
        __syncthreads();
    }
}

// threshold path: offsets = exclusive scan of counts, the row-tile table, the total row count.
// One workgroup; n <= 2048, eight experts per thread.  More rows than `capacity`: no tiles.
__global__ __launch_bounds__(256) void threshold_offsets_kernel(const int32_t *__restrict__ counts, int n, int TM,
                                                                int64_t capacity, int32_t *__restrict__ offsets,
                                                                int32_t *__restrict__ tile_expert,
                                                                int32_t *__restrict__ tile_row0,
                                                                int32_t *__restrict__ num_tiles,
                                                                int32_t *__restrict__ rows_total) {
    __shared__ int wave_r[4], wave_t[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int c[8], rows = 0, tiles = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int e = tid * 8 + j;
        c[j] = e < n ? counts[e] : 0;
        rows += c[j];
        tiles += (c[j] + TM - 1) / TM;
    }
    int ir = rows, it = tiles;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int vr = __shfl_up(ir, off), vt = __shfl_up(it, off);
        if (lane >= off) {
            ir += vr;
            it += vt;
        }
    }
    if (lane == 63) {
        wave_r[wave] = ir;
        wave_t[wave] = it;
    }
    __syncthreads();
    int r = ir - rows, tl = it - tiles;
    for (int w = 0; w < wave; ++w) {
        r += wave_r[w];
        tl += wave_t[w];
    }
    const int64_t total = (int64_t)wave_r[0] + wave_r[1] + wave_r[2] + wave_r[3];
    const bool fits = total <= capacity;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int e = tid * 8 + j;
        if (e < n) {
            offsets[e] = r;
            if (fits)
                for (int q = 0; q * TM < c[j]; ++q) {
                    tile_expert[tl] = e;
                    tile_row0[tl] = r + q * TM;
                    ++tl;
                }
            r += c[j];
        }
    }
    if (tid == 0) {
        offsets[n] = (int32_t)total;
        rows_total[0] = (int32_t)total;
        num_tiles[0] = fits ? wave_t[0] + wave_t[1] + wave_t[2] + wave_t[3] : 0;
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

// Eq.(1) with Eq.(16): one wavefront per token.  The lanes first list the token's kept experts in
// ascending order (row in the dispatch and gate value, 64 at a time in LDS), then every lane adds
// the listed rows for its columns, so the row loads are independent of each other.
// NC: float4 columns per lane (d/4 <= 64*NC).
// ADD: the backward pass's use of the same walk -- y[t] += the plain sum of the token's rows (G,
// denom and rows_total unused).
template <int NC, bool ADD>
__global__ __launch_bounds__(256) void combine_balanced_kernel(const float4 *__restrict__ out_rows,
                                                               const float *__restrict__ G,
                                                               const uint32_t *__restrict__ kept,
                                                               const int32_t *__restrict__ pos,
                                                               const float *__restrict__ denom,
                                                               const int32_t *__restrict__ offsets,
                                                               const int32_t *__restrict__ rows_total,
                                                               int64_t capacity, int64_t T, int n,
                                                               int kept_words, int d4, float4 *__restrict__ y) {
    __shared__ int l_row[4][64];
    __shared__ float l_g[4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t t = (int64_t)blockIdx.x * 4 + wave;
    if (t >= T) return;
    if (!ADD && rows_total && rows_total[0] > capacity) {   // the dispatch did not fit: no rows were computed
#pragma unroll
        for (int c = 0; c < NC; ++c)
            if (lane + 64 * c < d4) y[t * d4 + lane + 64 * c] = make_float4(0.f, 0.f, 0.f, 0.f);
        return;
    }
    const float dn = ADD ? 1.f : denom[t];
    const uint32_t bits = lane < kept_words ? kept[t * kept_words + lane] : 0u;   // kept_words <= 64
    const int cnt = __popc(bits);
    int inc = cnt;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int v = __shfl_up(inc, off);
        if (lane >= off) inc += v;
    }
    const int total = __shfl(inc, 63);
    const int before = inc - cnt;
    float4 acc[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) acc[c] = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int r0 = 0; r0 < total; r0 += 64) {
        int idx = before;
        uint32_t b = bits;
        while (b) {
            const int e = 32 * lane + __ffs(b) - 1;
            b &= b - 1;
            if (idx >= r0 && idx < r0 + 64) {
                l_row[wave][idx - r0] = offsets[e] + pos[t * n + e];
                l_g[wave][idx - r0] = ADD ? 1.f : G[t * n + e] / dn;
            }
            ++idx;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const int here = min(64, total - r0);
#pragma unroll 4
        for (int j = 0; j < here; ++j) {
            const int64_t row = l_row[wave][j];
            const float g = l_g[wave][j];
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const int col = lane + 64 * c;
                if (col < d4) {
                    const float4 v = out_rows[row * d4 + col];
                    acc[c].x = fmaf(g, v.x, acc[c].x);
                    acc[c].y = fmaf(g, v.y, acc[c].y);
                    acc[c].z = fmaf(g, v.z, acc[c].z);
                    acc[c].w = fmaf(g, v.w, acc[c].w);
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
#pragma unroll
    for (int c = 0; c < NC; ++c)
        if (lane + 64 * c < d4) {
            if (ADD) {
                const float4 v = y[t * d4 + lane + 64 * c];
                acc[c] = make_float4(v.x + acc[c].x, v.y + acc[c].y, v.z + acc[c].z, v.w + acc[c].w);
            }
            y[t * d4 + lane + 64 * c] = acc[c];
        }
}

// gate value of every dispatched row: row r belongs to the expert e with offsets[e] <= r <
// offsets[e+1] and holds token tokens[r]; G = G_sigma(t,e) / denom[t] as the combine forms it
__global__ __launch_bounds__(256) void balanced_row_gate_kernel(const float *__restrict__ G,
                                                                const float *__restrict__ denom,
                                                                const int32_t *__restrict__ tokens,
                                                                const int32_t *__restrict__ offsets, int n,
                                                                int64_t rows, float *__restrict__ row_gate) {
    const int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (r >= rows) return;
    int lo = 0, hi = n;   // the last e with offsets[e] <= r (never an empty expert)
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (offsets[mid] <= r) lo = mid; else hi = mid;
    }
    const int64_t t = tokens[r];
    row_gate[r] = G[t * n + lo] / denom[t];
}

// Backward of Eq.(16), Eq.(20) and Eq.(15) for one token per wavefront.  drow[r] = <dy_t, E_e(x_t)>
// of the token's row at expert e.  With D = denom and G_i = G_sigma_i M_i / D:
//   dG_sigma_i = M_i (dG_i - sum_j G_j dG_j) / D  +  w_b ((G_sigma_i > T_i) - M_i)
//   dlogit_i   = G_sigma_i (dG_sigma_i - sum_j G_sigma_j dG_sigma_j)
// (the masks are piecewise constant).  Sums in binary64, lanes strided over the experts, butterfly
// reduction (the same total in every lane).
__global__ __launch_bounds__(256) void balanced_gate_bwd_kernel(const float *__restrict__ G,
                                                                const uint32_t *__restrict__ kept,
                                                                const int32_t *__restrict__ pos,
                                                                const float *__restrict__ denom,
                                                                const int32_t *__restrict__ offsets,
                                                                const float *__restrict__ drow,
                                                                const float *__restrict__ thresholds,
                                                                float w_b, int64_t T, int n, int kept_words,
                                                                float *__restrict__ dlogit) {
    const int lane = threadIdx.x & 63;
    const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    const float dn = denom[t];
    const float *g = G + t * n;
    const int32_t *ps = pos + t * n;
    const uint32_t *kb = kept + t * kept_words;
    auto is_kept = [&](int i) { return ((kb[i >> 5] >> (i & 31)) & 1u) != 0u; };
    auto wave_sum = [&](double v) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
        return v;
    };
    double inner = 0.0;
    for (int i = lane; i < n; i += 64)
        if (is_kept(i)) inner += (double)(g[i] / dn) * (double)drow[offsets[i] + ps[i]];
    inner = wave_sum(inner);
    auto dsigma = [&](int i) {
        const bool kp = is_kept(i);
        double v = kp ? ((double)drow[offsets[i] + ps[i]] - inner) / (double)dn : 0.0;
        if (thresholds) v += (double)w_b * ((g[i] > thresholds[i] ? 1.0 : 0.0) - (kp ? 1.0 : 0.0));
        return v;
    };
    double u = 0.0;
    for (int i = lane; i < n; i += 64) u += (double)g[i] * dsigma(i);
    u = wave_sum(u);
    for (int i = lane; i < n; i += 64) dlogit[t * n + i] = (float)((double)g[i] * (dsigma(i) - u));
}

// d L_batchwise / d T_i = m_i - #{t : G_sigma(t,i) > T_i} (both masks are piecewise constant in T).
// A workgroup takes 64 experts (a lane each, rows read 256 bytes at a time), its four waves a
// quarter of the tokens each; kept_count[i] is the number the batchwise mask keeps (m for all).
__global__ __launch_bounds__(256) void threshold_grad_kernel(const float *__restrict__ G,
                                                             const float *__restrict__ thresholds, int64_t T,
                                                             int n, int m, float *__restrict__ dthr) {
    __shared__ int part[4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = blockIdx.x * 64 + lane;
    const float th = i < n ? thresholds[i] : 0.f;
    int cnt = 0;
    for (int64_t t = wave; t < T; t += 4) cnt += (i < n && G[t * n + i] > th) ? 1 : 0;
    part[wave][lane] = cnt;
    __syncthreads();
    if (wave == 0 && i < n) dthr[i] = (float)(m - (part[0][lane] + part[1][lane] + part[2][lane] + part[3][lane]));
}

static size_t b_up256(size_t v) { return (v + 255) & ~(size_t)255; }

struct BalancedLayout {
    size_t clean, Gt, pos, loss_part, counts, offsets, tile_expert, tile_row0, num_tiles, out_rows, ffn_ws,
        hidden, total;   // hidden: bf16 [rows, h] with MOE_FLAG_SAVE_HIDDEN and bf16 experts, else (size_t)-1
};

// the experts see `rows` dispatched rows, each one token: a flat layer of `rows` tokens with k = 1
static moe_config expert_view(const moe_config *cfg, int64_t rows) {
    moe_config f = *cfg;
    f.T = (int32_t)rows;
    f.k = 1;
    return f;
}

// rows: dispatched rows the buffers hold (k*T for the batchwise mask, the caller's capacity for
// the threshold mask)
static void balanced_layout(const moe_config *cfg, int64_t rows, BalancedLayout *L) {
    const size_t T = cfg->T, n = cfg->n;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off += b_up256(bytes ? bytes : 1);
        return at;
    };
    L->clean = take(T * n * 4);
    L->Gt = take(T * n * 4);
    L->pos = take(T * n * 4);
    L->loss_part = take(((T + 3) / 4) * 8);
    L->counts = take(n * 4);
    L->offsets = take((n + 1) * 4);
    const moe_config f = expert_view(cfg, rows);
    const size_t mt = (size_t)moe_max_tiles(&f) + 8;
    L->tile_expert = take(mt * 4);
    L->tile_row0 = take(mt * 4);
    L->num_tiles = take(16);
    L->out_rows = take((size_t)rows * cfg->d * 4);
    L->ffn_ws = take(moe_ffn_workspace_bytes(&f));
    const bool keep_hidden = (cfg->flags & MOE_FLAG_SAVE_HIDDEN) && cfg->expert_dtype == MOE_DTYPE_BF16;
    L->hidden = keep_hidden ? take((size_t)rows * cfg->h * 2) : (size_t)-1;
    L->total = off;
}

static int softmax_gate_check(const moe_config *cfg) {
    int st = check_config(cfg);
    if (st != MOE_OK) return st;
    if (cfg->a != 0) return MOE_EINVAL;
    if (cfg->n > kMaxBalancedExperts) return MOE_EUNSUPPORTED;
    if (cfg->d > 2048) return MOE_EUNSUPPORTED;                        // combine: 8 float4 per lane
    return MOE_OK;
}

static int balanced_check(const moe_config *cfg) {
    int st = softmax_gate_check(cfg);
    if (st != MOE_OK) return st;
    if (((int64_t)cfg->T * cfg->k) % cfg->n != 0) return MOE_EINVAL;   // m = k|X|/n must be whole
    return MOE_OK;
}

static int threshold_check(const moe_config *cfg, int64_t row_capacity) {
    int st = softmax_gate_check(cfg);
    if (st != MOE_OK) return st;
    if (row_capacity < 0 || row_capacity >= ((int64_t)1 << 31)) return MOE_EINVAL;
    if ((int64_t)cfg->T * cfg->n >= ((int64_t)1 << 31)) return MOE_EUNSUPPORTED;   // the row count is an int32
    return MOE_OK;
}

// Eq.(15) and its transposed copy; clears the kept bits
static int launch_softmax_gate(const moe_config *cfg, const float *x, const float *W_g, const float *gate_bias,
                               float *clean, float *gsigma, float *Gt, uint32_t *kept, hipStream_t s) {
    const int64_t T = cfg->T;
    const int n = cfg->n, kw = (n + 31) / 32;
    LogitsArgs la{};
    la.x = x; la.Wg = W_g; la.Wn = nullptr; la.bias = gate_bias; la.cleanb = clean; la.sp = nullptr;
    la.R = T; la.d = cfg->d; la.n = n;
    int st = launch_gate_logits(la, ceil_div(T, kGateBM), s);
    if (st != MOE_OK) return st;
    const unsigned rb = (unsigned)ceil_div(T, 4);
    if (n <= 256) hipLaunchKernelGGL(softmax_rows_kernel<4>, dim3(rb), dim3(256), 0, s, clean, T, n, gsigma, kept, kw);
    else if (n <= 512) hipLaunchKernelGGL(softmax_rows_kernel<8>, dim3(rb), dim3(256), 0, s, clean, T, n, gsigma, kept, kw);
    else if (n <= 1024) hipLaunchKernelGGL(softmax_rows_kernel<16>, dim3(rb), dim3(256), 0, s, clean, T, n, gsigma, kept, kw);
    else hipLaunchKernelGGL(softmax_rows_kernel<32>, dim3(rb), dim3(256), 0, s, clean, T, n, gsigma, kept, kw);
    MOE_LAUNCH_CHECK();
    hipLaunchKernelGGL(transpose_kernel, dim3((unsigned)ceil_div(T, 64), (unsigned)ceil_div(n, 64)), dim3(256), 0,
                       s, gsigma, T, n, Gt);
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}

struct SelectArgs {
    const float *Gt;
    int64_t T;
    int n, m, TM;
    int32_t *tokens;
    uint32_t *kept;
    int32_t *pos, *counts, *offsets, *tile_expert, *tile_row0, *num_tiles;
    const float *thresholds;
    int64_t capacity;
};

template <int MODE>
static int launch_select(const SelectArgs &a, hipStream_t s) {
    const int kw = (a.n + 31) / 32;
#define MOE_SELECT(KPT, VEC)                                                                                  \
    hipLaunchKernelGGL((select_columns_kernel<KPT, VEC, MODE>), dim3(a.n), dim3(256), 0, s, a.Gt, a.T, a.n, a.m, \
                       a.TM, a.tokens, a.kept, kw, a.pos, a.counts, a.offsets, a.tile_expert, a.tile_row0,     \
                       a.num_tiles, a.thresholds, a.capacity)
    const bool vec = a.T % 4 == 0;
    if (a.T <= 256 * 8) { if (vec) MOE_SELECT(8, true); else MOE_SELECT(8, false); }
    else { if (vec) MOE_SELECT(32, true); else MOE_SELECT(32, false); }
#undef MOE_SELECT
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}

static int launch_combine_balanced(const moe_config *cfg, const float *out_rows, const float *gsigma,
                                   const uint32_t *kept, const int32_t *pos, const float *denom,
                                   const int32_t *offsets, const int32_t *rows_total, int64_t capacity, float *y,
                                   hipStream_t s) {
    const int64_t T = cfg->T;
    const int n = cfg->n, kw = (n + 31) / 32, d4 = cfg->d / 4;
    const dim3 grid((unsigned)ceil_div(T, 4));
#define MOE_COMBINE(NC)                                                                                    \
    hipLaunchKernelGGL((combine_balanced_kernel<NC, false>), grid, dim3(256), 0, s, (const float4 *)out_rows, gsigma, \
                       kept, pos, denom, offsets, rows_total, capacity, T, n, kw, d4, (float4 *)y)
    if (d4 <= 64) MOE_COMBINE(1);
    else if (d4 <= 128) MOE_COMBINE(2);
    else if (d4 <= 256) MOE_COMBINE(4);
    else MOE_COMBINE(8);
#undef MOE_COMBINE
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}

// ---- pieces of the backward pass (the entry point sits with the other backward code) ----------
int balanced_forward_view(const moe_config *cfg, BalancedFwdView *v) {
    int st = balanced_check(cfg);
    if (st != MOE_OK) return st;
    BalancedLayout L;
    balanced_layout(cfg, (int64_t)cfg->T * cfg->k, &L);
    v->pos = L.pos; v->offsets = L.offsets; v->out_rows = L.out_rows; v->ffn_ws = L.ffn_ws;
    v->hidden = L.hidden; v->total = L.total;
    return MOE_OK;
}

int launch_balanced_row_gates(const float *gsigma, const float *denom, const int32_t *tokens,
                              const int32_t *offsets, int n, int64_t rows, float *row_gate, hipStream_t s) {
    if (rows == 0) return MOE_OK;
    hipLaunchKernelGGL(balanced_row_gate_kernel, dim3((unsigned)ceil_div(rows, 256)), dim3(256), 0, s, gsigma,
                       denom, tokens, offsets, n, rows, row_gate);
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}

int launch_balanced_gate_bwd(const moe_config *cfg, const float *gsigma, const uint32_t *kept, const int32_t *pos,
                             const float *denom, const int32_t *offsets, const float *drow,
                             const float *thresholds, float w_batchwise, float *dlogit, hipStream_t s) {
    hipLaunchKernelGGL(balanced_gate_bwd_kernel, dim3((unsigned)ceil_div((int64_t)cfg->T, 4)), dim3(256), 0, s,
                       gsigma, kept, pos, denom, offsets, drow, thresholds, w_batchwise, (int64_t)cfg->T, cfg->n,
                       (cfg->n + 31) / 32, dlogit);
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}

int launch_add_kept_rows(const moe_config *cfg, const float *rows_mat, const uint32_t *kept, const int32_t *pos,
                         const int32_t *offsets, float *dx, hipStream_t s) {
    const int64_t T = cfg->T;
    const int n = cfg->n, kw = (n + 31) / 32, d4 = cfg->d / 4;
    const dim3 grid((unsigned)ceil_div(T, 4));
#define MOE_ADD(NC)                                                                                          \
    hipLaunchKernelGGL((combine_balanced_kernel<NC, true>), grid, dim3(256), 0, s, (const float4 *)rows_mat,  \
                       (const float *)nullptr, kept, pos, (const float *)nullptr, offsets,                   \
                       (const int32_t *)nullptr, (int64_t)0, T, n, kw, d4, (float4 *)dx)
    if (d4 <= 64) MOE_ADD(1);
    else if (d4 <= 128) MOE_ADD(2);
    else if (d4 <= 256) MOE_ADD(4);
    else MOE_ADD(8);
#undef MOE_ADD
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}

static int record_event(void *const *ev, int i, hipStream_t s) {
    if (!ev || !ev[i]) return MOE_OK;
    MOE_HIP_TRY(hipEventRecord((hipEvent_t)ev[i], s));
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
    balanced_layout(cfg, (int64_t)cfg->T * cfg->k, &L);
    return L.total;
}

extern "C" size_t moe_threshold_workspace_bytes(const moe_config *cfg, int64_t row_capacity) {
    if (threshold_check(cfg, row_capacity) != MOE_OK) return 0;
    BalancedLayout L;
    balanced_layout(cfg, row_capacity, &L);
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
    balanced_layout(cfg, (int64_t)cfg->T * cfg->k, &L);
    if (workspace_bytes < L.total) return MOE_EWORKSPACE;
    if (cfg->T == 0) return MOE_OK;
    if (!x || !W_g) return MOE_EINVAL;
    if (!aligned16(x) || !aligned16(W_g) || !aligned16(gsigma) || !aligned16(workspace)) return MOE_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    char *ws = (char *)workspace;
    const int64_t T = cfg->T;
    const int n = cfg->n, kw = (n + 31) / 32;
    float *Gt = (float *)(ws + L.Gt);
    if ((st = launch_softmax_gate(cfg, x, W_g, gate_bias, (float *)(ws + L.clean), gsigma, Gt, kept, s)) != MOE_OK)
        return st;
    SelectArgs sa{};
    sa.Gt = Gt; sa.T = T; sa.n = n; sa.m = (int)(T * cfg->k / n);
    {   // the tile height the expert kernel will be launched with (it sees T*k rows with k = 1)
        const moe_config fv = expert_view(cfg, T * cfg->k);
        sa.TM = moe_tile_rows(&fv);
    }
    sa.tokens = tokens; sa.kept = kept; sa.pos = (int32_t *)(ws + L.pos); sa.counts = (int32_t *)(ws + L.counts);
    sa.offsets = (int32_t *)(ws + L.offsets); sa.tile_expert = (int32_t *)(ws + L.tile_expert);
    sa.tile_row0 = (int32_t *)(ws + L.tile_row0); sa.num_tiles = (int32_t *)(ws + L.num_tiles);
    if ((st = launch_select<SEL_BATCHWISE>(sa, s)) != MOE_OK) return st;
    const unsigned rb = (unsigned)ceil_div(T, 4);
    double *lp = thresholds ? (double *)(ws + L.loss_part) : nullptr;
    hipLaunchKernelGGL(balanced_rows_kernel, dim3(rb), dim3(256), 0, s, gsigma, kept, thresholds, T, n, kw, denom, lp);
    MOE_LAUNCH_CHECK();
    if (thresholds) {
        hipLaunchKernelGGL(sum_partials_kernel, dim3(1), dim3(256), 0, s, lp, (int64_t)rb, loss_batchwise);
        MOE_LAUNCH_CHECK();
    }
    return MOE_OK;
}

extern "C" int moe_layer_forward_balanced_profiled(const moe_config *cfg, const float *x, const float *W_g,
                                                   const float *gate_bias, const float *thresholds,
                                                   const void *W1, const void *W2, float *y, float *gsigma,
                                                   int32_t *tokens, uint32_t *kept, float *denom,
                                                   float *loss_batchwise, void *workspace,
                                                   size_t workspace_bytes, void *const *ev, void *stream) {
    hipStream_t s = (hipStream_t)stream;
    int st = balanced_check(cfg);
    if (st != MOE_OK) return st;
    if (cfg->T > 0 && (!W1 || !W2 || !y || !aligned16(y) || !aligned16(W1) || !aligned16(W2))) return MOE_EINVAL;
    if ((st = record_event(ev, 0, s)) != MOE_OK) return st;
    st = moe_gate_balanced(cfg, x, W_g, gate_bias, thresholds, gsigma, tokens, kept, denom,
                           loss_batchwise, workspace, workspace_bytes, stream);
    if (st != MOE_OK) return st;
    if ((st = record_event(ev, 1, s)) != MOE_OK) return st;
    if (cfg->T == 0) return MOE_OK;
    const int64_t rows = (int64_t)cfg->T * cfg->k;
    BalancedLayout L;
    balanced_layout(cfg, rows, &L);
    char *ws = (char *)workspace;
    const int32_t *offsets = (const int32_t *)(ws + L.offsets);
    float *out_rows = (float *)(ws + L.out_rows);
    // the routed-row list IS the per-expert token list
    const moe_config f = expert_view(cfg, rows);
    if ((st = record_event(ev, 2, s)) != MOE_OK) return st;
    st = expert_ffn_with_hidden(&f, x, tokens, offsets, (const int32_t *)(ws + L.tile_expert),
                                (const int32_t *)(ws + L.tile_row0), (const int32_t *)(ws + L.num_tiles), W1, W2,
                                out_rows, ws + L.ffn_ws, L.hidden != (size_t)-1 ? (uint16_t *)(ws + L.hidden) : nullptr, s);
    if (st != MOE_OK) return st;
    if ((st = record_event(ev, 3, s)) != MOE_OK) return st;
    st = launch_combine_balanced(cfg, out_rows, gsigma, kept, (const int32_t *)(ws + L.pos), denom, offsets,
                                 nullptr, rows, y, s);
    if (st != MOE_OK) return st;
    return record_event(ev, 4, s);
}

extern "C" int moe_layer_forward_balanced(const moe_config *cfg, const float *x, const float *W_g,
                                          const float *gate_bias, const float *thresholds,
                                          const void *W1, const void *W2, float *y, float *gsigma,
                                          int32_t *tokens, uint32_t *kept, float *denom,
                                          float *loss_batchwise, void *workspace,
                                          size_t workspace_bytes, void *stream) {
    return moe_layer_forward_balanced_profiled(cfg, x, W_g, gate_bias, thresholds, W1, W2, y, gsigma, tokens,
                                               kept, denom, loss_batchwise, workspace, workspace_bytes,
                                               nullptr, stream);
}

extern "C" int moe_layer_forward_threshold(const moe_config *cfg, const float *x, const float *W_g,
                                           const float *gate_bias, const float *thresholds, const void *W1,
                                           const void *W2, int64_t row_capacity, float *y, float *gsigma,
                                           int32_t *counts, int32_t *tokens, uint32_t *kept, float *denom,
                                           int32_t *rows_total, void *workspace, size_t workspace_bytes,
                                           void *stream) {
    int st = threshold_check(cfg, row_capacity);
    if (st != MOE_OK) return st;
    if (!thresholds || !gsigma || !counts || !tokens || !kept || !denom || !rows_total || !workspace)
        return MOE_EINVAL;
    BalancedLayout L;
    balanced_layout(cfg, row_capacity, &L);
    if (workspace_bytes < L.total) return MOE_EWORKSPACE;
    if (cfg->T == 0) return MOE_OK;
    if (!x || !W_g || !W1 || !W2 || !y) return MOE_EINVAL;
    if (!aligned16(x) || !aligned16(W_g) || !aligned16(gsigma) || !aligned16(workspace) || !aligned16(y) ||
        !aligned16(W1) || !aligned16(W2))
        return MOE_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    char *ws = (char *)workspace;
    const int64_t T = cfg->T;
    const int n = cfg->n, kw = (n + 31) / 32;
    float *Gt = (float *)(ws + L.Gt);
    if ((st = launch_softmax_gate(cfg, x, W_g, gate_bias, (float *)(ws + L.clean), gsigma, Gt, kept, s)) != MOE_OK)
        return st;
    SelectArgs sa{};
    sa.Gt = Gt; sa.T = T; sa.n = n; sa.m = 0;
    {
        const moe_config fv = expert_view(cfg, row_capacity);
        sa.TM = moe_tile_rows(&fv);
    }
    sa.tokens = tokens; sa.kept = kept; sa.pos = (int32_t *)(ws + L.pos); sa.counts = counts;
    sa.offsets = (int32_t *)(ws + L.offsets); sa.tile_expert = (int32_t *)(ws + L.tile_expert);
    sa.tile_row0 = (int32_t *)(ws + L.tile_row0); sa.num_tiles = (int32_t *)(ws + L.num_tiles);
    sa.thresholds = thresholds; sa.capacity = row_capacity;
    if ((st = launch_select<SEL_THR_COUNT>(sa, s)) != MOE_OK) return st;
    hipLaunchKernelGGL(threshold_offsets_kernel, dim3(1), dim3(256), 0, s, counts, n, sa.TM, row_capacity, sa.offsets,
                       sa.tile_expert, sa.tile_row0, sa.num_tiles, rows_total);
    MOE_LAUNCH_CHECK();
    if ((st = launch_select<SEL_THR_COMPACT>(sa, s)) != MOE_OK) return st;
    hipLaunchKernelGGL(balanced_rows_kernel, dim3((unsigned)ceil_div(T, 4)), dim3(256), 0, s, gsigma, kept,
                       (const float *)nullptr, T, n, kw, denom, (double *)nullptr);
    MOE_LAUNCH_CHECK();
    float *out_rows = (float *)(ws + L.out_rows);
    const moe_config f = expert_view(cfg, row_capacity);
    if (row_capacity > 0) {
        st = expert_ffn_with_hidden(&f, x, tokens, sa.offsets, sa.tile_expert, sa.tile_row0, sa.num_tiles, W1, W2,
                                    out_rows, ws + L.ffn_ws, nullptr, s);
        if (st != MOE_OK) return st;
    }
    return launch_combine_balanced(cfg, out_rows, gsigma, kept, sa.pos, denom, sa.offsets, rows_total, row_capacity,
                                   y, s);
}

extern "C" int moe_batchwise_loss_grad(const moe_config *cfg, const float *gsigma, const float *thresholds,
                                       float *dthresholds, void *stream) {
    int st = balanced_check(cfg);
    if (st != MOE_OK) return st;
    if (!gsigma || !thresholds || !dthresholds) return MOE_EINVAL;
    const int64_t T = cfg->T;
    const int n = cfg->n, m = (int)(T * cfg->k / n);
    hipLaunchKernelGGL(threshold_grad_kernel, dim3((unsigned)ceil_div(n, 64)), dim3(256), 0, (hipStream_t)stream,
                       gsigma, thresholds, T, n, m, dthresholds);
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}
