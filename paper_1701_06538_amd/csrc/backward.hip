// a6: backward pass of the flat layer (Section 2.1 "Training the Gating Network": plain
// back-propagation through the kept gate values, the experts and both balancing losses;
// Appendix D: the experts' hidden activations are recomputed, not stored).
//
// Objective: J = <dy, y> + w_importance CV^2(Importance) + w_load CV^2(Load).
//
//   bwd_prepare_kernel   per routed row: dout = gate * dy (bf16), x row (bf16), dgate = <dy, E(x)>
//   gg_rows_kernel       grouped bf16 MFMA GEMM over the ragged rows of each expert:
//                          hid = relu(xs W1)            dz = (dout W2^T) * [hid > 0]
//                          dxs = dz W1^T
//   gg_wgrad_kernel      (gemm_wgrad.hip) per expert, contraction over its rows: dW2 = hid^T dout, dW1 = xs^T dz
//   gate_bwd_rows_kernel per token: softmax-over-k backward, d/dclean and d/draw of Eq.(9) incl.
//                        the threshold element, H = clean + eps * sp
//   sg_kernel            fp32 MFMA GEMMs of the gate: dW_g = x^T dclean, dW_noise = x^T draw
//                        (split over tokens, partial sums added in a fixed order) and
//                        dx = dclean W_g^T + draw W_noise^T
//   dx_gather_add_kernel dx[t] += sum_s dxs[row of (t,s)]
#include "stages.h"

namespace moe {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

__device__ __forceinline__ uint32_t bf16_rne(float f) { return bf16_bits_of(f); }
__device__ __forceinline__ uint32_t pack2(float lo, float hi) { return pack_bf16_pair(lo, hi); }
__device__ __forceinline__ float bf16_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

// ---------------------------------------------------------------------------------------
// per routed row: dout, xs, dgate
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void bwd_prepare_kernel(const float *__restrict__ x,
                                                          const float *__restrict__ dy,
                                                          const float *__restrict__ out_sorted,
                                                          const float *__restrict__ gate,
                                                          const int32_t *__restrict__ perm, int64_t A,
                                                          int d, int k, int by_row,
                                                          uint16_t *__restrict__ xs,   // null: the forward pass kept these rows
                                                          uint16_t *__restrict__ dout,
                                                          float *__restrict__ dgate) {
    const int lane = threadIdx.x & 63;
    const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= A) return;
    // by_row: perm lists tokens, gate and dgate are indexed by the routed row itself
    const int64_t a = by_row ? r : perm[r];
    const int64_t t = by_row ? perm[r] : a / k;
    const float g = gate[a];
    float dot = 0.f;
    for (int c = lane * 4; c < d; c += 256) {
        const float4 vy = *reinterpret_cast<const float4 *>(dy + t * d + c);
        const float4 vo = stream_load4(reinterpret_cast<const float4 *>(out_sorted + r * d + c));   // read once here
        dot = fmaf(vy.x, vo.x, dot); dot = fmaf(vy.y, vo.y, dot);
        dot = fmaf(vy.z, vo.z, dot); dot = fmaf(vy.w, vo.w, dot);
        *reinterpret_cast<uint2 *>(dout + r * d + c) = make_uint2(pack2(g * vy.x, g * vy.y), pack2(g * vy.z, g * vy.w));
        if (xs) {
            const float4 vx = *reinterpret_cast<const float4 *>(x + t * d + c);
            *reinterpret_cast<uint2 *>(xs + r * d + c) = make_uint2(pack2(vx.x, vx.y), pack2(vx.z, vx.w));
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) dot += __shfl_xor(dot, off);
    if (lane == 0) dgate[a] = dot;
}

// The same quantities with one wavefront per token (flat layer): the token's dy (and x) row comes
// from HBM once and serves its k routed rows, found through inv_perm; per routed row the
// arithmetic and its order are those of bwd_prepare_kernel.
__global__ __launch_bounds__(256) void bwd_prepare_tokens_kernel(const float *__restrict__ x,
                                                                 const float *__restrict__ dy,
                                                                 const float *__restrict__ out_sorted,
                                                                 const float *__restrict__ gate,
                                                                 const int32_t *__restrict__ inv_perm,
                                                                 int64_t T, int d, int k,
                                                                 uint16_t *__restrict__ xs,   // null: kept by the forward pass
                                                                 uint16_t *__restrict__ dout,
                                                                 float *__restrict__ dgate) {
    const int lane = threadIdx.x & 63;
    const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    for (int j = 0; j < k; ++j) {
        const int64_t a = t * k + j;
        const int64_t r = inv_perm[a];
        const float g = gate[a];
        float dot = 0.f;
        for (int c = lane * 4; c < d; c += 256) {
            const float4 vy = *reinterpret_cast<const float4 *>(dy + t * d + c);
            const float4 vo = stream_load4(reinterpret_cast<const float4 *>(out_sorted + r * d + c));   // read once here
            dot = fmaf(vy.x, vo.x, dot); dot = fmaf(vy.y, vo.y, dot);
            dot = fmaf(vy.z, vo.z, dot); dot = fmaf(vy.w, vo.w, dot);
            *reinterpret_cast<uint2 *>(dout + r * d + c) = make_uint2(pack2(g * vy.x, g * vy.y), pack2(g * vy.z, g * vy.w));
            if (xs) {
                const float4 vx = *reinterpret_cast<const float4 *>(x + t * d + c);
                *reinterpret_cast<uint2 *>(xs + r * d + c) = make_uint2(pack2(vx.x, vx.y), pack2(vx.z, vx.w));
            }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) dot += __shfl_xor(dot, off);
        if (lane == 0) dgate[a] = dot;
    }
}

// ---------------------------------------------------------------------------------------
// bf16 MFMA block GEMM shared by the expert backward kernels: 128 x 128 tile, 4 waves (2 x 2),
// k-slabs of 32 staged in LDS with k contiguous for both operands.
// ---------------------------------------------------------------------------------------
constexpr int GBM = 128, GBN = 128, GKC = 32, GLD = GKC + 8;  // LDS row = 32 k + pad (bf16)

struct Tile16 {
    uint4 v[2];
};

// operand rows have k contiguous in memory: element (row, k) at src[row * ld + k]
__device__ __forceinline__ void load_kcontig(Tile16 &t, const uint16_t *src, int64_t ld, int row0,
                                             int rows_valid, int k0, int tid) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int r = (tid >> 2) + 64 * i, kq = (tid & 3) * 8;
        t.v[i] = r < rows_valid
                     ? *reinterpret_cast<const uint4 *>(src + (int64_t)(row0 + r) * ld + k0 + kq)
                     : make_uint4(0u, 0u, 0u, 0u);
    }
}
__device__ __forceinline__ void store_kcontig(const Tile16 &t, uint16_t (*S)[GLD], int tid) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int r = (tid >> 2) + 64 * i, kq = (tid & 3) * 8;
        *reinterpret_cast<uint4 *>(&S[r][kq]) = t.v[i];
    }
}
// operand rows are strided in k: element (row, k) at src[k * ld + row]
__device__ __forceinline__ void load_kstrided(Tile16 &t, const uint16_t *src, int64_t ld, int row0,
                                              int k0, int k_valid, int tid) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int k = (tid >> 4) + 16 * i, rs = (tid & 15) * 8;
        t.v[i] = (k0 + k) < k_valid
                     ? *reinterpret_cast<const uint4 *>(src + (int64_t)(k0 + k) * ld + row0 + rs)
                     : make_uint4(0u, 0u, 0u, 0u);
    }
}
__device__ __forceinline__ void store_kstrided(const Tile16 &t, uint16_t (*S)[GLD], int tid) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int k = (tid >> 4) + 16 * i, rs = (tid & 15) * 8;
        const uint32_t w[4] = {t.v[i].x, t.v[i].y, t.v[i].z, t.v[i].w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            S[rs + 2 * j][k] = (uint16_t)(w[j] & 0xffffu);
            S[rs + 2 * j + 1][k] = (uint16_t)(w[j] >> 16);
        }
    }
}

__device__ __forceinline__ void mma_slab(v16f (&acc)[2][2], uint16_t (*As)[GLD], uint16_t (*Bs)[GLD],
                                         int wm, int wn, int lane) {
    const int l32 = lane & 31, kg = lane >> 5;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        v8bf a[2], b[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            a[i] = __builtin_bit_cast(v8bf, *reinterpret_cast<const uint4 *>(&As[wm * 64 + 32 * i + l32][16 * ks + 8 * kg]));
            b[i] = __builtin_bit_cast(v8bf, *reinterpret_cast<const uint4 *>(&Bs[wn * 64 + 32 * i + l32][16 * ks + 8 * kg]));
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
}

// C[rows of expert e, N] = A[rows, K] * B_e   over the row tiles of a 128-row tile table
template <bool B_KN, int EPI>
__global__ __launch_bounds__(256) void gg_rows_kernel(GGRows p) {
    __shared__ __attribute__((aligned(16))) uint16_t As[2][GBM][GLD];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[2][GBN][GLD];
    const int tile = blockIdx.x;
    if (tile >= *p.num_tiles) return;
    const int e = p.tile_expert[tile];
    const int row0 = p.tile_row0[tile];
    const int rows = min(p.tile_rows > 0 ? min(GBM, p.tile_rows) : GBM, p.offsets[e + 1] - row0);
    const int col0 = blockIdx.y * GBN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, wm = wave >> 1, wn = wave & 1;
    const uint16_t *Bw = p.B + (size_t)e * p.K * p.N;

    v16f acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    Tile16 ta, tb;
    auto load = [&](int k0) {
        load_kcontig(ta, p.A, p.K, row0, rows, k0, tid);
        if (B_KN) load_kstrided(tb, Bw, p.N, col0, k0, p.K, tid);
        else load_kcontig(tb, Bw, p.K, col0, GBN, k0, tid);
    };
    auto store = [&](int buf) {
        store_kcontig(ta, As[buf], tid);
        if (B_KN) store_kstrided(tb, Bs[buf], tid);
        else store_kcontig(tb, Bs[buf], tid);
    };
    load(0);
    store(0);
    __syncthreads();
    for (int k0 = 0; k0 < p.K; k0 += GKC) {
        const int buf = (k0 / GKC) & 1;
        const bool more = k0 + GKC < p.K;
        if (more) load(k0 + GKC);
        mma_slab(acc, As[buf], Bs[buf], wm, wn, lane);
        if (more) store(buf ^ 1);
        __syncthreads();
    }
    const int l32 = lane & 31, half = lane >> 5;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = wm * 64 + 32 * i + 8 * (r / 4) + 4 * half + (r % 4);
            if (row >= rows) continue;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int col = col0 + wn * 64 + 32 * j + l32;
                const size_t at = (size_t)(row0 + row) * p.N + col;
                float v = acc[i][j][r];
                if (EPI == EPI_RELU_BF16) {
                    reinterpret_cast<uint16_t *>(p.C)[at] = (uint16_t)bf16_rne(fmaxf(v, 0.f));
                } else if (EPI == EPI_MASK_BF16) {
                    // relu'(z) with relu'(0) = 0: the stored hidden value is positive iff z > 0
                    const bool on = (p.mask[at] & 0x7fffu) != 0 && (p.mask[at] & 0x8000u) == 0;
                    reinterpret_cast<uint16_t *>(p.C)[at] = (uint16_t)bf16_rne(on ? v : 0.f);
                } else {
                    reinterpret_cast<float *>(p.C)[at] = v;
                }
            }
        }
}

// ---------------------------------------------------------------------------------------
// gate: gradients of the two CV^2 losses with respect to Importance and Load
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void loss_grad_kernel(const double *__restrict__ sums64, int n,
                                                        float w_imp, float w_load,
                                                        float *__restrict__ gI, float *__restrict__ gL) {
    __shared__ double red[2][256];
    for (int which = 0; which < 2; ++which) {
        const double *v = sums64 + (size_t)which * n;
        double s = 0.0, s2 = 0.0;
        for (int i = threadIdx.x; i < n; i += 256) {
            s += v[i];
            s2 += v[i] * v[i];
        }
        red[0][threadIdx.x] = s;
        red[1][threadIdx.x] = s2;
        __syncthreads();
        for (int o = 128; o > 0; o >>= 1) {
            if ((int)threadIdx.x < o) {
                red[0][threadIdx.x] += red[0][threadIdx.x + o];
                red[1][threadIdx.x] += red[1][threadIdx.x + o];
            }
            __syncthreads();
        }
        const double S = red[0][0], Q = red[1][0];
        __syncthreads();
        const double w = which ? (double)w_load : (double)w_imp;
        float *out = which ? gL : gI;
        // d CV^2 / d v_i = 2 n v_i / S^2 - 2 n sum(v^2) / S^3   (population variance)
        for (int i = threadIdx.x; i < n; i += 256)
            out[i] = (float)(w * (2.0 * n * v[i] / (S * S) - 2.0 * n * Q / (S * S * S)));
    }
}

struct GateBwdArgs {
    const float *cleanb, *sp, *eps;   // [T, n]
    const int32_t *idx;               // [T, k]
    const float *gate, *dgate;        // [T, k]
    const int32_t *next_idx;          // [T]
    const float *gI, *gL;             // [n]
    float *dclean, *draw;             // [T, n]
    int64_t T;
    int n, k;
    // a secondary gate of the hierarchical layer: row t of cleanb/sp/dclean/draw belongs to row
    // row_map[t] of eps/idx/gate/dgate/next_idx and to the group g with
    // group_offsets[g] <= t < group_offsets[g+1], whose Load gradient is gL[g*n ..]; null = flat
    const int32_t *row_map;
    const int32_t *group_offsets;
    int groups;
};

// NG > 0: n <= 256 * NG (n is a multiple of 4): a lane owns NG groups of four adjacent experts
// (16-byte loads and stores) and keeps their terms of the first pass in registers for the second;
// NG = 0: any n, one expert per lane and step, the terms recomputed.
template <int NG>
__global__ __launch_bounds__(256) void gate_bwd_rows_kernel(GateBwdArgs p) {
    const int lane = threadIdx.x & 63;
    const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= p.T) return;
    const int n = p.n, k = p.k;
    const float *c_row = p.cleanb + t * n, *s_row = p.sp + t * n;
    const int64_t ot = p.row_map ? (int64_t)p.row_map[t] : t;
    const float *gL_row = p.gL;
    if (p.group_offsets) {
        int lo = 0, hi = p.groups;                 // last group whose first row is <= t
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if ((int64_t)p.group_offsets[mid] <= t) lo = mid;
            else hi = mid;
        }
        gL_row = p.gL + (size_t)lo * n;
    }
    const float *e_row = p.eps ? p.eps + ot * n : nullptr;
    int ki[kMaxK];
    float g[kMaxK], dH[kMaxK];
    float inner = 0.f;
#pragma unroll
    for (int s = 0; s < kMaxK; ++s) {
        ki[s] = s < k ? p.idx[ot * k + s] : -1;
        g[s] = s < k ? p.gate[ot * k + s] : 0.f;
        const float dg = s < k ? p.dgate[ot * k + s] + (p.gI ? p.gI[ki[s]] : 0.f) : 0.f;
        dH[s] = dg;
        inner = fmaf(g[s], dg, inner);
    }
#pragma unroll
    for (int s = 0; s < kMaxK; ++s) dH[s] = g[s] * (dH[s] - inner);   // softmax over the kept logits

    const bool with_load = k < n;
    int j_in = -1, j_out = -1;
    float thr_in = 0.f, thr_out = 0.f;
    if (with_load) {
        j_in = p.next_idx[ot];
#pragma unroll
        for (int s = 0; s < kMaxK; ++s)
            if (s == k - 1) j_out = ki[s];
        thr_in = e_row ? __fmaf_rn(e_row[j_in], s_row[j_in], c_row[j_in]) : c_row[j_in];
        thr_out = e_row ? __fmaf_rn(e_row[j_out], s_row[j_out], c_row[j_out]) : c_row[j_out];
    }
    auto kept_dh = [&](int i, float &dh) {   // is expert i one of the kept, and its softmax term
        bool kept = false;
        dh = 0.f;
#pragma unroll
        for (int s = 0; s < kMaxK; ++s)
            if (ki[s] == i) {
                kept = true;
                dh = dH[s];
            }
        return kept;
    };
    // c = gL * phi(u) / sp, u = (clean - threshold) / sp: the Load term of expert i (Eq.(9))
    auto load_term = [&](bool kept, float clean, float sp, float gl, float &u) {
        u = (clean - (kept ? thr_in : thr_out)) / sp;
        return gl * 0.3989422804014327f * expf(-0.5f * u * u) / sp;
    };
    float S_in = 0.f, S_out = 0.f;   // sums of c over the kept and over the other experts
    if (NG > 0) {
        float4 cv[NG > 0 ? NG : 1], uv[NG > 0 ? NG : 1], sv[NG > 0 ? NG : 1];
#pragma unroll
        for (int q = 0; q < NG; ++q) {
            const int i0 = 4 * lane + 256 * q;
            cv[q] = uv[q] = make_float4(0.f, 0.f, 0.f, 0.f);
            sv[q] = make_float4(1.f, 1.f, 1.f, 1.f);
            if (i0 >= n) continue;
            sv[q] = *reinterpret_cast<const float4 *>(s_row + i0);
            if (!with_load) continue;
            const float4 c4 = *reinterpret_cast<const float4 *>(c_row + i0);
            const float4 g4 = *reinterpret_cast<const float4 *>(gL_row + i0);
            const float cl[4] = {c4.x, c4.y, c4.z, c4.w}, gl[4] = {g4.x, g4.y, g4.z, g4.w};
            const float sp[4] = {sv[q].x, sv[q].y, sv[q].z, sv[q].w};
            float c[4], u[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float dh;
                const bool kept = kept_dh(i0 + e, dh);
                c[e] = load_term(kept, cl[e], sp[e], gl[e], u[e]);
                if (kept) S_in += c[e];
                else S_out += c[e];
            }
            cv[q] = make_float4(c[0], c[1], c[2], c[3]);
            uv[q] = make_float4(u[0], u[1], u[2], u[3]);
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            S_in += __shfl_xor(S_in, off);
            S_out += __shfl_xor(S_out, off);
        }
#pragma unroll
        for (int q = 0; q < NG; ++q) {
            const int i0 = 4 * lane + 256 * q;
            if (i0 >= n) continue;
            const float4 e4 = e_row ? *reinterpret_cast<const float4 *>(e_row + i0) : make_float4(0.f, 0.f, 0.f, 0.f);
            const float ev[4] = {e4.x, e4.y, e4.z, e4.w};
            const float c[4] = {cv[q].x, cv[q].y, cv[q].z, cv[q].w}, u[4] = {uv[q].x, uv[q].y, uv[q].z, uv[q].w};
            const float sp[4] = {sv[q].x, sv[q].y, sv[q].z, sv[q].w};
            float dc[4], dr[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float dh;
                kept_dh(i0 + e, dh);
                if (with_load && i0 + e == j_in) dh -= S_in;     // the threshold of the kept experts
                if (with_load && i0 + e == j_out) dh -= S_out;   // the threshold of all the others
                dc[e] = c[e] + dh;
                dr[e] = fmaf(dh, ev[e], -c[e] * u[e]) * -expm1f(-sp[e]);   // softplus' = sigmoid(raw) = 1 - exp(-sp), without the cancellation at small sp
            }
            *reinterpret_cast<float4 *>(p.dclean + t * n + i0) = make_float4(dc[0], dc[1], dc[2], dc[3]);
            *reinterpret_cast<float4 *>(p.draw + t * n + i0) = make_float4(dr[0], dr[1], dr[2], dr[3]);
        }
        return;
    }
    if (with_load) {
        for (int i = lane; i < n; i += 64) {
            float dh, u;
            const bool kept = kept_dh(i, dh);
            const float c = load_term(kept, c_row[i], s_row[i], gL_row[i], u);
            if (kept) S_in += c;
            else S_out += c;
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            S_in += __shfl_xor(S_in, off);
            S_out += __shfl_xor(S_out, off);
        }
    }
    for (int i = lane; i < n; i += 64) {
        float dh;
        const bool kept = kept_dh(i, dh);
        const float sp = s_row[i];
        float c = 0.f, u = 0.f;
        if (with_load) {
            c = load_term(kept, c_row[i], sp, gL_row[i], u);
            if (i == j_in) dh -= S_in;
            if (i == j_out) dh -= S_out;
        }
        const float ev = e_row ? e_row[i] : 0.f;
        p.dclean[t * n + i] = c + dh;
        p.draw[t * n + i] = fmaf(dh, ev, -c * u) * -expm1f(-sp);
    }
}

static int launch_gate_bwd_rows(const GateBwdArgs &a, int64_t rows, hipStream_t s) {
    if (rows <= 0) return MOE_OK;
    const dim3 grid((unsigned)ceil_div(rows, 4));
#define MOE_GBR(NG) hipLaunchKernelGGL(gate_bwd_rows_kernel<NG>, grid, dim3(256), 0, s, a)
    if (a.n % 4 != 0 || a.n > 2048) MOE_GBR(0);
    else if (a.n <= 256) MOE_GBR(1);
    else if (a.n <= 512) MOE_GBR(2);
    else if (a.n <= 1024) MOE_GBR(4);
    else MOE_GBR(8);
#undef MOE_GBR
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}

// ---------------------------------------------------------------------------------------
// fp32 MFMA GEMM for the gate: C[M,N] (+)= sum over segments of A_s * B_s
// ---------------------------------------------------------------------------------------
struct SGArgs {
    const float *A[2];
    const float *B[2];
    float *C;
    int M, N, K;      // K per segment
    int lda, ldb, ldc;
    int nseg;
    int ksplit;       // blockIdx.z = which * ksplit + split (A_MK only)
    size_t c_which_stride, c_split_stride;
    // optional row range on the device (rows lo = range[range_idx] .. range[range_idx+1] of the
    // row-indexed operands): with A_MK the contraction runs over those rows (K = their number),
    // otherwise they are the rows of A and C (M = their number; tiles past the end exit)
    const int32_t *range;
    int range_idx;
    // several ranges in one launch.  A_MK: blockIdx.z = g, rows range[g] .. range[g+1] are contracted
    // into C + g * c_group_stride (ksplit must be 1).  Otherwise: blockIdx.x indexes a table of
    // 128-row tiles that never straddle ranges (tile_group, tile_row0, num_tiles); tile t covers
    // rows tile_row0[t] .. of range g = tile_group[t] and multiplies by B + g * b_group_stride.
    int range_groups;
    size_t c_group_stride, b_group_stride;
    const int32_t *tile_group, *tile_row0, *num_tiles;
};

constexpr int SBM = 128, SBN = 128, SKC = 32, SAS = SKC + 4;

typedef float v4f32 __attribute__((ext_vector_type(4)));
typedef float v2f32 __attribute__((ext_vector_type(2)));

// A_MK: A(m,k) = A[k*lda + m] (m contiguous; used for x^T), else A(m,k) = A[m*lda + k].
// B_NK: B(k,n) = B[n*ldb + k] (k contiguous; used for W^T), else B(k,n) = B[k*ldb + n].
// M, N, K, lda, ldb, ldc are multiples of 4.
//
// 128 x 128 tile, four waves x (32 rows x four 32x32 tiles of v_mfma_f32_32x32x2f32).  An operand
// whose rows are contiguous in k is staged in LDS as [row][k parity][k/2] (a lane's 16-byte read
// feeds four consecutive k-steps); one that is contiguous in the other index is staged as
// [k][row] and read one element per k-step -- either way the global 16-byte loads go to LDS
// without a scattering transpose.  All loads are unconditional (clamped addresses, values past
// the end of k replaced by zero with a select), slab s+1 is stored and slab s+2 fetched in the
// middle of slab s, operands are read one group of four k-steps ahead and the barrier sits before
// the slab's last group.  The epilogue goes through LDS so rows leave as 16-byte stores.
template <bool A_MK, bool B_NK>
__global__ __launch_bounds__(256) void sg_kernel(SGArgs p) {
    constexpr int OPB = SBM * SAS * 4;   // bytes of one operand buffer (the larger layout)
    constexpr int CS = SBN + 4;
    static_assert(SBM * CS * 4 <= 4 * OPB, "the output tile reuses the operand buffers");
    __shared__ __attribute__((aligned(16))) char smem[4 * OPB];
    float (*A_mk)[SBM][SAS] = reinterpret_cast<float (*)[SBM][SAS]>(smem);
    float (*A_km)[SKC][SBM] = reinterpret_cast<float (*)[SKC][SBM]>(smem);
    float (*B_nk)[SBN][SAS] = reinterpret_cast<float (*)[SBN][SAS]>(smem + 2 * OPB);
    float (*B_kn)[SKC][SBN] = reinterpret_cast<float (*)[SKC][SBN]>(smem + 2 * OPB);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    int m0 = blockIdx.x * SBM;
    const int n0 = blockIdx.y * SBN;
    int which = 0, split = 0;
    if (A_MK && !p.range_groups) {
        which = blockIdx.z / p.ksplit;
        split = blockIdx.z % p.ksplit;
    }
    int M_ = p.M, K_ = p.K;
    const float *A0 = p.A[0], *A1 = p.A[1], *B0 = p.B[0], *B1 = p.B[1];
    float *C_ = p.C;
    if (p.range && !A_MK && p.tile_row0) {
        if ((int)blockIdx.x >= *p.num_tiles) return;
        const int g = p.tile_group[blockIdx.x];
        m0 = p.tile_row0[blockIdx.x];
        M_ = p.range[g + 1];
        B0 += (size_t)g * p.b_group_stride;
        B1 += (size_t)g * p.b_group_stride;
    } else if (p.range) {
        const int gi = p.range_idx + (p.range_groups ? (int)blockIdx.z : 0);
        const int lo = p.range[gi], hi = p.range[gi + 1];
        if (A_MK) {
            K_ = hi - lo;
            A0 += (size_t)lo * p.lda;
            B0 += (size_t)lo * p.ldb;
            B1 += (size_t)lo * p.ldb;
            if (p.range_groups) C_ += (size_t)blockIdx.z * p.c_group_stride;
        } else {
            M_ = hi - lo;
            if (m0 >= M_) return;
            A0 += (size_t)lo * p.lda;
            A1 += (size_t)lo * p.lda;
            C_ += (size_t)lo * p.ldc;
        }
    }
    const int kper = A_MK ? ((K_ + p.ksplit - 1) / p.ksplit + SKC - 1) / SKC * SKC : K_;
    const int kbeg = split * kper, kend = min(K_, kbeg + kper);
    const int per_seg = kend > kbeg ? (kend - kbeg + SKC - 1) / SKC : 0;
    const int nslab = per_seg * (A_MK ? 1 : p.nseg);

    v16f acc[4];
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[c][r] = 0.f;

    // staging coordinates
    const int rk = tid >> 5, r4 = (tid & 31) * 4;    // [k][row] operands: k = rk + 8 i, rows r4..r4+3
    const int rr = tid >> 3, kq = (tid & 7) * 4;     // [row][k] operands: row = rr + 32 i, k = kq..kq+3
    v4f32 a_reg[4], b_reg[4];
    auto load_global = [&](int slab) {
        const int sgm = A_MK ? 0 : slab / per_seg;
        const int k0 = kbeg + (slab - sgm * per_seg) * SKC;
        const float *A = (A_MK || sgm == 0) ? A0 : A1;
        const float *B = (A_MK ? which : sgm) == 0 ? B0 : B1;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (A_MK) {
                const int k = k0 + rk + 8 * i;
                const v4f32 v = *reinterpret_cast<const v4f32 *>(A + (size_t)min(k, kend - 1) * p.lda + min(m0 + r4, M_ - 4));
                a_reg[i] = k < kend ? v : v4f32{0.f, 0.f, 0.f, 0.f};
            } else {
                const int k = k0 + kq;
                const v4f32 v = *reinterpret_cast<const v4f32 *>(A + (size_t)min(m0 + rr + 32 * i, M_ - 1) * p.lda + min(k, kend - 4));
                a_reg[i] = k < kend ? v : v4f32{0.f, 0.f, 0.f, 0.f};
            }
            if (B_NK) {
                const int k = k0 + kq;
                const v4f32 v = *reinterpret_cast<const v4f32 *>(B + (size_t)min(n0 + rr + 32 * i, p.N - 1) * p.ldb + min(k, kend - 4));
                b_reg[i] = k < kend ? v : v4f32{0.f, 0.f, 0.f, 0.f};
            } else {
                const int k = k0 + rk + 8 * i;
                const v4f32 v = *reinterpret_cast<const v4f32 *>(B + (size_t)min(k, kend - 1) * p.ldb + min(n0 + r4, p.N - 4));
                b_reg[i] = k < kend ? v : v4f32{0.f, 0.f, 0.f, 0.f};
            }
        }
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (A_MK) {
                *reinterpret_cast<v4f32 *>(&A_km[buf][rk + 8 * i][r4]) = a_reg[i];
            } else {
                float *row = &A_mk[buf][rr + 32 * i][0];
                *reinterpret_cast<v2f32 *>(row + kq / 2) = v2f32{a_reg[i].x, a_reg[i].z};
                *reinterpret_cast<v2f32 *>(row + SKC / 2 + kq / 2) = v2f32{a_reg[i].y, a_reg[i].w};
            }
            if (B_NK) {
                float *row = &B_nk[buf][rr + 32 * i][0];
                *reinterpret_cast<v2f32 *>(row + kq / 2) = v2f32{b_reg[i].x, b_reg[i].z};
                *reinterpret_cast<v2f32 *>(row + SKC / 2 + kq / 2) = v2f32{b_reg[i].y, b_reg[i].w};
            } else {
                *reinterpret_cast<v4f32 *>(&B_kn[buf][rk + 8 * i][r4]) = b_reg[i];
            }
        }
    };
    float a_grp[2][4], b_grp[2][4][4];
    auto read_group = [&](int slot, int buf, int kk4) {
        if (A_MK) {
#pragma unroll
            for (int u = 0; u < 4; ++u) a_grp[slot][u] = A_km[buf][2 * (kk4 + u) + half][wave * 32 + l32];
        } else {
            const v4f32 a4 = *reinterpret_cast<const v4f32 *>(&A_mk[buf][wave * 32 + l32][half * (SKC / 2) + kk4]);
#pragma unroll
            for (int u = 0; u < 4; ++u) a_grp[slot][u] = a4[u];
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (B_NK) {
                const v4f32 b4 = *reinterpret_cast<const v4f32 *>(&B_nk[buf][32 * c + l32][half * (SKC / 2) + kk4]);
#pragma unroll
                for (int u = 0; u < 4; ++u) b_grp[slot][u][c] = b4[u];
            } else {
#pragma unroll
                for (int u = 0; u < 4; ++u) b_grp[slot][u][c] = B_kn[buf][2 * (kk4 + u) + half][32 * c + l32];
            }
        }
    };

    if (nslab > 0) {
        constexpr int NG = SKC / 8;
        load_global(0);
        store_lds(0);
        load_global(min(1, nslab - 1));
        __syncthreads();
        read_group(0, 0, 0);
        for (int sl = 0; sl < nslab; ++sl) {
            const int buf = sl & 1;
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                if (g == NG - 1) {
                    __syncthreads();
                    read_group((g + 1) & 1, buf ^ 1, 0);   // after the last slab: unused
                } else {
                    read_group((g + 1) & 1, buf, 4 * (g + 1));
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        acc[c] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_grp[g & 1][u], b_grp[g & 1][u][c], acc[c], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (g == NG / 2 - 1) {
                    store_lds(buf ^ 1);
                    load_global(min(sl + 2, nslab - 1));
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
    }
    __syncthreads();   // every wave is done with the operand buffers (also the unused last reads)

    float *Ct = reinterpret_cast<float *>(smem);
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            Ct[(wave * 32 + 8 * (r / 4) + 4 * half + (r % 4)) * CS + 32 * c + l32] = acc[c][r];
    __syncthreads();
    float *C = C_ + (A_MK ? which * p.c_which_stride + split * p.c_split_stride : 0);
    const int cq = tid & 31, r0 = tid >> 5;     // 32 float4 per row, 8 rows per pass
    const int col = n0 + 4 * cq;
    for (int pass0 = 0; pass0 < SBM / 8; pass0 += 4) {
        v4f32 t[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) t[u] = *reinterpret_cast<const v4f32 *>(Ct + (r0 + 8 * (pass0 + u)) * CS + 4 * cq);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int row = m0 + r0 + 8 * (pass0 + u);
            if (row < M_ && col < p.N) *reinterpret_cast<v4f32 *>(C + (size_t)row * p.ldc + col) = t[u];
        }
    }
}

// out[i] = sum over splits (ascending) of part[split][i]
__global__ __launch_bounds__(256) void split_sum_kernel(const float *__restrict__ part, int splits,
                                                        size_t stride, size_t count,
                                                        float *__restrict__ out) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= count) return;
    float s = 0.f;
    for (int q = 0; q < splits; ++q) s += part[(size_t)q * stride + i];
    out[i] = s;
}

__global__ __launch_bounds__(256) void dx_gather_add_kernel(float4 *__restrict__ dx,
                                                            const float4 *__restrict__ dxs,
                                                            const int32_t *__restrict__ inv_perm,
                                                            int64_t T, int d4, int k) {
    const int lane = threadIdx.x & 63;
    const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    int rows[kMaxK];
#pragma unroll
    for (int s = 0; s < kMaxK; ++s) rows[s] = s < k ? inv_perm[t * k + s] : 0;
    for (int c = lane; c < d4; c += 64) {
        float4 acc = dx[t * d4 + c];
#pragma unroll
        for (int s = 0; s < kMaxK; ++s)
            if (s < k) {
                const float4 v = stream_load4(dxs + (int64_t)rows[s] * d4 + c);   // each row is read once
                acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
            }
        dx[t * d4 + c] = acc;
    }
}

int launch_gg_rows128(const GGRows &p, bool b_kn, int epi, int64_t max_tiles, hipStream_t st) {
    if (p.K % GKC || p.N % GBN) return MOE_EUNSUPPORTED;
    if (max_tiles <= 0) return MOE_OK;
    const dim3 grid((unsigned)max_tiles, (unsigned)(p.N / GBN));
    if (b_kn && epi == EPI_RELU_BF16) hipLaunchKernelGGL((gg_rows_kernel<true, EPI_RELU_BF16>), grid, dim3(256), 0, st, p);
    else if (b_kn && epi == EPI_F32) hipLaunchKernelGGL((gg_rows_kernel<true, EPI_F32>), grid, dim3(256), 0, st, p);
    else return MOE_EUNSUPPORTED;
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}

static size_t up256(size_t v) { return (v + 255) & ~(size_t)255; }

struct BwdLayout {
    size_t xs, dout, hid, dz, dxs, dgate, dclean, draw, gI, gL, wpart, tile_expert, tile_row0,
        num_tiles, order, mom[4], total;
    int ksplit;
};

static int bwd_layout(const moe_config *cfg, BwdLayout *L) {
    const size_t T = cfg->T, n = cfg->n, A = T * (size_t)cfg->k, d = cfg->d, h = cfg->h;
    size_t off = 0;
    auto take = [&](size_t b) {
        const size_t at = off;
        off = up256(off + (b ? b : 1));
        return at;
    };
    const size_t es = cfg->expert_dtype == MOE_DTYPE_BF16 ? 2 : 4;   // fp32 experts keep fp32 rows
    L->xs = take(A * d * es);
    L->dout = take(A * d * es);
    L->hid = take(A * h * 2);
    L->dz = take(A * h * es);
    L->dxs = take(A * d * 4);
    L->dgate = take(A * 4);
    L->dclean = take(T * n * 4);
    L->draw = take(T * n * 4);
    L->gI = take(n * 4);
    L->gL = take(n * 4);
    // tokens per split of the weight-gradient GEMM: enough workgroups to fill the chip
    const int64_t tiles = ceil_div(cfg->d, SBM) * ceil_div(cfg->n, SBN) * 2;
    int ks = (int)ceil_div(1024, tiles);
    const int maxks = (int)ceil_div(cfg->T > 0 ? cfg->T : 1, 256);
    if (ks > maxks) ks = maxks;
    if (ks < 1) ks = 1;
    L->ksplit = ks;
    L->wpart = take((size_t)ks * 2 * d * n * 4);
    const size_t MT = (size_t)ceil_div((int64_t)A, kFfnBwdTileRows) + n + 8;   // the shortest tiles any kernel here asks for
    L->tile_expert = take(MT * 4);
    L->tile_row0 = take(MT * 4);
    L->num_tiles = take(16);
    L->order = take(n * 4);
    // MOE_FLAG_ADAM_MOMENTS: per-block sums of squares of dW1 [d,h] and dW2 [h,d] (see GGWgrad)
    const bool mom = (cfg->flags & MOE_FLAG_ADAM_MOMENTS) && cfg->expert_dtype == MOE_DTYPE_BF16;
    L->mom[0] = mom ? take(n * (h / 256) * d * 4) : (size_t)-1;
    L->mom[1] = mom ? take(n * (d / 256) * h * 4) : (size_t)-1;
    L->mom[2] = mom ? take(n * (d / 256) * h * 4) : (size_t)-1;
    L->mom[3] = mom ? take(n * (h / 256) * d * 4) : (size_t)-1;
    L->total = off;
    return MOE_OK;
}

int launch_build_tiles(const int32_t *offsets, int n, int tile_rows, int32_t *tile_expert,
                       int32_t *tile_row0, int32_t *num_tiles, hipStream_t st);

// fp32 experts: the same per-row preparation without rounding
__global__ __launch_bounds__(256) void bwd_prepare_f32_kernel(const float *__restrict__ x,
                                                              const float *__restrict__ dy,
                                                              const float *__restrict__ out_sorted,
                                                              const float *__restrict__ gate,
                                                              const int32_t *__restrict__ perm, int64_t A,
                                                              int d, int k, int by_row,
                                                              float *__restrict__ xs,
                                                              float *__restrict__ dout,
                                                              float *__restrict__ dgate) {
    const int lane = threadIdx.x & 63;
    const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= A) return;
    const int64_t a = by_row ? r : perm[r];
    const int64_t t = by_row ? perm[r] : a / k;
    const float g = gate[a];
    float dot = 0.f;
    for (int c = lane * 4; c < d; c += 256) {
        const float4 vy = *reinterpret_cast<const float4 *>(dy + t * d + c);
        const float4 vo = stream_load4(reinterpret_cast<const float4 *>(out_sorted + r * d + c));   // read once here
        dot = fmaf(vy.x, vo.x, dot); dot = fmaf(vy.y, vo.y, dot);
        dot = fmaf(vy.z, vo.z, dot); dot = fmaf(vy.w, vo.w, dot);
        *reinterpret_cast<float4 *>(dout + r * d + c) = make_float4(g * vy.x, g * vy.y, g * vy.z, g * vy.w);
        *reinterpret_cast<float4 *>(xs + r * d + c) = *reinterpret_cast<const float4 *>(x + t * d + c);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) dot += __shfl_xor(dot, off);
    if (lane == 0) dgate[a] = dot;
}

// dz = dh * [hid > 0]   (relu'(0) = 0: the stored hidden value is positive iff z > 0)
__global__ __launch_bounds__(256) void relu_mask_f32_kernel(float4 *__restrict__ dz, const float4 *__restrict__ hid,
                                                            int64_t count4) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= count4) return;
    float4 v = dz[i];
    const float4 m = hid[i];
    v.x = m.x > 0.f ? v.x : 0.f; v.y = m.y > 0.f ? v.y : 0.f;
    v.z = m.z > 0.f ? v.z : 0.f; v.w = m.w > 0.f ? v.w : 0.f;
    dz[i] = v;
}

// The experts' share of the backward pass for fp32 experts, entirely on the fp32 matrix cores:
// the grouped forms of sg_kernel (a group = an expert's rows) serve all four GEMMs.  hid are the
// hidden activations the fp32 forward pass keeps in its expert workspace.
struct ExpertBwdF32 {
    const float *x, *dy, *out_sorted, *gate;
    const int32_t *perm, *offsets;
    const float *W1, *W2, *hid;
    float *xs, *dout, *dz, *dxs, *dgate;
    int32_t *tile_expert, *tile_row0, *num_tiles;
    float *dW1, *dW2;
    bool by_row;   // perm lists tokens; gate and dgate are per routed row (balanced gating)
};

static int run_expert_backward_f32(const moe_config *cfg, const ExpertBwdF32 &b, hipStream_t s) {
    const int64_t A = (int64_t)cfg->T * cfg->k;
    const int d = cfg->d, h = cfg->h, n = cfg->n, k = cfg->k;
    if (n > 65535) return MOE_EUNSUPPORTED;   // an expert per blockIdx.z
    int st;
    hipLaunchKernelGGL(bwd_prepare_f32_kernel, dim3((unsigned)ceil_div(A, 4)), dim3(256), 0, s, b.x, b.dy,
                       b.out_sorted, b.gate, b.perm, A, d, k, b.by_row ? 1 : 0, b.xs, b.dout, b.dgate);
    MOE_LAUNCH_CHECK();
    if ((st = launch_build_tiles(b.offsets, n, SBM, b.tile_expert, b.tile_row0, b.num_tiles, s)) != MOE_OK) return st;
    const unsigned max_tiles = (unsigned)(ceil_div(A, SBM) + n);
    auto rows_form = [&](const float *Arows, int K, const float *Bw, int N, float *C) {
        SGArgs r{};
        r.A[0] = Arows; r.B[0] = Bw; r.C = C;
        r.M = 0; r.N = N; r.K = K; r.lda = K; r.ldb = K; r.ldc = N; r.nseg = 1; r.ksplit = 1;
        r.range = b.offsets; r.b_group_stride = (size_t)K * N;
        r.tile_group = b.tile_expert; r.tile_row0 = b.tile_row0; r.num_tiles = b.num_tiles;
        hipLaunchKernelGGL((sg_kernel<false, true>), dim3(max_tiles, ceil_div(N, SBN), 1), dim3(256), 0, s, r);
    };
    auto wgrad_form = [&](const float *Arows, int M, const float *Brows, int N, float *C) {
        SGArgs w{};
        w.A[0] = Arows; w.B[0] = Brows; w.C = C;
        w.M = M; w.N = N; w.K = 0; w.lda = M; w.ldb = N; w.ldc = N; w.nseg = 1; w.ksplit = 1;
        w.range = b.offsets; w.range_idx = 0; w.range_groups = n; w.c_group_stride = (size_t)M * N;
        hipLaunchKernelGGL((sg_kernel<true, false>), dim3(ceil_div(M, SBM), ceil_div(N, SBN), n), dim3(256), 0, s, w);
    };
    rows_form(b.dout, d, b.W2, h, b.dz);          // dh[r, j] = sum_c dout[r, c] W2[j, c]
    MOE_LAUNCH_CHECK();
    hipLaunchKernelGGL(relu_mask_f32_kernel, dim3((unsigned)ceil_div(A * h / 4, 256)), dim3(256), 0, s,
                       (float4 *)b.dz, (const float4 *)b.hid, A * h / 4);
    MOE_LAUNCH_CHECK();
    wgrad_form(b.hid, h, b.dout, d, b.dW2);       // dW2_e = hid_e^T dout_e
    MOE_LAUNCH_CHECK();
    wgrad_form(b.xs, d, b.dz, h, b.dW1);          // dW1_e = xs_e^T dz_e
    MOE_LAUNCH_CHECK();
    rows_form(b.dz, h, b.W1, d, b.dxs);           // dxs[r, c] = sum_j dz[r, j] W1[c, j]
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}

// The experts' share of a backward pass, for any assignment list (flat or hierarchical gate):
// Eq.(1) per routed row, the two-layer expert's backward GEMMs and both weight gradients.
struct ExpertBwd {
    const float *x, *dy, *out_sorted, *gate;   // gate [T*k] in assignment order
    const int32_t *perm, *offsets;
    const void *W1, *W2;
    const uint16_t *saved_hid;                 // hidden activations kept by the forward pass, or null
    uint16_t *xs, *dout, *hid, *dz;            // workspace (hid unused when saved_hid is given)
    float *dxs, *dgate;                        // out: [T*k, d] expert part of dx per routed row; [T*k]
    int32_t *tile_expert, *tile_row0, *num_tiles, *order;
    float *dW1, *dW2;
    float *mom[4];                             // optional sums of squares for the optimiser, or nulls
    bool by_row;                               // perm lists tokens; gate and dgate are per routed row
    const uint16_t *saved_xs;                  // routed input rows (bf16) kept by the forward pass, or null
    const int32_t *inv_perm;                   // flat layer: sorted row of each (token, slot), or null
};

static int run_expert_backward(const moe_config *cfg, const ExpertBwd &b, hipStream_t s) {
    const int64_t A = (int64_t)cfg->T * cfg->k;
    const int d = cfg->d, h = cfg->h, n = cfg->n, k = cfg->k;
    int st;
    const uint16_t *xs = b.saved_xs ? b.saved_xs : b.xs;
    if (b.inv_perm && !b.by_row)
        hipLaunchKernelGGL(bwd_prepare_tokens_kernel, dim3((unsigned)ceil_div(cfg->T, 4)), dim3(256), 0, s, b.x,
                           b.dy, b.out_sorted, b.gate, b.inv_perm, (int64_t)cfg->T, d, k,
                           b.saved_xs ? nullptr : b.xs, b.dout, b.dgate);
    else
        hipLaunchKernelGGL(bwd_prepare_kernel, dim3((unsigned)ceil_div(A, 4)), dim3(256), 0, s, b.x, b.dy,
                           b.out_sorted, b.gate, b.perm, A, d, k, b.by_row ? 1 : 0, b.saved_xs ? nullptr : b.xs,
                           b.dout, b.dgate);
    MOE_LAUNCH_CHECK();
    const uint16_t *hid = b.saved_hid;
    if (!hid) {   // Appendix D: recompute the hidden activations
        if ((st = launch_build_tiles(b.offsets, n, GBM, b.tile_expert, b.tile_row0, b.num_tiles, s)) != MOE_OK) return st;
        const unsigned max_tiles = (unsigned)(ceil_div(A, GBM) + n);
        GGRows g1{xs, (const uint16_t *)b.W1, b.hid, nullptr, d, h, b.offsets, b.tile_expert, b.tile_row0, b.num_tiles};
        if ((st = launch_gg_rows128(g1, true, EPI_RELU_BF16, max_tiles, s)) != MOE_OK) return st;
        hid = b.hid;
    }
    if (ffn_bwd_rows_applies(cfg)) {
        // about one tile of rows per expert: both row products in one launch that streams the
        // expert's matrices once (the forward kernel's regime, run backwards)
        if ((st = launch_build_tiles(b.offsets, n, kFfnBwdTileRows, b.tile_expert, b.tile_row0, b.num_tiles, s)) != MOE_OK)
            return st;
        FfnBwdRows fr{b.dout, hid, b.W1, b.W2, b.dz, b.dxs, b.offsets, b.tile_expert, b.tile_row0, b.num_tiles};
        if ((st = launch_ffn_bwd_rows(fr, ceil_div(A, kFfnBwdTileRows) + n, s)) != MOE_OK) return st;
        if ((st = launch_expert_order(b.offsets, n, b.order, s)) != MOE_OK) return st;
        GGWgrad w2{hid, b.dout, b.dW2, h, d, b.offsets, b.order, b.mom[2], b.mom[3]};
        if ((st = launch_gg_wgrad(w2, n, s)) != MOE_OK) return st;
        GGWgrad w1{xs, b.dz, b.dW1, d, h, b.offsets, b.order, b.mom[0], b.mom[1]};
        return launch_gg_wgrad(w1, n, s);
    }
    // the two compute-bound GEMMs of the expert backward run on 256-row tiles
    if ((st = launch_build_tiles(b.offsets, n, 256, b.tile_expert, b.tile_row0, b.num_tiles, s)) != MOE_OK) return st;
    const int64_t max_tiles256 = ceil_div(A, 256) + n;
    GGRows g2{b.dout, (const uint16_t *)b.W2, b.dz, hid, d, h, b.offsets, b.tile_expert, b.tile_row0, b.num_tiles};
    if ((st = launch_gg_rows256(g2, EPI_MASK_BF16, max_tiles256, s)) != MOE_OK) return st;
    if ((st = launch_expert_order(b.offsets, n, b.order, s)) != MOE_OK) return st;
    GGWgrad w2{hid, b.dout, b.dW2, h, d, b.offsets, b.order, b.mom[2], b.mom[3]};
    if ((st = launch_gg_wgrad(w2, n, s)) != MOE_OK) return st;
    GGWgrad w1{xs, b.dz, b.dW1, d, h, b.offsets, b.order, b.mom[0], b.mom[1]};
    if ((st = launch_gg_wgrad(w1, n, s)) != MOE_OK) return st;
    GGRows g5{b.dz, (const uint16_t *)b.W1, b.dxs, nullptr, h, d, b.offsets, b.tile_expert, b.tile_row0, b.num_tiles};
    return launch_gg_rows256(g5, EPI_F32, max_tiles256, s);
}

}  // namespace moe

using namespace moe;

namespace moe {
// An empty batch still owes the caller fully written outputs: every gradient is zero.
__global__ __launch_bounds__(256) void zero_f32x4_kernel(float4 *out, size_t count4) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < count4; i += (size_t)gridDim.x * 256)
        out[i] = make_float4(0.f, 0.f, 0.f, 0.f);
}
static int launch_zero(float *out, size_t count, hipStream_t s) {   // count: a multiple of 4
    if (count == 0) return MOE_OK;
    const size_t c4 = count / 4;
    const unsigned grid = (unsigned)(c4 < 256 * 2048 ? ceil_div((int64_t)c4, 256) : 2048);
    hipLaunchKernelGGL(zero_f32x4_kernel, dim3(grid), dim3(256), 0, s, reinterpret_cast<float4 *>(out), c4);
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}
static int hier_moments_offsets(const moe_config *cfg, size_t off[4]);
int backward_moments_offsets(const moe_config *cfg, size_t off[4]) {
    if (check_config(cfg) != MOE_OK) return MOE_EINVAL;
    if (cfg->a != 0) return hier_moments_offsets(cfg, off);
    BwdLayout L;
    bwd_layout(cfg, &L);
    for (int q = 0; q < 4; ++q) {
        if (L.mom[q] == (size_t)-1) return MOE_EINVAL;
        off[q] = L.mom[q];
    }
    return MOE_OK;
}
}  // namespace moe

extern "C" size_t moe_backward_workspace_bytes(const moe_config *cfg) {
    if (check_config(cfg) != MOE_OK || cfg->a != 0) return 0;
    BwdLayout L;
    bwd_layout(cfg, &L);
    return L.total;
}

extern "C" int moe_layer_backward(const moe_config *cfg, const float *x, const float *W_g,
                                  const float *W_noise, const float *eps, const void *W1,
                                  const void *W2, const float *dy, const int32_t *topk_idx,
                                  const float *topk_gate, const void *fwd_workspace, float *dx,
                                  float *dW_g, float *dW_noise, float *dW1, float *dW2,
                                  void *workspace, size_t workspace_bytes, void *stream) {
    moe_workspace_layout F;
    int st = moe_get_workspace_layout(cfg, &F);
    if (st != MOE_OK) return st;
    if (cfg->a != 0) return MOE_EUNSUPPORTED;           // flat layer only
    const bool f32_experts = cfg->expert_dtype != MOE_DTYPE_BF16;
    if (!f32_experts && (cfg->d % 256 != 0 || cfg->h % 256 != 0)) return MOE_EUNSUPPORTED;
    if (cfg->d % 4 != 0 || cfg->h % 4 != 0 || cfg->n % 4 != 0) return MOE_EUNSUPPORTED;
    if (!W_g || !W_noise || !W1 || !W2 || !fwd_workspace || !dW_g || !dW_noise || !dW1 || !dW2 || !workspace)
        return MOE_EINVAL;
    if (cfg->T > 0 && (!x || !dy || !topk_idx || !topk_gate || !dx)) return MOE_EINVAL;   // [T, .] tensors
    if (!aligned16(x) || !aligned16(dy) || !aligned16(dx) || !aligned16(W1) || !aligned16(W2) ||
        !aligned16(dW1) || !aligned16(dW2) || !aligned16(dW_g) || !aligned16(dW_noise) ||
        !aligned16(workspace) || !aligned16(fwd_workspace) || (eps && !aligned16(eps)))
        return MOE_EINVAL;
    BwdLayout L;
    bwd_layout(cfg, &L);
    if (workspace_bytes < L.total) return MOE_EWORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    const int64_t T = cfg->T, A = T * cfg->k;
    const int d = cfg->d, h = cfg->h, n = cfg->n, k = cfg->k;
    if (T == 0) {
        MOE_TRY(launch_zero(dW_g, (size_t)d * n, s));
        MOE_TRY(launch_zero(dW_noise, (size_t)d * n, s));
        MOE_TRY(launch_zero(dW1, (size_t)n * d * h, s));
        return launch_zero(dW2, (size_t)n * d * h, s);
    }
    char *fw = (char *)fwd_workspace;   // read-only here
    char *ws = (char *)workspace;
    const float *cleanb = (const float *)(fw + F.cleanb), *sp = (const float *)(fw + F.sp);
    const int32_t *next_idx = (const int32_t *)(fw + F.next_idx);
    const int32_t *offsets = (const int32_t *)(fw + F.offsets);
    const int32_t *perm = (const int32_t *)(fw + F.perm), *inv_perm = (const int32_t *)(fw + F.inv_perm);
    const float *out_sorted = (const float *)(fw + F.out_sorted);
    const double *sums64 = (const double *)(fw + F.aux_ws);
    uint16_t *xs = (uint16_t *)(ws + L.xs), *dout = (uint16_t *)(ws + L.dout);
    const bool saved_hidden = F.hidden != (size_t)-1;
    uint16_t *hid = saved_hidden ? (uint16_t *)(fw + F.hidden) : (uint16_t *)(ws + L.hid);
    uint16_t *dz = (uint16_t *)(ws + L.dz);
    float *dxs = (float *)(ws + L.dxs), *dgate = (float *)(ws + L.dgate);
    float *dclean = (float *)(ws + L.dclean), *draw = (float *)(ws + L.draw);
    float *gI = (float *)(ws + L.gI), *gL = (float *)(ws + L.gL), *wpart = (float *)(ws + L.wpart);
    int32_t *tile_expert = (int32_t *)(ws + L.tile_expert), *tile_row0 = (int32_t *)(ws + L.tile_row0);
    int32_t *num_tiles = (int32_t *)(ws + L.num_tiles);

    if (f32_experts) {
        ExpertBwdF32 ef{x, dy, out_sorted, topk_gate, perm, offsets, (const float *)W1, (const float *)W2,
                        (const float *)(fw + F.ffn_ws), (float *)xs, (float *)dout, (float *)dz, dxs, dgate,
                        tile_expert, tile_row0, num_tiles, dW1, dW2};
        if ((st = run_expert_backward_f32(cfg, ef, s)) != MOE_OK) return st;
    } else {
        ExpertBwd eb{x, dy, out_sorted, topk_gate, perm, offsets, W1, W2, saved_hidden ? hid : nullptr,
                     xs, dout, saved_hidden ? nullptr : hid, dz, dxs, dgate, tile_expert, tile_row0, num_tiles,
                     (int32_t *)(ws + L.order), dW1, dW2, {nullptr, nullptr, nullptr, nullptr}};
        for (int q = 0; q < 4; ++q)
            if (L.mom[q] != (size_t)-1) eb.mom[q] = (float *)(ws + L.mom[q]);
        if (F.xs != (size_t)-1) eb.saved_xs = (const uint16_t *)(fw + F.xs);
        eb.inv_perm = inv_perm;
        if ((st = run_expert_backward(cfg, eb, s)) != MOE_OK) return st;
    }

    // gate
    hipLaunchKernelGGL(loss_grad_kernel, dim3(1), dim3(256), 0, s, sums64, n, cfg->w_importance,
                       cfg->w_load, gI, gL);
    MOE_LAUNCH_CHECK();
    GateBwdArgs gb{cleanb, sp, eps, topk_idx, topk_gate, dgate, next_idx, gI, gL, dclean, draw, T, n, k};
    if ((st = launch_gate_bwd_rows(gb, T, s)) != MOE_OK) return st;

    // dW_g = x^T dclean, dW_noise = x^T draw: split over tokens, then a fixed-order sum
    SGArgs wa{};
    wa.A[0] = x; wa.B[0] = dclean; wa.B[1] = draw; wa.C = wpart;
    wa.M = d; wa.N = n; wa.K = (int)T; wa.lda = d; wa.ldb = n; wa.ldc = n; wa.nseg = 1;
    wa.ksplit = L.ksplit;
    wa.c_split_stride = (size_t)2 * d * n;
    wa.c_which_stride = (size_t)d * n;
    hipLaunchKernelGGL((sg_kernel<true, false>), dim3(ceil_div(d, SBM), ceil_div(n, SBN), 2 * L.ksplit),
                       dim3(256), 0, s, wa);
    MOE_LAUNCH_CHECK();
    hipLaunchKernelGGL(split_sum_kernel, dim3((unsigned)ceil_div((int64_t)d * n, 256)), dim3(256), 0, s,
                       wpart, L.ksplit, (size_t)2 * d * n, (size_t)d * n, dW_g);
    MOE_LAUNCH_CHECK();
    hipLaunchKernelGGL(split_sum_kernel, dim3((unsigned)ceil_div((int64_t)d * n, 256)), dim3(256), 0, s,
                       wpart + (size_t)d * n, L.ksplit, (size_t)2 * d * n, (size_t)d * n, dW_noise);
    MOE_LAUNCH_CHECK();

    // dx = dclean W_g^T + draw W_noise^T  (+ the experts' part)
    SGArgs xa{};
    xa.A[0] = dclean; xa.A[1] = draw; xa.B[0] = W_g; xa.B[1] = W_noise; xa.C = dx;
    xa.M = (int)T; xa.N = d; xa.K = n; xa.lda = n; xa.ldb = n; xa.ldc = d; xa.nseg = 2; xa.ksplit = 1;
    hipLaunchKernelGGL((sg_kernel<false, true>), dim3((unsigned)ceil_div(T, SBM), ceil_div(d, SBN), 1),
                       dim3(256), 0, s, xa);
    MOE_LAUNCH_CHECK();
    hipLaunchKernelGGL(dx_gather_add_kernel, dim3((unsigned)ceil_div(T, 4)), dim3(256), 0, s,
                       (float4 *)dx, (const float4 *)dxs, inv_perm, T, d / 4, k);
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}

// ---------------------------------------------------------------------------------------
// strictly balanced gating (Appendix F): backward through Eq.(16), Eq.(20), Eq.(15) and the experts
// ---------------------------------------------------------------------------------------
extern "C" size_t moe_backward_balanced_workspace_bytes(const moe_config *cfg) {
    BalancedFwdView V;
    if (balanced_forward_view(cfg, &V) != MOE_OK) return 0;
    BwdLayout L;
    bwd_layout(cfg, &L);
    return L.total;
}

extern "C" int moe_layer_backward_balanced(const moe_config *cfg, const float *x, const float *W_g,
                                           const float *thresholds, const void *W1, const void *W2,
                                           const float *dy, const float *gsigma, const int32_t *tokens,
                                           const uint32_t *kept, const float *denom,
                                           const void *fwd_workspace, float w_batchwise, float *dx,
                                           float *dW_g, float *dW1, float *dW2, void *workspace,
                                           size_t workspace_bytes, void *stream) {
    BalancedFwdView V;
    int st = balanced_forward_view(cfg, &V);
    if (st != MOE_OK) return st;
    const bool f32_experts = cfg->expert_dtype != MOE_DTYPE_BF16;
    if (!f32_experts && (cfg->d % 256 != 0 || cfg->h % 256 != 0)) return MOE_EUNSUPPORTED;
    if (cfg->d % 4 != 0 || cfg->h % 4 != 0 || cfg->n % 4 != 0) return MOE_EUNSUPPORTED;
    if (!W_g || !W1 || !W2 || !fwd_workspace || !dW_g || !dW1 || !dW2 || !workspace) return MOE_EINVAL;
    if (cfg->T > 0 && (!x || !dy || !gsigma || !tokens || !kept || !denom || !dx)) return MOE_EINVAL;   // [T, .] tensors
    if (w_batchwise != 0.f && !thresholds) return MOE_EINVAL;
    if (!aligned16(x) || !aligned16(dy) || !aligned16(dx) || !aligned16(W1) || !aligned16(W2) ||
        !aligned16(dW1) || !aligned16(dW2) || !aligned16(dW_g) || !aligned16(W_g) || !aligned16(gsigma) ||
        !aligned16(workspace) || !aligned16(fwd_workspace))
        return MOE_EINVAL;
    BwdLayout L;
    bwd_layout(cfg, &L);
    if (workspace_bytes < L.total) return MOE_EWORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    const int64_t T = cfg->T, A = T * cfg->k;
    const int d = cfg->d, n = cfg->n;
    if (T == 0) {
        MOE_TRY(launch_zero(dW_g, (size_t)d * n, s));
        MOE_TRY(launch_zero(dW1, (size_t)n * d * cfg->h, s));
        return launch_zero(dW2, (size_t)n * d * cfg->h, s);
    }
    const char *fw = (const char *)fwd_workspace;   // read-only here
    char *ws = (char *)workspace;
    const int32_t *pos = (const int32_t *)(fw + V.pos), *offsets = (const int32_t *)(fw + V.offsets);
    const float *out_rows = (const float *)(fw + V.out_rows);
    float *dxs = (float *)(ws + L.dxs), *drow = (float *)(ws + L.dgate);
    float *dlogit = (float *)(ws + L.dclean), *row_gate = (float *)(ws + L.draw);   // A <= T*n floats
    float *wpart = (float *)(ws + L.wpart);
    int32_t *tile_expert = (int32_t *)(ws + L.tile_expert), *tile_row0 = (int32_t *)(ws + L.tile_row0);
    int32_t *num_tiles = (int32_t *)(ws + L.num_tiles);

    // the experts: an expert's rows are its kept tokens, in the order of `tokens`
    if ((st = launch_balanced_row_gates(gsigma, denom, tokens, offsets, n, A, row_gate, s)) != MOE_OK) return st;
    if (f32_experts) {
        ExpertBwdF32 ef{x, dy, out_rows, row_gate, tokens, offsets, (const float *)W1, (const float *)W2,
                        (const float *)(fw + V.ffn_ws), (float *)(ws + L.xs), (float *)(ws + L.dout),
                        (float *)(ws + L.dz), dxs, drow, tile_expert, tile_row0, num_tiles, dW1, dW2, true};
        if ((st = run_expert_backward_f32(cfg, ef, s)) != MOE_OK) return st;
    } else {
        const uint16_t *saved = V.hidden != (size_t)-1 ? (const uint16_t *)(fw + V.hidden) : nullptr;
        ExpertBwd eb{x, dy, out_rows, row_gate, tokens, offsets, W1, W2, saved, (uint16_t *)(ws + L.xs),
                     (uint16_t *)(ws + L.dout), (uint16_t *)(ws + L.hid), (uint16_t *)(ws + L.dz), dxs, drow,
                     tile_expert, tile_row0, num_tiles, (int32_t *)(ws + L.order), dW1, dW2,
                     {nullptr, nullptr, nullptr, nullptr}, true};
        for (int q = 0; q < 4; ++q)
            if (L.mom[q] != (size_t)-1) eb.mom[q] = (float *)(ws + L.mom[q]);
        if ((st = run_expert_backward(cfg, eb, s)) != MOE_OK) return st;
    }

    // the gate: d/dlogits per token, then the two GEMMs
    if ((st = launch_balanced_gate_bwd(cfg, gsigma, kept, pos, denom, offsets, drow,
                                       w_batchwise != 0.f ? thresholds : nullptr, w_batchwise, dlogit, s)) != MOE_OK)
        return st;
    SGArgs wa{};
    wa.A[0] = x; wa.B[0] = dlogit; wa.C = wpart;
    wa.M = d; wa.N = n; wa.K = (int)T; wa.lda = d; wa.ldb = n; wa.ldc = n; wa.nseg = 1;
    wa.ksplit = L.ksplit;
    wa.c_split_stride = (size_t)d * n;
    hipLaunchKernelGGL((sg_kernel<true, false>), dim3(ceil_div(d, SBM), ceil_div(n, SBN), L.ksplit), dim3(256), 0,
                       s, wa);
    MOE_LAUNCH_CHECK();
    hipLaunchKernelGGL(split_sum_kernel, dim3((unsigned)ceil_div((int64_t)d * n, 256)), dim3(256), 0, s, wpart,
                       L.ksplit, (size_t)d * n, (size_t)d * n, dW_g);
    MOE_LAUNCH_CHECK();
    SGArgs xa{};
    xa.A[0] = dlogit; xa.B[0] = W_g; xa.C = dx;
    xa.M = (int)T; xa.N = d; xa.K = n; xa.lda = n; xa.ldb = n; xa.ldc = d; xa.nseg = 1; xa.ksplit = 1;
    hipLaunchKernelGGL((sg_kernel<false, true>), dim3((unsigned)ceil_div(T, SBM), ceil_div(d, SBN), 1), dim3(256),
                       0, s, xa);
    MOE_LAUNCH_CHECK();
    return launch_add_kept_rows(cfg, dxs, kept, pos, offsets, dx, s);
}

// ---------------------------------------------------------------------------------------
// hierarchical layer (Appendix B): backward through Eq.(12)-(14)
// ---------------------------------------------------------------------------------------
namespace moe {

// Eq.(12),(13): gate(t,p,s) = G_primary(t,p) * G_secondary(t,p,s) feeds Eq.(1) and Importance_H.
// One thread per (token, primary slot): product rule into both levels.
__global__ __launch_bounds__(256) void hier_dgate_kernel(const float *__restrict__ dgate,
                                                         const int32_t *__restrict__ topk_idx,
                                                         const float *__restrict__ gI,
                                                         const float *__restrict__ p_gate,
                                                         const float *__restrict__ s_gate, int64_t Ap,
                                                         int k_s, float *__restrict__ dGp,
                                                         float *__restrict__ dGs) {
    const int64_t ap = (int64_t)blockIdx.x * 256 + threadIdx.x;     // t * k_p + p
    if (ap >= Ap) return;
    const float gp = p_gate[ap];
    float acc = 0.f;
    for (int s = 0; s < k_s; ++s) {
        const int64_t at = ap * k_s + s;                            // = t * k + p * k_s + s
        const float dg = dgate[at] + gI[topk_idx[at]];
        dGs[at] = dg * gp;
        acc = fmaf(dg, s_gate[at], acc);
    }
    dGp[ap] = acc;
}

// Eq.(14): Load_H(i,j) = Load_p(i) * Load_i(j) / |X^(i)|.  One workgroup per group i:
// dLoad_s[i][j] = gL[i][j] * Load_p(i) / |X^(i)|,  dLoad_p[i] = sum_j gL[i][j] * Load_i(j) / |X^(i)|,
// the secondary loads re-summed from the forward pass's per-block partial rows, in order.
__global__ __launch_bounds__(256) void hier_load_grads_kernel(const float *__restrict__ gL,
                                                              const double *__restrict__ p_sums,
                                                              const float *__restrict__ s_partials,
                                                              const int32_t *__restrict__ p_counts,
                                                              const int32_t *__restrict__ p_tile_offsets,
                                                              int a, int b, int sub,
                                                              float *__restrict__ dLoad_p,
                                                              float *__restrict__ dLoad_s) {
    __shared__ double red[256];
    const int i = blockIdx.x, tid = threadIdx.x;
    const int cnt = p_counts[i];
    const double inv = cnt > 0 ? 1.0 / (double)cnt : 0.0;
    const double lp = p_sums[a + i];
    const int blk0 = p_tile_offsets[i] * sub, blk1 = p_tile_offsets[i + 1] * sub;
    double acc = 0.0;
    for (int j = tid; j < b; j += 256) {
        double ls = 0.0;
        for (int blk = blk0; blk < blk1; ++blk) ls += (double)s_partials[((size_t)blk * 2 + 1) * b + j];
        const double g = (double)gL[(size_t)i * b + j];
        dLoad_s[(size_t)i * b + j] = (float)(g * lp * inv);
        acc += g * ls * inv;
    }
    red[tid] = acc;
    __syncthreads();
    if (tid == 0) {
        double t = 0.0;
        for (int q = 0; q < 256; ++q) t += red[q];
        dLoad_p[i] = (float)t;
    }
}

// xg[r] = x[row_src[r] / div]  (fp32 rows in routed order); one wavefront per row
__global__ __launch_bounds__(256) void gather_rows_f32_kernel(const float4 *__restrict__ x,
                                                              const int32_t *__restrict__ row_src, int div,
                                                              int64_t rows, int d4, float4 *__restrict__ out) {
    const int lane = threadIdx.x & 63;
    const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= rows) return;
    const int64_t t = row_src[r] / div;
    for (int c = lane; c < d4; c += 64) out[r * d4 + c] = x[t * d4 + c];
}

struct HierBwdLayout {
    size_t xs, dout, hid, dz, dxs, dgate, gI, gL, tile_expert, tile_row0, num_tiles, order;
    size_t dGp, dGs, dLoad_p, dLoad_s, dclean_p, draw_p, dclean_s, draw_s, xg, dxg, wpart, mom[4], total;
    int ksplit;
};

static void hier_bwd_layout(const moe_config *cfg, HierBwdLayout *L) {
    const size_t T = cfg->T, n = cfg->n, A = T * (size_t)cfg->k, d = cfg->d, h = cfg->h;
    const size_t a = cfg->a, b = cfg->b, Ap = T * (size_t)cfg->k_primary;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off = up256(off + (bytes ? bytes : 1));
        return at;
    };
    L->xs = take(A * d * 2);
    L->dout = take(A * d * 2);
    L->hid = take(A * h * 2);
    L->dz = take(A * h * 2);
    L->dxs = take(A * d * 4);
    L->dgate = take(A * 4);
    L->gI = take(n * 4);
    L->gL = take(n * 4);
    const size_t MT = (size_t)ceil_div((int64_t)A, kFfnBwdTileRows) + n + 8;   // the shortest tiles any kernel here asks for
    L->tile_expert = take(MT * 4);
    L->tile_row0 = take(MT * 4);
    L->num_tiles = take(16);
    L->order = take(n * 4);
    L->dGp = take(Ap * 4);
    L->dGs = take(A * 4);
    L->dLoad_p = take(a * 4);
    L->dLoad_s = take(n * 4);
    L->dclean_p = take(T * a * 4);
    L->draw_p = take(T * a * 4);
    L->dclean_s = take(Ap * b * 4);
    L->draw_s = take(Ap * b * 4);
    L->xg = take(Ap * d * 4);
    L->dxg = take(Ap * d * 4);
    const int64_t tiles = ceil_div(cfg->d, SBM) * ceil_div(cfg->a, SBN) * 2;
    int ks = (int)ceil_div(1024, tiles);
    const int maxks = (int)ceil_div(cfg->T > 0 ? cfg->T : 1, 256);
    if (ks > maxks) ks = maxks;
    if (ks < 1) ks = 1;
    L->ksplit = ks;
    L->wpart = take((size_t)ks * 2 * d * a * 4);
    // MOE_FLAG_ADAM_MOMENTS: per-block sums of squares of dW1 [d,h] and dW2 [h,d] (see GGWgrad)
    const bool mom = (cfg->flags & MOE_FLAG_ADAM_MOMENTS) && cfg->expert_dtype == MOE_DTYPE_BF16;
    L->mom[0] = mom ? take(n * (h / 256) * d * 4) : (size_t)-1;
    L->mom[1] = mom ? take(n * (d / 256) * h * 4) : (size_t)-1;
    L->mom[2] = mom ? take(n * (d / 256) * h * 4) : (size_t)-1;
    L->mom[3] = mom ? take(n * (h / 256) * d * 4) : (size_t)-1;
    L->total = off;
}

static int hier_moments_offsets(const moe_config *cfg, size_t off[4]) {
    HierBwdLayout L;
    hier_bwd_layout(cfg, &L);
    for (int q = 0; q < 4; ++q) {
        if (L.mom[q] == (size_t)-1) return MOE_EINVAL;
        off[q] = L.mom[q];
    }
    return MOE_OK;
}

static int hier_bwd_check(const moe_config *cfg) {
    int st = check_config(cfg);
    if (st != MOE_OK) return st;
    if (cfg->a <= 0) return MOE_EINVAL;
    if (cfg->expert_dtype != MOE_DTYPE_BF16) return MOE_EUNSUPPORTED;
    if (cfg->d % 256 != 0 || cfg->h % 256 != 0) return MOE_EUNSUPPORTED;
    if (cfg->a % 32 != 0 || cfg->b % 32 != 0) return MOE_EUNSUPPORTED;   // k-slabs of the gate GEMMs
    return MOE_OK;
}

}  // namespace moe

extern "C" size_t moe_backward_hier_workspace_bytes(const moe_config *cfg) {
    if (hier_bwd_check(cfg) != MOE_OK) return 0;
    HierBwdLayout L;
    hier_bwd_layout(cfg, &L);
    return L.total;
}

extern "C" int moe_layer_backward_hier(const moe_config *cfg, const float *x, const float *Wg_p,
                                       const float *Wn_p, const float *eps_p, const float *Wg_s,
                                       const float *Wn_s, const float *eps_s, const void *W1,
                                       const void *W2, const float *dy, const int32_t *topk_idx,
                                       const float *topk_gate, const void *fwd_workspace, float *dx,
                                       float *dWg_p, float *dWn_p, float *dWg_s, float *dWn_s,
                                       float *dW1, float *dW2, void *workspace, size_t workspace_bytes,
                                       void *stream) {
    int st = hier_bwd_check(cfg);
    if (st != MOE_OK) return st;
    moe_workspace_layout F;
    if ((st = moe_get_workspace_layout(cfg, &F)) != MOE_OK) return st;
    if (!Wg_p || !Wn_p || !Wg_s || !Wn_s || !W1 || !W2 || !fwd_workspace || !dWg_p || !dWn_p || !dWg_s ||
        !dWn_s || !dW1 || !dW2 || !workspace)
        return MOE_EINVAL;
    if (cfg->T > 0 && (!x || !dy || !topk_idx || !topk_gate || !dx)) return MOE_EINVAL;   // [T, .] tensors
    const void *ptrs[] = {x, Wg_p, Wn_p, Wg_s, Wn_s, W1, W2, dy, fwd_workspace, dx, dWg_p, dWn_p, dWg_s, dWn_s,
                          dW1, dW2, workspace};
    for (const void *q : ptrs)
        if (!aligned16(q)) return MOE_EINVAL;
    if ((eps_p && !aligned16(eps_p)) || (eps_s && !aligned16(eps_s))) return MOE_EINVAL;
    HierBwdLayout L;
    hier_bwd_layout(cfg, &L);
    if (workspace_bytes < L.total) return MOE_EWORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    const int64_t T = cfg->T, A = T * cfg->k, Ap = T * cfg->k_primary;
    const int d = cfg->d, n = cfg->n, a = cfg->a, b = cfg->b, k_p = cfg->k_primary, k_s = cfg->k_secondary;
    if (T == 0) {
        MOE_TRY(launch_zero(dWg_p, (size_t)d * a, s));
        MOE_TRY(launch_zero(dWn_p, (size_t)d * a, s));
        MOE_TRY(launch_zero(dWg_s, (size_t)a * d * b, s));
        MOE_TRY(launch_zero(dWn_s, (size_t)a * d * b, s));
        MOE_TRY(launch_zero(dW1, (size_t)n * d * cfg->h, s));
        return launch_zero(dW2, (size_t)n * d * cfg->h, s);
    }
    char *fw = (char *)fwd_workspace;   // read-only here
    char *ws = (char *)workspace;

    // experts (the flat kernels on the k_p * k_s assignments of every token)
    const bool saved_hidden = F.hidden != (size_t)-1;
    float *dgate = (float *)(ws + L.dgate), *dxs = (float *)(ws + L.dxs);
    ExpertBwd eb{x, dy, (const float *)(fw + F.out_sorted), topk_gate, (const int32_t *)(fw + F.perm),
                 (const int32_t *)(fw + F.offsets), W1, W2,
                 saved_hidden ? (const uint16_t *)(fw + F.hidden) : nullptr, (uint16_t *)(ws + L.xs),
                 (uint16_t *)(ws + L.dout), (uint16_t *)(ws + L.hid), (uint16_t *)(ws + L.dz), dxs, dgate,
                 (int32_t *)(ws + L.tile_expert), (int32_t *)(ws + L.tile_row0), (int32_t *)(ws + L.num_tiles),
                 (int32_t *)(ws + L.order), dW1, dW2, {nullptr, nullptr, nullptr, nullptr}};
    for (int q = 0; q < 4; ++q)
        if (L.mom[q] != (size_t)-1) eb.mom[q] = (float *)(ws + L.mom[q]);
    if ((st = run_expert_backward(cfg, eb, s)) != MOE_OK) return st;

    // Eq.(13),(14): gradients of both CV^2 with respect to Importance_H and Load_H, then into the levels
    float *gI = (float *)(ws + L.gI), *gL = (float *)(ws + L.gL);
    hipLaunchKernelGGL(loss_grad_kernel, dim3(1), dim3(256), 0, s, (const double *)(fw + F.aux_ws), n,
                       cfg->w_importance, cfg->w_load, gI, gL);
    MOE_LAUNCH_CHECK();
    const float *p_gate = (const float *)(fw + F.p_gate), *s_gate = (const float *)(fw + F.s_gate);
    const int32_t *p_idx = (const int32_t *)(fw + F.p_idx), *s_idx = (const int32_t *)(fw + F.s_idx);
    const int32_t *p_offsets = (const int32_t *)(fw + F.p_offsets), *p_perm = (const int32_t *)(fw + F.p_perm);
    const int32_t *p_inv_perm = (const int32_t *)(fw + F.p_inv_perm);
    float *dGp = (float *)(ws + L.dGp), *dGs = (float *)(ws + L.dGs);
    float *dLoad_p = (float *)(ws + L.dLoad_p), *dLoad_s = (float *)(ws + L.dLoad_s);
    hipLaunchKernelGGL(hier_dgate_kernel, dim3((unsigned)ceil_div(Ap, 256)), dim3(256), 0, s, dgate, topk_idx, gI,
                       p_gate, s_gate, Ap, k_s, dGp, dGs);
    MOE_LAUNCH_CHECK();
    hipLaunchKernelGGL(hier_load_grads_kernel, dim3((unsigned)a), dim3(256), 0, s, gL,
                       (const double *)(fw + F.p_aux_ws), (const float *)(fw + F.partials),
                       (const int32_t *)(fw + F.p_counts), (const int32_t *)(fw + F.p_tile_offsets), a, b,
                       kGateBM / gate_rows_per_block(Ap, b), dLoad_p, dLoad_s);
    MOE_LAUNCH_CHECK();

    // primary gate: rows = tokens
    float *dclean_p = (float *)(ws + L.dclean_p), *draw_p = (float *)(ws + L.draw_p);
    GateBwdArgs gp{(const float *)(fw + F.p_cleanb), (const float *)(fw + F.p_sp), eps_p, p_idx, p_gate, dGp,
                   (const int32_t *)(fw + F.p_next_idx), nullptr, dLoad_p, dclean_p, draw_p, T, a, k_p};
    if ((st = launch_gate_bwd_rows(gp, T, s)) != MOE_OK) return st;
    float *wpart = (float *)(ws + L.wpart);
    SGArgs wa{};
    wa.A[0] = x; wa.B[0] = dclean_p; wa.B[1] = draw_p; wa.C = wpart;
    wa.M = d; wa.N = a; wa.K = (int)T; wa.lda = d; wa.ldb = a; wa.ldc = a; wa.nseg = 1;
    wa.ksplit = L.ksplit;
    wa.c_split_stride = (size_t)2 * d * a;
    wa.c_which_stride = (size_t)d * a;
    hipLaunchKernelGGL((sg_kernel<true, false>), dim3(ceil_div(d, SBM), ceil_div(a, SBN), 2 * L.ksplit), dim3(256),
                       0, s, wa);
    MOE_LAUNCH_CHECK();
    hipLaunchKernelGGL(split_sum_kernel, dim3((unsigned)ceil_div((int64_t)d * a, 256)), dim3(256), 0, s, wpart,
                       L.ksplit, (size_t)2 * d * a, (size_t)d * a, dWg_p);
    MOE_LAUNCH_CHECK();
    hipLaunchKernelGGL(split_sum_kernel, dim3((unsigned)ceil_div((int64_t)d * a, 256)), dim3(256), 0, s,
                       wpart + (size_t)d * a, L.ksplit, (size_t)2 * d * a, (size_t)d * a, dWn_p);
    MOE_LAUNCH_CHECK();
    SGArgs xa{};
    xa.A[0] = dclean_p; xa.A[1] = draw_p; xa.B[0] = Wg_p; xa.B[1] = Wn_p; xa.C = dx;
    xa.M = (int)T; xa.N = d; xa.K = a; xa.lda = a; xa.ldb = a; xa.ldc = d; xa.nseg = 2; xa.ksplit = 1;
    hipLaunchKernelGGL((sg_kernel<false, true>), dim3((unsigned)ceil_div(T, SBM), ceil_div(d, SBN), 1), dim3(256), 0,
                       s, xa);
    MOE_LAUNCH_CHECK();

    // secondary gates: rows = (token, primary slot) pairs in the forward pass's group order
    float *dclean_s = (float *)(ws + L.dclean_s), *draw_s = (float *)(ws + L.draw_s);
    GateBwdArgs gs{(const float *)(fw + F.cleanb), (const float *)(fw + F.sp), eps_s, s_idx, s_gate, dGs,
                   (const int32_t *)(fw + F.next_idx), nullptr, dLoad_s, dclean_s, draw_s, Ap, b, k_s,
                   p_perm, p_offsets, a};
    if ((st = launch_gate_bwd_rows(gs, Ap, s)) != MOE_OK) return st;
    float *xg = (float *)(ws + L.xg), *dxg = (float *)(ws + L.dxg);
    hipLaunchKernelGGL(gather_rows_f32_kernel, dim3((unsigned)ceil_div(Ap, 4)), dim3(256), 0, s, (const float4 *)x,
                       p_perm, k_p, Ap, d / 4, (float4 *)xg);
    MOE_LAUNCH_CHECK();
    // every group's two weight gradients over its own rows (one launch each, a group per blockIdx.z),
    // then every group's rows of dx on the forward pass's 128-row tiles, which never straddle groups
    for (int which = 0; which < 2; ++which) {
        SGArgs wg{};
        wg.A[0] = xg; wg.B[0] = which ? draw_s : dclean_s;
        wg.C = which ? dWn_s : dWg_s;
        wg.M = d; wg.N = b; wg.K = 0; wg.lda = d; wg.ldb = b; wg.ldc = b; wg.nseg = 1; wg.ksplit = 1;
        wg.range = p_offsets; wg.range_idx = 0; wg.range_groups = a; wg.c_group_stride = (size_t)d * b;
        hipLaunchKernelGGL((sg_kernel<true, false>), dim3(ceil_div(d, SBM), ceil_div(b, SBN), a), dim3(256), 0, s, wg);
        MOE_LAUNCH_CHECK();
    }
    {
        SGArgs xr{};
        xr.A[0] = dclean_s; xr.A[1] = draw_s; xr.B[0] = Wg_s; xr.B[1] = Wn_s; xr.C = dxg;
        xr.M = 0; xr.N = d; xr.K = b; xr.lda = b; xr.ldb = b; xr.ldc = d; xr.nseg = 2; xr.ksplit = 1;
        xr.range = p_offsets; xr.b_group_stride = (size_t)d * b;
        xr.tile_group = (const int32_t *)(fw + F.p_tile_group);
        xr.tile_row0 = (const int32_t *)(fw + F.p_tile_row0);
        xr.num_tiles = (const int32_t *)(fw + F.p_num_tiles);
        const unsigned max_tiles_p = (unsigned)(ceil_div(Ap, kGateBM) + a);
        hipLaunchKernelGGL((sg_kernel<false, true>), dim3(max_tiles_p, ceil_div(d, SBN), 1), dim3(256), 0, s, xr);
        MOE_LAUNCH_CHECK();
    }
    // dx = primary part (written above) + secondary rows + expert rows
    hipLaunchKernelGGL(dx_gather_add_kernel, dim3((unsigned)ceil_div(T, 4)), dim3(256), 0, s, (float4 *)dx,
                       (const float4 *)dxg, p_inv_perm, T, d / 4, k_p);
    MOE_LAUNCH_CHECK();
    hipLaunchKernelGGL(dx_gather_add_kernel, dim3((unsigned)ceil_div(T, 4)), dim3(256), 0, s, (float4 *)dx,
                       (const float4 *)dxs, (const int32_t *)(fw + F.inv_perm), T, d / 4, cfg->k);
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}
