// a1: noisy top-k gating (Section 2.1, Eq.(3)-(5)) and the per-block partial sums of
// Importance (Eq.(6)) and Load (Eq.(8)-(10), Appendix A).
//
// Two kernels:
//  * gate_logits_kernel  -- clean = x W_g (+bias), sp = Softplus(x W_noise) as an fp32 GEMM on
//    the matrix cores.  v_mfma_f32_32x32x2f32 accumulates its two k-slices one after the other
//    with a single rounding each, i.e. exactly acc = fma(x_j, W_ji, acc) for ascending j, so
//    as long as every output keeps ONE accumulator chain over the whole of d the result has
//    the bits of the sequential fused chain that defines the gate's arithmetic.
//  * gate_topk_kernel    -- one wavefront per row: H = fma(eps, sp, clean), per-lane sorted
//    candidate lists merged by k+1 wave-wide arg-max rounds (ties to the lower index), softmax
//    over the kept logits, then P(x,i) for every expert and the block's partial sums.
#include "stages.h"

namespace moe {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));

// ---------------------------------------------------------------------------------------
// Softplus in binary64, rounded once to fp32.  Fixed operation sequence:
//   a = min(|z|, 64); q = rint(a*log2e); r = fma(-q, ln2, a); E = 2^-q * T13(-r)
//   (T13 = degree-13 Taylor polynomial of exp, Horner with fma);
//   v = 2 + E; y = reciprocal of v by a linear guess (5/6 - v/6) and four Newton steps;
//   s = E*y; L = 2*s*A13(s*s) with A13 = sum_{j<=13} u^j/(2j+1) (Horner with fma);
//   result = (float)(max(z,0) + L).
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ float softplus_spec(float zf) {
    const double z = (double)zf;
    double a = fabs(z);
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
    const double E = ldexp(p, -(int)q);
    const double v = 2.0 + E;
    double y = __fma_rn(-1.0 / 6.0, v, 5.0 / 6.0);
    double e;
    e = __fma_rn(-v, y, 1.0); y = __fma_rn(y, e, y);
    e = __fma_rn(-v, y, 1.0); y = __fma_rn(y, e, y);
    e = __fma_rn(-v, y, 1.0); y = __fma_rn(y, e, y);
    e = __fma_rn(-v, y, 1.0); y = __fma_rn(y, e, y);
    const double s = __dmul_rn(E, y);
    const double s2 = __dmul_rn(s, s);
    double t = 1.0 / 27.0;
    t = __fma_rn(t, s2, 1.0 / 25.0);
    t = __fma_rn(t, s2, 1.0 / 23.0);
    t = __fma_rn(t, s2, 1.0 / 21.0);
    t = __fma_rn(t, s2, 1.0 / 19.0);
    t = __fma_rn(t, s2, 1.0 / 17.0);
    t = __fma_rn(t, s2, 1.0 / 15.0);
    t = __fma_rn(t, s2, 1.0 / 13.0);
    t = __fma_rn(t, s2, 1.0 / 11.0);
    t = __fma_rn(t, s2, 1.0 / 9.0);
    t = __fma_rn(t, s2, 1.0 / 7.0);
    t = __fma_rn(t, s2, 1.0 / 5.0);
    t = __fma_rn(t, s2, 1.0 / 3.0);
    t = __fma_rn(t, s2, 1.0);
    const double L = __dmul_rn(2.0, __dmul_rn(s, t));
    const double zpos = z > 0.0 ? z : 0.0;
    return (float)__dadd_rn(zpos, L);
}

// ---------------------------------------------------------------------------------------
// logits GEMM
// ---------------------------------------------------------------------------------------

constexpr int BM = kGateBM;  // 128 rows: 4 waves x 32


// RN: the block tile is BM x (32*RN) columns of ONE of the two matrices.  VEC: n is a multiple of
// four, so weight rows can be read 16 bytes at a time.
// Every global load of the main loop is unconditional: rows past the end of the tile and columns
// past n re-read a valid element instead (their products only reach outputs that are never
// stored).  A conditional load would put a join, and with it a wait for the load, between the
// load and the matrix work that is supposed to hide it.
// KC: depth of the k-slab staged in LDS.
template <int RN, bool VEC, int KC>
__global__ __launch_bounds__(256) void gate_logits_kernel(LogitsArgs p) {
    constexpr int BN = 32 * RN;
    constexpr int ASTR = KC + 4;  // floats per LDS row of the x tile: [parity][KC/2] + pad
    constexpr int APT = KC / 4;   // threads per x row (one float4 each)
    constexpr int ARP = 256 / APT, APASS = BM / ARP;   // x rows per pass, passes
    constexpr int A_BYTES = 2 * BM * ASTR * 4, B_BYTES = 2 * KC * BN * 4;
    // the epilogue stages EC of the RN column tiles at a time in the (then dead) operand buffers
    constexpr int EC = BM * (BN + 4) * 4 <= A_BYTES + B_BYTES ? RN
                       : BM * (BN / 2 + 4) * 4 <= A_BYTES + B_BYTES ? RN / 2 : RN / 4;
    constexpr int CS = 32 * EC + 4;   // floats per LDS row of the staged output tile
    static_assert(EC >= 1 && BM * CS * 4 <= A_BYTES + B_BYTES, "the output tile reuses the operand buffers");
    __shared__ __attribute__((aligned(16))) char smem[A_BYTES + B_BYTES];
    float (*As)[BM][ASTR] = reinterpret_cast<float (*)[BM][ASTR]>(smem);
    float (*Bs)[KC][BN] = reinterpret_cast<float (*)[KC][BN]>(smem + A_BYTES);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;

    int group = 0;
    int64_t row0 = (int64_t)blockIdx.x * BM;
    int rows;
    if (p.tile_row0) {
        if ((int)blockIdx.x >= *p.num_tiles) return;
        group = p.tile_group[blockIdx.x];
        row0 = p.tile_row0[blockIdx.x];
        rows = (int)min((int64_t)BM, (int64_t)p.group_offsets[group + 1] - row0);
    } else {
        rows = (int)min((int64_t)BM, p.R - row0);
    }
    if (rows <= 0) return;
    const int NT = (p.n + BN - 1) / BN;
    const int which = blockIdx.y / NT;
    const int col0 = (blockIdx.y % NT) * BN;
    const int d = p.d, n = p.n;
    const float *W = (which ? p.Wn : p.Wg) + (size_t)group * d * n;

    // global -> register staging
    const int a_r = tid / APT, a_k = (tid % APT) * 4;       // + ARP*i rows
    const float *a_src[APASS];
#pragma unroll
    for (int i = 0; i < APASS; ++i) {
        const int r = min(a_r + ARP * i, rows - 1);
        const int64_t tok = p.row_src ? (int64_t)(p.row_src[row0 + r] / p.row_div) : row0 + r;
        a_src[i] = p.x + tok * d + a_k;
    }
    constexpr int BQ = BN / 4;                  // float4 per B row
    constexpr int BROWS = 256 / BQ;             // B rows covered per pass
    constexpr int BPASS = KC / BROWS;
    const int b_k = tid / BQ, b_c = (tid % BQ) * 4;
    const float *b_src[4];   // VEC: [0] only
    if (VEC) {
        b_src[0] = W + (size_t)b_k * n + min(col0 + b_c, n - 4);
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) b_src[j] = W + (size_t)b_k * n + min(col0 + b_c + j, n - 1);
    }

    static_assert(BPASS >= 1, "slab too shallow for this tile width");
    v4f a_reg[APASS], b_reg[BPASS];
    auto load_global = [&](int k0) {
#pragma unroll
        for (int i = 0; i < APASS; ++i) a_reg[i] = *reinterpret_cast<const v4f *>(a_src[i] + k0);
#pragma unroll
        for (int i = 0; i < BPASS; ++i) {
            const size_t off = (size_t)(k0 + BROWS * i) * n;
            if (VEC)
                b_reg[i] = *reinterpret_cast<const v4f *>(b_src[0] + off);
            else
                b_reg[i] = v4f{b_src[0][off], b_src[1][off], b_src[2][off], b_src[3][off]};
        }
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int i = 0; i < APASS; ++i) {
            float *row = &As[buf][a_r + ARP * i][0];
            // k parity 0 -> first half of the row, parity 1 -> second half
            *reinterpret_cast<v2f *>(row + a_k / 2) = v2f{a_reg[i].x, a_reg[i].z};
            *reinterpret_cast<v2f *>(row + KC / 2 + a_k / 2) = v2f{a_reg[i].y, a_reg[i].w};
        }
#pragma unroll
        for (int i = 0; i < BPASS; ++i)
            *reinterpret_cast<v4f *>(&Bs[buf][b_k + BROWS * i][b_c]) = b_reg[i];
    };

    v16f acc[RN];
#pragma unroll
    for (int c = 0; c < RN; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[c][r] = 0.f;

    // Main loop, software-pipelined at three levels.  (1) Global -> registers: the loads of slab
    // s+2 are issued as soon as the registers holding slab s+1 have been stored to LDS, in the
    // middle of slab s, so they have a whole slab of matrix work to arrive.  (2) Registers -> LDS:
    // that store also sits in the middle of slab s, far ahead of the barrier that publishes it.
    // (3) LDS -> operand registers: operands are read one group (four k-steps) ahead, and the
    // barrier comes BEFORE the slab's last group, whose operands are already in registers: the
    // first reads of the next slab are in flight while that group runs, so no wave waits on LDS
    // with the matrix pipe empty.
    constexpr int NG = KC / 8;          // operand groups per slab
    constexpr int PG = NG / 2 - 1;      // group after which slab s+1 is stored and s+2 fetched
    v4f a_grp[2];
    float b_grp[2][4][RN];
    auto read_group = [&](int slot, int buf, int kk4) {
        const float *a_row = &As[buf][wave * 32 + l32][half * (KC / 2)];
        const float *b_col = &Bs[buf][half][l32];
        a_grp[slot] = *reinterpret_cast<const v4f *>(a_row + kk4);
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int c = 0; c < RN; ++c) b_grp[slot][u][c] = b_col[2 * (kk4 + u) * BN + 32 * c];
    };
    load_global(0);
    store_lds(0);
    load_global(min(KC, d - KC));
    __syncthreads();
    read_group(0, 0, 0);
    for (int k0 = 0; k0 < d; k0 += KC) {
        const int buf = (k0 / KC) & 1;
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
                for (int c = 0; c < RN; ++c)
                    acc[c] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_grp[g & 1][u], b_grp[g & 1][u][c],
                                                                  acc[c], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if (g == PG) {
                // unconditional (a conditional load or store would put a wait at the join);
                // past the last slab they re-read a valid slab and fill a buffer nobody reads
                store_lds(buf ^ 1);
                load_global(min(k0 + 2 * KC, d - KC));
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }

    // Epilogue.  The accumulators go through LDS (the operand buffers are dead after the last
    // barrier of the loop) so that every lane then owns four adjacent columns of a row: rows leave
    // as 16-byte stores, and the softplus chains of a lane's values are independent straight-line
    // code that the scheduler can interleave.
    float *Ct = reinterpret_cast<float *>(smem);
    float *out = which ? p.sp : p.cleanb;
    constexpr int EQ = 8 * EC;              // float4 per staged row
    constexpr int RPP = 256 / EQ;           // rows per pass
    const int cq = tid % EQ, rr = tid / EQ;
    const bool add_bias = !which && p.bias;
#pragma unroll
    for (int c0 = 0; c0 < RN; c0 += EC) {
        if (c0) __syncthreads();
#pragma unroll
        for (int c = 0; c < EC; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int i = wave * 32 + 8 * (r / 4) + 4 * half + (r % 4);
                Ct[i * CS + 32 * c + l32] = acc[c0 + c][r];
            }
        __syncthreads();
        const int col = col0 + 32 * c0 + 4 * cq;
        float bias[4] = {0.f, 0.f, 0.f, 0.f};
        if (add_bias) {
#pragma unroll
            for (int j = 0; j < 4; ++j) bias[j] = p.bias[min(col + j, n - 1)];
        }
        // four passes at a time: all LDS reads first, then the arithmetic, then the stores
        constexpr int PB = 4;
        static_assert((BM / RPP) % PB == 0, "passes come in batches");
        for (int pass0 = 0; pass0 < BM / RPP; pass0 += PB) {
            v4f t[PB];
#pragma unroll
            for (int u = 0; u < PB; ++u)
                t[u] = *reinterpret_cast<const v4f *>(Ct + (rr + (pass0 + u) * RPP) * CS + 4 * cq);
            if (which) {
#pragma unroll
                for (int u = 0; u < PB; ++u)
#pragma unroll
                    for (int j = 0; j < 4; ++j) t[u][j] = softplus_spec(t[u][j]);
            } else if (add_bias) {
#pragma unroll
                for (int u = 0; u < PB; ++u)
#pragma unroll
                    for (int j = 0; j < 4; ++j) t[u][j] = __fadd_rn(t[u][j], bias[j]);
            }
#pragma unroll
            for (int u = 0; u < PB; ++u) {
                const int i = rr + (pass0 + u) * RPP;
                if (i < rows) {
                    float *dst = out + (row0 + i) * (int64_t)n + col;
                    if (VEC) {
                        if (col < n) *reinterpret_cast<v4f *>(dst) = t[u];
                    } else {
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            if (col + j < n) dst[j] = t[u][j];
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// top-k, softmax, P(x,i) and partial sums
// ---------------------------------------------------------------------------------------

// Phi(u), the standard normal CDF of Eq.(9), in fp32: erfc(x) = t exp(-x^2 + P(t)), t = 1/(1 + x/2),
// with P a degree-10 fit derived by gen_phi_coeffs.py (relative error below 1e-6 wherever Phi
// matters; the sums of P(x,.) over a batch need far less).
__device__ __forceinline__ float normal_cdf(float u) {
    const float x = fabsf(u) * 0.70710678118654752f;
    const float t = __builtin_amdgcn_rcpf(fmaf(0.5f, x, 1.0f));   // v_rcp_f32 (1 ulp); the argument is >= 1
    float p = 8.192740381e-03f;
    p = fmaf(p, t, 1.299090832e-01f);
    p = fmaf(p, t, -7.351043820e-01f);
    p = fmaf(p, t, 1.386106610e+00f);
    p = fmaf(p, t, -1.062397480e+00f);
    p = fmaf(p, t, 2.468332201e-01f);
    p = fmaf(p, t, -1.777072996e-01f);
    p = fmaf(p, t, 9.546407312e-02f);
    p = fmaf(p, t, 3.741950989e-01f);
    p = fmaf(p, t, 1.000020504e+00f);
    p = fmaf(p, t, -1.265512228e+00f);
    const float half_erfc = 0.5f * t * __expf(fmaf(-x, x, p));   // = Phi(-|u|)
    return u < 0.f ? half_erfc : 1.0f - half_erfc;
}

// 1 / (noise standard deviation) for the argument of Phi in Eq.(9): the hardware reciprocal (1 ulp)
// in place of a correctly rounded division, which changes Phi by less than 1e-7.  Deviations below
// 1e-30 (Softplus of a logit under -69; the reciprocal instruction does not take denormals) are
// raised to 1e-30: the argument is then +-inf-like or exactly 0 either way.
__device__ __forceinline__ float load_inv_sigma(float sp) { return __builtin_amdgcn_rcpf(fmaxf(sp, 1e-30f)); }

// Selection key: one unsigned 64-bit integer per (logit, expert) whose order is the order the
// top-k must follow: larger logit first, equal logits -> lower expert index first, +0 = -0.
// High word: the logit's bits mapped monotonically to unsigned; low word: 0x7fffffff - index.
// Key 0 is below every real key (logits are finite) and marks an empty slot.
__device__ __forceinline__ uint64_t sel_key(float h, int i) {
    uint32_t u = __float_as_uint(h + 0.0f);   // -0 -> +0
    u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
    return ((uint64_t)u << 32) | (uint32_t)(0x7fffffff - i);
}
__device__ __forceinline__ float key_logit(uint64_t key) {
    uint32_t u = (uint32_t)(key >> 32);
    u = (u & 0x80000000u) ? (u & 0x7fffffffu) : ~u;
    return __uint_as_float(u);
}
__device__ __forceinline__ int key_index(uint64_t key) { return 0x7fffffff - (int)(uint32_t)key; }

// Maximum of one 32-bit value per lane over the whole wavefront, returned wave-uniform.  Four
// data-parallel-primitive steps (swap within pairs, within quads, mirror within 8 and within 16
// lanes) leave every 16-lane row holding its maximum; the four rows meet in scalar registers.
// No LDS permutes and no waits: the chain is a dozen short-latency instructions.
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, true));    // quad_perm [1,0,3,2]
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, true));    // quad_perm [2,3,0,1]
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xF, 0xF, true));   // row_half_mirror
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xF, 0xF, true));   // row_mirror
    const uint32_t r0 = __builtin_amdgcn_readlane((int)v, 0), r1 = __builtin_amdgcn_readlane((int)v, 16);
    const uint32_t r2 = __builtin_amdgcn_readlane((int)v, 32), r3 = __builtin_amdgcn_readlane((int)v, 48);
    return max(max(r0, r1), max(r2, r3));
}

// Largest selection key of the wavefront.  Keys are unique (the index is part of the key), so the
// maximum is found in two 32-bit passes: the largest logit word, then the largest index word among
// the lanes that hold that logit.  An all-empty wavefront (every key 0) gives 0.
__device__ __forceinline__ uint64_t wave_max_key(uint64_t key) {
    const uint32_t hi = (uint32_t)(key >> 32), lo = (uint32_t)key;
    const uint32_t hmax = wave_max_u32(hi);
    const uint32_t lmax = wave_max_u32(hi == hmax ? lo : 0u);
    return ((uint64_t)hmax << 32) | lmax;
}

// The same pointer in scalar registers (all lanes hold the same value): loads through it can use
// scalar-base addressing with one 32-bit lane offset.
__device__ __forceinline__ const float *uniform_ptr(const float *ptr) {
    const uint64_t v = reinterpret_cast<uint64_t>(ptr);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const float *>(((uint64_t)hi << 32) | lo);
}

// L >= k+1 candidate slots per lane; NCH >= ceil(n/64) register chunks: a lane holds the whole of
// its share of a row (clean, softplus, H) in registers, so the row is read from memory once, all
// loads are in flight together, and both passes (top-k, then P(x,i)) run from registers.  The
// per-expert sums of G(x) and P(x,.) also stay in registers across the rows a wave walks.
template <int L, int NCH>
__global__ __launch_bounds__(256, 2) void gate_topk_kernel(TopkArgs p) {
    extern __shared__ float lds_acc[];  // Importance per wave [4][n] | Load of the block [n]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: row pointers stay uniform
    const int n = p.n, k = p.k;
    const int RPB = p.rows_per_block;
    const int SUB = kGateBM / RPB;

    int64_t rb, re;
    if (p.tile_row0) {
        const int tile = blockIdx.x / SUB;
        if (tile >= *p.num_tiles) return;
        const int g = p.tile_group[tile];
        const int64_t t0 = p.tile_row0[tile];
        const int64_t tend = min(t0 + kGateBM, (int64_t)p.group_offsets[g + 1]);
        rb = min(t0 + (int64_t)(blockIdx.x % SUB) * RPB, tend);
        re = min(rb + RPB, tend);
    } else {
        rb = (int64_t)blockIdx.x * RPB;
        re = min(rb + RPB, p.R);
    }
    const int kp1 = (k < n) ? k + 1 : k;
    // Load: every expert of every row contributes, so the sums stay in registers.  Importance:
    // only the k kept experts of a row contribute, so k lanes add their gate values to the
    // wave's own LDS array (distinct addresses inside one instruction, rows in order: the sum
    // of each entry is a fixed sequence of fp32 additions).
    float acc_load[NCH];
#pragma unroll
    for (int q = 0; q < NCH; ++q) acc_load[q] = 0.f;
    float *imp_w = lds_acc + wave * n;
    for (int i = tid; i < 4 * n; i += 256) lds_acc[i] = 0.f;
    __syncthreads();

#pragma unroll 1
    for (int64_t r = rb + wave; r < re; r += 4) {
        const float *c_row = uniform_ptr(p.cleanb + r * n);
        const float *s_row = uniform_ptr(p.sp + r * n);
        const int64_t orow = p.row_map ? p.row_map[r] : r;
        const float *e_row = p.eps ? uniform_ptr(p.eps + orow * n) : nullptr;

        // Unconditional loads from a wave-uniform row pointer plus a clamped lane offset: lanes past
        // the end of the row re-read its last element (they are masked out of the selection and of
        // the sums below), so no load sits behind a branch.
        float cv[NCH], sv[NCH], hv[NCH];
#pragma unroll
        for (int q = 0; q < NCH; ++q) {
            const unsigned i = min((unsigned)(lane + 64 * q), (unsigned)(n - 1));
            cv[q] = c_row[i];
            sv[q] = s_row[i];
        }
        if (e_row) {
#pragma unroll
            for (int q = 0; q < NCH; ++q)
                hv[q] = e_row[min((unsigned)(lane + 64 * q), (unsigned)(n - 1))];
#pragma unroll
            for (int q = 0; q < NCH; ++q) hv[q] = __fmaf_rn(hv[q], sv[q], cv[q]);
        } else {
#pragma unroll
            for (int q = 0; q < NCH; ++q) hv[q] = cv[q];
        }

        // per-lane sorted candidate list: branch-free compare-exchange insertion
        uint64_t lk[L];
#pragma unroll
        for (int j = 0; j < L; ++j) lk[j] = 0;
#pragma unroll
        for (int q = 0; q < NCH; ++q) {
            const int i = lane + 64 * q;
            uint64_t key = i < n ? sel_key(hv[q], i) : 0;
#pragma unroll
            for (int j = 0; j < L; ++j) {
                const bool up = key > lk[j];
                const uint64_t lo = up ? lk[j] : key;
                lk[j] = up ? key : lk[j];
                key = lo;
            }
            // long rows: one element at a time, or the keys of the whole row are built up front
            // and spill
            if (NCH >= 16) __builtin_amdgcn_sched_barrier(0);
        }
        // k+1 rounds: wave-wide maximum of the list heads (keys are unique), the owner pops
        float tv[L];
        int ti[L];
#pragma unroll
        for (int j = 0; j < L; ++j) {
            tv[j] = -INFINITY;
            ti[j] = 0x7fffffff;
            if (j < kp1) {
                const uint64_t v = wave_max_key(lk[0]);
                tv[j] = key_logit(v);
                ti[j] = key_index(v);
                const bool pop = lk[0] == v;
#pragma unroll
                for (int q = 0; q + 1 < L; ++q) lk[q] = pop ? lk[q + 1] : lk[q];
                lk[L - 1] = pop ? 0 : lk[L - 1];
            }
        }
        // Eq.(3): softmax over the kept logits
        float g[L];
        float sum = 0.f;
#pragma unroll
        for (int j = 0; j < L; ++j) {
            g[j] = (j < k) ? expf(tv[j] - tv[0]) : 0.f;
            sum += g[j];
        }
        const float inv = 1.0f / sum;
#pragma unroll
        for (int j = 0; j < L; ++j) g[j] *= inv;
        {
            // lane j < k owns slot j: it writes the slot's outputs and adds its gate value
            int my_i = ti[0];
            float my_g = g[0];
#pragma unroll
            for (int j = 1; j < L; ++j)
                if (j < k && lane == j) {
                    my_i = ti[j];
                    my_g = g[j];
                }
            if (lane < k) {
                p.idx[orow * k + lane] = my_i;
                p.gate[orow * k + lane] = my_g;
                unsafeAtomicAdd(&imp_w[my_i], my_g);
            }
        }
        // Eq.(9): P(x,i) for every expert; threshold = (k+1)-th H for kept experts, k-th otherwise.
        // "kept" is H_i >= the k-th kept logit: where that misjudges a tie, the (k+1)-th logit
        // equals the k-th and both thresholds coincide.
        float thr_in = 0.f, thr_out = 0.f;
        int nxt = -1;
#pragma unroll
        for (int j = 0; j < L; ++j) {
            if (j == k && k < n) {
                thr_in = tv[j];
                nxt = ti[j];
            }
            if (j == k - 1) thr_out = tv[j];
        }
        if (lane == 0 && p.next_idx) p.next_idx[orow] = nxt;
        if (k < n) {
#pragma unroll
            for (int q = 0; q < NCH; ++q) {
                const int i = lane + 64 * q;
                const float u = (cv[q] - (hv[q] >= thr_out ? thr_in : thr_out)) * load_inv_sigma(sv[q]);
                const float P = normal_cdf(u);
                acc_load[q] += i < n ? P : 0.f;
                if (NCH >= 16 && (q & 3) == 3) __builtin_amdgcn_sched_barrier(0);
            }
        } else {
#pragma unroll
            for (int q = 0; q < NCH; ++q) acc_load[q] += (lane + 64 * q) < n ? 1.0f : 0.f;
        }
    }
    // the four waves' sums, added in wave order
    float *load_s = lds_acc + 4 * n;
    for (int w = 0; w < 4; ++w) {
        if (wave == w) {
#pragma unroll
            for (int q = 0; q < NCH; ++q) {
                const int i = lane + 64 * q;
                if (i < n) load_s[i] = (w ? load_s[i] : 0.f) + acc_load[q];
            }
        }
        __syncthreads();
    }
    float *out = p.partials + (size_t)blockIdx.x * 2 * n;
    for (int i = tid; i < n; i += 256) {
        out[i] = (((0.f + lds_acc[i]) + lds_acc[n + i]) + lds_acc[2 * n + i]) + lds_acc[3 * n + i];
        out[n + i] = load_s[i];
    }
}

// Long rows (n > 1024): the four wavefronts of a workgroup share one row; a row is NCK chunks of
// 2048 columns and a wave owns a quarter of every chunk, so a lane holds NCH = 8 logits at a time
// (the one-wave-per-row kernel would need 32 and spills).  Rows of up to 2048 experts are one chunk
// that stays in registers for both passes; longer rows walk their chunks twice.  Each
// wave finds the k+1 best of its quarter, the 4(k+1) candidates meet in LDS, every wave merges
// them (identically) into the row's k+1 best, and then evaluates P(x,i) on its own quarter.  A
// wave keeps the same columns for every row of the workgroup, so the Load sums need no exchange
// at all; Importance is added by the first wave alone, row after row.
template <int L, int NCH, int NCK>   // NCK chunks of 256 * NCH columns cover the row
__global__ __launch_bounds__(256, 2) void gate_topk_wide_kernel(TopkArgs p) {
    constexpr int CW = 256 * NCH;                 // columns of one chunk
    extern __shared__ float lds_imp[];            // Importance of the block [n]
    __shared__ uint64_t cand[2][4][L];            // per row parity, per wave
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = p.n, k = p.k;
    const int RPB = p.rows_per_block;
    const int SUB = kGateBM / RPB;

    int64_t rb, re;
    if (p.tile_row0) {
        const int tile = blockIdx.x / SUB;
        if (tile >= *p.num_tiles) return;
        const int g = p.tile_group[tile];
        const int64_t t0 = p.tile_row0[tile];
        const int64_t tend = min(t0 + kGateBM, (int64_t)p.group_offsets[g + 1]);
        rb = min(t0 + (int64_t)(blockIdx.x % SUB) * RPB, tend);
        re = min(rb + RPB, tend);
    } else {
        rb = (int64_t)blockIdx.x * RPB;
        re = min(rb + RPB, p.R);
    }
    const int kp1 = (k < n) ? k + 1 : k;
    const int col_base = wave * 64 * NCH;         // this wave's quarter of every chunk
    float acc_load[NCK][NCH];
#pragma unroll
    for (int cb = 0; cb < NCK; ++cb)
#pragma unroll
        for (int q = 0; q < NCH; ++q) acc_load[cb][q] = 0.f;
    for (int i = tid; i < n; i += 256) lds_imp[i] = 0.f;
    __syncthreads();

#pragma unroll 1
    for (int64_t r = rb; r < re; ++r) {
        const int par = (int)(r - rb) & 1;
        const float *c_row = uniform_ptr(p.cleanb + r * n);
        const float *s_row = uniform_ptr(p.sp + r * n);
        const int64_t orow = p.row_map ? p.row_map[r] : r;
        const float *e_row = p.eps ? uniform_ptr(p.eps + orow * n) : nullptr;

        // one chunk of this wave's columns: clean, Softplus and H (unconditional clamped loads)
        float cv[NCH], sv[NCH], hv[NCH];
        auto load_chunk = [&](int cb) {
#pragma unroll
            for (int q = 0; q < NCH; ++q) {
                const unsigned i = min((unsigned)(cb * CW + col_base + lane + 64 * q), (unsigned)(n - 1));
                cv[q] = c_row[i];
                sv[q] = s_row[i];
            }
            if (e_row) {
#pragma unroll
                for (int q = 0; q < NCH; ++q)
                    hv[q] = e_row[min((unsigned)(cb * CW + col_base + lane + 64 * q), (unsigned)(n - 1))];
#pragma unroll
                for (int q = 0; q < NCH; ++q) hv[q] = __fmaf_rn(hv[q], sv[q], cv[q]);
            } else {
#pragma unroll
                for (int q = 0; q < NCH; ++q) hv[q] = cv[q];
            }
        };

        // this wave's k+1 best over all its chunks: per-lane sorted lists, then wave-wide maxima
        uint64_t lk[L];
#pragma unroll
        for (int j = 0; j < L; ++j) lk[j] = 0;
#pragma unroll 1
        for (int cb = 0; cb < NCK; ++cb) {
            load_chunk(cb);
#pragma unroll
            for (int q = 0; q < NCH; ++q) {
                const int i = cb * CW + col_base + lane + 64 * q;
                uint64_t key = i < n ? sel_key(hv[q], i) : 0;
#pragma unroll
                for (int j = 0; j < L; ++j) {
                    const bool up = key > lk[j];
                    const uint64_t lo = up ? lk[j] : key;
                    lk[j] = up ? key : lk[j];
                    key = lo;
                }
            }
        }
        uint64_t mine = 0;   // lane j keeps the quarter's j-th best
#pragma unroll
        for (int j = 0; j < L; ++j) {
            if (j < kp1) {
                const uint64_t v = wave_max_key(lk[0]);
                mine = lane == j ? v : mine;
                const bool pop = lk[0] == v;
#pragma unroll
                for (int q = 0; q + 1 < L; ++q) lk[q] = pop ? lk[q + 1] : lk[q];
                lk[L - 1] = pop ? 0 : lk[L - 1];
            }
        }
        if (lane < L) cand[par][wave][lane] = lane < kp1 ? mine : 0;
        __syncthreads();
        // every wave merges the 4L candidates the same way
        uint64_t ck = lane < 4 * L ? cand[par][lane / L][lane % L] : 0;
        float tv[L];
        int ti[L];
#pragma unroll
        for (int j = 0; j < L; ++j) {
            tv[j] = -INFINITY;
            ti[j] = 0x7fffffff;
            if (j < kp1) {
                const uint64_t v = wave_max_key(ck);
                tv[j] = key_logit(v);
                ti[j] = key_index(v);
                ck = ck == v ? 0 : ck;
            }
        }
        // Eq.(3): softmax over the kept logits
        float g[L];
        float sum = 0.f;
#pragma unroll
        for (int j = 0; j < L; ++j) {
            g[j] = (j < k) ? expf(tv[j] - tv[0]) : 0.f;
            sum += g[j];
        }
        const float inv = 1.0f / sum;
#pragma unroll
        for (int j = 0; j < L; ++j) g[j] *= inv;
        float thr_in = 0.f, thr_out = 0.f;
        int nxt = -1;
#pragma unroll
        for (int j = 0; j < L; ++j) {
            if (j == k && k < n) {
                thr_in = tv[j];
                nxt = ti[j];
            }
            if (j == k - 1) thr_out = tv[j];
        }
        if (wave == 0) {
            int my_i = ti[0];
            float my_g = g[0];
#pragma unroll
            for (int j = 1; j < L; ++j)
                if (j < k && lane == j) {
                    my_i = ti[j];
                    my_g = g[j];
                }
            if (lane < k) {
                p.idx[orow * k + lane] = my_i;
                p.gate[orow * k + lane] = my_g;
                unsafeAtomicAdd(&lds_imp[my_i], my_g);
            }
            if (lane == 0 && p.next_idx) p.next_idx[orow] = nxt;
        }
        // Eq.(9) on this wave's columns.  A single chunk is still in registers; several chunks are
        // fetched again (the same loads and the same fused multiply-add give the same H).
        if (k < n) {
#pragma unroll 1
            for (int cb = 0; cb < NCK; ++cb) {
                if (NCK > 1) load_chunk(cb);
#pragma unroll
                for (int q = 0; q < NCH; ++q) {
                    const int i = cb * CW + col_base + lane + 64 * q;
                    const float u = (cv[q] - (hv[q] >= thr_out ? thr_in : thr_out)) * load_inv_sigma(sv[q]);
                    const float P = normal_cdf(u);
                    acc_load[cb][q] += i < n ? P : 0.f;
                }
            }
        } else {
#pragma unroll
            for (int cb = 0; cb < NCK; ++cb)
#pragma unroll
                for (int q = 0; q < NCH; ++q) acc_load[cb][q] += (cb * CW + col_base + lane + 64 * q) < n ? 1.0f : 0.f;
        }
    }
    __syncthreads();
    float *out = p.partials + (size_t)blockIdx.x * 2 * n;
    for (int i = tid; i < n; i += 256) out[i] = lds_imp[i];
#pragma unroll
    for (int cb = 0; cb < NCK; ++cb)
#pragma unroll
        for (int q = 0; q < NCH; ++q) {
            const int i = cb * CW + col_base + lane + 64 * q;
            if (i < n) out[n + i] = acc_load[cb][q];
        }
}

// Eq.(12): global expert id and gate product for every (token, primary slot, secondary slot)
__global__ __launch_bounds__(256) void hier_compose_kernel(const int32_t *__restrict__ p_idx,
                                                           const float *__restrict__ p_gate,
                                                           const int32_t *__restrict__ s_idx,
                                                           const float *__restrict__ s_gate,
                                                           int64_t T, int k_p, int k_s, int b,
                                                           int32_t *__restrict__ idx,
                                                           float *__restrict__ gate) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;   // over T*k_p*k_s
    if (i >= T * k_p * k_s) return;
    const int64_t ap = i / k_s;                                  // primary assignment t*k_p + p
    idx[i] = p_idx[ap] * b + s_idx[i];
    gate[i] = p_gate[ap] * s_gate[i];
}

int launch_hier_compose(const int32_t *p_idx, const float *p_gate, const int32_t *s_idx,
                        const float *s_gate, int64_t T, int k_p, int k_s, int b, int32_t *idx,
                        float *gate, hipStream_t st) {
    const int64_t total = T * k_p * k_s;
    if (total <= 0) return MOE_OK;
    hipLaunchKernelGGL(hier_compose_kernel, dim3((unsigned)ceil_div(total, 256)), dim3(256), 0, st,
                       p_idx, p_gate, s_idx, s_gate, T, k_p, k_s, b, idx, gate);
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------
template <int RN, int KC = 32>
static void launch_logits_rn(const LogitsArgs &a, int64_t row_tiles, hipStream_t st) {
    // without a noise matrix only the clean half of the grid exists
    dim3 grid((unsigned)row_tiles, (a.Wn ? 2u : 1u) * (unsigned)ceil_div(a.n, 32 * RN));
    if (a.n % 4 == 0) hipLaunchKernelGGL((gate_logits_kernel<RN, true, KC>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((gate_logits_kernel<RN, false, KC>), grid, dim3(256), 0, st, a);
}

int launch_gate_logits(const LogitsArgs &a, int64_t row_tiles, hipStream_t st) {
    if (row_tiles <= 0) return MOE_OK;
    if (a.n <= 32) launch_logits_rn<1>(a, row_tiles, st);
    else if (a.n <= 64) launch_logits_rn<2>(a, row_tiles, st);
    // few tiles: narrower column tiles so that every CU holds at least two workgroups
    else if (row_tiles * 2 * ceil_div(a.n, 128) < 1024) launch_logits_rn<2>(a, row_tiles, st);
    // wide flat gates with many rounds of tiles: 256-column tiles over 16-deep slabs (same LDS and
    // register budget, two workgroups per CU) halve the prologues and epilogues per flop: 3 % at
    // 2048 and 512 experts; slower for the grouped secondary gates of the hierarchical layer
    else if (a.n % 256 == 0 && a.n >= 512 && !a.tile_row0) launch_logits_rn<8, 16>(a, row_tiles, st);
    else launch_logits_rn<4>(a, row_tiles, st);
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}

template <int L>
static int launch_topk_nch(const TopkArgs &a, unsigned blocks, size_t lds, hipStream_t st) {
    const size_t wide_lds = (size_t)a.n * sizeof(float);
    if (a.n <= 64) hipLaunchKernelGGL((gate_topk_kernel<L, 1>), dim3(blocks), dim3(256), lds, st, a);
    else if (a.n <= 128) hipLaunchKernelGGL((gate_topk_kernel<L, 2>), dim3(blocks), dim3(256), lds, st, a);
    else if (a.n <= 256) hipLaunchKernelGGL((gate_topk_kernel<L, 4>), dim3(blocks), dim3(256), lds, st, a);
    else if (a.n <= 512) hipLaunchKernelGGL((gate_topk_kernel<L, 8>), dim3(blocks), dim3(256), lds, st, a);
    else if (a.n <= 1024) hipLaunchKernelGGL((gate_topk_kernel<L, 16>), dim3(blocks), dim3(256), lds, st, a);
    else if (a.n <= 2048) hipLaunchKernelGGL((gate_topk_wide_kernel<L, 8, 1>), dim3(blocks), dim3(256), wide_lds, st, a);
    else if (a.n <= 4096) hipLaunchKernelGGL((gate_topk_wide_kernel<L, 8, 2>), dim3(blocks), dim3(256), wide_lds, st, a);
    else if (a.n <= 8192) hipLaunchKernelGGL((gate_topk_wide_kernel<L, 8, 4>), dim3(blocks), dim3(256), wide_lds, st, a);
    else {
        static LdsLimitOnce lds_once;   // 64 KB of Importance sums beside the candidate exchange
        MOE_TRY(lds_once.set((const void *)gate_topk_wide_kernel<L, 8, 8>, wide_lds));
        hipLaunchKernelGGL((gate_topk_wide_kernel<L, 8, 8>), dim3(blocks), dim3(256), wide_lds, st, a);
    }
    return MOE_OK;
}

int launch_gate_topk(const TopkArgs &a, int64_t blocks, hipStream_t st) {
    if (blocks <= 0) return MOE_OK;
    const size_t lds = (size_t)5 * a.n * sizeof(float);
    if (a.k + 1 <= 3) MOE_TRY(launch_topk_nch<3>(a, (unsigned)blocks, lds, st));
    else if (a.k + 1 <= 5) MOE_TRY(launch_topk_nch<5>(a, (unsigned)blocks, lds, st));
    else MOE_TRY(launch_topk_nch<9>(a, (unsigned)blocks, lds, st));
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}

}  // namespace moe

using namespace moe;

namespace moe {
// Rows one top-k workgroup (4 waves) walks: few rows per block when the batch is small, so that
// every CU holds several blocks and row latency is hidden; more when the partial-sum traffic
// (one [2][n] row per block) would otherwise rival the logits themselves.
int gate_rows_per_block(int64_t rows, int n) {
    return (rows * (int64_t)n <= ((int64_t)1 << 22)) ? 8 : 32;
}
}  // namespace moe

extern "C" int64_t moe_gate_partial_rows(const moe_config *cfg) {
    if (!cfg || cfg->T <= 0) return 0;
    return ceil_div(cfg->T, gate_rows_per_block(cfg->T, cfg->n));
}

extern "C" int moe_gate(const moe_config *cfg, const float *x, const float *W_g,
                        const float *W_noise, const float *gate_bias, const float *eps,
                        int32_t *topk_idx, float *topk_gate, float *cleanb, float *sp,
                        int32_t *next_idx, float *partials, void *stream) {
    int st = check_config(cfg);
    if (st != MOE_OK) return st;
    if (cfg->a != 0) return MOE_EINVAL;  // flat entry point; hierarchical layers use moe_gate_hier
    if (!x || !W_g || !W_noise || !topk_idx || !topk_gate || !cleanb || !sp || !partials)
        return MOE_EINVAL;
    if (!aligned16(x) || !aligned16(W_g) || !aligned16(W_noise) || !aligned16(cleanb) ||
        !aligned16(sp) || (eps && !aligned16(eps)))
        return MOE_EINVAL;
    st = check_gate_level(cfg->T, cfg->d, cfg->n, cfg->k);
    if (st != MOE_OK) return st;

    LogitsArgs la{};
    la.x = x; la.Wg = W_g; la.Wn = W_noise; la.bias = gate_bias;
    la.cleanb = cleanb; la.sp = sp;
    la.R = cfg->T; la.d = cfg->d; la.n = cfg->n;
    st = launch_gate_logits(la, ceil_div(cfg->T, kGateBM), (hipStream_t)stream);
    if (st != MOE_OK) return st;

    TopkArgs ta{};
    ta.cleanb = cleanb; ta.sp = sp; ta.eps = eps;
    ta.R = cfg->T; ta.n = cfg->n; ta.k = cfg->k;
    ta.idx = topk_idx; ta.gate = topk_gate; ta.next_idx = next_idx; ta.partials = partials;
    ta.rows_per_block = gate_rows_per_block(cfg->T, cfg->n);
    return launch_gate_topk(ta, moe_gate_partial_rows(cfg), (hipStream_t)stream);
}
