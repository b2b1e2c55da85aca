// a3: the experts.  E_i(x) = relu(x W1_i) W2_i (Appendix C: one ReLU hidden layer, no biases),
// evaluated only for the (token, expert) pairs the gate kept (Section 2) and batched per expert
// (Section 3.1).
//
// bf16 path (ffn_bf16_kernel): one workgroup = one row tile (<= 64 gathered rows of ONE expert).
// The expert's 2 x d x h bf16 weights are streamed exactly once per tile straight from global
// memory into matrix-core operands: each lane loads an 8(k) x BW(column) block of the row-major
// weight matrix and transposes it in registers with byte permutes, so the plain
// "input x hidden" / "hidden x output" layouts need no repacking and no LDS staging.  The x tile
// and then the hidden tile live in LDS (the hidden layer never reaches HBM); accumulation is
// fp32 in v_mfma_f32_32x32x16_bf16.
//
// fp32 path (ffn_f32_mfma_kernel): LDS-tiled grouped GEMM on the fp32 matrix cores, hidden layer
// kept in a workspace.
#include "stages.h"

namespace moe {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));

constexpr int kFfnTM = 64;  // rows per tile
// Cache policy of the four-wave kernel's weight loads (it runs when experts have one tile each, so
// every weight byte is used once): the non-temporal bit of the buffer instruction's policy field.
#ifndef FFN4_AUX
#define FFN4_AUX 2
#endif
#ifndef FFN_STAGES1
#define FFN_STAGES1 2
#define FFN_STAGES2 2
#endif

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) { return pack_bf16_pair(lo, hi); }

// 16 bytes of expert output.  The rows are written once and read back by the combine after the
// whole launch: a streaming store keeps them from displacing weights in L2.
__device__ __forceinline__ void store_out4(float *dst, v4f v) {
    MOE_STREAM_STORE(v, reinterpret_cast<v4f *>(dst));
}


// XCD-aware tile order: consecutive workgroup ids go to different XCDs (one L2 each), so
// workgroup b takes tile (b % 8) * ceil(num/8) + b / 8: tiles of one expert, which are adjacent
// in the table, then run at the same time behind the same L2 and the expert's weights cross
// the fabric once.
__device__ __forceinline__ int xcd_tile(int bid, int num_tiles) {
    const int per = (num_tiles + 7) >> 3;
    const int tile = (bid & 7) * per + (bid >> 3);
    return ((bid >> 3) < per && tile < num_tiles) ? tile : -1;
}

// A workgroup's tile: expert, first sorted row, rows (<= TM).  All wave-uniform and kept in scalar
// registers (they give the weight stream a scalar buffer descriptor).  The row count comes from
// the NEXT table entry, fetched in the same round trip as this one, instead of from the offsets
// array one dependent round trip later: tiles of one expert are consecutive and only its last one
// is short, and the next expert's first row is where this expert's rows end (experts in between
// have none).  Only the table's very last tile has to look at the offsets.
struct TileCoord {
    int e, row0, rows;
};
template <class Args>
__device__ __forceinline__ bool load_tile(const Args &p, int TM, TileCoord &t) {
    const int num = *p.num_tiles;
    const int tile = xcd_tile(blockIdx.x, num);
    if (tile < 0) return false;
    const bool has_next = tile + 1 < num;
    const int nx = has_next ? tile + 1 : tile;
    const int e = p.tile_expert[tile], row0 = p.tile_row0[tile];
    const int e2 = p.tile_expert[nx], r2 = p.tile_row0[nx];
    t.e = __builtin_amdgcn_readfirstlane(e);
    t.row0 = __builtin_amdgcn_readfirstlane(row0);
    int rows;
    if (has_next) rows = e2 == e ? TM : r2 - row0;
    else rows = min(TM, p.offsets[t.e + 1] - t.row0);
    t.rows = __builtin_amdgcn_readfirstlane(rows);
    return true;
}

// One 32-deep k-step of B-operand data for 8 adjacent columns of a row-major [K, N] bf16
// matrix: lane (c = lane % 16, g = lane / 16) holds rows k0+8g .. k0+8g+7, columns col .. col+7,
// fetched as eight 16-byte loads (the vector memory pipe moves 16 B per lane per instruction at
// the same address-processing cost as 4 B, so nothing narrower is ever issued for weights).
struct BFrag {
    uint32_t r[8][4];
};

// Column j of the block as a v_mfma_f32_16x16x32_bf16 B operand (8 consecutive k in one lane):
// a register transpose done with byte permutes.
__device__ __forceinline__ v8bf bfrag_column(const BFrag &f, int j) {
    const uint32_t sel = (j & 1) ? 0x07060302u : 0x05040100u;
    uint4 o;
    o.x = __builtin_amdgcn_perm(f.r[1][j >> 1], f.r[0][j >> 1], sel);
    o.y = __builtin_amdgcn_perm(f.r[3][j >> 1], f.r[2][j >> 1], sel);
    o.z = __builtin_amdgcn_perm(f.r[5][j >> 1], f.r[4][j >> 1], sel);
    o.w = __builtin_amdgcn_perm(f.r[7][j >> 1], f.r[6][j >> 1], sel);
    return __builtin_bit_cast(v8bf, o);
}

// A software-pipelined stream of weight fragments: STAGES k-steps of 32 stay in flight per
// wave, so the weights (read once per tile) arrive ahead of the matrix cores.  The k loop is
// fully unrolled: with no loop-carried registers the compiler's wait counts stay exact.
template <int K, int LD, int STAGES>   // LD: elements per row of the weight matrix
struct WeightStream {
    static_assert(K % (32 * STAGES) == 0, "k extent must be a multiple of the pipeline depth");
    BFrag f[STAGES];
    __amdgpu_buffer_rsrc_t rsrc;   // the expert's matrix as a buffer: scalar base, so the whole stream
    uint32_t lane_off;             // needs one address VGPR (this lane's first element, in bytes)

    __device__ __forceinline__ void load(int s, int k0) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const v4u v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, lane_off, (uint32_t)(k0 + i) * LD * 2u, 0);
            f[s].r[i][0] = v.x; f[s].r[i][1] = v.y; f[s].r[i][2] = v.z; f[s].r[i][3] = v.w;
        }
    }
    // W: the matrix (bytes long); the stream covers rows [row0, row0 + K), columns col .. col + 7
    __device__ __forceinline__ void start(const uint16_t *W, uint32_t bytes, int row0, int col, int g) {
        rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(W), 0, bytes, 0x00020000);
        lane_off = (uint32_t)((row0 + 8 * g) * LD + col) * 2u;
#pragma unroll
        for (int s = 0; s < STAGES; ++s) load(s, 32 * s);
    }

    // acc[rt][j] += A[16rt + c, 0:K] * W[0:K, col + j]   (A bf16 in LDS, row stride lda)
    __device__ __forceinline__ void run(v4f (&acc)[4][8], const uint16_t *A_lds, int lda, int c,
                                        int g) {
        const uint16_t *ap = A_lds + (size_t)c * lda + 8 * g;
        auto mma_half = [&](const v8bf (&b)[4], int j0, int kk) {
#pragma unroll
            for (int rt = 0; rt < 4; ++rt) {
                const v8bf a = __builtin_bit_cast(
                    v8bf, *reinterpret_cast<const uint4 *>(ap + (size_t)(16 * rt) * lda + kk));
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[rt][j0 + j] =
                        __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b[j], acc[rt][j0 + j], 0, 0, 0);
            }
        };
        auto step = [&](int s, int kk, bool reload) {
            // first four columns: transpose, multiply
            v8bf b[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = bfrag_column(f[s], j);
            mma_half(b, 0, kk);
            // last four columns: transpose (the fragment's last reads), refill the fragment's
            // registers at once so the loads have ~STAGES k-steps of matrix work to arrive,
            // then multiply
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = bfrag_column(f[s], 4 + j);
            __builtin_amdgcn_sched_barrier(0);
            if (reload) load(s, kk + 32 * STAGES);
            __builtin_amdgcn_sched_barrier(0);
            mma_half(b, 4, kk);
            __builtin_amdgcn_sched_barrier(0);
        };
#pragma unroll
        for (int k0 = 0; k0 < K - 32 * STAGES; k0 += 32 * STAGES) {
#pragma unroll
            for (int s = 0; s < STAGES; ++s) step(s, k0 + 32 * s, true);
        }
#pragma unroll
        for (int s = 0; s < STAGES; ++s) step(s, K - 32 * STAGES + 32 * s, false);
    }
};


template <int D, int H>
__global__ __launch_bounds__(512) void ffn_bf16_kernel(FfnArgs p) {
    constexpr int TM = kFfnTM;
    constexpr int XS = D + 8;   // bf16 elements per LDS row of the x tile
    constexpr int HS = H + 8;   // ... of the hidden tile (aliases the x tile)
    constexpr int PS = D + 4;   // fp32 elements per LDS row of the split-k partial sums
    static_assert(H == 8 * 128, "eight waves own 128 hidden columns each");
    static_assert(D == 4 * 128, "four column groups of 128 outputs, two k halves");
    static_assert(TM * PS * 4 <= TM * HS * 2, "partial sums reuse the hidden tile's LDS");
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];

    TileCoord tc;
    if (!load_tile(p, TM, tc)) return;
    const int e = tc.e, row0 = tc.row0, rows = tc.rows;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g = lane >> 4;

    const uint16_t *W1 = (const uint16_t *)p.W1 + (size_t)e * D * H;
    const uint16_t *W2 = (const uint16_t *)p.W2 + (size_t)e * H * D;

    // gather the tile's token rows (rounded to bf16, nearest even).  Order of issue: row ids,
    // then the first weight fragments (they do not depend on x), then the token rows, so the
    // two dependent round trips of the gather overlap the weights' first trip.
    WeightStream<D, H, FFN_STAGES1> s1;
    const int col1 = 128 * wave + 8 * c;
    {
        constexpr int F4 = D / 4;                 // float4 per row
        constexpr int RPP = 512 / F4;             // rows per pass
        constexpr int PASSES = TM / RPP;
        const int c4 = tid % F4, rr = tid / F4;
        int tok[PASSES];
#pragma unroll
        for (int i = 0; i < PASSES; ++i) {
            const int r = min(rr + i * RPP, rows - 1);      // clamped: padding rows re-read a valid row
            tok[i] = p.perm[row0 + r];
        }
        s1.start(W1, (uint32_t)(D * H * 2), 0, col1, g);
        float4 v[PASSES];
#pragma unroll
        for (int i = 0; i < PASSES; ++i) {
            const int t = p.k_shift >= 0 ? (tok[i] >> p.k_shift) : (tok[i] / p.k);
            v[i] = *reinterpret_cast<const float4 *>(p.x + (size_t)t * D + 4 * c4);
        }
#pragma unroll
        for (int i = 0; i < PASSES; ++i) {
            const int r = rr + i * RPP;
            const bool live = r < rows;
            *reinterpret_cast<uint2 *>(lds + (size_t)r * XS + 4 * c4) =
                make_uint2(live ? pack_bf16x2(v[i].x, v[i].y) : 0u, live ? pack_bf16x2(v[i].z, v[i].w) : 0u);
        }
    }
    __syncthreads();
    if (p.xs_out) {   // training: keep the rounded input rows for the backward pass (the tile is only read from here on)
        constexpr int U4 = D / 8;
        for (int i = tid; i < TM * U4; i += 512) {
            const int r = i / U4, cc = i % U4;
            if (r < rows)
                MOE_STREAM_STORE(*reinterpret_cast<const v4u *>(lds + (size_t)r * XS + 8 * cc),   // kept for the backward pass: written once
                                 reinterpret_cast<v4u *>(p.xs_out + (size_t)(row0 + r) * D + 8 * cc));
        }
    }

    // hidden = relu(x W1): wave w owns hidden columns [128w, 128w+128)
    const int cg = wave & 3, kh = wave >> 2;
    WeightStream<H / 2, D, FFN_STAGES2> s2;
    const int col2 = 128 * cg + 8 * c;
    {
        v4f acc[4][8];
#pragma unroll
        for (int rt = 0; rt < 4; ++rt)
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[rt][j] = v4f{0.f, 0.f, 0.f, 0.f};
        s1.run(acc, lds, XS, c, g);
        // second matrix starts streaming during the hand-over below
        s2.start(W2, (uint32_t)(D * H * 2), (H / 2) * kh, col2, g);
        __syncthreads();  // every wave is done reading the x tile; the hidden tile overwrites it
#pragma unroll
        for (int rt = 0; rt < 4; ++rt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = 16 * rt + 4 * g + r;
                uint4 w;
                w.x = pack_bf16x2(fmaxf(acc[rt][0][r], 0.f), fmaxf(acc[rt][1][r], 0.f));
                w.y = pack_bf16x2(fmaxf(acc[rt][2][r], 0.f), fmaxf(acc[rt][3][r], 0.f));
                w.z = pack_bf16x2(fmaxf(acc[rt][4][r], 0.f), fmaxf(acc[rt][5][r], 0.f));
                w.w = pack_bf16x2(fmaxf(acc[rt][6][r], 0.f), fmaxf(acc[rt][7][r], 0.f));
                *reinterpret_cast<uint4 *>(lds + (size_t)row * HS + col1) = w;
            }
        __syncthreads();
    }
    if (p.hid_out) {   // training: keep the hidden activations for the backward pass
        constexpr int U4 = H / 8;   // 16-byte pieces per row
        for (int i = tid; i < TM * U4; i += 512) {
            const int r = i / U4, cc = i % U4;
            if (r < rows)
                MOE_STREAM_STORE(*reinterpret_cast<const v4u *>(lds + (size_t)r * HS + 8 * cc),   // kept for the backward pass: written once
                                 reinterpret_cast<v4u *>(p.hid_out + (size_t)(row0 + r) * H + 8 * cc));
        }
    }

    // out = hidden W2: wave (cg, kh) owns output columns [128cg, +128) and hidden units
    // [512kh, +512); the two k halves are added through LDS.
    {
        v4f acc[4][8];
#pragma unroll
        for (int rt = 0; rt < 4; ++rt)
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[rt][j] = v4f{0.f, 0.f, 0.f, 0.f};
        s2.run(acc, lds + (H / 2) * kh, HS, c, g);
        __syncthreads();  // the hidden tile is dead; its LDS now carries the partial sums
        float *part = reinterpret_cast<float *>(lds);
        if (kh == 1) {
#pragma unroll
            for (int rt = 0; rt < 4; ++rt)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float *dst = part + (size_t)(16 * rt + 4 * g + r) * PS + col2;
                    *reinterpret_cast<float4 *>(dst) =
                        make_float4(acc[rt][0][r], acc[rt][1][r], acc[rt][2][r], acc[rt][3][r]);
                    *reinterpret_cast<float4 *>(dst + 4) =
                        make_float4(acc[rt][4][r], acc[rt][5][r], acc[rt][6][r], acc[rt][7][r]);
                }
        }
        __syncthreads();
        if (kh == 0) {
#pragma unroll
            for (int rt = 0; rt < 4; ++rt)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = 16 * rt + 4 * g + r;
                    if (row >= rows) continue;
                    const float *src = part + (size_t)row * PS + col2;
                    const float4 p0 = *reinterpret_cast<const float4 *>(src);
                    const float4 p1 = *reinterpret_cast<const float4 *>(src + 4);
                    float *dst = p.out + (size_t)(row0 + row) * D + col2;
                    store_out4(dst, v4f{acc[rt][0][r] + p0.x, acc[rt][1][r] + p0.y, acc[rt][2][r] + p0.z,
                                        acc[rt][3][r] + p0.w});
                    store_out4(dst + 4, v4f{acc[rt][4][r] + p1.x, acc[rt][5][r] + p1.y, acc[rt][6][r] + p1.z,
                                            acc[rt][7][r] + p1.w});
                }
        }
    }
}

// ---------------------------------------------------------------------------------------
// Four-wave variant: one wave per SIMD with the whole 512-register budget.  Each wave owns 256
// hidden columns in the first GEMM (accumulators in AGPRs) and 128 output columns over the full
// hidden dimension in the second, so there is no split-k exchange, half as many waves meet at the
// barriers, and the registers left over hold three (first GEMM) and six (second GEMM) k-steps of
// weights in flight.
// ---------------------------------------------------------------------------------------
template <int K, int LD, int STAGES, int NG>   // NG groups of 128 columns per wave
struct WeightStream4 {
    static constexpr int NSTEPS = K / 32;
    BFrag f[STAGES][NG];
    __amdgpu_buffer_rsrc_t rsrc;   // the matrix as a buffer: scalar base, one 32-bit lane offset
    uint32_t lane_off;

    __device__ __forceinline__ void load(int s, int q, int k0) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const v4u v = __builtin_amdgcn_raw_buffer_load_b128(
                rsrc, lane_off, (uint32_t)(k0 + i) * LD * 2u + 256u * (uint32_t)q, FFN4_AUX);
            f[s][q].r[i][0] = v.x; f[s][q].r[i][1] = v.y; f[s][q].r[i][2] = v.z; f[s][q].r[i][3] = v.w;
        }
    }
    __device__ __forceinline__ void start(const uint16_t *W, uint32_t bytes, int col, int g) {
        rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(W), 0, bytes, 0x00020000);
        lane_off = (uint32_t)((8 * g) * LD + col) * 2u;
#pragma unroll
        for (int s = 0; s < STAGES; ++s)
#pragma unroll
            for (int q = 0; q < NG; ++q) load(s, q, 32 * s);
    }

    __device__ __forceinline__ void run(v4f (&acc)[NG][4][8], const uint16_t *A_lds, int lda, int c, int g) {
        const uint16_t *ap = A_lds + (size_t)c * lda + 8 * g;
#pragma unroll
        for (int step = 0; step < NSTEPS; ++step) {
            const int s = step % STAGES, kk = 32 * step;
            const bool reload = step + STAGES < NSTEPS;
            v8bf a[4];
#pragma unroll
            for (int rt = 0; rt < 4; ++rt)
                a[rt] = __builtin_bit_cast(v8bf, *reinterpret_cast<const uint4 *>(ap + (size_t)(16 * rt) * lda + kk));
#pragma unroll
            for (int q = 0; q < NG; ++q) {
                v8bf b[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) b[j] = bfrag_column(f[s][q], j);
                __builtin_amdgcn_sched_barrier(0);
                if (reload) load(s, q, kk + 32 * STAGES);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int j = 0; j < 8; ++j)
#pragma unroll
                    for (int rt = 0; rt < 4; ++rt)
                        acc[q][rt][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[rt], b[j], acc[q][rt][j], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
};

#ifndef FFN4_STAGES1
#define FFN4_STAGES1 2
#define FFN4_STAGES2 6
#endif

template <int D, int H>
__global__ __launch_bounds__(256) void ffn_bf16_w4_kernel(FfnArgs p) {
    constexpr int TM = kFfnTM;
    constexpr int XS = D + 8, HS = H + 8;
    static_assert(H == 4 * 256 && D == 4 * 128, "four waves: 256 hidden / 128 output columns each");
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];

    TileCoord tc;
    if (!load_tile(p, TM, tc)) return;
    const int e = tc.e, row0 = tc.row0, rows = tc.rows;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g = lane >> 4;
    const uint16_t *W1 = (const uint16_t *)p.W1 + (size_t)e * D * H;
    const uint16_t *W2 = (const uint16_t *)p.W2 + (size_t)e * H * D;

    WeightStream4<D, H, FFN4_STAGES1, 2> s1;
    const int col1 = 256 * wave + 8 * c;
    {
        constexpr int F4 = D / 4, RPP = 256 / F4, HALF = TM / RPP / 2;
        const int c4 = tid % F4, rr = tid / F4;
        int tok[2 * HALF];
#pragma unroll
        for (int i = 0; i < 2 * HALF; ++i) tok[i] = p.perm[row0 + min(rr + i * RPP, rows - 1)];
        s1.start(W1, (uint32_t)(D * H * 2), col1, g);
#pragma unroll
        for (int hb = 0; hb < 2; ++hb) {
            float4 v[HALF];
#pragma unroll
            for (int i = 0; i < HALF; ++i) {
                const int a = tok[hb * HALF + i];
                const int t = p.k_shift >= 0 ? (a >> p.k_shift) : (a / p.k);
                v[i] = *reinterpret_cast<const float4 *>(p.x + (size_t)t * D + 4 * c4);
            }
#pragma unroll
            for (int i = 0; i < HALF; ++i) {
                const int r = rr + (hb * HALF + i) * RPP;
                const bool live = r < rows;
                *reinterpret_cast<uint2 *>(lds + (size_t)r * XS + 4 * c4) =
                    make_uint2(live ? pack_bf16x2(v[i].x, v[i].y) : 0u, live ? pack_bf16x2(v[i].z, v[i].w) : 0u);
            }
        }
    }
    __syncthreads();
    if (p.xs_out) {   // training: keep the rounded input rows for the backward pass
        constexpr int U4 = D / 8;
        for (int i = tid; i < TM * U4; i += 256) {
            const int r = i / U4, cc = i % U4;
            if (r < rows)
                MOE_STREAM_STORE(*reinterpret_cast<const v4u *>(lds + (size_t)r * XS + 8 * cc),   // kept for the backward pass: written once
                                 reinterpret_cast<v4u *>(p.xs_out + (size_t)(row0 + r) * D + 8 * cc));
        }
    }

    WeightStream4<H, D, FFN4_STAGES2, 1> s2;
    const int col2 = 128 * wave + 8 * c;
    {
        v4f acc[2][4][8];
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int rt = 0; rt < 4; ++rt)
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[q][rt][j] = v4f{0.f, 0.f, 0.f, 0.f};
        s1.run(acc, lds, XS, c, g);
        s2.start(W2, (uint32_t)(D * H * 2), col2, g);
        __syncthreads();  // the hidden tile overwrites the x tile
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int rt = 0; rt < 4; ++rt)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = 16 * rt + 4 * g + r;
                    uint4 w;
                    w.x = pack_bf16x2(fmaxf(acc[q][rt][0][r], 0.f), fmaxf(acc[q][rt][1][r], 0.f));
                    w.y = pack_bf16x2(fmaxf(acc[q][rt][2][r], 0.f), fmaxf(acc[q][rt][3][r], 0.f));
                    w.z = pack_bf16x2(fmaxf(acc[q][rt][4][r], 0.f), fmaxf(acc[q][rt][5][r], 0.f));
                    w.w = pack_bf16x2(fmaxf(acc[q][rt][6][r], 0.f), fmaxf(acc[q][rt][7][r], 0.f));
                    *reinterpret_cast<uint4 *>(lds + (size_t)row * HS + col1 + 128 * q) = w;
                }
        __syncthreads();
    }
    if (p.hid_out) {
        constexpr int U4 = H / 8;
        for (int i = tid; i < TM * U4; i += 256) {
            const int r = i / U4, cc = i % U4;
            if (r < rows)
                MOE_STREAM_STORE(*reinterpret_cast<const v4u *>(lds + (size_t)r * HS + 8 * cc),   // kept for the backward pass: written once
                                 reinterpret_cast<v4u *>(p.hid_out + (size_t)(row0 + r) * H + 8 * cc));
        }
    }
    {
        v4f acc[1][4][8];
#pragma unroll
        for (int rt = 0; rt < 4; ++rt)
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[0][rt][j] = v4f{0.f, 0.f, 0.f, 0.f};
        s2.run(acc, lds, HS, c, g);
#pragma unroll
        for (int rt = 0; rt < 4; ++rt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = 16 * rt + 4 * g + r;
                if (row >= rows) continue;
                float *dst = p.out + (size_t)(row0 + row) * D + col2;
                store_out4(dst, v4f{acc[0][rt][0][r], acc[0][rt][1][r], acc[0][rt][2][r], acc[0][rt][3][r]});
                store_out4(dst + 4, v4f{acc[0][rt][4][r], acc[0][rt][5][r], acc[0][rt][6][r], acc[0][rt][7][r]});
            }
    }
}

// ---------------------------------------------------------------------------------------
// Backward through the two layers of an expert for routed rows, where experts hold about one tile
// of rows (the forward pass's four-wave regime): dz = (dout W2^T) * [hid > 0] (bf16, kept for the
// weight gradient) and dxs = dz W1^T in ONE launch that streams both matrices once per tile, the
// dz tile staying in LDS between the products -- the forward kernel run backwards.  Both products
// contract over the CONTIGUOUS index of the row-major weight matrices, so a lane's 16-byte load
// is a matrix-core operand as it stands (no register transpose): the weights are the A operand
// (16 weight rows x 32 k per instruction), the tile's rows the B operand, and a lane ends up with
// four consecutive output columns of one tile row.
// ---------------------------------------------------------------------------------------
// Cache policy of the backward kernel's weight loads (measured on 16384 experts of 16 rows:
// 6.3-6.8 ms from process to process with plain loads or with the first-level cache bypassed alike,
// 7.7 ms non-temporal: the half lines a wave instruction fetches must find their line again).
#ifndef FFNB_AUX
#define FFNB_AUX 1
#endif
template <int K, int LD, int STAGES, int NB>   // NB blocks of 16 weight rows per wave, row pitch LD
struct WeightRowsStream {
    // A wave instruction fetches 64 bytes of each of 16 weight rows (four lanes per row), half a
    // cache line: the stream therefore moves in steps of 64 k, the two halves of every line
    // requested back to back, so that the second is served by the first one's fill instead of
    // fetching the line again after a streaming load has let go of it.
    static constexpr int NSUPER = K / 64;
    v4u f[STAGES][NB][2];
    __amdgpu_buffer_rsrc_t rsrc;
    uint32_t lane_off;

    __device__ __forceinline__ void load(int s, int jj, int k0) {
#pragma unroll
        for (int u = 0; u < 2; ++u)
            f[s][jj][u] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, lane_off, (uint32_t)(16 * jj * LD + k0 + 32 * u) * 2u,
                                                                FFNB_AUX);
    }
    // W: the matrix (bytes long); this wave's rows start at wrow0; lane (m, g) reads row wrow0 + 16 jj + m
    __device__ __forceinline__ void start(const uint16_t *W, uint32_t bytes, int wrow0, int m, int g) {
        rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(W), 0, bytes, 0x00020000);
        lane_off = (uint32_t)((wrow0 + m) * LD + 8 * g) * 2u;
#pragma unroll
        for (int s = 0; s < STAGES; ++s)
#pragma unroll
            for (int jj = 0; jj < NB; ++jj) load(s, jj, 64 * s);
    }
    // acc[jj][rt] (+)= W[wrow0 + 16 jj + (0..15), 0:K] * A[16 rt + (0..15), 0:K]^T   (A bf16 in LDS, row stride lda)
    __device__ __forceinline__ void run(v4f (&acc)[NB][4], const uint16_t *A_lds, int lda, int c, int g) {
        const uint16_t *ap = A_lds + (size_t)c * lda + 8 * g;
#pragma unroll
        for (int ss = 0; ss < NSUPER; ++ss) {
            const int s = ss % STAGES, kk = 64 * ss;
            const bool reload = ss + STAGES < NSUPER;
            v8bf b[2][4];
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int rt = 0; rt < 4; ++rt)
                    b[u][rt] = __builtin_bit_cast(
                        v8bf, *reinterpret_cast<const uint4 *>(ap + (size_t)(16 * rt) * lda + kk + 32 * u));
#pragma unroll
            for (int j0 = 0; j0 < NB; j0 += 8) {
#pragma unroll
                for (int u = 0; u < 2; ++u)
#pragma unroll
                    for (int jj = j0; jj < j0 + 8; ++jj) {
                        const v8bf a = __builtin_bit_cast(v8bf, f[s][jj][u]);
#pragma unroll
                        for (int rt = 0; rt < 4; ++rt)
                            acc[jj][rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b[u][rt], acc[jj][rt], 0, 0, 0);
                    }
                __builtin_amdgcn_sched_barrier(0);
                // the sixteen fragments just multiplied are refilled at once: STAGES steps to arrive
                if (reload) {
#pragma unroll
                    for (int jj = j0; jj < j0 + 8; ++jj) load(s, jj, kk + 64 * STAGES);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
};

#ifndef FFNB_STAGES1
#define FFNB_STAGES1 1
#define FFNB_STAGES2 3
#endif

template <int D, int H>
__global__ __launch_bounds__(256) void ffn_bwd_rows_w4_kernel(FfnBwdRows p) {
    constexpr int TM = kFfnTM;
    constexpr int XS = D + 8, HS = H + 8;
    static_assert(H == 4 * 256 && D == 4 * 128, "four waves: 256 hidden / 128 input columns each");
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];

    TileCoord tc;
    if (!load_tile(p, TM, tc)) return;
    const int e = tc.e, row0 = tc.row0, rows = tc.rows;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g = lane >> 4;
    const uint16_t *W1 = (const uint16_t *)p.W1 + (size_t)e * D * H;   // [D][H]: row = input column
    const uint16_t *W2 = (const uint16_t *)p.W2 + (size_t)e * H * D;   // [H][D]: row = hidden unit

    // first product: dz_pre[row, j] = sum_c dout[row, c] W2[j, c]; this wave's hidden units 256 wave ..
    WeightRowsStream<D, D, FFNB_STAGES1, 16> s1;
    s1.start(W2, (uint32_t)(D * H * 2), 256 * wave, c, g);
    {
        // the tile's dout rows (bf16, adjacent in the sorted order) into LDS; rows past the end as zeros
        constexpr int CH = D / 8;                       // 16-byte pieces per row
        constexpr int PASSES = TM * CH / 256, HALF = PASSES / 2;
        static_assert(TM * CH % 512 == 0, "two equal halves of whole passes");
#pragma unroll
        for (int hb = 0; hb < 2; ++hb) {
            v4u v[HALF];
#pragma unroll
            for (int i = 0; i < HALF; ++i) {
                const int idx = tid + 256 * (hb * HALF + i), r = idx / CH, ch = idx % CH;
                v[i] = MOE_STREAM_LOAD(reinterpret_cast<const v4u *>(p.dout + (size_t)(row0 + min(r, rows - 1)) * D + 8 * ch));
            }
#pragma unroll
            for (int i = 0; i < HALF; ++i) {
                const int idx = tid + 256 * (hb * HALF + i), r = idx / CH, ch = idx % CH;
                *reinterpret_cast<v4u *>(lds + (size_t)r * XS + 8 * ch) = r < rows ? v[i] : v4u{0u, 0u, 0u, 0u};
            }
        }
    }
    __syncthreads();

    WeightRowsStream<H, H, FFNB_STAGES2, 8> s2;
    {
        v4f acc[16][4];
#pragma unroll
        for (int jj = 0; jj < 16; ++jj)
#pragma unroll
            for (int rt = 0; rt < 4; ++rt) acc[jj][rt] = v4f{0.f, 0.f, 0.f, 0.f};
        s1.run(acc, lds, XS, c, g);
        // second product: dxs[row, cc] = sum_j dz[row, j] W1[cc, j]; this wave's input columns 128 wave ..
        s2.start(W1, (uint32_t)(D * H * 2), 128 * wave, c, g);
        __syncthreads();  // the dz tile overwrites the dout tile
        // lane (row c of block rt, g) holds hidden units 256 wave + 16 jj + 4 g + (0..3) of its row
#pragma unroll
        for (int jj = 0; jj < 16; ++jj)
#pragma unroll
            for (int rt = 0; rt < 4; ++rt)
                *reinterpret_cast<uint2 *>(lds + (size_t)(16 * rt + c) * HS + 256 * wave + 16 * jj + 4 * g) =
                    make_uint2(pack_bf16x2(acc[jj][rt][0], acc[jj][rt][1]), pack_bf16x2(acc[jj][rt][2], acc[jj][rt][3]));
        __syncthreads();
    }
    {
        // ReLU'(z) = [hid > 0] (hid is the ReLU's output: positive or +0), applied to whole rows as
        // they leave for the weight-gradient kernel; the masked tile stays in LDS for the second product
        constexpr int CH = H / 8;
        for (int i = tid; i < rows * CH; i += 256) {
            const int r = i / CH, ch = i % CH;
            const v4u hv = MOE_STREAM_LOAD(reinterpret_cast<const v4u *>(p.hid + (size_t)(row0 + r) * H + 8 * ch));
            v4u zv = *reinterpret_cast<const v4u *>(lds + (size_t)r * HS + 8 * ch);
#pragma unroll
            for (int w = 0; w < 4; ++w)
                zv[w] &= ((hv[w] & 0x7fffu) ? 0xffffu : 0u) | ((hv[w] & 0x7fff0000u) ? 0xffff0000u : 0u);
            *reinterpret_cast<v4u *>(lds + (size_t)r * HS + 8 * ch) = zv;
            *reinterpret_cast<v4u *>(p.dz + (size_t)(row0 + r) * H + 8 * ch) = zv;
        }
        __syncthreads();
    }
    {
        v4f acc[8][4];
#pragma unroll
        for (int cc = 0; cc < 8; ++cc)
#pragma unroll
            for (int rt = 0; rt < 4; ++rt) acc[cc][rt] = v4f{0.f, 0.f, 0.f, 0.f};
        s2.run(acc, lds, HS, c, g);
#pragma unroll
        for (int rt = 0; rt < 4; ++rt) {
            const int row = 16 * rt + c;
            if (row >= rows) continue;
#pragma unroll
            for (int cc = 0; cc < 8; ++cc)
                store_out4(p.dxs + (size_t)(row0 + row) * D + 128 * wave + 16 * cc + 4 * g, acc[cc][rt]);
        }
    }
}

static_assert(kFfnBwdTileRows == kFfnTM, "the backward kernel uses the forward kernel's tile height");
bool ffn_bwd_rows_applies(const moe_config *cfg) {
    return cfg->expert_dtype == MOE_DTYPE_BF16 && cfg->d == 512 && cfg->h == 1024 &&
           (int64_t)cfg->T * cfg->k <= (int64_t)cfg->n * kFfnTM;
}

int launch_ffn_bwd_rows(const FfnBwdRows &a, int64_t max_tiles, hipStream_t st) {
    if (max_tiles <= 0) return MOE_OK;
    static LdsLimitOnce lds_once;
    constexpr size_t lds = (size_t)kFfnTM * (1024 + 8) * sizeof(uint16_t);
    MOE_TRY(lds_once.set((const void *)ffn_bwd_rows_w4_kernel<512, 1024>, lds));
    const unsigned grid = (unsigned)(ceil_div(max_tiles, 8) * 8);
    hipLaunchKernelGGL((ffn_bwd_rows_w4_kernel<512, 1024>), dim3(grid), dim3(256), lds, st, a);
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}

// ---------------------------------------------------------------------------------------
// fp32 experts: C[rows, N] = act(A[rows, K] W_e[K, N]) per row tile; A rows either gathered
// from x through perm or read from the sorted hidden buffer.
// ---------------------------------------------------------------------------------------
// On the fp32 matrix cores: 64 x 64 tile, four waves of one 32 x 32 block each
// (v_mfma_f32_32x32x2f32: a lane supplies A(row = lane % 32, k) and B(k, col = lane % 32) for
// k = lane / 32 of the instruction's two k values).  k-slabs of 32 double-buffered in LDS, the next
// slab prefetched into registers under the current one's 16 matrix instructions.  Which two k values
// an instruction takes is free as long as both operands agree: step (j, u) uses k = 8j + u from
// lanes 0-31 and 8j + 4 + u from lanes 32-63, so a lane's A values for four steps are one 16-byte
// LDS read.  Every output keeps one accumulator over the whole of K (a sequential fp32 fma chain).
typedef float v16f32 __attribute__((ext_vector_type(16)));
template <bool GATHER, bool RELU>
__global__ __launch_bounds__(256) void ffn_f32_mfma_kernel(FfnArgs p, const float *A, const float *Wall,
                                                           float *C, int K, int N) {
    constexpr int TM = kFfnTM, TN = 64, TK = 32, AS = TK + 4, BS = TN + 8;
    static_assert(TM == 64, "four waves cover 64 x 64");
    __shared__ __attribute__((aligned(16))) float As[2][TM][AS];   // [row][k]; 36-float rows: conflict-free 16-byte reads
    __shared__ __attribute__((aligned(16))) float Bs[2][TK][BS];   // [k][col]; 72-float rows: k and k+4 hit different bank halves
    const int num_tiles = *p.num_tiles;
    const int tile = blockIdx.x;
    if (tile >= num_tiles) return;
    const int e = p.tile_expert[tile];
    const int row0 = p.tile_row0[tile];
    const int rows = min(TM, p.offsets[e + 1] - row0);
    if (rows <= 0) return;
    const int col0 = blockIdx.y * TN;
    const float *W = Wall + (size_t)e * K * N;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31, wm = wave >> 1, wn = wave & 1;

    // loaders: A 64 rows x 32 k and B 32 k x 64 cols, two float4 per thread each
    const int ar = tid >> 3, akq = (tid & 7) * 4;
    const int bk = tid >> 4, bc = (tid & 15) * 4;
    const float *a_src[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int r = min(ar + 32 * i, rows - 1);   // rows past the end re-read a valid row; their results are not stored
        const int64_t src_row = GATHER ? (int64_t)(p.perm[row0 + r] / p.k) : (int64_t)(row0 + r);
        a_src[i] = A + src_row * K;
    }
    const bool b_in = col0 + bc < N;
    // Two register sets: the slab stored to LDS in step s was requested two steps earlier, so a
    // global round trip has two slabs of matrix work to hide behind (these launches are small and
    // latency-sized: with one set the loop ran at the memory latency per slab).
    float4 areg[2][2], breg[2][2];
    auto load_slab = [&](int s, float4 (&ar_)[2], float4 (&br_)[2]) {
        const int k0 = s * TK;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int ka = k0 + akq, kb = k0 + bk + 16 * i;
            const float4 av = *reinterpret_cast<const float4 *>(a_src[i] + min(ka, K - 4));
            ar_[i] = ka < K ? av : make_float4(0.f, 0.f, 0.f, 0.f);
            const float4 bv = *reinterpret_cast<const float4 *>(W + (size_t)min(kb, K - 1) * N + (b_in ? col0 + bc : 0));
            br_[i] = (kb < K && b_in) ? bv : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    };
    auto store_slab = [&](int buf, const float4 (&ar_)[2], const float4 (&br_)[2]) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            *reinterpret_cast<float4 *>(&As[buf][ar + 32 * i][akq]) = ar_[i];
            *reinterpret_cast<float4 *>(&Bs[buf][bk + 16 * i][bc]) = br_[i];
        }
    };
    v16f32 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    const int nslab = (K + TK - 1) / TK;
    load_slab(0, areg[0], breg[0]);
    store_slab(0, areg[0], breg[0]);
    load_slab(min(1, nslab - 1), areg[0], breg[0]);      // clamped: a short K re-reads a valid slab nobody uses
    load_slab(min(2, nslab - 1), areg[1], breg[1]);
    __syncthreads();
    // step s: multiply slab s from LDS, store slab s+1 (held in `ra`, `rb`), request slab s+3 into them
    auto step = [&](int s, float4 (&ra)[2], float4 (&rb)[2]) {
        const int buf = s & 1;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float4 a4 = *reinterpret_cast<const float4 *>(&As[buf][32 * wm + l32][8 * j + 4 * half]);
            const float av[4] = {a4.x, a4.y, a4.z, a4.w};
#pragma unroll
            for (int u = 0; u < 4; ++u)
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av[u], Bs[buf][8 * j + 4 * half + u][32 * wn + l32], acc, 0, 0, 0);
        }
        if (s + 1 < nslab) store_slab(buf ^ 1, ra, rb);
        if (s + 3 < nslab) load_slab(s + 3, ra, rb);
        __syncthreads();
    };
    for (int s = 0; s < nslab; s += 2) {
        step(s, areg[0], breg[0]);
        if (s + 1 < nslab) step(s + 1, areg[1], breg[1]);
    }
    const int c = col0 + 32 * wn + l32;
    if (c < N) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = 32 * wm + 8 * (r / 4) + 4 * half + (r % 4);
            if (row < rows) C[(size_t)(row0 + row) * N + c] = RELU ? fmaxf(acc[r], 0.f) : acc[r];
        }
    }
}

// routed rows of x, rounded to bf16: xs[r] = bf16(x[perm[r] / k]); one wavefront per row.
// rows_used[0]: rows the dispatch really holds (offsets[n]); perm is defined only below it.
__global__ __launch_bounds__(256) void gather_bf16_kernel(const float *__restrict__ x,
                                                          const int32_t *__restrict__ perm, int64_t A,
                                                          const int32_t *__restrict__ rows_used, int d, int k,
                                                          uint16_t *__restrict__ xs) {
    const int lane = threadIdx.x & 63;
    const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= A || r >= rows_used[0]) return;
    const int64_t t = perm[r] / k;
    for (int c = lane * 4; c < d; c += 256) {
        const float4 v = *reinterpret_cast<const float4 *>(x + t * d + c);
        *reinterpret_cast<uint2 *>(xs + r * d + c) = make_uint2(pack_bf16x2(v.x, v.y), pack_bf16x2(v.z, v.w));
    }
}

int ffn_tile_rows(const moe_config *cfg);
static size_t ffn_up256(size_t v) { return (v + 255) & ~(size_t)255; }

// bf16 experts of any shape with d and h multiples of 128: gather, then two grouped GEMMs with
// the hidden layer (bf16) in the workspace -- the plain path beside the fused kernel, which is
// built for the paper's 512 x 1024 experts.
static int launch_expert_ffn_general(const moe_config *cfg, const FfnArgs &a, int64_t max_tiles,
                                     hipStream_t st) {
    if (cfg->d % 128 || cfg->h % 128) return MOE_EUNSUPPORTED;
    const int64_t A = (int64_t)cfg->T * cfg->k;
    uint16_t *xs = a.xs_out ? a.xs_out : reinterpret_cast<uint16_t *>(a.hidden);
    uint16_t *hid = a.hid_out ? a.hid_out
                              : reinterpret_cast<uint16_t *>(reinterpret_cast<char *>(a.hidden) +
                                                             ffn_up256((size_t)A * cfg->d * 2));
    hipLaunchKernelGGL(gather_bf16_kernel, dim3((unsigned)ceil_div(A, 4)), dim3(256), 0, st, a.x, a.perm, A,
                       a.offsets + cfg->n, cfg->d, cfg->k, xs);
    MOE_LAUNCH_CHECK();
    GGRows g1{xs, (const uint16_t *)a.W1, hid, nullptr, cfg->d, cfg->h, a.offsets, a.tile_expert,
              a.tile_row0, a.num_tiles, ffn_tile_rows(cfg)};
    int rc = launch_gg_rows128(g1, true, EPI_RELU_BF16, max_tiles, st);
    if (rc != MOE_OK) return rc;
    GGRows g2{hid, (const uint16_t *)a.W2, a.out, nullptr, cfg->h, cfg->d, a.offsets, a.tile_expert,
              a.tile_row0, a.num_tiles, ffn_tile_rows(cfg)};
    return launch_gg_rows128(g2, true, EPI_F32, max_tiles, st);
}

// Rows per tile of the dispatch table (one height for every shape today; the callers ask per config).
int ffn_tile_rows(const moe_config *) { return kFfnTM; }

int launch_expert_ffn(const moe_config *cfg, const FfnArgs &a, int64_t max_tiles, hipStream_t st) {
    if (max_tiles <= 0) return MOE_OK;
    if (cfg->expert_dtype == MOE_DTYPE_BF16) {
        if (cfg->d != 512 || cfg->h != 1024) return launch_expert_ffn_general(cfg, a, max_tiles, st);
        static LdsLimitOnce lds8, lds4;
        const unsigned grid = (unsigned)(ceil_div(max_tiles, 8) * 8);
        constexpr size_t lds = (size_t)kFfnTM * (1024 + 8) * sizeof(uint16_t);
        // One tile per expert (<= 64 rows on average): every tile streams its weights from HBM, and
        // the four-wave kernel's deeper load pipeline pays.  Several tiles per expert: the tiles
        // share weights through L2 and the eight-wave kernel is marginally faster.
        const bool four_waves = (int64_t)cfg->T * cfg->k <= (int64_t)cfg->n * kFfnTM;
        if (four_waves) MOE_TRY(lds4.set((const void *)ffn_bf16_w4_kernel<512, 1024>, lds));
        else MOE_TRY(lds8.set((const void *)ffn_bf16_kernel<512, 1024>, lds));
        if (four_waves) hipLaunchKernelGGL((ffn_bf16_w4_kernel<512, 1024>), dim3(grid), dim3(256), lds, st, a);
        else hipLaunchKernelGGL((ffn_bf16_kernel<512, 1024>), dim3(grid), dim3(512), lds, st, a);
        MOE_LAUNCH_CHECK();
        return MOE_OK;
    }
    if (cfg->d % 4 || cfg->h % 4) return MOE_EUNSUPPORTED;
    dim3 g1((unsigned)max_tiles, (unsigned)ceil_div(cfg->h, 64));
    hipLaunchKernelGGL((ffn_f32_mfma_kernel<true, true>), g1, dim3(256), 0, st, a, a.x,
                       (const float *)a.W1, a.hidden, cfg->d, cfg->h);
    MOE_LAUNCH_CHECK();
    dim3 g2((unsigned)max_tiles, (unsigned)ceil_div(cfg->d, 64));
    hipLaunchKernelGGL((ffn_f32_mfma_kernel<false, false>), g2, dim3(256), 0, st, a, a.hidden,
                       (const float *)a.W2, a.out, cfg->h, cfg->d);
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}

}  // namespace moe

using namespace moe;

extern "C" int32_t moe_tile_rows(const moe_config *cfg) { return ffn_tile_rows(cfg); }

extern "C" int64_t moe_max_tiles(const moe_config *cfg) {
    if (check_config(cfg) != MOE_OK) return 0;
    const int64_t A = (int64_t)cfg->T * cfg->k;
    return ceil_div(A, ffn_tile_rows(cfg)) + (cfg->n < A ? cfg->n : A);
}

extern "C" size_t moe_ffn_workspace_bytes(const moe_config *cfg) {
    if (check_config(cfg) != MOE_OK) return 0;
    const size_t A = (size_t)cfg->T * cfg->k;
    if (cfg->expert_dtype == MOE_DTYPE_BF16) {
        if (cfg->d == 512 && cfg->h == 1024) return 0;                       // fused kernel
        return ffn_up256(A * cfg->d * 2) + ffn_up256(A * cfg->h * 2);        // bf16 rows of x, hidden layer
    }
    return A * cfg->h * sizeof(float);
}

namespace moe {
int expert_ffn_with_hidden(const moe_config *cfg, const float *x, const int32_t *perm,
                           const int32_t *offsets, const int32_t *tile_expert,
                           const int32_t *tile_row0, const int32_t *num_tiles, const void *W1,
                           const void *W2, float *out_sorted, void *workspace, uint16_t *hid_out,
                           hipStream_t st, uint16_t *xs_out) {
    int rc = check_config(cfg);
    if (rc != MOE_OK) return rc;
    if (!x || !perm || !offsets || !tile_expert || !tile_row0 || !num_tiles || !W1 || !W2 ||
        !out_sorted)
        return MOE_EINVAL;
    if (!aligned16(x) || !aligned16(W1) || !aligned16(W2) || !aligned16(out_sorted))
        return MOE_EINVAL;
    if (moe_ffn_workspace_bytes(cfg) > 0 && (!workspace || !aligned16(workspace))) return MOE_EINVAL;
    FfnArgs a{};
    a.x = x; a.perm = perm; a.offsets = offsets;
    a.tile_expert = tile_expert; a.tile_row0 = tile_row0; a.num_tiles = num_tiles;
    a.W1 = W1; a.W2 = W2; a.out = out_sorted; a.hidden = (float *)workspace;
    a.hid_out = hid_out;
    a.xs_out = cfg->expert_dtype == MOE_DTYPE_BF16 ? xs_out : nullptr;
    a.d = cfg->d; a.h = cfg->h; a.k = cfg->k;
    a.k_shift = (cfg->k & (cfg->k - 1)) == 0 ? __builtin_ctz(cfg->k) : -1;
    return launch_expert_ffn(cfg, a, moe_max_tiles(cfg), st);
}
}  // namespace moe

extern "C" int moe_expert_ffn(const moe_config *cfg, const float *x, const int32_t *perm,
                              const int32_t *offsets, const int32_t *tile_expert,
                              const int32_t *tile_row0, const int32_t *num_tiles, const void *W1,
                              const void *W2, float *out_sorted, void *workspace, void *stream) {
    return expert_ffn_with_hidden(cfg, x, perm, offsets, tile_expert, tile_row0, num_tiles, W1, W2,
                                  out_sorted, workspace, nullptr, (hipStream_t)stream);
}
