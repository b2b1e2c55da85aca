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
// fp32 path (ffn_f32_kernel): plain LDS-tiled grouped GEMM, hidden layer kept in a workspace.
#include "stages.h"

namespace moe {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

constexpr int kFfnTM = 64;  // rows per tile

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);  // inputs are finite
    return u >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    return f32_to_bf16_rne(lo) | (f32_to_bf16_rne(hi) << 16);
}


// XCD-aware tile order: consecutive workgroup ids go to different XCDs (one L2 each), so
// workgroup b takes tile (b % 8) * ceil(num/8) + b / 8: tiles of one expert, which are adjacent
// in the table, then share an L2.
__device__ __forceinline__ int xcd_tile(int bid, int num_tiles) {
    const int per = (num_tiles + 7) >> 3;
    const int tile = (bid & 7) * per + (bid >> 3);
    return ((bid >> 3) < per && tile < num_tiles) ? tile : -1;
}

// One 16-deep k-step of B-operand data for BW adjacent columns: rows k0+8g .. k0+8g+7.
template <int BW>
struct BFrag {
    uint32_t r[8][BW / 2];
};

template <int BW>
__device__ __forceinline__ void load_bfrag(BFrag<BW> &f, const uint16_t *W, int ld, int k0, int g,
                                           int col) {
    const uint16_t *src = W + (size_t)(k0 + 8 * g) * ld + col;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        if constexpr (BW == 2) {
            f.r[i][0] = *reinterpret_cast<const uint32_t *>(src + (size_t)i * ld);
        } else if constexpr (BW == 4) {
            const uint2 v = *reinterpret_cast<const uint2 *>(src + (size_t)i * ld);
            f.r[i][0] = v.x;
            f.r[i][1] = v.y;
        } else {
            const uint4 v = *reinterpret_cast<const uint4 *>(src + (size_t)i * ld);
            f.r[i][0] = v.x; f.r[i][1] = v.y; f.r[i][2] = v.z; f.r[i][3] = v.w;
        }
    }
}

// Column j of the block as an MFMA B operand: 8 consecutive k in one lane.
template <int BW>
__device__ __forceinline__ v8bf bfrag_column(const BFrag<BW> &f, int j) {
    const uint32_t sel = (j & 1) ? 0x07060302u : 0x05040100u;
    uint4 o;
    o.x = __builtin_amdgcn_perm(f.r[1][j >> 1], f.r[0][j >> 1], sel);
    o.y = __builtin_amdgcn_perm(f.r[3][j >> 1], f.r[2][j >> 1], sel);
    o.z = __builtin_amdgcn_perm(f.r[5][j >> 1], f.r[4][j >> 1], sel);
    o.w = __builtin_amdgcn_perm(f.r[7][j >> 1], f.r[6][j >> 1], sel);
    return __builtin_bit_cast(v8bf, o);
}

// acc[rt][j] += A[rows 32rt.., K] * W[K, col0 + BW*q + j]   (A bf16 in LDS, row stride lda)
template <int BW, int K>
__device__ __forceinline__ void wave_gemm(v16f (&acc)[2][BW], const uint16_t *A_lds, int lda,
                                          const uint16_t *W, int ldw, int col, int q, int g) {
    BFrag<BW> f0, f1;
    load_bfrag<BW>(f0, W, ldw, 0, g, col);
    load_bfrag<BW>(f1, W, ldw, 16, g, col);
    const uint16_t *a0p = A_lds + (size_t)q * lda + 8 * g;
    const uint16_t *a1p = a0p + (size_t)32 * lda;
    auto step = [&](BFrag<BW> &f, int k0) {
        const v8bf a0 = __builtin_bit_cast(v8bf, *reinterpret_cast<const uint4 *>(a0p + k0));
        const v8bf a1 = __builtin_bit_cast(v8bf, *reinterpret_cast<const uint4 *>(a1p + k0));
        v8bf b[BW];
#pragma unroll
        for (int j = 0; j < BW; ++j) b[j] = bfrag_column<BW>(f, j);
        if (k0 + 32 < K) load_bfrag<BW>(f, W, ldw, k0 + 32, g, col);
#pragma unroll
        for (int j = 0; j < BW; ++j) {
            acc[0][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b[j], acc[0][j], 0, 0, 0);
            acc[1][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b[j], acc[1][j], 0, 0, 0);
        }
    };
#pragma unroll 1
    for (int k0 = 0; k0 < K; k0 += 32) {
        step(f0, k0);
        step(f1, k0 + 16);
    }
}

template <int D, int H>
__global__ __launch_bounds__(512) void ffn_bf16_kernel(FfnArgs p) {
    constexpr int TM = kFfnTM;
    constexpr int XS = D + 8;   // bf16 elements per LDS row of the x tile
    constexpr int HS = H + 8;   // ... of the hidden tile (aliases the x tile)
    constexpr int BW1 = H / 256;  // 8 waves x 32 lanes x BW1 columns = H
    constexpr int BW2 = D / 256;
    static_assert(BW1 == 2 || BW1 == 4 || BW1 == 8, "hidden size");
    static_assert(BW2 == 2 || BW2 == 4 || BW2 == 8, "model width");
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];

    const int tile = xcd_tile(blockIdx.x, *p.num_tiles);
    if (tile < 0) return;
    const int e = p.tile_expert[tile];
    const int row0 = p.tile_row0[tile];
    const int rows = min(TM, p.offsets[e + 1] - row0);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int q = lane & 31, g = lane >> 5;

    // gather the tile's token rows, round to bf16 (nearest even)
    {
        constexpr int F4 = D / 4;                 // float4 per row
        constexpr int RPP = 512 / F4;             // rows per pass
        const int c4 = tid % F4, rr = tid / F4;
#pragma unroll 4
        for (int r = rr; r < TM; r += RPP) {
            uint2 packed = make_uint2(0u, 0u);
            if (r < rows) {
                const int tok = p.perm[row0 + r] / p.k;
                const float4 v = *reinterpret_cast<const float4 *>(p.x + (size_t)tok * D + 4 * c4);
                packed.x = pack_bf16x2(v.x, v.y);
                packed.y = pack_bf16x2(v.z, v.w);
            }
            *reinterpret_cast<uint2 *>(lds + (size_t)r * XS + 4 * c4) = packed;
        }
    }
    __syncthreads();

    const uint16_t *W1 = (const uint16_t *)p.W1 + (size_t)e * D * H;
    const uint16_t *W2 = (const uint16_t *)p.W2 + (size_t)e * H * D;

    // hidden = relu(x W1): wave owns hidden columns [32*BW1*wave, +32*BW1)
    {
        v16f acc[2][BW1];
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
#pragma unroll
            for (int j = 0; j < BW1; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[rt][j][r] = 0.f;
        const int col = 32 * BW1 * wave + BW1 * q;
        wave_gemm<BW1, D>(acc, lds, XS, W1, H, col, q, g);
        __syncthreads();  // every wave is done reading the x tile; the hidden tile overwrites it
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = 32 * rt + 8 * (r / 4) + 4 * g + (r % 4);
                uint32_t w[BW1 / 2];
#pragma unroll
                for (int j = 0; j < BW1; j += 2)
                    w[j / 2] = pack_bf16x2(fmaxf(acc[rt][j][r], 0.f), fmaxf(acc[rt][j + 1][r], 0.f));
                uint16_t *dst = lds + (size_t)row * HS + col;
                if constexpr (BW1 == 2) *reinterpret_cast<uint32_t *>(dst) = w[0];
                else if constexpr (BW1 == 4) *reinterpret_cast<uint2 *>(dst) = make_uint2(w[0], w[1]);
                else *reinterpret_cast<uint4 *>(dst) = make_uint4(w[0], w[1], w[2], w[3]);
            }
        __syncthreads();
    }

    // out = hidden W2: wave owns output columns [32*BW2*wave, +32*BW2)
    {
        v16f acc[2][BW2];
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
#pragma unroll
            for (int j = 0; j < BW2; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[rt][j][r] = 0.f;
        const int col = 32 * BW2 * wave + BW2 * q;
        wave_gemm<BW2, H>(acc, lds, HS, W2, D, col, q, g);
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = 32 * rt + 8 * (r / 4) + 4 * g + (r % 4);
                if (row >= rows) continue;
                float *dst = p.out + (size_t)(row0 + row) * D + col;
                if constexpr (BW2 == 2) {
                    *reinterpret_cast<float2 *>(dst) = make_float2(acc[rt][0][r], acc[rt][1][r]);
                } else {
#pragma unroll
                    for (int j = 0; j < BW2; j += 4)
                        *reinterpret_cast<float4 *>(dst + j) = make_float4(
                            acc[rt][j][r], acc[rt][j + 1][r], acc[rt][j + 2][r], acc[rt][j + 3][r]);
                }
            }
    }
}

// ---------------------------------------------------------------------------------------
// fp32 experts: C[rows, N] = act(A[rows, K] W_e[K, N]) per row tile; A rows either gathered
// from x through perm or read from the sorted hidden buffer.
// ---------------------------------------------------------------------------------------
template <bool GATHER, bool RELU>
__global__ __launch_bounds__(256) void ffn_f32_kernel(FfnArgs p, const float *A, const float *Wall,
                                                      float *C, int K, int N) {
    constexpr int TM = kFfnTM, TN = 64, TK = 16;
    __shared__ float As[TK][TM + 4];
    __shared__ float Bs[TK][TN + 4];
    const int num_tiles = *p.num_tiles;
    const int tile = blockIdx.x;
    if (tile >= num_tiles) return;
    const int e = p.tile_expert[tile];
    const int row0 = p.tile_row0[tile];
    const int rows = min(TM, p.offsets[e + 1] - row0);
    const int col0 = blockIdx.y * TN;
    const float *W = Wall + (size_t)e * K * N;
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;

    // A loader: 64 rows x 16 k, one float4 along k per thread
    const int ar = tid >> 2, ak = (tid & 3) * 4;
    const float *a_src = nullptr;
    if (ar < rows) {
        const int64_t src_row = GATHER ? (int64_t)(p.perm[row0 + ar] / p.k) : (int64_t)(row0 + ar);
        a_src = A + src_row * K + ak;
    }
    // B loader: 16 k x 64 cols, one float4 along cols per thread
    const int bk = tid >> 4, bc = (tid & 15) * 4;

    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += TK) {
        float4 av = make_float4(0.f, 0.f, 0.f, 0.f);
        if (a_src && k0 + ak < K) av = *reinterpret_cast<const float4 *>(a_src + k0);
        As[ak + 0][ar] = av.x; As[ak + 1][ar] = av.y; As[ak + 2][ar] = av.z; As[ak + 3][ar] = av.w;
        float4 bv = make_float4(0.f, 0.f, 0.f, 0.f);
        if (k0 + bk < K && col0 + bc < N)
            bv = *reinterpret_cast<const float4 *>(W + (size_t)(k0 + bk) * N + col0 + bc);
        *reinterpret_cast<float4 *>(&Bs[bk][bc]) = bv;
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < TK; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = ty * 4 + i;
        if (r >= rows) continue;
        const int c = col0 + tx * 4;
        if (c >= N) continue;
        float4 o = make_float4(acc[i][0], acc[i][1], acc[i][2], acc[i][3]);
        if (RELU) {
            o.x = fmaxf(o.x, 0.f); o.y = fmaxf(o.y, 0.f); o.z = fmaxf(o.z, 0.f); o.w = fmaxf(o.w, 0.f);
        }
        *reinterpret_cast<float4 *>(C + (size_t)(row0 + r) * N + c) = o;
    }
}

int launch_expert_ffn(const moe_config *cfg, const FfnArgs &a, int64_t max_tiles, hipStream_t st) {
    if (max_tiles <= 0) return MOE_OK;
    if (cfg->expert_dtype == MOE_DTYPE_BF16) {
        if (cfg->d != 512 || cfg->h != 1024) return MOE_EUNSUPPORTED;
        constexpr size_t lds = (size_t)kFfnTM * (1024 + 8) * sizeof(uint16_t);
        static bool attr_set = false;
        if (!attr_set) {
            MOE_HIP_TRY(hipFuncSetAttribute((const void *)ffn_bf16_kernel<512, 1024>,
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
            attr_set = true;
        }
        const unsigned grid = (unsigned)(ceil_div(max_tiles, 8) * 8);
        hipLaunchKernelGGL((ffn_bf16_kernel<512, 1024>), dim3(grid), dim3(512), lds, st, a);
        MOE_LAUNCH_CHECK();
        return MOE_OK;
    }
    if (cfg->d % 4 || cfg->h % 4) return MOE_EUNSUPPORTED;
    dim3 g1((unsigned)max_tiles, (unsigned)ceil_div(cfg->h, 64));
    hipLaunchKernelGGL((ffn_f32_kernel<true, true>), g1, dim3(256), 0, st, a, a.x,
                       (const float *)a.W1, a.hidden, cfg->d, cfg->h);
    MOE_LAUNCH_CHECK();
    dim3 g2((unsigned)max_tiles, (unsigned)ceil_div(cfg->d, 64));
    hipLaunchKernelGGL((ffn_f32_kernel<false, false>), g2, dim3(256), 0, st, a, a.hidden,
                       (const float *)a.W2, a.out, cfg->h, cfg->d);
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}

}  // namespace moe

using namespace moe;

extern "C" int32_t moe_tile_rows(const moe_config *) { return kFfnTM; }

extern "C" int64_t moe_max_tiles(const moe_config *cfg) {
    if (check_config(cfg) != MOE_OK) return 0;
    const int64_t A = (int64_t)cfg->T * cfg->k;
    return ceil_div(A, kFfnTM) + (cfg->n < A ? cfg->n : A);
}

extern "C" size_t moe_ffn_workspace_bytes(const moe_config *cfg) {
    if (check_config(cfg) != MOE_OK) return 0;
    if (cfg->expert_dtype == MOE_DTYPE_BF16) return 0;
    return (size_t)cfg->T * cfg->k * cfg->h * sizeof(float);
}

extern "C" int moe_expert_ffn(const moe_config *cfg, const float *x, const int32_t *perm,
                              const int32_t *offsets, const int32_t *tile_expert,
                              const int32_t *tile_row0, const int32_t *num_tiles, const void *W1,
                              const void *W2, float *out_sorted, void *workspace, void *stream) {
    int st = check_config(cfg);
    if (st != MOE_OK) return st;
    if (!x || !perm || !offsets || !tile_expert || !tile_row0 || !num_tiles || !W1 || !W2 ||
        !out_sorted)
        return MOE_EINVAL;
    if (!aligned16(x) || !aligned16(W1) || !aligned16(W2) || !aligned16(out_sorted))
        return MOE_EINVAL;
    if (cfg->expert_dtype == MOE_DTYPE_F32 && (!workspace || !aligned16(workspace)))
        return MOE_EINVAL;
    FfnArgs a{};
    a.x = x; a.perm = perm; a.offsets = offsets;
    a.tile_expert = tile_expert; a.tile_row0 = tile_row0; a.num_tiles = num_tiles;
    a.W1 = W1; a.W2 = W2; a.out = out_sorted; a.hidden = (float *)workspace;
    a.d = cfg->d; a.h = cfg->h; a.k = cfg->k;
    return launch_expert_ffn(cfg, a, moe_max_tiles(cfg), (hipStream_t)stream);
}
