// Compute-bound grouped GEMM of the expert backward pass (Section 2.1: plain back-propagation
// through the experts): C[rows of expert e, N] = A[rows, K] * B_e^T with B_e stored [N, K]
// (k contiguous), i.e. dz = (dout W2^T) * relu'  and  dxs = dz W1^T.
//
// One workgroup = a 256 x 256 tile of C: 256 rows of ONE expert (a row tile of a 256-row tile
// table) by 256 columns.  Four waves, one per SIMD, each a 128 x 128 quarter held as 4 x 4
// v_mfma_f32_32x32x16_bf16 accumulators (256 AGPRs): with this wave tile the LDS read traffic is
// half a KB per matrix instruction, which the LDS can sustain beside the slab stores.  Operand
// slabs of 32 k go global -> registers -> LDS (k contiguous for both operands, rows padded to 80
// bytes so 16-byte reads are conflict free); the three-level software pipeline is the one of the
// gate's logits kernel: slab s+1 is stored and slab s+2 fetched in the middle of slab s, operand
// registers are read one k-step ahead, and the barrier sits before the slab's last k-step.
// Work items are ordered column-tile-fastest and handed out XCD by XCD, so the column tiles of
// one row tile (same A rows) and the row tiles of one expert (same weights) share an L2.
#include "stages.h"

namespace moe {

typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));

constexpr int RT = 256;            // tile rows and columns
#ifndef GG_RKC
#define GG_RKC 64
#endif
constexpr int RKC = GG_RKC;        // slab depth
constexpr int RLD = RKC + 8;       // bf16 elements per LDS row (+16 bytes: 16-byte reads of 8 rows hit 32 banks)



// NW wavefronts: four own 128 x 128 each (256 accumulators, one wave per SIMD), eight own 128 x 64
// (two waves per SIMD: one's LDS reads and stores run under the other's matrix work).
template <int EPI, int NW>
__global__ __launch_bounds__(64 * NW, 1) void gg_rows256_kernel(GGRows p, int col_tiles) {
    constexpr int NT = 64 * NW;          // threads
    constexpr int NJ = NW == 8 ? 2 : 4;  // 32-column fragments per wave
    constexpr int WCOLS = 32 * NJ;       // columns per wave
    constexpr int SLAB = RT * RLD * 2;                       // bytes of one operand slab
    __shared__ __attribute__((aligned(16))) char smem[4 * SLAB];
    uint16_t (*As)[RT][RLD] = reinterpret_cast<uint16_t (*)[RT][RLD]>(smem);
    uint16_t (*Bs)[RT][RLD] = reinterpret_cast<uint16_t (*)[RT][RLD]>(smem + 2 * SLAB);

    // work item = row tile * col_tiles + column tile, handed out XCD by XCD
    const int num_items = *p.num_tiles * col_tiles;
    const int per = (num_items + 7) >> 3;
    const int item = (blockIdx.x & 7) * per + (blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= per || item >= num_items) return;
    const int tile = item / col_tiles;
    const int col0 = (item % col_tiles) * RT;
    const int e = p.tile_expert[tile];
    const int row0 = p.tile_row0[tile];
    const int rows = min(RT, p.offsets[e + 1] - row0);
    const int K = p.K, N = p.N;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = NW == 8 ? wave >> 2 : wave >> 1, wn = NW == 8 ? wave & 3 : wave & 1;
    const int l32 = lane & 31, kg = lane >> 5;
    const uint16_t *Bw = p.B + (size_t)e * K * N;

    // staging: a slab row is CPR 16-byte chunks handled by CPR adjacent threads (with 64-deep
    // slabs that is one whole 128-byte line per row); SP passes of SR rows cover the tile.  Rows
    // past the end of the tile re-read its last row (never stored).
    constexpr int CPR = RKC / 8, SR = NT / CPR, SP = RT / SR;
    const int s_row = tid / CPR, s_kq = (tid % CPR) * 8;
    const uint16_t *a_src[SP], *b_src[SP];
#pragma unroll
    for (int i = 0; i < SP; ++i) {
        a_src[i] = p.A + (size_t)(row0 + min(s_row + SR * i, rows - 1)) * K + s_kq;
        b_src[i] = Bw + (size_t)(col0 + s_row + SR * i) * K + s_kq;
    }
    v4u a_reg[SP], b_reg[SP];
    auto load_global = [&](int k0) {
#pragma unroll
        for (int i = 0; i < SP; ++i) a_reg[i] = *reinterpret_cast<const v4u *>(a_src[i] + k0);
#pragma unroll
        for (int i = 0; i < SP; ++i) b_reg[i] = *reinterpret_cast<const v4u *>(b_src[i] + k0);
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int i = 0; i < SP; ++i) *reinterpret_cast<v4u *>(&As[buf][s_row + SR * i][s_kq]) = a_reg[i];
#pragma unroll
        for (int i = 0; i < SP; ++i) *reinterpret_cast<v4u *>(&Bs[buf][s_row + SR * i][s_kq]) = b_reg[i];
    };

    v16f acc[4][NJ];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // operands of one k-step of 16: four row fragments, four column fragments
    v4u a_op[2][4], b_op[2][NJ];
    auto read_ops = [&](int slot, int buf, int ks) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            a_op[slot][i] = *reinterpret_cast<const v4u *>(&As[buf][128 * wm + 32 * i + l32][16 * ks + 8 * kg]);
#pragma unroll
        for (int j = 0; j < NJ; ++j)
            b_op[slot][j] = *reinterpret_cast<const v4u *>(&Bs[buf][WCOLS * wn + 32 * j + l32][16 * ks + 8 * kg]);
    };

    constexpr int NS = RKC / 16;   // k-steps per slab
    load_global(0);
    store_lds(0);
    load_global(min(RKC, K - RKC));
    __syncthreads();
    read_ops(0, 0, 0);
    for (int k0 = 0; k0 < K; k0 += RKC) {
        const int buf = (k0 / RKC) & 1;
#pragma unroll
        for (int ks = 0; ks < NS; ++ks) {
            if (ks == NS - 1) {
                __syncthreads();
                read_ops((ks + 1) & 1, buf ^ 1, 0);   // after the last slab: unused
            } else {
                read_ops((ks + 1) & 1, buf, ks + 1);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(   // the transposed product
                        __builtin_bit_cast(v8bf, b_op[ks & 1][j]), __builtin_bit_cast(v8bf, a_op[ks & 1][i]),
                        acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if (ks == NS / 2 - 1) {
                // unconditional: past the last slab they re-read a valid slab into a dead buffer
                store_lds(buf ^ 1);
                load_global(min(k0 + 2 * RKC, K - RKC));
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }

    // Epilogue through LDS, half a tile (128 rows) at a time: the waves that own the half write
    // their accumulators into a [128][256] fp32 image (the operand slabs are dead), then every wave
    // stores whole rows -- 1 KB (fp32) or 512 B (bf16) contiguous per row instead of the 32-byte
    // pieces a lane's own columns would make; the relu mask is read the same way.
    constexpr int CS = RT + 4;                       // fp32 words per staged row (rows stay 16-byte aligned)
    static_assert(128 * CS * 4 <= 4 * SLAB, "the staged half tile fits the operand buffers");
    float *Ct = reinterpret_cast<float *>(smem);
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) {
        __syncthreads();   // the operand buffers (hf = 0) / the first half's image (hf = 1) are no longer read
        if (wm == hf) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (128 * hf + 32 * i >= rows) continue;   // a short tile: nothing of this strip is stored
#pragma unroll
                for (int j = 0; j < NJ; ++j)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        *reinterpret_cast<v4f *>(&Ct[(32 * i + l32) * CS + WCOLS * wn + 32 * j + 8 * q + 4 * kg]) =
                            v4f{acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
            }
        }
        __syncthreads();
        if (EPI == EPI_F32) {
            float *C = reinterpret_cast<float *>(p.C);
            for (int r = wave; r < 128; r += NW) {          // a wavefront per row: 64 lanes x 16 bytes
                const int row = 128 * hf + r;
                if (row < rows)
                    MOE_STREAM_STORE(*reinterpret_cast<const v4f *>(&Ct[r * CS + 4 * lane]),   // read once, by the row gather
                                     reinterpret_cast<v4f *>(C + (size_t)(row0 + row) * N + col0 + 4 * lane));
            }
        } else {
            uint16_t *C = reinterpret_cast<uint16_t *>(p.C);
            const int c8 = 8 * (lane & 31);
            for (int r = 2 * wave + (lane >> 5); r < 128; r += 2 * NW) {   // half a wavefront per row: 32 lanes x 8 columns
                const int row = 128 * hf + r;
                if (row >= rows) continue;
                const size_t at = (size_t)(row0 + row) * N + col0 + c8;
                const v4f lo = *reinterpret_cast<const v4f *>(&Ct[r * CS + c8]);
                const v4f hi = *reinterpret_cast<const v4f *>(&Ct[r * CS + c8 + 4]);
                float v[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                if (EPI == EPI_MASK_BF16) {
                    // relu'(z) with relu'(0) = 0: the stored hidden value is positive iff z > 0
                    const v4u m = *reinterpret_cast<const v4u *>(p.mask + at);
#pragma unroll
                    for (int t = 0; t < 4; ++t) {   // a bf16 is positive iff its bits, moved to the top of a word, are > 0 as an integer
                        v[2 * t] = (int32_t)(m[t] << 16) > 0 ? v[2 * t] : 0.f;
                        v[2 * t + 1] = (int32_t)(m[t] & 0xffff0000u) > 0 ? v[2 * t + 1] : 0.f;
                    }
                } else {
#pragma unroll
                    for (int t = 0; t < 8; ++t) v[t] = fmaxf(v[t], 0.f);
                }
                v4u o;
#pragma unroll
                for (int t = 0; t < 4; ++t) o[t] = pack_bf16_pair(v[2 * t], v[2 * t + 1]);
                *reinterpret_cast<v4u *>(C + at) = o;
            }
        }
    }
}

// p's tile table must hold 256-row tiles; max_tiles bounds *p.num_tiles.
int launch_gg_rows256(const GGRows &p, int epi, int64_t max_tiles, hipStream_t st) {
    if (p.N % RT || p.K % RKC || p.K < RKC) return MOE_EUNSUPPORTED;
    const int col_tiles = p.N / RT;
    const unsigned grid = (unsigned)(ceil_div(max_tiles * col_tiles, 8) * 8);
    if (grid == 0) return MOE_OK;
#ifndef GG_NW
#define GG_NW 8
#endif
    constexpr int NW = GG_NW;
    if (epi == EPI_MASK_BF16) hipLaunchKernelGGL((gg_rows256_kernel<EPI_MASK_BF16, NW>), dim3(grid), dim3(64 * NW), 0, st, p, col_tiles);
    else if (epi == EPI_F32) hipLaunchKernelGGL((gg_rows256_kernel<EPI_F32, NW>), dim3(grid), dim3(64 * NW), 0, st, p, col_tiles);
    else hipLaunchKernelGGL((gg_rows256_kernel<EPI_RELU_BF16, NW>), dim3(grid), dim3(64 * NW), 0, st, p, col_tiles);
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}

}  // namespace moe
