// Weight gradients of the experts (backward of Appendix C's two-layer expert):
//   C_e[M, N] = sum over the rows r of expert e of A[r, :]^T B[r, :]
// (dW2 = hid^T dout, dW1 = xs^T dz), both operands row-major in the rows being contracted.
//
// One workgroup of eight wavefronts owns a 256 x 256 block of C_e, each wavefront 128 x 64 as 8 x 4
// v_mfma_f32_16x16x32_bf16 tiles (128 accumulators, two wavefronts per SIMD so that one's LDS and
// vector work runs under the other's matrix work).  The matrix cores want, per lane, eight
// CONSECUTIVE contracted rows of one column, but memory has the columns consecutive: the
// transposing LDS reads described at the kernel deliver exactly that from row-major slabs.
// Pipeline per 32 contracted rows: slab s is multiplied from LDS while slab s+1 is stored into
// the other LDS buffer and slab s+2 is in flight from memory; every load and store is
// unconditional (clamped rows, selected values).  Per slab the wavefronts read 96 KB of LDS and
// write 32 KB, about as many LDS cycles as the 1024 cycles of matrix work per SIMD.
#include "stages.h"

namespace moe {

typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));


constexpr int WG_TILE = 256;    // rows and columns of C per workgroup
constexpr int WG_K = 32;        // contracted rows per slab
// Operand staging: the slabs go to LDS as they are in memory
// (row = contracted row, columns contiguous; 16-byte stores, a wavefront per row), and gfx950's
// ds_read_b64_tr_b16 hands every lane four CONSECUTIVE contracted rows of one column: within a
// block of 16 lanes, lane j receives element j % 4 of the 8 bytes addressed by lanes j / 4,
// j / 4 + 4, j / 4 + 8, j / 4 + 12.  Lane i of block b therefore addresses row 8 b + 4 half + i / 4,
// columns 4 (i % 4) .. + 3 of the 16-column tile, and two such reads (half = 0, 1) make one
// matrix-core operand (k = 8 b .. 8 b + 7 of the slab in lane group b).  No register transpose and
// no scattered LDS stores.  B is the matrix instruction's first operand, so a lane holds four
// consecutive columns of one row of C:
//   acc[i][j][r] = C[m0 + 128 wm + 16 i + c][n0 + 64 wn + 16 j + 4 g + r].
constexpr int WT_PITCH = 2 * WG_TILE + 32;            // bytes per slab row of one panel: 136 words = 8 mod 64 banks
constexpr int WT_PANEL = WG_K * WT_PITCH;
constexpr int WT_STAGE = 2 * WT_PANEL;
constexpr int WT_CS = WG_TILE + 4;                    // fp32 words per row of the epilogue's image of half a block
constexpr int WT_LDS = 2 * WT_STAGE > 128 * WT_CS * 4 ? 2 * WT_STAGE : 128 * WT_CS * 4;

typedef short v4s __attribute__((ext_vector_type(4)));
typedef short v8s __attribute__((ext_vector_type(8)));

__device__ __forceinline__ v8bf read_tr_operand(const char *panel_tile) {
    // panel_tile: this lane's address for half 0; half 1 is four slab rows further
    const v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((v4s __attribute__((address_space(3))) *)panel_tile);
    const v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (v4s __attribute__((address_space(3))) *)(panel_tile + 4 * WT_PITCH));
    return __builtin_bit_cast(v8bf, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

__global__ __launch_bounds__(512) void gg_wgrad_kernel(GGWgrad p) {
    extern __shared__ __attribute__((aligned(16))) char stage_mem[];   // two stages
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tiles_m = p.M / WG_TILE, tiles_n = p.N / WG_TILE, per_e = tiles_m * tiles_n;
    const int n_experts = gridDim.x / per_e;
    int rank = blockIdx.x / per_e, sub = blockIdx.x % per_e;
    // A workgroup contracts ALL rows of its expert, so with a skewed gate the workgroups differ
    // widely in length: the experts are taken by decreasing row count (longest first), rank r on
    // XCD r % 8 (workgroup i goes to XCD i % 8), so that the long ones start first, spread over the
    // chip, and the workgroups of one expert share one L2's copy of its rows.
    if (n_experts % 8 == 0) {
        const int xcd = blockIdx.x % 8, slot = blockIdx.x / 8, round = slot / per_e;
        rank = round * 8 + ((round & 1) ? 7 - xcd : xcd);   // serpentine: the XCDs' row totals stay close
        sub = slot % per_e;
    }
    const int e = p.order[rank];
    const int m0 = (sub / tiles_n) * WG_TILE, n0 = (sub % tiles_n) * WG_TILE;
    const int r0 = p.offsets[e], r1 = p.offsets[e + 1];

    v4f acc[8][4];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = v4f{0.f, 0.f, 0.f, 0.f};

    // staging role: a wavefront moves slab rows wave, wave + 8, wave + 16, wave + 24; lanes 0-31 the
    // 32 16-byte chunks of the A panel's row, lanes 32-63 those of the B panel's
    const bool is_b = lane >= 32;
    const int chunk = lane & 31;
    const uint16_t *src = is_b ? p.B + n0 + 8 * chunk : p.A + m0 + 8 * chunk;
    const int64_t ld = is_b ? p.N : p.M;
    const int st_off = (is_b ? WT_PANEL : 0) + 16 * chunk;      // + row * WT_PITCH

    // multiply role
    const int c = lane & 15, g = lane >> 4;
    const int wm = wave >> 2, wn = wave & 3;
    const int rd = (8 * g + (c >> 2)) * WT_PITCH + 8 * (c & 3);  // this lane's row and 8-byte piece within a tile
    const int a_off = rd + 2 * (128 * wm);                       // + 32 * i for tile i
    const int b_off = WT_PANEL + rd + 2 * (64 * wn);             // + 32 * j for tile j

    const int nslab = (r1 - r0 + WG_K - 1) / WG_K;
    v4u raw[4];
    auto fetch = [&](int s) {   // slab s (clamped) -> registers; rows past the end re-read a valid row
        const int row = r0 + min(s, nslab - 1) * WG_K + wave;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            raw[i] = *reinterpret_cast<const v4u *>(src + (int64_t)min(row + 8 * i, r1 - 1) * ld);
    };
    auto put = [&](int s, char *buf) {   // rows past the end become zeros
        const int row = r0 + s * WG_K + wave;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const bool in = row + 8 * i < r1;
            v4u z;
            z.x = in ? raw[i].x : 0u; z.y = in ? raw[i].y : 0u;
            z.z = in ? raw[i].z : 0u; z.w = in ? raw[i].w : 0u;
            *reinterpret_cast<v4u *>(buf + st_off + (wave + 8 * i) * WT_PITCH) = z;
        }
    };

    if (nslab > 0) {
        fetch(0);
        put(0, stage_mem);
        fetch(1);
        __syncthreads();
        for (int s = 0; s < nslab; ++s) {
            const char *cur = stage_mem + (s & 1) * WT_STAGE;
            v8bf a[8], b[4];
#pragma unroll
            for (int i = 0; i < 8; ++i) a[i] = read_tr_operand(cur + a_off + 32 * i);
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = read_tr_operand(cur + b_off + 32 * j);
            put(s + 1, stage_mem + ((s + 1) & 1) * WT_STAGE);     // past the last slab: zeros nobody reads
            fetch(s + 2);
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
            __syncthreads();
        }
    }

    // The block leaves through LDS, 128 rows at a time (the operand stages are dead): the four
    // wavefronts that own the half write their accumulators into a [128][256] image, then every
    // wavefront stores whole 1 KB rows instead of the 64-byte pieces its own lanes would make.
    float *Ce = p.C + (size_t)e * p.M * p.N;
    float *Ct = reinterpret_cast<float *>(stage_mem);
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) {
        __syncthreads();
        if (wm == hf) {
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    *reinterpret_cast<v4f *>(&Ct[(16 * i + c) * WT_CS + 64 * wn + 16 * j + 4 * g]) = acc[i][j];
        }
        __syncthreads();
        for (int r = wave; r < 128; r += 8)
            // the gradient is written once and read once, much later, by the optimiser: a streaming store
            MOE_STREAM_STORE(*reinterpret_cast<const v4f *>(&Ct[r * WT_CS + 4 * lane]),
                             reinterpret_cast<v4f *>(Ce + (size_t)(m0 + 128 * hf + r) * p.N + n0 + 4 * lane));
    }
    // Optional: this block's share of the row and column sums of squares of the gradient, which
    // the factored second-moment estimator of the optimiser needs (Appendix D) -- taken here, where
    // the gradient is in registers, instead of re-reading it from memory.
    // rowpart [n][N/256][M], colpart [n][M/256][N]; every partial is written by exactly one
    // workgroup and summed by the consumer in a fixed order.
    if (p.rowpart) {
        float *red = reinterpret_cast<float *>(stage_mem);        // the operand stages are dead
        float *rrow = red;                                        // [4 wn][256 rows]
        float *rcol = red + 4 * WG_TILE;                          // [2 wm][256 cols]
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            float rs = 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) rs = fmaf(acc[i][j][r], acc[i][j][r], rs);
            rs += __shfl_xor(rs, 16);                                                  // over g
            rs += __shfl_xor(rs, 32);
            if (g == 0) rrow[wn * WG_TILE + 128 * wm + 16 * i + c] = rs;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float cs = 0.f;
#pragma unroll
                for (int i = 0; i < 8; ++i) cs = fmaf(acc[i][j][r], acc[i][j][r], cs);
#pragma unroll
                for (int off = 1; off < 16; off <<= 1) cs += __shfl_xor(cs, off);    // over c
                if (c == 0) rcol[wm * WG_TILE + 64 * wn + 16 * j + 4 * g + r] = cs;
            }
        __syncthreads();
        const int tn = n0 / WG_TILE, tm = m0 / WG_TILE;
        if (tid < WG_TILE) {
            const float v = ((rrow[tid] + rrow[WG_TILE + tid]) + rrow[2 * WG_TILE + tid]) + rrow[3 * WG_TILE + tid];
            p.rowpart[((size_t)e * tiles_n + tn) * p.M + m0 + tid] = v;
        } else {
            const int cc = tid - WG_TILE;
            p.colpart[((size_t)e * tiles_m + tm) * p.N + n0 + cc] = rcol[cc] + rcol[WG_TILE + cc];
        }
    }
}

// A workgroup ranks 64 experts (one per lane); its four waves each compare them against a quarter
// of every 2048-expert chunk, and the four partial ranks are added at the end.
__global__ __launch_bounds__(256) void expert_order_kernel(const int32_t *__restrict__ offsets, int n,
                                                           int32_t *__restrict__ order) {
    __shared__ __attribute__((aligned(16))) int cs[2048];   // counts of a chunk of experts (-1 past the end)
    __shared__ int part[4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int e = blockIdx.x * 64 + lane;
    const int c = e < n ? offsets[e + 1] - offsets[e] : 0;
    int rank = 0;
    for (int o0 = 0; o0 < n; o0 += 2048) {
        const int m = min(2048, n - o0);
        __syncthreads();
        for (int i = threadIdx.x; i < 2048; i += 256) cs[i] = i < m ? offsets[o0 + i + 1] - offsets[o0 + i] : -1;
        __syncthreads();
        const int lo = 512 * wave, hi = min(lo + 512, (m + 3) & ~3);
        // every lane reads the same four counts per step (a broadcast 16-byte LDS read)
#pragma unroll 4
        for (int i = lo; i < hi; i += 4) {
            const int4 v = *reinterpret_cast<const int4 *>(&cs[i]);
            const int j = o0 + i;
            rank += (v.x > c || (v.x == c && j < e)) + (v.y > c || (v.y == c && j + 1 < e)) +
                    (v.z > c || (v.z == c && j + 2 < e)) + (v.w > c || (v.w == c && j + 3 < e));
        }
    }
    part[wave][lane] = rank;
    __syncthreads();
    if (wave == 0 && e < n) order[part[0][lane] + part[1][lane] + part[2][lane] + part[3][lane]] = e;
}

int launch_expert_order(const int32_t *offsets, int n, int32_t *order, hipStream_t st) {
    if (n <= 0) return MOE_OK;
    hipLaunchKernelGGL(expert_order_kernel, dim3((unsigned)ceil_div(n, 64)), dim3(256), 0, st, offsets, n, order);
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}

int launch_gg_wgrad(const GGWgrad &p, int n, hipStream_t st) {
    if (p.M % WG_TILE || p.N % WG_TILE) return MOE_EUNSUPPORTED;
    if (n <= 0) return MOE_OK;
    const unsigned grid = (unsigned)((p.M / WG_TILE) * (p.N / WG_TILE) * n);
    constexpr int lds = WT_LDS;
    static LdsLimitOnce lds_once;
    MOE_TRY(lds_once.set((const void *)gg_wgrad_kernel, lds));
    hipLaunchKernelGGL(gg_wgrad_kernel, dim3(grid), dim3(512), lds, st, p);
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}

}  // namespace moe
