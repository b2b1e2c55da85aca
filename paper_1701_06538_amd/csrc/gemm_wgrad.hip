// Weight gradients of the experts (backward of Appendix C's two-layer expert):
//   C_e[M, N] = sum over the rows r of expert e of A[r, :]^T B[r, :]
// (dW2 = hid^T dout, dW1 = xs^T dz), both operands row-major in the rows being contracted.
//
// One workgroup of eight wavefronts owns a 256 x 256 block of C_e, each wavefront 128 x 64 as 8 x 4
// v_mfma_f32_16x16x32_bf16 tiles (128 accumulators, two wavefronts per SIMD so that one's LDS and
// vector work runs under the other's matrix work).  The matrix cores want, per lane, eight
// CONSECUTIVE contracted rows of one column, but memory has the columns consecutive.  So every
// thread loads a 4 x 8 block (four 16-byte loads), transposes it in registers with byte permutes
// and writes eight 8-byte column pieces to LDS; the operand reads are then plain 16-byte LDS
// reads, and the wavefronts share one copy of both panels.  Column 8c+j of a 128-column group is
// stored in slot 16j+c (80-byte slots), so that a lane ends up holding four consecutive columns of
// a row of C and a pair of wavefronts fills whole 32-byte pieces.
// Pipeline per 32 contracted rows: slab s is multiplied from LDS while slab s+1 is transposed into
// the other LDS buffer and slab s+2 is in flight from memory; every load and store is
// unconditional (clamped rows, selected values).  The kernel is bound by LDS traffic: per slab the
// wavefronts read 96 KB and write 32 KB, about 1700 cycles, against 1024 cycles of matrix work.
#include "stages.h"

namespace moe {

typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef uint32_t v4u __attribute__((ext_vector_type(4)));
typedef uint32_t v2u __attribute__((ext_vector_type(2)));

#ifdef MOE_WGRAD_TIMING
__device__ long long g_wgrad_timing[8192 * 4];
#define WG_STAMP(i) do { if (threadIdx.x == 0 && blockIdx.x < 8192) g_wgrad_timing[blockIdx.x * 4 + (i)] = (i) == 3 ? (long long)nslab : wall_clock64(); } while (0)
extern "C" int moe_debug_read_wgrad_timing(long long *host_out) {
    return (int)hipMemcpyFromSymbol(host_out, HIP_SYMBOL(g_wgrad_timing), sizeof(long long) * 8192 * 4);
}
#else
#define WG_STAMP(i) do { } while (0)
#endif

constexpr int WG_TILE = 256;    // rows and columns of C per workgroup
constexpr int WG_K = 32;        // contracted rows per slab
constexpr int WG_SLOT = 80;     // bytes per staged column: 32 rows of bf16 + 16 bytes of padding
constexpr int WG_STAGE = 2 * WG_TILE * WG_SLOT;   // both panels

__global__ __launch_bounds__(512) void gg_wgrad_kernel(GGWgrad p) {
    extern __shared__ __attribute__((aligned(16))) char stage_mem[];   // two stages
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // A workgroup contracts ALL rows of its expert, so with a skewed gate the workgroups differ
    // widely in length: the experts are taken by decreasing row count (longest first), rank r on
    // XCD r % 8 (workgroup i goes to XCD i % 8), so that the long ones start first, spread over the
    // chip, and the workgroups of one expert share one L2's copy of its rows.
    const int tiles_m = p.M / WG_TILE, tiles_n = p.N / WG_TILE, per_e = tiles_m * tiles_n;
    const int n_experts = gridDim.x / per_e;
    int rank = blockIdx.x / per_e, sub = blockIdx.x % per_e;
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

    // staging role: rows 4*sg .. 4*sg+3 of the slab, columns 8*cb .. 8*cb+7 of panel A (cb < 32) or B
    const int sg = lane & 7, cb = wave * 8 + (lane >> 3);
    const bool is_b = cb >= 32;
    const int cbl = cb & 31;
    const uint16_t *src = is_b ? p.B + n0 + 8 * cbl : p.A + m0 + 8 * cbl;
    const int64_t ld = is_b ? p.N : p.M;
    // slot of column 8*cbl + j within its panel: group of 128 columns, then 16*j + (cbl % 16)
    const int slot0 = (is_b ? WG_TILE : 0) + 128 * (cbl >> 4) + (cbl & 15);
    const int st_off = slot0 * WG_SLOT + 8 * sg;        // + 16*j*WG_SLOT for column j

    // multiply role: wave (wm, wn) owns rows 128 wm .. +127 of the block and, of the 128-column group
    // wn / 2, the columns 8 c + 4 (wn % 2) + j, j < 4: slots 16 (4 (wn % 2) + j) + c
    const int c = lane & 15, g = lane >> 4;
    const int wm = wave >> 2, wn = wave & 3;
    const int a_off = (128 * wm + c) * WG_SLOT + 16 * g;                // + 16*i*WG_SLOT for tile i
    const int b_off = (WG_TILE + 128 * (wn >> 1) + 64 * (wn & 1) + c) * WG_SLOT + 16 * g;

    const int nslab = (r1 - r0 + WG_K - 1) / WG_K;
    v4u raw[4];
    auto fetch = [&](int s) {   // slab s (clamped) -> registers; rows past the end re-read a valid row
        const int row = r0 + min(s, nslab - 1) * WG_K + 4 * sg;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            raw[i] = *reinterpret_cast<const v4u *>(src + (int64_t)min(row + i, r1 - 1) * ld);
    };
    auto put = [&](int s, char *buf) {   // transpose the 4 x 8 block, zero the rows past the end
        const int row = r0 + s * WG_K + 4 * sg;
        v4u z[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const bool in = row + i < r1;
            z[i].x = in ? raw[i].x : 0u; z[i].y = in ? raw[i].y : 0u;
            z[i].z = in ? raw[i].z : 0u; z[i].w = in ? raw[i].w : 0u;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t sel = (j & 1) ? 0x07060302u : 0x05040100u;
            const int w = j >> 1;
            v2u o;
            o.x = __builtin_amdgcn_perm(z[1][w], z[0][w], sel);
            o.y = __builtin_amdgcn_perm(z[3][w], z[2][w], sel);
            *reinterpret_cast<v2u *>(buf + st_off + 16 * j * WG_SLOT) = o;
        }
    };

    WG_STAMP(0);
    if (nslab > 0) {
        fetch(0);
        put(0, stage_mem);
        fetch(1);
        __syncthreads();
        for (int s = 0; s < nslab; ++s) {
            const char *cur = stage_mem + (s & 1) * WG_STAGE;
            v8bf a[8], b[4];
#pragma unroll
            for (int i = 0; i < 8; ++i)
                a[i] = __builtin_bit_cast(v8bf, *reinterpret_cast<const v4u *>(cur + a_off + 16 * i * WG_SLOT));
#pragma unroll
            for (int j = 0; j < 4; ++j)
                b[j] = __builtin_bit_cast(v8bf, *reinterpret_cast<const v4u *>(cur + b_off + 16 * j * WG_SLOT));
            put(s + 1, stage_mem + ((s + 1) & 1) * WG_STAGE);     // past the last slab: zeros nobody reads
            fetch(s + 2);
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
            __syncthreads();
        }
    }

    WG_STAMP(1);
    WG_STAMP(3);
    // acc[i][j][q] = C[m0 + 128 wm + 8 (4g + q) + i][n0 + 128 (wn/2) + 8 c + 4 (wn%2) + j]
    float *Ce = p.C + (size_t)e * p.M * p.N;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int row = m0 + 128 * wm + 8 * (4 * g + q) + i;
            float *dst = Ce + (size_t)row * p.N + n0 + 128 * (wn >> 1) + 8 * c + 4 * (wn & 1);
            *reinterpret_cast<v4f *>(dst) = v4f{acc[i][0][q], acc[i][1][q], acc[i][2][q], acc[i][3][q]};
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
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float rs = 0.f;
#pragma unroll
                for (int j = 0; j < 4; ++j) rs = fmaf(acc[i][j][q], acc[i][j][q], rs);
#pragma unroll
                for (int off = 1; off < 16; off <<= 1) rs += __shfl_xor(rs, off);    // over c
                if (c == 0) rrow[wn * WG_TILE + 128 * wm + 8 * (4 * g + q) + i] = rs;
            }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float cs = 0.f;
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q) cs = fmaf(acc[i][j][q], acc[i][j][q], cs);
            cs += __shfl_xor(cs, 16);                                                  // over g
            cs += __shfl_xor(cs, 32);
            if (g == 0) rcol[wm * WG_TILE + 128 * (wn >> 1) + 8 * c + 4 * (wn & 1) + j] = cs;
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
    WG_STAMP(2);
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
    constexpr int lds = 2 * WG_STAGE;
    static bool attr_set = false;
    if (!attr_set) {
        MOE_HIP_TRY(hipFuncSetAttribute((const void *)gg_wgrad_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds));
        attr_set = true;
    }
    hipLaunchKernelGGL(gg_wgrad_kernel, dim3(grid), dim3(512), lds, st, p);
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}

}  // namespace moe
