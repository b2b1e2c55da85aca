// a2: dispatch bookkeeping -- a deterministic stable counting sort of the T*k assignments by
// expert id.  Skipping experts with G(x)_i = 0 (Section 2) and giving each expert one combined
// batch (Section 3.1) both come down to this permutation.
//
//   route_hist_kernel    chunk c of the assignment list -> LDS histogram -> hist[c][e]
//   route_colscan_kernel per expert: exclusive scan over chunks (in place), counts[e]
//   route_offsets_kernel one block: offsets = scan(counts); row-tile table for the expert kernel
//   route_scatter_kernel one wavefront per chunk walks its assignments in order; the rank of an
//                        assignment among equal experts inside a 64-wide step comes from
//                        ballots over the bits of the expert id, so no atomics decide positions
#include "stages.h"
#include "device_bodies.h"

namespace moe {


void route_chunking(int64_t A, int *chunk, int *num_chunks) {
    int64_t c = ceil_div(ceil_div(A, 512), 64) * 64;
    if (c < 64) c = 64;
    if (c > 4096) c = 4096;
    *chunk = (int)c;
    *num_chunks = (int)ceil_div(A, c);
}

size_t route_ws_bytes(int64_t A, int n) {
    int chunk, nc;
    route_chunking(A, &chunk, &nc);
    return (size_t)(nc > 0 ? nc : 1) * n * sizeof(int32_t);
}

__global__ __launch_bounds__(256) void route_hist_kernel(RouteArgs p) {
    extern __shared__ int lds_hist[];
    const int n = p.n;
    for (int e = threadIdx.x; e < n; e += 256) lds_hist[e] = 0;
    __syncthreads();
    const int64_t a0 = (int64_t)blockIdx.x * p.chunk;
    const int64_t a1 = min(a0 + p.chunk, p.A);
    for (int64_t a = a0 + threadIdx.x; a < a1; a += 256) {
        const int e = p.idx[a];
        if (e >= 0 && e < n) atomicAdd(&lds_hist[e], 1);  // integer counts: order-independent
    }
    __syncthreads();
    int32_t *out = p.hist + (size_t)blockIdx.x * n;
    for (int e = threadIdx.x; e < n; e += 256) out[e] = lds_hist[e];
}

// Per expert, the exclusive scan of the chunk histograms over the chunks (in place) and the
// total.  A workgroup covers 32 experts x 8 chunk groups: every thread first sums its group of
// chunks (independent loads), the eight group sums are scanned in LDS, then every thread rewrites
// its chunks with the running prefix.
__global__ __launch_bounds__(256) void route_colscan_kernel(RouteArgs p) {
    __shared__ int grp[8][33];
    const int ex = threadIdx.x & 31, cg = threadIdx.x >> 5;
    const int e = blockIdx.x * 32 + ex;
    const int per = (p.num_chunks + 7) / 8;
    const int c0 = cg * per, c1 = min(p.num_chunks, c0 + per);
    int sum = 0;
    if (e < p.n) {
#pragma unroll 8
        for (int c = c0; c < c1; ++c) sum += p.hist[(size_t)c * p.n + e];   // independent loads, eight in flight
    }
    grp[cg][ex] = sum;
    __syncthreads();
    int run = 0;
    for (int q = 0; q < cg; ++q) run += grp[q][ex];
    if (e < p.n) {
        for (int cb = c0; cb < c1; cb += 8) {   // eight cells at a time: the loads first, then the running prefix
            int v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = cb + u < c1 ? p.hist[(size_t)(cb + u) * p.n + e] : 0;
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (cb + u < c1) {
                    p.hist[(size_t)(cb + u) * p.n + e] = run;
                    run += v[u];
                }
        }
        if (cg == 7) {
            int total = 0;
            for (int q = 0; q < 8; ++q) total += grp[q][ex];
            p.counts[e] = total;
        }
    }
}

// Block-wide inclusive scan of one int per thread (1024 threads = 16 waves).
__device__ __forceinline__ int block_inclusive_scan(int v, int *wave_sums) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_up(v, off);
        if (lane >= off) v += o;
    }
    if (lane == 63) wave_sums[wave] = v;
    __syncthreads();
    int add = 0;
    for (int w = 0; w < wave; ++w) add += wave_sums[w];
    __syncthreads();
    return v + add;
}

__global__ __launch_bounds__(1024) void route_offsets_kernel(RouteArgs p) {
    __shared__ int wave_sums[16];
    __shared__ int carry[2];
    const int n = p.n, TM = p.tile_rows;
    if (threadIdx.x == 0) {
        carry[0] = 0;
        carry[1] = 0;
    }
    __syncthreads();
    for (int base = 0; base < n; base += 1024) {
        const int e = base + threadIdx.x;
        const int cnt = e < n ? p.counts[e] : 0;
        const int tiles = (cnt + TM - 1) / TM;
        const int c0 = carry[0], c1 = carry[1];
        const int inc_rows = block_inclusive_scan(cnt, wave_sums);
        const int inc_tiles = block_inclusive_scan(tiles, wave_sums);
        if (e < n) {
            const int off = c0 + inc_rows - cnt;
            const int toff = c1 + inc_tiles - tiles;
            p.offsets[e] = off;
            if (p.tile_offsets) p.tile_offsets[e] = toff;
            for (int j = 0; j < tiles; ++j) {
                p.tile_expert[toff + j] = e;
                p.tile_row0[toff + j] = off + j * TM;
            }
        }
        __syncthreads();
        if (threadIdx.x == 1023) {
            carry[0] = c0 + inc_rows;
            carry[1] = c1 + inc_tiles;
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        p.offsets[n] = carry[0];
        if (p.tile_offsets) p.tile_offsets[n] = carry[1];
        p.num_tiles[0] = carry[1];
    }
}

__global__ __launch_bounds__(64) void route_scatter_kernel(RouteArgs p, int nbits) {
    extern __shared__ int lds_cursor[];
    const int n = p.n, lane = threadIdx.x;
    for (int e = lane; e < n; e += 64) lds_cursor[e] = 0;
    __syncthreads();
    const int32_t *base_row = p.hist + (size_t)blockIdx.x * n;
    const int64_t a0 = (int64_t)blockIdx.x * p.chunk;
    const int64_t a1 = min(a0 + p.chunk, p.A);
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
    for (int64_t s = a0; s < a1; s += 64) {
        const int64_t a = s + lane;
        int e = (a < a1) ? p.idx[a] : -1;
        const bool active = e >= 0 && e < n;
        unsigned long long same = __ballot(active);
        for (int b = 0; b < nbits; ++b) {
            const bool bit = (e >> b) & 1;
            const unsigned long long bal = __ballot(active && bit);
            same &= bit ? bal : ~bal;
        }
        if (active) {
            const int rank = __popcll(same & lt_mask);
            const int cnt = __popcll(same);
            const int before = lds_cursor[e];
            const int pos = p.offsets[e] + base_row[e] + before + rank;
            p.perm[pos] = (int32_t)a;
            p.inv_perm[a] = pos;
            if (rank == cnt - 1) lds_cursor[e] = before + cnt;  // issued after every lane's read
        }
    }
}

__global__ __launch_bounds__(256) void route_small_kernel(RouteArgs p, int nbits) {
    extern __shared__ int lds_s[];
    route_small_body(p, nbits, blockIdx.x, lds_s);
}

// Row-tile table for another tile height, from an existing offsets array (one workgroup).
__global__ __launch_bounds__(1024) void build_tiles_kernel(const int32_t *__restrict__ offsets, int n,
                                                           int TM, int32_t *__restrict__ tile_expert,
                                                           int32_t *__restrict__ tile_row0,
                                                           int32_t *__restrict__ num_tiles) {
    __shared__ int wave_sums[16];
    __shared__ int carry;
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    for (int base = 0; base < n; base += 1024) {
        const int e = base + threadIdx.x;
        const int off = e < n ? offsets[e] : 0;
        const int cnt = e < n ? offsets[e + 1] - off : 0;
        const int tiles = (cnt + TM - 1) / TM;
        const int c0 = carry;
        const int inc = block_inclusive_scan(tiles, wave_sums);
        if (e < n) {
            const int toff = c0 + inc - tiles;
            for (int j = 0; j < tiles; ++j) {
                tile_expert[toff + j] = e;
                tile_row0[toff + j] = off + j * TM;
            }
        }
        __syncthreads();
        if (threadIdx.x == 1023) carry = c0 + inc;
        __syncthreads();
    }
    if (threadIdx.x == 0) num_tiles[0] = carry;
}

int launch_build_tiles(const int32_t *offsets, int n, int tile_rows, int32_t *tile_expert,
                       int32_t *tile_row0, int32_t *num_tiles, hipStream_t st) {
    hipLaunchKernelGGL(build_tiles_kernel, dim3(1), dim3(1024), 0, st, offsets, n, tile_rows,
                       tile_expert, tile_row0, num_tiles);
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}

bool route_is_small(int64_t A, int n) { return n <= kSmallMaxN && A <= 65536; }

int launch_route(RouteArgs a, hipStream_t st) {
    int nbits = 0;
    while ((1 << nbits) < a.n) ++nbits;
    if (route_is_small(a.A, a.n)) {
        const unsigned blocks = (unsigned)(a.A > 0 ? ceil_div(a.A, kSmallChunk) : 1);
        hipLaunchKernelGGL(route_small_kernel, dim3(blocks), dim3(256), (size_t)6 * a.n * sizeof(int),
                           st, a, nbits);
        MOE_LAUNCH_CHECK();
        return MOE_OK;
    }
    route_chunking(a.A, &a.chunk, &a.num_chunks);
    const size_t lds = (size_t)a.n * sizeof(int);
    if (a.num_chunks > 0) {
        hipLaunchKernelGGL(route_hist_kernel, dim3(a.num_chunks), dim3(256), lds, st, a);
        MOE_LAUNCH_CHECK();
    }
    hipLaunchKernelGGL(route_colscan_kernel, dim3((unsigned)ceil_div(a.n, 32)), dim3(256), 0, st, a);
    MOE_LAUNCH_CHECK();
    hipLaunchKernelGGL(route_offsets_kernel, dim3(1), dim3(1024), 0, st, a);
    MOE_LAUNCH_CHECK();
    if (a.num_chunks > 0) {
        hipLaunchKernelGGL(route_scatter_kernel, dim3(a.num_chunks), dim3(64), lds, st, a, nbits);
        MOE_LAUNCH_CHECK();
    }
    return MOE_OK;
}

}  // namespace moe

using namespace moe;

extern "C" size_t moe_route_workspace_bytes(const moe_config *cfg) {
    if (check_config(cfg) != MOE_OK) return 0;
    return route_ws_bytes((int64_t)cfg->T * cfg->k, cfg->n);
}

static int route_with_scratch(const moe_config *cfg, const int32_t *topk_idx, int32_t *counts,
                              int32_t *offsets, int32_t *perm, int32_t *inv_perm, int32_t *tile_expert,
                              int32_t *tile_row0, int32_t *num_tiles, void *workspace, void *stream) {
    RouteArgs a{};
    a.idx = topk_idx;
    a.A = (int64_t)cfg->T * cfg->k;
    a.n = cfg->n;
    a.tile_rows = moe_tile_rows(cfg);
    a.counts = counts; a.offsets = offsets; a.perm = perm; a.inv_perm = inv_perm;
    a.tile_expert = tile_expert; a.tile_row0 = tile_row0; a.num_tiles = num_tiles;
    a.tile_offsets = nullptr;
    a.hist = (int32_t *)workspace;
    return launch_route(a, (hipStream_t)stream);
}

extern "C" int moe_route(const moe_config *cfg, const int32_t *topk_idx, int32_t *counts,
                         int32_t *offsets, int32_t *perm, int32_t *inv_perm, int32_t *tile_expert,
                         int32_t *tile_row0, int32_t *num_tiles, void *workspace, void *stream) {
    int st = check_config(cfg);
    if (st != MOE_OK) return st;
    if (!topk_idx || !counts || !offsets || !perm || !inv_perm || !tile_expert || !tile_row0 ||
        !num_tiles || !workspace)
        return MOE_EINVAL;
    return route_with_scratch(cfg, topk_idx, counts, offsets, perm, inv_perm, tile_expert, tile_row0,
                              num_tiles, workspace, stream);
}

// ---- moe_route for callers that cannot allocate -----------------------------------------
// The chunk histograms live in a device array that is part of the library image: every GPU the
// library runs on holds its own copy until the process ends.  The array's name is only a
// host-side stand-in; its device address is looked up once per device and that address is what
// the kernels receive.
constexpr size_t kRouteScratchBytes = MOE_ROUTE_STATIC_MAX_WORKSPACE_BYTES;   // 4 MiB: 512 chunks x 2048 experts
static __device__ __align__(256) int32_t scratch[kRouteScratchBytes / sizeof(int32_t)];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
int32_t *g_scratch_ptr[kMaxDevices] = {};

int route_scratch_for_current_device(int32_t **out) {
    int dev = 0;
    MOE_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return MOE_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        MOE_HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return MOE_EHIP;
        g_scratch_ptr[dev] = (int32_t *)ptr;
    }
    *out = g_scratch_ptr[dev];
    return MOE_OK;
}
}  // namespace

extern "C" int moe_route_static(const moe_config *cfg, const int32_t *topk_idx, int32_t *counts,
                                int32_t *offsets, int32_t *perm, int32_t *inv_perm,
                                int32_t *tile_expert, int32_t *tile_row0, int32_t *num_tiles,
                                void *stream) {
    int st = check_config(cfg);
    if (st != MOE_OK) return st;
    if (!topk_idx || !counts || !offsets || !perm || !inv_perm || !tile_expert || !tile_row0 || !num_tiles)
        return MOE_EINVAL;
    if (route_ws_bytes((int64_t)cfg->T * cfg->k, cfg->n) > kRouteScratchBytes) return MOE_EWORKSPACE;
    int32_t *ptr = nullptr;
    if ((st = route_scratch_for_current_device(&ptr)) != MOE_OK) return st;
    // every histogram cell a kernel reads is written earlier in the same call (route_hist_kernel
    // fills all num_chunks x n cells), so nothing of the previous call's contents has to be cleared
    return route_with_scratch(cfg, topk_idx, counts, offsets, perm, inv_perm, tile_expert, tile_row0,
                              num_tiles, ptr, stream);
}
