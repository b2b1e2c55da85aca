// Fused launches of the layer forward for small problems, where the stages between the big
// kernels are bound by launch latency rather than by work.  Two independent stages share one
// grid (blocks of the second stage follow the blocks of the first), so that the sums behind the
// balancing losses (Eq.(6),(10)) ride along with routing, and their last step and the CV^2
// (Eq.(7),(11)) ride along with the combine (Eq.(1)).  Each block runs the unchanged body of its
// own stage, so results are identical to the separate launches.
#include "stages.h"
#include "device_bodies.h"

namespace moe {

// blocks [0, route_blocks): routing of one 1024-assignment chunk each;
// blocks [route_blocks, +col_blocks*chunks): level-1 sums of the gate's partial rows.
__global__ __launch_bounds__(256) void route_small_sums_kernel(RouteArgs p, int nbits, int route_blocks,
                                                               const float *__restrict__ partials,
                                                               int64_t prow, double *__restrict__ level2,
                                                               int col_blocks) {
    extern __shared__ int lds_s[];
    const int b = blockIdx.x;
    if (b < route_blocks) {
        route_small_body(p, nbits, b, lds_s);
    } else {
        const int q = b - route_blocks;
        reduce_partials_body(partials, prow, p.n, level2, q % col_blocks, q / col_blocks);
    }
}

// block 0 (dispatched first, so it runs beside the others from the start) finishes the sums and
// evaluates the two CV^2; blocks 1 .. combine_blocks combine four tokens each.
__global__ __launch_bounds__(256) void combine_losses_kernel(const float4 *__restrict__ out_sorted,
                                                             const float *__restrict__ gate,
                                                             const int32_t *__restrict__ inv_perm,
                                                             float4 *__restrict__ y, int64_t T, int d4,
                                                             int k, int combine_blocks,
                                                             const double *__restrict__ level2,
                                                             int chunks, int n, double *__restrict__ sums64,
                                                             float *__restrict__ importance,
                                                             float *__restrict__ load, float w_importance,
                                                             float w_load, float *__restrict__ losses) {
    if (blockIdx.x > 0) {
        combine_body(out_sorted, gate, inv_perm, y, T, d4, k, (int64_t)blockIdx.x - 1);
        return;
    }
    finish_sums_body(level2, chunks, n, sums64, importance, load, threadIdx.x, 256);
    __threadfence_block();
    __syncthreads();   // the block's own sums64 writes are visible to all of its threads
    cv2_body(sums64, n, w_importance, w_load, losses);
}

int launch_route_small_sums(RouteArgs a, const float *partials, int64_t prow, double *aux_ws,
                            hipStream_t st) {
    int nbits = 0;
    while ((1 << nbits) < a.n) ++nbits;
    const int route_blocks = (int)(a.A > 0 ? ceil_div(a.A, kSmallChunk) : 1);
    const int chunks = (int)ceil_div(prow > 0 ? prow : 1, kAuxChunkRows);
    const int col_blocks = (int)ceil_div(2 * a.n, 32);
    double *level2 = aux_ws + 2 * (size_t)a.n;
    hipLaunchKernelGGL(route_small_sums_kernel, dim3((unsigned)(route_blocks + col_blocks * chunks)),
                       dim3(256), (size_t)6 * a.n * sizeof(int), st, a, nbits, route_blocks, partials,
                       prow, level2, col_blocks);
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}

int launch_combine_losses(const float *out_sorted, const float *gate, const int32_t *inv_perm, float *y,
                          int64_t T, int d, int k, int64_t prow, int n, double *aux_ws, float w_imp,
                          float w_load, float *importance, float *load, float *losses, hipStream_t st) {
    const int combine_blocks = (int)ceil_div(T, 4);
    const int chunks = (int)ceil_div(prow > 0 ? prow : 1, kAuxChunkRows);
    hipLaunchKernelGGL(combine_losses_kernel, dim3((unsigned)(combine_blocks + 1)), dim3(256), 0, st,
                       (const float4 *)out_sorted, gate, inv_perm, (float4 *)y, T, d / 4, k,
                       combine_blocks, aux_ws + 2 * (size_t)n, chunks, n, aux_ws, importance, load,
                       w_imp, w_load, losses);
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}

}  // namespace moe
