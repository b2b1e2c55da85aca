// a5: Importance(X) = sum_x G(x) (Eq.(6)), Load(X) = sum_x P(x,.) (Eq.(10)) and the two
// CV^2 losses (Eq.(7),(11)).  The gating kernel leaves per-block fp32 partial sums; here they
// are added in a fixed order in fp64 and the coefficient of variation (population variance,
// no epsilon) is evaluated in fp64.
#include "stages.h"
#include "device_bodies.h"

namespace moe {

__global__ __launch_bounds__(256) void reduce_partials_kernel(const float *__restrict__ partials,
                                                              int64_t rows, int n,
                                                              double *__restrict__ level2) {
    reduce_partials_body(partials, rows, n, level2, blockIdx.x, blockIdx.y);
}

__global__ __launch_bounds__(256) void finish_sums_kernel(const double *__restrict__ level2,
                                                          int chunks, int n,
                                                          double *__restrict__ sums64,
                                                          float *__restrict__ importance,
                                                          float *__restrict__ load) {
    finish_sums_body(level2, chunks, n, sums64, importance, load, blockIdx.x * 256 + threadIdx.x, gridDim.x * 256);
}

__global__ __launch_bounds__(256) void cv2_kernel(const double *__restrict__ sums64, int n,
                                                  float w_importance, float w_load,
                                                  float *__restrict__ losses) {
    cv2_body(sums64, n, w_importance, w_load, losses);
}

int launch_aux_losses(const float *partials, int64_t rows, int n, float w_imp, float w_load,
                      float *importance, float *load, float *losses, double *ws, hipStream_t st) {
    const int chunks = (int)ceil_div(rows > 0 ? rows : 1, kAuxChunkRows);
    double *sums64 = ws;                  // [2n]
    double *level2 = ws + 2 * (size_t)n;  // [chunks][2n]
    hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)ceil_div(2 * n, 32), (unsigned)chunks),
                       dim3(256), 0, st, partials, rows, n, level2);
    MOE_LAUNCH_CHECK();
    hipLaunchKernelGGL(finish_sums_kernel, dim3((unsigned)ceil_div(2 * n, 256)), dim3(256), 0, st,
                       level2, chunks, n, sums64, importance, load);
    MOE_LAUNCH_CHECK();
    hipLaunchKernelGGL(cv2_kernel, dim3(1), dim3(256), 0, st, sums64, n, w_imp, w_load, losses);
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}

int launch_partial_sums(const float *partials, int64_t rows, int n, double *ws, hipStream_t st) {
    const int chunks = (int)ceil_div(rows > 0 ? rows : 1, kAuxChunkRows);
    double *sums64 = ws;
    double *level2 = ws + 2 * (size_t)n;
    hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)ceil_div(2 * n, 32), (unsigned)chunks),
                       dim3(256), 0, st, partials, rows, n, level2);
    MOE_LAUNCH_CHECK();
    hipLaunchKernelGGL(finish_sums_kernel, dim3((unsigned)ceil_div(2 * n, 256)), dim3(256), 0, st,
                       level2, chunks, n, sums64, (float *)nullptr, (float *)nullptr);
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}

// Eq.(13)-(14), one thread per expert e = i*b + j:
//   Importance_H = sum of the gate products routed to e (rows offsets[e]..offsets[e+1], in order)
//   Load_H       = Load_primary_i * Load_i(X^(i))_j / |X^(i)|, the secondary load being the sum of
//                  the partial rows of group i's tiles, in order.
__global__ __launch_bounds__(256) void hier_losses_kernel(HierLossArgs p) {
    const int n = p.a * p.b;
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= n) return;
    const int i = e / p.b, j = e % p.b;
    // both sums fetch eight terms at a time (independent loads) and add them in ascending order
    double imp = 0.0;
    const int r1 = p.offsets[e + 1];
    for (int r0 = p.offsets[e]; r0 < r1; r0 += 8) {
        int a[8];
        float g[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) a[u] = p.perm[min(r0 + u, r1 - 1)];
#pragma unroll
        for (int u = 0; u < 8; ++u) g[u] = p.gate[a[u]];
#pragma unroll
        for (int u = 0; u < 8; ++u) imp += r0 + u < r1 ? (double)g[u] : 0.0;
    }
    double ls = 0.0;
    const int blk0 = p.p_tile_offsets[i] * p.sub, blk1 = p.p_tile_offsets[i + 1] * p.sub;
    for (int b0 = blk0; b0 < blk1; b0 += 8) {
        float t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) t[u] = p.s_partials[((size_t)min(b0 + u, blk1 - 1) * 2 + 1) * p.b + j];
#pragma unroll
        for (int u = 0; u < 8; ++u) ls += b0 + u < blk1 ? (double)t[u] : 0.0;
    }
    const int cnt = p.p_counts[i];
    const double ld = cnt > 0 ? p.p_sums[p.a + i] * ls / (double)cnt : 0.0;
    p.sums64[e] = imp;
    p.sums64[n + e] = ld;
    p.importance[e] = (float)imp;
    p.load[e] = (float)ld;
}

int launch_hier_losses(const HierLossArgs &a, float w_imp, float w_load, float *losses, hipStream_t st) {
    const int n = a.a * a.b;
    hipLaunchKernelGGL(hier_losses_kernel, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, st, a);
    MOE_LAUNCH_CHECK();
    hipLaunchKernelGGL(cv2_kernel, dim3(1), dim3(256), 0, st, a.sums64, n, w_imp, w_load, losses);
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}

size_t aux_ws_bytes(int64_t rows, int n) {
    const int64_t chunks = ceil_div(rows > 0 ? rows : 1, kAuxChunkRows);
    return (size_t)(2 * (size_t)n * (1 + chunks)) * sizeof(double);
}

}  // namespace moe
