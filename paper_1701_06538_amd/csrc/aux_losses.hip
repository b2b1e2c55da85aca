// a5: Importance(X) = sum_x G(x) (Eq.(6)), Load(X) = sum_x P(x,.) (Eq.(10)) and the two
// CV^2 losses (Eq.(7),(11)).  The gating kernel leaves per-block fp32 partial sums; here they
// are added in a fixed order in fp64 and the coefficient of variation (population variance,
// no epsilon) is evaluated in fp64.
#include "stages.h"

namespace moe {

// Level 1: level2[chunk][i] = sum of partials[r][i] over the chunk's 128 rows (i runs over the
// 2n importance|load columns).  A block covers 32 columns x 8 row groups, every thread adds its
// 16 rows (all loads independent) in fp64, the eight group sums are added in ascending order.
constexpr int kAuxChunkRows = 128;

__global__ __launch_bounds__(256) void reduce_partials_kernel(const float *__restrict__ partials,
                                                              int64_t rows, int n,
                                                              double *__restrict__ level2) {
    __shared__ double part[8][33];
    const int cx = threadIdx.x & 31, rg = threadIdx.x >> 5;
    const int i = blockIdx.x * 32 + cx;
    const int64_t r0 = (int64_t)blockIdx.y * kAuxChunkRows;
    double acc = 0.0;
    if (i < 2 * n) {
        const float *col = partials + i;
        float v[kAuxChunkRows / 8];
#pragma unroll
        for (int q = 0; q < kAuxChunkRows / 8; ++q) {
            const int64_t r = r0 + rg + 8 * q;
            v[q] = r < rows ? col[r * 2 * n] : 0.f;
        }
#pragma unroll
        for (int q = 0; q < kAuxChunkRows / 8; ++q) acc += (double)v[q];
    }
    part[rg][cx] = acc;
    __syncthreads();
    if (rg == 0 && i < 2 * n) {
        double s = part[0][cx];
#pragma unroll
        for (int q = 1; q < 8; ++q) s += part[q][cx];
        level2[(size_t)blockIdx.y * 2 * n + i] = s;
    }
}

// Level 2 (one block): add the chunk sums in ascending chunk order, publish Importance and Load,
// then the two CV^2.
__global__ __launch_bounds__(256) void finish_sums_kernel(const double *__restrict__ level2,
                                                          int chunks, int n,
                                                          double *__restrict__ sums64,
                                                          float *__restrict__ importance,
                                                          float *__restrict__ load) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= 2 * n) return;
    double s = 0.0;
    for (int c = 0; c < chunks; ++c) s += level2[(size_t)c * 2 * n + i];
    sums64[i] = s;
    if (!importance) return;
    if (i < n) importance[i] = (float)s;
    else load[i - n] = (float)s;
}

// one block: CV^2 of v[0..n) in fp64
__device__ double block_cv2(const double *v, int n, double *scratch) {
    double s = 0.0, s2 = 0.0;
    for (int i = threadIdx.x; i < n; i += 256) s += v[i];
    scratch[threadIdx.x] = s;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) scratch[threadIdx.x] += scratch[threadIdx.x + o];
        __syncthreads();
    }
    const double mean = scratch[0] / n;
    __syncthreads();
    for (int i = threadIdx.x; i < n; i += 256) {
        const double dlt = v[i] - mean;
        s2 += dlt * dlt;
    }
    scratch[threadIdx.x] = s2;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) scratch[threadIdx.x] += scratch[threadIdx.x + o];
        __syncthreads();
    }
    const double var = scratch[0] / n;
    __syncthreads();
    return var / (mean * mean);
}

__global__ __launch_bounds__(256) void cv2_kernel(const double *__restrict__ sums64, int n,
                                                  float w_importance, float w_load,
                                                  float *__restrict__ losses) {
    __shared__ double scratch[256];
    const double ci = block_cv2(sums64, n, scratch);
    const double cl = block_cv2(sums64 + n, n, scratch);
    if (threadIdx.x == 0) {
        losses[0] = (float)((double)w_importance * ci);
        losses[1] = (float)((double)w_load * cl);
        losses[2] = (float)ci;
        losses[3] = (float)cl;
    }
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
    double imp = 0.0;
    for (int r = p.offsets[e]; r < p.offsets[e + 1]; ++r) imp += (double)p.gate[p.perm[r]];
    double ls = 0.0;
    const int blk0 = p.p_tile_offsets[i] * p.sub, blk1 = p.p_tile_offsets[i + 1] * p.sub;
    for (int blk = blk0; blk < blk1; ++blk) ls += (double)p.s_partials[((size_t)blk * 2 + 1) * p.b + j];
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
