// a5: Importance(X) = sum_x G(x) (Eq.(6)), Load(X) = sum_x P(x,.) (Eq.(10)) and the two
// CV^2 losses (Eq.(7),(11)).  The gating kernel leaves per-block fp32 partial sums; here they
// are added in a fixed order in fp64 and the coefficient of variation (population variance,
// no epsilon) is evaluated in fp64.
#include "stages.h"

namespace moe {

// sums64[which*n + i] = sum over rows r of partials[r][which][i], added in a fixed order:
// a block covers 32 columns x 8 row groups; each thread adds rows rg, rg+8, ... in fp64 and the
// eight group sums are added in ascending group order.
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float *__restrict__ partials,
                                                              int64_t rows, int n,
                                                              float *__restrict__ importance,
                                                              float *__restrict__ load,
                                                              double *__restrict__ sums64) {
    __shared__ double part[8][33];
    const int cx = threadIdx.x & 31, rg = threadIdx.x >> 5;
    const int i = blockIdx.x * 32 + cx;
    double acc = 0.0;
    if (i < 2 * n) {
        const float *col = partials + i;
        int64_t r = rg;
        for (; r + 24 < rows; r += 32) {
            const float v0 = col[r * 2 * n], v1 = col[(r + 8) * 2 * n];
            const float v2 = col[(r + 16) * 2 * n], v3 = col[(r + 24) * 2 * n];
            acc += (double)v0;
            acc += (double)v1;
            acc += (double)v2;
            acc += (double)v3;
        }
        for (; r < rows; r += 8) acc += (double)col[r * 2 * n];
    }
    part[rg][cx] = acc;
    __syncthreads();
    if (rg == 0 && i < 2 * n) {
        double s = part[0][cx];
#pragma unroll
        for (int q = 1; q < 8; ++q) s += part[q][cx];
        sums64[i] = s;
        if (i < n) importance[i] = (float)s;
        else load[i - n] = (float)s;
    }
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
                      float *importance, float *load, float *losses, double *sums64,
                      hipStream_t st) {
    hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)ceil_div(2 * n, 32)), dim3(256), 0,
                       st, partials, rows, n, importance, load, sums64);
    MOE_LAUNCH_CHECK();
    hipLaunchKernelGGL(cv2_kernel, dim3(1), dim3(256), 0, st, sums64, n, w_imp, w_load, losses);
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}

}  // namespace moe
