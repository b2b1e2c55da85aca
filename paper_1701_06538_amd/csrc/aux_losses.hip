// a5: Importance(X) = sum_x G(x) (Eq.(6)), Load(X) = sum_x P(x,.) (Eq.(10)) and the two
// CV^2 losses (Eq.(7),(11)).  The gating kernel leaves per-block fp32 partial sums; here they
// are added in a fixed order in fp64 and the coefficient of variation (population variance,
// no epsilon) is evaluated in fp64.
#include "stages.h"

namespace moe {

// out[which][i] = sum over rows r in [row_begin(i-group), row_end) of partials[r][which][i]
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float *__restrict__ partials,
                                                              int64_t rows, int n,
                                                              float *__restrict__ importance,
                                                              float *__restrict__ load,
                                                              double *__restrict__ sums64) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= 2 * n) return;
    double acc = 0.0;
    for (int64_t r = 0; r < rows; ++r) acc += (double)partials[r * 2 * n + i];
    sums64[i] = acc;
    if (i < n) importance[i] = (float)acc;
    else load[i - n] = (float)acc;
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
    hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)ceil_div(2 * n, 256)), dim3(256), 0,
                       st, partials, rows, n, importance, load, sums64);
    MOE_LAUNCH_CHECK();
    hipLaunchKernelGGL(cv2_kernel, dim3(1), dim3(256), 0, st, sums64, n, w_imp, w_load, losses);
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}

}  // namespace moe
