// a4: y_t = sum_s gate[t,s] * out_sorted[inv_perm[t*k+s]]  (Eq.(1); with products of primary
// and secondary gates it is Eq.(12)).  One wavefront per token, 16-byte accesses, slots
// accumulated in ascending s so the result does not depend on scheduling.
#include "stages.h"

namespace moe {

__global__ __launch_bounds__(256) void combine_kernel(const float4 *__restrict__ out_sorted,
                                                      const float *__restrict__ gate,
                                                      const int32_t *__restrict__ inv_perm,
                                                      float4 *__restrict__ y, int64_t T, int d4, int k) {
    const int lane = threadIdx.x & 63;
    const int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    int rows[kMaxK];
    float g[kMaxK];
#pragma unroll
    for (int s = 0; s < kMaxK; ++s) {
        rows[s] = s < k ? inv_perm[t * k + s] : 0;
        g[s] = s < k ? gate[t * k + s] : 0.f;
    }
    for (int c = lane; c < d4; c += 64) {
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int s = 0; s < kMaxK; ++s) {
            if (s < k) {
                const float4 v = out_sorted[(int64_t)rows[s] * d4 + c];
                acc.x = fmaf(g[s], v.x, acc.x);
                acc.y = fmaf(g[s], v.y, acc.y);
                acc.z = fmaf(g[s], v.z, acc.z);
                acc.w = fmaf(g[s], v.w, acc.w);
            }
        }
        y[t * d4 + c] = acc;
    }
}

int launch_combine(const float *out_sorted, const float *gate, const int32_t *inv_perm, float *y,
                   int64_t T, int d, int k, hipStream_t st) {
    if (T <= 0) return MOE_OK;
    hipLaunchKernelGGL(combine_kernel, dim3((unsigned)ceil_div(T, 4)), dim3(256), 0, st,
                       (const float4 *)out_sorted, gate, inv_perm, (float4 *)y, T, d / 4, k);
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}

}  // namespace moe

using namespace moe;

extern "C" int moe_combine(const moe_config *cfg, const float *out_sorted, const float *topk_gate,
                           const int32_t *inv_perm, float *y, void *stream) {
    int st = check_config(cfg);
    if (st != MOE_OK) return st;
    if (!out_sorted || !topk_gate || !inv_perm || !y) return MOE_EINVAL;
    if (!aligned16(out_sorted) || !aligned16(y)) return MOE_EINVAL;
    return launch_combine(out_sorted, topk_gate, inv_perm, y, cfg->T, cfg->d, cfg->k,
                          (hipStream_t)stream);
}
