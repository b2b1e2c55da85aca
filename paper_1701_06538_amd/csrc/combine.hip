// a4: y_t = sum_s gate[t,s] * out_sorted[inv_perm[t*k+s]]  (Eq.(1); with products of primary
// and secondary gates it is Eq.(12)).  One wavefront per token, 16-byte accesses, slots
// accumulated in ascending s so the result does not depend on scheduling.
#include "stages.h"
#include "device_bodies.h"

namespace moe {

__global__ __launch_bounds__(256) void combine_kernel(const float4 *__restrict__ out_sorted,
                                                      const float *__restrict__ gate,
                                                      const int32_t *__restrict__ inv_perm,
                                                      float4 *__restrict__ y, int64_t T, int d4, int k) {
    combine_body(out_sorted, gate, inv_perm, y, T, d4, k, blockIdx.x);
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
