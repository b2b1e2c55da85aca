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

// Eq.(1) fused with what the language models put behind the layer (Appendix C, "Model
// Architecture"): out = x + keep * sigmoid(y) / (1 - drop_prob).  keep: one byte per activation
// (the dropout draw, an input), or null for no dropout; x: the layer's input, or null for no
// residual connection.
__global__ __launch_bounds__(256) void combine_epilogue_kernel(const float4 *__restrict__ out_sorted,
                                                               const float *__restrict__ gate,
                                                               const int32_t *__restrict__ inv_perm,
                                                               const float4 *__restrict__ x,
                                                               const uint32_t *__restrict__ keep,
                                                               float inv_keep_prob, float4 *__restrict__ y,
                                                               int64_t T, int d4, int k) {
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
        // the mask and the residual are requested first, so that they travel with the expert rows
        // instead of after the arithmetic on them; rows, mask and y are touched once: streaming
        uint32_t m = 0xffffffffu;
        float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
        if (keep) m = __builtin_nontemporal_load(keep + t * d4 + c);   // four mask bytes
        if (x) r = x[t * d4 + c];
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int s = 0; s < kMaxK; ++s) {
            if (s < k) {
                const float4 v = stream_load4(out_sorted + (int64_t)rows[s] * d4 + c);
                acc.x = fmaf(g[s], v.x, acc.x);
                acc.y = fmaf(g[s], v.y, acc.y);
                acc.z = fmaf(g[s], v.z, acc.z);
                acc.w = fmaf(g[s], v.w, acc.w);
            }
        }
        float4 o;
        o.x = inv_keep_prob / (1.0f + expf(-acc.x));
        o.y = inv_keep_prob / (1.0f + expf(-acc.y));
        o.z = inv_keep_prob / (1.0f + expf(-acc.z));
        o.w = inv_keep_prob / (1.0f + expf(-acc.w));
        o.x = ((m & 0xffu) ? o.x : 0.f) + r.x;
        o.y = ((m & 0xff00u) ? o.y : 0.f) + r.y;
        o.z = ((m & 0xff0000u) ? o.z : 0.f) + r.z;
        o.w = ((m & 0xff000000u) ? o.w : 0.f) + r.w;
        stream_store4(y + t * d4 + c, o);
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

extern "C" int moe_combine_epilogue(const moe_config *cfg, const float *out_sorted, const float *topk_gate,
                                    const int32_t *inv_perm, const float *x, const uint8_t *keep,
                                    float drop_prob, float *y, void *stream) {
    int st = check_config(cfg);
    if (st != MOE_OK) return st;
    if (!out_sorted || !topk_gate || !inv_perm || !y) return MOE_EINVAL;
    if (!aligned16(out_sorted) || !aligned16(y) || (x && !aligned16(x)) || (keep && ((uintptr_t)keep & 3u)))
        return MOE_EINVAL;
    if (!(drop_prob >= 0.f && drop_prob < 1.f) || (!keep && drop_prob != 0.f)) return MOE_EINVAL;
    if (cfg->T <= 0) return MOE_OK;
    hipLaunchKernelGGL(combine_epilogue_kernel, dim3((unsigned)ceil_div(cfg->T, 4)), dim3(256), 0,
                       (hipStream_t)stream, (const float4 *)out_sorted, topk_gate, inv_perm, (const float4 *)x,
                       (const uint32_t *)keep, 1.0f / (1.0f - drop_prob), (float4 *)y, (int64_t)cfg->T, cfg->d / 4,
                       cfg->k);
    MOE_LAUNCH_CHECK();
    return MOE_OK;
}
