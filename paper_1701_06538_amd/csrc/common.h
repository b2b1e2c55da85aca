// Internal helpers of the HIP library (host-side checks, launch error capture, small device
// utilities).  Not part of the ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "../../include/moe.h"

namespace moe {

extern thread_local int g_last_hip_error;

inline int hip_fail(hipError_t e) {
    g_last_hip_error = (int)e;
    return MOE_EHIP;
}

#define MOE_HIP_TRY(expr)                                   \
    do {                                                    \
        hipError_t e__ = (expr);                            \
        if (e__ != hipSuccess) return ::moe::hip_fail(e__); \
    } while (0)

// after a kernel launch: catches bad launch configurations without synchronising
#define MOE_LAUNCH_CHECK() MOE_HIP_TRY(hipGetLastError())

// Raises a kernel's dynamic-LDS limit the first time it is needed.  Entry points may be called
// from several host threads (distinct streams and buffers), so the "first time" is a
// std::call_once; the attribute call's status is kept and reported by every caller.
struct LdsLimitOnce {
    std::once_flag flag;
    hipError_t status = hipSuccess;
    int set(const void *kernel, size_t bytes) {
        std::call_once(flag, [&] {
            status = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
        });
        return status == hipSuccess ? (int)MOE_OK : hip_fail(status);
    }
};
#define MOE_TRY(expr)                    \
    do {                                 \
        const int rc__ = (expr);         \
        if (rc__ != MOE_OK) return rc__; \
    } while (0)

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Shape checks shared by every entry point.  Returns MOE_OK or the status to report.
int check_config(const moe_config *cfg);
// Checks of one gating level (n experts, k kept).
int check_gate_level(int64_t T, int d, int n, int k);

constexpr int kGateBM = 128;       // rows per block tile of the logits kernel
constexpr int kMaxK = 8;
constexpr int kMaxExperts = 16384;   // route histograms live in 64 KB of LDS
constexpr int kMaxGateExperts = 16384;  // experts of one gating level (the wide top-k kernel walks 2048-column chunks)
constexpr int kMaxBalancedExperts = 2048;  // strictly balanced gating: one column-selection workgroup per expert, softmax rows in registers

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Accesses to data that crosses HBM exactly once per call (expert weights with one tile per expert,
// expert output rows, the layer output): the non-temporal hint keeps them from displacing what is
// re-read (token rows, weights shared by several tiles) in L2.  Measured on the expert kernel at
// 16384 experts: 6.1 -> 5.4 ms.
#define MOE_STREAM_LOAD(ptr) __builtin_nontemporal_load(ptr)
#define MOE_STREAM_STORE(val, ptr) __builtin_nontemporal_store((val), (ptr))
typedef float f32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 stream_load4(const float4 *p) {
    const f32x4_t v = MOE_STREAM_LOAD(reinterpret_cast<const f32x4_t *>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void stream_store4(float4 *p, float4 v) {
    MOE_STREAM_STORE((f32x4_t{v.x, v.y, v.z, v.w}), reinterpret_cast<f32x4_t *>(p));
}

// Two fp32 values rounded to bf16 (nearest, ties to even) and packed, lo in bits 0-15: one
// v_cvt_pk_bf16_f32 on gfx950.  For every finite input, denormals included, the result equals
// the integer form (bits + 0x7fff + bit 16, shifted right by 16); NaNs are quieted, and no
// input here is one.
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16_pair(float lo, float hi) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{lo, hi}, bf16x2_t));
}
__device__ __forceinline__ uint32_t bf16_bits_of(float f) { return pack_bf16_pair(f, 0.f) & 0xffffu; }

}  // namespace moe
