// Host-side pieces of the ABI: status strings, shape validation, workspace layout and the
// composition of the five stages into moe_layer_forward (Eq.(1)-(11) end to end, one stream,
// no host synchronisation: counts, offsets and the tile table stay on the device).
#include "stages.h"

namespace moe {

thread_local int g_last_hip_error = 0;

int check_gate_level(int64_t T, int d, int n, int k) {
    if (T < 0 || d <= 0 || n <= 0 || k <= 0) return MOE_EINVAL;
    if (k > n) return MOE_EINVAL;
    if (k > kMaxK) return MOE_EUNSUPPORTED;
    if (d % 32 != 0) return MOE_EUNSUPPORTED;
    if (n > kMaxGateExperts) return MOE_EUNSUPPORTED;
    return MOE_OK;
}

int check_config(const moe_config *cfg) {
    if (!cfg) return MOE_EINVAL;
    if (cfg->T < 0 || cfg->d <= 0 || cfg->h <= 0 || cfg->n <= 0 || cfg->k <= 0) return MOE_EINVAL;
    if (cfg->k > cfg->n) return MOE_EINVAL;
    if (cfg->expert_dtype != MOE_DTYPE_F32 && cfg->expert_dtype != MOE_DTYPE_BF16) return MOE_EINVAL;
    if (cfg->a < 0 || cfg->b < 0) return MOE_EINVAL;
    if (cfg->a > 0) {
        if (cfg->b <= 0 || cfg->k_primary <= 0 || cfg->k_secondary <= 0) return MOE_EINVAL;
        if ((int64_t)cfg->a * cfg->b != cfg->n) return MOE_EINVAL;
        if (cfg->k_primary * cfg->k_secondary != cfg->k) return MOE_EINVAL;
        if (cfg->k_primary > cfg->a || cfg->k_secondary > cfg->b) return MOE_EINVAL;
    } else if (cfg->b != 0 || cfg->k_primary != 0 || cfg->k_secondary != 0) {
        return MOE_EINVAL;
    }
    if (cfg->k > kMaxK) return MOE_EUNSUPPORTED;
    if (cfg->n > kMaxExperts) return MOE_EUNSUPPORTED;
    if (cfg->d % 32 != 0 || cfg->h % 4 != 0) return MOE_EUNSUPPORTED;
    if ((int64_t)cfg->T * cfg->k * (int64_t)(cfg->d > cfg->h ? cfg->d : cfg->h) >= (int64_t)1 << 40)
        return MOE_EUNSUPPORTED;
    if ((int64_t)cfg->T * cfg->k >= (int64_t)1 << 31) return MOE_EUNSUPPORTED;
    return MOE_OK;
}

}  // namespace moe

using namespace moe;

extern "C" int moe_version(void) { return 100; }

extern "C" const char *moe_strerror(int status) {
    switch (status) {
        case MOE_OK: return "ok";
        case MOE_EINVAL: return "invalid argument (null/misaligned pointer or inconsistent shape)";
        case MOE_EUNSUPPORTED: return "shape or dtype outside what the kernels support";
        case MOE_EWORKSPACE: return "workspace too small";
        case MOE_EHIP: return "a HIP runtime call failed (see moe_last_hip_error)";
        default: return "unknown status";
    }
}

extern "C" int moe_last_hip_error(void) { return g_last_hip_error; }
