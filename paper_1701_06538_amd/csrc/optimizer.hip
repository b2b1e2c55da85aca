// Adam with beta1 = 0 and a factored second-moment estimator for the expert matrices (Appendix D):
// per matrix [R, C] only the row-wise and column-wise averages of the second-moment matrix are kept
// (R + C numbers instead of R*C); the estimator used in the step is their outer product divided by
// their common mean.  Three launches, all bound by HBM traffic:
//
//   adam_moments_kernel   one pass over the gradients: a workgroup takes 64 whole rows of one
//                         matrix, finishes their row sums of squares and writes its share of the
//                         column sums (per row block, so that the order of addition is fixed)
//   adam_vectors_kernel   per matrix: the two vectors' recursion, their mean, the step's scale
//   adam_update_kernel    elementwise update of the fp32 parameters and refresh of the bf16 copy
#include "stages.h"

namespace moe {

constexpr int kAdamRB = 64;   // rows per workgroup of the moments pass

struct AdamMat {
    const float *G;     // [count, R, C]
    int R, C, count;
    double *rowsum;     // [count, R]
    double *colpart;    // [count, ceil(R/64), C]
};

// Rows of up to 256*NJ floats: a wavefront owns whole rows (w, w+4, ... of the block), so a row sum
// is one wave reduction and goes straight to memory; the four waves' column sums meet in LDS and
// are added in wave order.  blockIdx.x = row block, blockIdx.y = expert.
template <int NJ>
__global__ __launch_bounds__(256) void adam_moments_kernel(AdamMat m) {
    extern __shared__ double col_part[];            // [4][C]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int R = m.R, C = m.C, C4 = C >> 2;
    const int rb = blockIdx.x, e = blockIdx.y;
    const int nrb = (R + kAdamRB - 1) / kAdamRB;
    const int r0 = rb * kAdamRB, rows = min(kAdamRB, R - r0);
    const float4 *G = reinterpret_cast<const float4 *>(m.G + ((size_t)e * R + r0) * C);
    double cs[NJ][4];
#pragma unroll
    for (int j = 0; j < NJ; ++j) cs[j][0] = cs[j][1] = cs[j][2] = cs[j][3] = 0.0;
    int c4[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) c4[j] = min(lane + 64 * j, C4 - 1);     // clamped: masked below
#pragma unroll 2
    for (int r = wave; r < rows; r += 4) {
        float4 g[NJ];
#pragma unroll
        for (int j = 0; j < NJ; ++j) g[j] = G[(size_t)r * C4 + c4[j]];
        double rs = 0.0;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const bool on = lane + 64 * j < C4;
            const double q0 = on ? (double)g[j].x * g[j].x : 0.0, q1 = on ? (double)g[j].y * g[j].y : 0.0,
                         q2 = on ? (double)g[j].z * g[j].z : 0.0, q3 = on ? (double)g[j].w * g[j].w : 0.0;
            cs[j][0] += q0; cs[j][1] += q1; cs[j][2] += q2; cs[j][3] += q3;
            rs += (q0 + q1) + (q2 + q3);
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) rs += __shfl_xor(rs, off);
        if (lane == 0) m.rowsum[(size_t)e * R + r0 + r] = rs;
    }
#pragma unroll
    for (int j = 0; j < NJ; ++j)
        if (lane + 64 * j < C4) {
            double *dst = col_part + (size_t)wave * C + 4 * (lane + 64 * j);
            dst[0] = cs[j][0]; dst[1] = cs[j][1]; dst[2] = cs[j][2]; dst[3] = cs[j][3];
        }
    __syncthreads();
    double *colpart = m.colpart + ((size_t)e * nrb + rb) * C;
    for (int c = tid; c < C; c += 256)
        colpart[c] = ((col_part[c] + col_part[C + c]) + col_part[2 * C + c]) + col_part[3 * C + c];
}

// Any row length: every wavefront takes a quarter of each row (blockIdx.x = row block,
// blockIdx.y = expert).
__global__ __launch_bounds__(256) void adam_moments_wide_kernel(AdamMat m) {
    __shared__ double row_part[kAdamRB][4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int R = m.R, C = m.C, C4 = C >> 2;
    const int rb = blockIdx.x, e = blockIdx.y;
    const int nrb = (R + kAdamRB - 1) / kAdamRB;
    const int r0 = rb * kAdamRB, rows = min(kAdamRB, R - r0);
    const float4 *G = reinterpret_cast<const float4 *>(m.G + ((size_t)e * R + r0) * C);
    double *colpart = m.colpart + ((size_t)e * nrb + rb) * C;

    for (int c0 = 0; c0 < C4; c0 += 256) {          // column panels of 1024
        const int c4 = c0 + tid;
        const bool on = c4 < C4;
        double cs[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll 4
        for (int r = 0; r < rows; ++r) {
            float4 g = make_float4(0.f, 0.f, 0.f, 0.f);
            if (on) g = G[(size_t)r * C4 + c4];
            const double q0 = (double)g.x * g.x, q1 = (double)g.y * g.y, q2 = (double)g.z * g.z,
                         q3 = (double)g.w * g.w;
            cs[0] += q0; cs[1] += q1; cs[2] += q2; cs[3] += q3;
            double rs = (q0 + q1) + (q2 + q3);
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) rs += __shfl_xor(rs, off);
            if (lane == 0) {
                if (c0 == 0) row_part[r][wave] = rs;
                else row_part[r][wave] += rs;       // same wave, same slot: ordered
            }
        }
        if (on) {
            colpart[4 * c4] = cs[0];
            colpart[4 * c4 + 1] = cs[1];
            colpart[4 * c4 + 2] = cs[2];
            colpart[4 * c4 + 3] = cs[3];
        }
    }
    __syncthreads();
    if (tid < rows)
        m.rowsum[(size_t)e * R + r0 + tid] =
            ((row_part[tid][0] + row_part[tid][1]) + row_part[tid][2]) + row_part[tid][3];
}

struct AdamVec {
    const double *rowsum, *colpart;      // own moments pass: rowsum [count, R], colpart [count, nrb, C]
    const float *rowpart_f, *colpart_f;  // or the weight-gradient kernel's: [count, nrp, R], [count, ncp, C]
    int nrp, ncp;
    float *v_row, *v_col;   // [count, R], [count, C]
    float *scale;           // [count]: 1 / (mean(v_row) * (1 - beta2^step)), or -1 when the mean is 0
    int R, C;
    float beta2, bias_corr;   // bias_corr = 1 - beta2^step
};

__global__ __launch_bounds__(256) void adam_vectors_kernel(AdamVec a) {
    __shared__ double red[256];
    const int e = blockIdx.x, tid = threadIdx.x;
    const int R = a.R, C = a.C, nrb = (R + kAdamRB - 1) / kAdamRB;
    const double b2 = (double)a.beta2, ob2 = 1.0 - b2;
    double msum = 0.0;
    for (int r = tid; r < R; r += 256) {
        double rsum = 0.0;
        if (a.rowpart_f) {
            for (int q = 0; q < a.nrp; ++q) rsum += (double)a.rowpart_f[((size_t)e * a.nrp + q) * R + r];
        } else {
            rsum = a.rowsum[(size_t)e * R + r];
        }
        const double v = b2 * (double)a.v_row[(size_t)e * R + r] + ob2 * (rsum / C);
        const float vf = (float)v;
        a.v_row[(size_t)e * R + r] = vf;
        msum += (double)vf;
    }
    for (int c = tid; c < C; c += 256) {
        double s = 0.0;
        if (a.colpart_f) {
            for (int q = 0; q < a.ncp; ++q) s += (double)a.colpart_f[((size_t)e * a.ncp + q) * C + c];
        } else {
            for (int rb = 0; rb < nrb; ++rb) s += a.colpart[((size_t)e * nrb + rb) * C + c];
        }
        a.v_col[(size_t)e * C + c] = (float)(b2 * (double)a.v_col[(size_t)e * C + c] + ob2 * (s / R));
    }
    red[tid] = msum;
    __syncthreads();
    if (tid == 0) {
        double t = 0.0;
        for (int i = 0; i < 256; ++i) t += red[i];
        const double mean = t / R;
        a.scale[e] = mean > 0.0 ? (float)(1.0 / (mean * (double)a.bias_corr)) : -1.0f;
    }
}

struct AdamUpd {
    const float *G;
    float *master;          // [count, R, C] fp32 parameters
    uint16_t *copy;         // bf16 copy or null
    const float *v_row, *v_col, *scale;
    int R, C;
    float lr, eps;
};


// one workgroup per 4 rows of one matrix (blockIdx.y = matrix)
__global__ __launch_bounds__(256) void adam_update_kernel(AdamUpd a) {
    const int e = blockIdx.y, C4 = a.C >> 2;
    const float s = a.scale[e];
    const bool moves = s >= 0.f;                       // no gradient history: the parameters stay
    if (!moves && !a.copy) return;
    const float *vcol = a.v_col + (size_t)e * a.C;
    for (int rr = 0; rr < 4; ++rr) {
        const int r = blockIdx.x * 4 + rr;
        if (r >= a.R) return;
        const float vr = a.v_row[(size_t)e * a.R + r] * s;
        const size_t base = ((size_t)e * a.R + r) * C4;
        for (int c4 = threadIdx.x; c4 < C4; c4 += 256) {
            // gradient and parameter cross HBM once per step: streaming loads and stores
            const float4 g = stream_load4(reinterpret_cast<const float4 *>(a.G) + base + c4);
            float4 w = stream_load4(reinterpret_cast<const float4 *>(a.master) + base + c4);
            const float4 vc = reinterpret_cast<const float4 *>(vcol)[c4];
            if (moves) {
                w.x -= a.lr * g.x / (sqrtf(vr * vc.x) + a.eps);
                w.y -= a.lr * g.y / (sqrtf(vr * vc.y) + a.eps);
                w.z -= a.lr * g.z / (sqrtf(vr * vc.z) + a.eps);
                w.w -= a.lr * g.w / (sqrtf(vr * vc.w) + a.eps);
                stream_store4(reinterpret_cast<float4 *>(a.master) + base + c4, w);
            }
            if (a.copy)
                reinterpret_cast<uint2 *>(a.copy)[base + c4] =
                    make_uint2(pack_bf16_pair(w.x, w.y), pack_bf16_pair(w.z, w.w));   // round to nearest even
        }
    }
}

static size_t adam_up256(size_t v) { return (v + 255) & ~(size_t)255; }

struct AdamLayout {
    size_t rowsum[2], colpart[2], scale[2], total;
};

static void adam_layout(const moe_config *cfg, AdamLayout *L) {
    const size_t n = cfg->n, d = cfg->d, h = cfg->h;
    const size_t R[2] = {d, h}, C[2] = {h, d};
    size_t off = 0;
    for (int w = 0; w < 2; ++w) {
        L->rowsum[w] = off;
        off = adam_up256(off + n * R[w] * 8);
        L->colpart[w] = off;
        off = adam_up256(off + n * ((R[w] + kAdamRB - 1) / kAdamRB) * C[w] * 8);
        L->scale[w] = off;
        off = adam_up256(off + n * 4);
    }
    L->total = off;
}

static int adam_check(const moe_config *cfg) {
    int st = check_config(cfg);
    if (st != MOE_OK) return st;
    if (cfg->d % 4 || cfg->h % 4) return MOE_EUNSUPPORTED;
    if (cfg->n > 65535) return MOE_EUNSUPPORTED;          // matrices ride on gridDim.y
    return MOE_OK;
}

}  // namespace moe

using namespace moe;

extern "C" size_t moe_adam_workspace_bytes(const moe_config *cfg) {
    if (adam_check(cfg) != MOE_OK) return 0;
    AdamLayout L;
    adam_layout(cfg, &L);
    return L.total;
}

extern "C" int moe_expert_adam_step(const moe_config *cfg, const moe_adam_params *hp, const float *dW1,
                                    const float *dW2, float *W1_master, float *W2_master, void *W1_copy,
                                    void *W2_copy, float *v_row1, float *v_col1, float *v_row2,
                                    float *v_col2, const void *backward_workspace, void *workspace,
                                    size_t workspace_bytes, void *stream) {
    int st = adam_check(cfg);
    if (st != MOE_OK) return st;
    if (!hp || !dW1 || !dW2 || !W1_master || !W2_master || !v_row1 || !v_col1 || !v_row2 || !v_col2 || !workspace)
        return MOE_EINVAL;
    if (hp->step < 1 || !(hp->beta2 >= 0.f && hp->beta2 < 1.f) || !(hp->eps >= 0.f)) return MOE_EINVAL;
    if ((W1_copy == nullptr) != (W2_copy == nullptr)) return MOE_EINVAL;
    if (W1_copy && cfg->expert_dtype != MOE_DTYPE_BF16) return MOE_EINVAL;
    if (!aligned16(dW1) || !aligned16(dW2) || !aligned16(W1_master) || !aligned16(W2_master) ||
        !aligned16(v_col1) || !aligned16(v_col2) || !aligned16(workspace) || (W1_copy && !aligned16(W1_copy)) ||
        (W2_copy && !aligned16(W2_copy)))
        return MOE_EINVAL;
    AdamLayout L;
    adam_layout(cfg, &L);
    if (workspace_bytes < L.total) return MOE_EWORKSPACE;
    size_t mom_off[4] = {0, 0, 0, 0};
    if (backward_workspace) {
        if (!(cfg->flags & MOE_FLAG_ADAM_MOMENTS) || cfg->d % 256 || cfg->h % 256) return MOE_EINVAL;
        if ((st = backward_moments_offsets(cfg, mom_off)) != MOE_OK) return st;
    }
    hipStream_t s = (hipStream_t)stream;
    char *ws = (char *)workspace;
    const int n = cfg->n;
    const float bias_corr = (float)(1.0 - pow((double)hp->beta2, (double)hp->step));
    const float *G[2] = {dW1, dW2};
    float *M[2] = {W1_master, W2_master};
    uint16_t *Cp[2] = {(uint16_t *)W1_copy, (uint16_t *)W2_copy};
    float *vr[2] = {v_row1, v_row2}, *vc[2] = {v_col1, v_col2};
    const int R[2] = {cfg->d, cfg->h}, C[2] = {cfg->h, cfg->d};
    for (int w = 0; w < 2; ++w) {
        double *rowsum = (double *)(ws + L.rowsum[w]), *colpart = (double *)(ws + L.colpart[w]);
        float *scale = (float *)(ws + L.scale[w]);
        AdamMat am{G[w], R[w], C[w], n, rowsum, colpart};
        const float *rp = nullptr, *cp = nullptr;
        if (backward_workspace) {   // the weight-gradient kernels already summed the squares per block
            rp = (const float *)((const char *)backward_workspace + mom_off[2 * w]);
            cp = (const float *)((const char *)backward_workspace + mom_off[2 * w + 1]);
        }
        const dim3 mgrid((unsigned)ceil_div(R[w], kAdamRB), (unsigned)n);
        if (!backward_workspace) {
        const size_t mlds = (size_t)4 * C[w] * sizeof(double);
        if (C[w] <= 1024) hipLaunchKernelGGL(adam_moments_kernel<4>, mgrid, dim3(256), mlds, s, am);
        else if (C[w] <= 2048) {
            static LdsLimitOnce lds_once;
            MOE_TRY(lds_once.set((const void *)adam_moments_kernel<8>, (size_t)4 * 2048 * 8));
            hipLaunchKernelGGL(adam_moments_kernel<8>, mgrid, dim3(256), mlds, s, am);
        } else hipLaunchKernelGGL(adam_moments_wide_kernel, mgrid, dim3(256), 0, s, am);
        MOE_LAUNCH_CHECK();
        }
        AdamVec av{rowsum, colpart, rp, cp, C[w] / 256, R[w] / 256, vr[w], vc[w], scale, R[w], C[w], hp->beta2, bias_corr};
        hipLaunchKernelGGL(adam_vectors_kernel, dim3((unsigned)n), dim3(256), 0, s, av);
        MOE_LAUNCH_CHECK();
        AdamUpd au{G[w], M[w], Cp[w], vr[w], vc[w], scale, R[w], C[w], hp->lr, hp->eps};
        hipLaunchKernelGGL(adam_update_kernel, dim3((unsigned)ceil_div(R[w], 4), (unsigned)n), dim3(256), 0, s, au);
        MOE_LAUNCH_CHECK();
    }
    return MOE_OK;
}
