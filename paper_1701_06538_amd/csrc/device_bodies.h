// Device-side bodies of the small latency-bound kernels.  Each is used by its own kernel and by
// the fused launches of the layer forward (fused.hip), where blocks of two independent stages
// share one grid so that neither pays a launch of its own.
#pragma once
#include "stages.h"

namespace moe {

// Small problems (n <= 512, A <= 65536) in ONE launch: every workgroup rebuilds the two
// histograms it needs by reading the whole (L2-resident) assignment list -- totals, and counts
// of everything ahead of its own 1024-assignment chunk -- so no cross-workgroup scan is needed;
// it then scatters its chunk with the same ordered, ballot-ranked walk, one 256-assignment
// sub-chunk per wave.
constexpr int kSmallChunk = 1024;
constexpr int kSmallMaxN = 512;

// `block` is the index of the 1024-assignment chunk; lds_s holds total[n] | before[n] | wavehist[4][n].
__device__ __forceinline__ void route_small_body(const RouteArgs &p, int nbits, int block, int *lds_s) {
    __shared__ int wave_sums[4];
    const int n = p.n, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int *total = lds_s, *before = lds_s + n, *wh = lds_s + 2 * n;
    for (int i = tid; i < 6 * n; i += 256) lds_s[i] = 0;
    __syncthreads();
    const int64_t c0 = (int64_t)block * kSmallChunk;
    const int64_t c1 = min(c0 + kSmallChunk, p.A);
    // One LDS atomic per assignment: it falls before the chunk, into one of the chunk's four
    // 256-assignment quarters, or after the chunk (that last bin temporarily lives in total[]).
    auto count_one = [&](int64_t a, int e) {
        if (e >= 0 && e < n) {
            int *bin = a < c0 ? &before[e] : a < c1 ? &wh[((a - c0) >> 8) * n + e] : &total[e];
            atomicAdd(bin, 1);   // integer counts: order-independent
        }
    };
    if ((reinterpret_cast<uintptr_t>(p.idx) & 15) == 0) {
        // 16-byte loads, eight in flight per thread: the whole list takes A / 8192 round trips
        const int64_t n4 = p.A >> 2;
        const int4 *idx4 = reinterpret_cast<const int4 *>(p.idx);
        for (int64_t base = 0; base < n4; base += 256 * 8) {
            int4 ev8[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int64_t g = base + 256 * u + tid;
                ev8[u] = g < n4 ? idx4[g] : make_int4(-1, -1, -1, -1);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int64_t a = 4 * (base + 256 * u + tid);
                count_one(a, ev8[u].x);
                count_one(a + 1, ev8[u].y);
                count_one(a + 2, ev8[u].z);
                count_one(a + 3, ev8[u].w);
            }
        }
        const int64_t a = 4 * n4 + tid;
        if (a < p.A) count_one(a, p.idx[a]);
    } else {
        for (int64_t base = 0; base < p.A; base += 256 * 8) {
            int ev8[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {   // eight independent loads in flight
                const int64_t a = base + 256 * u + tid;
                ev8[u] = a < p.A ? p.idx[a] : -1;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) count_one(base + 256 * u + tid, ev8[u]);
        }
    }
    __syncthreads();
    // totals = before + the chunk's quarters + after
    for (int e = tid; e < n; e += 256)
        total[e] += before[e] + wh[e] + wh[n + e] + wh[2 * n + e] + wh[3 * n + e];
    __syncthreads();
    // exclusive scan of the totals over experts: two adjacent experts per thread
    const int TM = p.tile_rows;
    {
        const int e0 = 2 * tid, e1 = 2 * tid + 1;
        const int v0 = e0 < n ? total[e0] : 0, v1 = e1 < n ? total[e1] : 0;
        const int t0 = (v0 + TM - 1) / TM, t1 = (v1 + TM - 1) / TM;
        int rows_inc = v0 + v1, tiles_inc = t0 + t1;
        // block scan over 256 threads (4 waves)
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int o = __shfl_up(rows_inc, off);
            const int o2 = __shfl_up(tiles_inc, off);
            if (lane >= off) {
                rows_inc += o;
                tiles_inc += o2;
            }
        }
        if (lane == 63) wave_sums[wave] = rows_inc;
        __syncthreads();
        int add = 0;
        for (int w = 0; w < wave; ++w) add += wave_sums[w];
        __syncthreads();
        if (lane == 63) wave_sums[wave] = tiles_inc;
        __syncthreads();
        int tadd = 0;
        for (int w = 0; w < wave; ++w) tadd += wave_sums[w];
        rows_inc += add;
        tiles_inc += tadd;
        const int off0 = rows_inc - v0 - v1, off1 = off0 + v0;
        const int toff0 = tiles_inc - t0 - t1, toff1 = toff0 + t0;
        // cursors: offsets + assignments ahead of this chunk + earlier waves of this chunk
        if (e0 < n) {
            int run = off0 + before[e0];
            for (int w = 0; w < 4; ++w) {
                const int v = wh[w * n + e0];
                wh[w * n + e0] = run;
                run += v;
            }
        }
        if (e1 < n) {
            int run = off1 + before[e1];
            for (int w = 0; w < 4; ++w) {
                const int v = wh[w * n + e1];
                wh[w * n + e1] = run;
                run += v;
            }
        }
        if (block == 0) {
            if (e0 < n) {
                p.counts[e0] = v0;
                p.offsets[e0] = off0;
                if (p.tile_offsets) p.tile_offsets[e0] = toff0;
                for (int j = 0; j < t0; ++j) {
                    p.tile_expert[toff0 + j] = e0;
                    p.tile_row0[toff0 + j] = off0 + j * TM;
                }
            }
            if (e1 < n) {
                p.counts[e1] = v1;
                p.offsets[e1] = off1;
                if (p.tile_offsets) p.tile_offsets[e1] = toff1;
                for (int j = 0; j < t1; ++j) {
                    p.tile_expert[toff1 + j] = e1;
                    p.tile_row0[toff1 + j] = off1 + j * TM;
                }
            }
            if (tid == 255) {
                p.offsets[n] = rows_inc;
                if (p.tile_offsets) p.tile_offsets[n] = tiles_inc;
                p.num_tiles[0] = tiles_inc;
            }
        }
    }
    __syncthreads();
    // ordered scatter of this wave's 256 assignments
    int *my = wh + wave * n;
    const int64_t a0 = c0 + 256 * wave;
    int ev[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const int64_t a = a0 + 64 * s + lane;
        int e = -1;
        if (a < c1) {
            e = p.idx[a];
            if (e < 0 || e >= n) e = -1;
        }
        ev[s] = e;
    }
    const unsigned long long lt_mask = (1ull << lane) - 1ull;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const int64_t a = a0 + 64 * s + lane;
        const int ex = ev[s];
        const bool active = ex >= 0;
        unsigned long long same = __ballot(active);
        for (int b = 0; b < nbits; ++b) {
            const bool bit = (ex >> b) & 1;
            const unsigned long long bal = __ballot(active && bit);
            same &= bit ? bal : ~bal;
        }
        if (active) {
            const int rank = __popcll(same & lt_mask);
            const int c = __popcll(same);
            const int before_me = my[ex];
            const int pos = before_me + rank;
            p.perm[pos] = (int32_t)a;
            p.inv_perm[a] = pos;
            if (rank == c - 1) my[ex] = before_me + c;  // issued after every lane's read
        }
    }
}


// ---------------------------------------------------------------------------------------
// Importance / Load sums and CV^2 (Eq.(6),(7),(10),(11))
// ---------------------------------------------------------------------------------------

// Level 1: level2[chunk][i] = sum of partials[r][i] over the chunk's 128 rows (i runs over the
// 2n importance|load columns).  A block covers 32 columns x 8 row groups, every thread adds its
// 16 rows (all loads independent) in fp64, the eight group sums are added in ascending order.
constexpr int kAuxChunkRows = 128;

__device__ __forceinline__ void reduce_partials_body(const float *__restrict__ partials, int64_t rows,
                                                     int n, double *__restrict__ level2, int bx, int by) {
    __shared__ double part[8][33];
    const int cx = threadIdx.x & 31, rg = threadIdx.x >> 5;
    const int i = bx * 32 + cx;
    const int64_t r0 = (int64_t)by * kAuxChunkRows;
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
        level2[(size_t)by * 2 * n + i] = s;
    }
}

// Level 2: add the chunk sums in ascending chunk order, publish Importance and Load.  Thread
// `first` of `stride` handles columns first, first + stride, ...
__device__ __forceinline__ void finish_sums_body(const double *__restrict__ level2, int chunks, int n,
                                                 double *__restrict__ sums64,
                                                 float *__restrict__ importance,
                                                 float *__restrict__ load, int first, int stride) {
    for (int i = first; i < 2 * n; i += stride) {
        double s = 0.0;
        for (int c = 0; c < chunks; ++c) s += level2[(size_t)c * 2 * n + i];
        sums64[i] = s;
        if (!importance) continue;
        if (i < n) importance[i] = (float)s;
        else load[i - n] = (float)s;
    }
}

// sum over the block's 256 threads in a fixed order: butterfly inside each wavefront, then the
// four wavefront sums in ascending order
__device__ __forceinline__ double block_sum256(double v, double *scratch4) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    if ((threadIdx.x & 63) == 0) scratch4[threadIdx.x >> 6] = v;
    __syncthreads();
    const double t = ((scratch4[0] + scratch4[1]) + scratch4[2]) + scratch4[3];
    __syncthreads();
    return t;
}

// one block of 256 threads: CV^2 of v[0..n) in fp64 (population variance, no epsilon)
__device__ __forceinline__ double block_cv2(const double *v, int n, double *scratch4) {
    // a thread's elements are fetched eight at a time (independent loads, one round trip) and
    // added in ascending order, so the sum does not depend on how the loads are batched
    double s = 0.0, s2 = 0.0;
    for (int i0 = threadIdx.x; i0 < n; i0 += 8 * 256) {
        double t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) t[u] = i0 + 256 * u < n ? v[i0 + 256 * u] : 0.0;
#pragma unroll
        for (int u = 0; u < 8; ++u) s += t[u];
    }
    const double mean = block_sum256(s, scratch4) / n;
    for (int i0 = threadIdx.x; i0 < n; i0 += 8 * 256) {
        double t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) t[u] = i0 + 256 * u < n ? v[i0 + 256 * u] - mean : 0.0;
#pragma unroll
        for (int u = 0; u < 8; ++u) s2 += t[u] * t[u];
    }
    const double var = block_sum256(s2, scratch4) / n;
    return var / (mean * mean);
}

__device__ __forceinline__ void cv2_body(const double *__restrict__ sums64, int n, float w_importance,
                                         float w_load, float *__restrict__ losses) {
    __shared__ double scratch[4];
    const double ci = block_cv2(sums64, n, scratch);
    const double cl = block_cv2(sums64 + n, n, scratch);
    if (threadIdx.x == 0) {
        losses[0] = (float)((double)w_importance * ci);
        losses[1] = (float)((double)w_load * cl);
        losses[2] = (float)ci;
        losses[3] = (float)cl;
    }
}

// ---------------------------------------------------------------------------------------
// combine (Eq.(1)): block `block` handles tokens 4*block .. 4*block+3, one wavefront each
// ---------------------------------------------------------------------------------------
// One token with k = KC known at compile time (KC = 0: any k up to kMaxK, slot by slot): the row
// loads of a column are all issued before the first multiply-add waits for one of them.
template <int KC>
__device__ __forceinline__ void combine_token(const float4 *__restrict__ out_sorted,
                                              const float *__restrict__ gate,
                                              const int32_t *__restrict__ inv_perm,
                                              float4 *__restrict__ y, int64_t t, int d4, int k, int lane) {
    constexpr int KN = KC ? KC : kMaxK;
    int rows[KN];
    float g[KN];
#pragma unroll
    for (int s = 0; s < KN; ++s) {
        rows[s] = s < k ? inv_perm[t * k + s] : 0;
        g[s] = s < k ? gate[t * k + s] : 0.f;
    }
    auto column = [&](int c) {
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        if (KC) {
            float4 v[KN];
#pragma unroll
            for (int s = 0; s < KN; ++s)   // every expert output row is read exactly once: streaming loads
                v[s] = stream_load4(out_sorted + (int64_t)rows[s] * d4 + c);
#pragma unroll
            for (int s = 0; s < KN; ++s) {
                acc.x = fmaf(g[s], v[s].x, acc.x);
                acc.y = fmaf(g[s], v[s].y, acc.y);
                acc.z = fmaf(g[s], v[s].z, acc.z);
                acc.w = fmaf(g[s], v[s].w, acc.w);
            }
        } else {
#pragma unroll
            for (int s = 0; s < KN; ++s) {
                if (s < k) {
                    const float4 v = stream_load4(out_sorted + (int64_t)rows[s] * d4 + c);
                    acc.x = fmaf(g[s], v.x, acc.x);
                    acc.y = fmaf(g[s], v.y, acc.y);
                    acc.z = fmaf(g[s], v.z, acc.z);
                    acc.w = fmaf(g[s], v.w, acc.w);
                }
            }
        }
        stream_store4(y + t * d4 + c, acc);
    };
    if (d4 == 128) {
        // the paper's d = 512: both 16-byte columns of a lane at once
#pragma unroll
        for (int i = 0; i < 2; ++i) column(lane + 64 * i);
    } else {
        for (int c = lane; c < d4; c += 64) column(c);
    }
}

__device__ __forceinline__ void combine_body(const float4 *__restrict__ out_sorted,
                                             const float *__restrict__ gate,
                                             const int32_t *__restrict__ inv_perm,
                                             float4 *__restrict__ y, int64_t T, int d4, int k,
                                             int64_t block) {
    const int lane = threadIdx.x & 63;
    const int64_t t = block * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    // slots in ascending order in every form: the same sequence of fused multiply-adds
    if (k == 4) combine_token<4>(out_sorted, gate, inv_perm, y, t, d4, k, lane);
    else if (k == 2) combine_token<2>(out_sorted, gate, inv_perm, y, t, d4, k, lane);
    else if (k == 1) combine_token<1>(out_sorted, gate, inv_perm, y, t, d4, k, lane);
    else combine_token<0>(out_sorted, gate, inv_perm, y, t, d4, k, lane);
}

}  // namespace moe
