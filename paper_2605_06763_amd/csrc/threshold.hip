// Built-in threshold selection (appendix "Threshold Oracle Comparison"): a reservoir of R <= 256
// past keys per (sequence, KV head), kept uniform by reservoir sampling, and tau estimated from
// the query's dot products with it.
//
// Reservoir sampling in parallel.  Algorithm R processes positions in arrival order: position
// i < R fills slot i; position i >= R draws j uniform in [0, i] and overwrites slot j if j < R.
// The final occupant of a slot is therefore the LARGEST position that chose it, so any batch of
// positions can be handled by independent threads with an atomic max per accepted draw.  The
// draw is a counter-based hash of (seed, stream = sequence*H_kv + KV head, position): the
// splitmix64 finaliser, top 32 bits, j = floor(hash * (i+1) / 2^32).
#include "lvr_internal.h"

namespace {

__device__ __forceinline__ uint32_t hash32(uint64_t seed, uint64_t stream, uint64_t counter) {
    uint64_t z = seed + stream * 0xD1B54A32D192ED03ull + counter * 0x9E3779B97F4A7C15ull;
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    z ^= z >> 31;
    return (uint32_t)(z >> 32);
}

__global__ void reservoir_reset_kernel(int32_t *res, int total) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < total) res[i] = -1;
}

__global__ void reservoir_update_kernel(int32_t *res, int R, uint64_t seed, int64_t pos0, int64_t count) {
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= count) return;
    const int bh = blockIdx.y;
    const int64_t i = pos0 + k;
    int64_t j;
    if (i < R)
        j = i;
    else
        j = (int64_t)(((uint64_t)hash32(seed, (uint64_t)bh, (uint64_t)i) * (uint64_t)(i + 1)) >> 32);
    if (j < R) atomicMax(&res[(int64_t)bh * R + j], (int32_t)i);
}

// One 256-thread workgroup per query head: scores of the reservoir keys (16 lanes per row),
// bitonic sort in LDS (descending), then the rule.
template <typename KT>
__global__ void __launch_bounds__(256)
threshold_kernel(const void *__restrict__ K, const int32_t *__restrict__ pos_slot, const int32_t *__restrict__ res,
                 const float *__restrict__ q, float *__restrict__ tau_out, int R, int64_t cap_rows, int64_t n_total,
                 int n_q_heads, int n_kv_heads, int G, int mode, float param) {
    __shared__ float s[256];
    const int64_t hq = blockIdx.x;
    const int b = (int)(hq / n_q_heads), h = (int)(hq % n_q_heads);
    const int bh = b * n_kv_heads + h / G;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, sub = lane >> 4, li = lane & 15;
    float qv[8];
    {
        const float *qh = q + hq * LVR_D + li * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) qv[e] = qh[e];
    }
    const char *Kb = static_cast<const char *>(K) + (int64_t)bh * cap_rows * LVR_D * sizeof(KT);
    const int32_t *pslot = pos_slot ? pos_slot + (int64_t)bh * cap_rows : nullptr;
    const int32_t *rb = res + (int64_t)bh * R;
    for (int j0 = 0; j0 < 256; j0 += 16) {
        const int j = j0 + wave * 4 + sub;
        int pos = (j < R) ? rb[j] : -1;
        const bool valid = pos >= 0 && pos < n_total;
        if (!valid) pos = 0;
        const int64_t slot = pslot ? (int64_t)pslot[pos] : pos;
        float x[8];
        lvr_load8<KT>(Kb, n_total > 0 ? slot : 0, li, x);
        float d = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) d += qv[e] * x[e];
        d = lvr_row16_sum(d);
        if (li == 0) s[j] = valid ? d : -INFINITY;
    }
    __syncthreads();
    // bitonic sort, descending
    for (int k = 2; k <= 256; k <<= 1) {
        for (int jj = k >> 1; jj > 0; jj >>= 1) {
            const int partner = t ^ jj;
            if (partner > t) {
                const float a = s[t], c = s[partner];
                const bool desc = (t & k) == 0;
                if (desc ? (a < c) : (a > c)) {
                    s[t] = c;
                    s[partner] = a;
                }
            }
            __syncthreads();
        }
    }
    if (t == 0) {
        int m = 0;
        while (m < 256 && s[m] != -INFINITY) ++m;   // valid scores sort first
        float tau = -INFINITY;
        if (m > 0) {
            tau = s[0];
            if (mode == LVR_TAU_SAMPLE_MEAN_MAX) {
                double mean = 0.0;
                for (int i = 0; i < m; ++i) mean += (double)s[i];
                tau = (float)(0.5 * ((double)s[0] + mean / (double)m));
            } else if (mode == LVR_TAU_SAMPLE_GAP) {
                int best = 0;
                float gap = -1.0f;
                for (int i = 0; i + 1 < m; ++i) {
                    const float g = s[i] - s[i + 1];
                    if (g > gap) {
                        gap = g;
                        best = i;
                    }
                }
                tau = s[best];
            } else if (mode == LVR_TAU_SAMPLE_TOPK || mode == LVR_TAU_BUDGET) {
                int k = mode == LVR_TAU_SAMPLE_TOPK ? (int)param : (int)ceil((double)param * (double)m);
                if (k < 1) k = 1;
                if (k > m) k = m;
                tau = s[k - 1];
            }
        }
        tau_out[hq] = tau;
    }
}

}  // namespace

hipError_t lvr_launch_reservoir_reset(lvr_index *ix, hipStream_t st) {
    if (!ix->reservoir) return hipSuccess;
    const int total = lvr_n_bh(ix) * ix->cfg.reservoir_size;
    hipLaunchKernelGGL(reservoir_reset_kernel, dim3((total + 255) / 256), dim3(256), 0, st, ix->reservoir, total);
    return hipGetLastError();
}

hipError_t lvr_launch_reservoir_update(lvr_index *ix, int64_t pos0, int64_t count, hipStream_t st) {
    if (!ix->reservoir || count <= 0) return hipSuccess;
    dim3 grid((unsigned)((count + 255) / 256), (unsigned)lvr_n_bh(ix));
    hipLaunchKernelGGL(reservoir_update_kernel, grid, dim3(256), 0, st, ix->reservoir, ix->cfg.reservoir_size,
                       (uint64_t)ix->cfg.seed, pos0, count);
    return hipGetLastError();
}

hipError_t lvr_launch_threshold(lvr_index *ix, const float *q, int mode, float param, float *tau_out, hipStream_t st) {
    const int n_bhq = lvr_n_bhq(ix);
    if (ix->cfg.kv_dtype == LVR_BF16)
        hipLaunchKernelGGL(threshold_kernel<lvr_bf16_t>, dim3((unsigned)n_bhq), dim3(256), 0, st, ix->K, ix->pos_slot,
                           ix->reservoir, q, tau_out, ix->cfg.reservoir_size, ix->cap_rows, ix->n_total,
                           ix->cfg.n_q_heads, ix->cfg.n_kv_heads, ix->G, mode, param);
    else
        hipLaunchKernelGGL(threshold_kernel<lvr_f32_t>, dim3((unsigned)n_bhq), dim3(256), 0, st, ix->K, ix->pos_slot,
                           ix->reservoir, q, tau_out, ix->cfg.reservoir_size, ix->cap_rows, ix->n_total,
                           ix->cfg.n_q_heads, ix->cfg.n_kv_heads, ix->G, mode, param);
    return hipGetLastError();
}
