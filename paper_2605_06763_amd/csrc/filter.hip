// Exact-filter kernel: the dot-product check that closes both query algorithms of Sec. 4.2
// ("Candidates then undergo an exact dot-product check"; Alg. 3 / Alg. 4, the line that forms
// L*).  It streams the key rows of the groups that survived the bound test, plus the rows of
// the not-yet-indexed buffer (Sec. 4.3), computes <q_h, k> in fp32 for the G query heads that
// share the KV head (each row is read once), and emits the token positions with
// <q_h, k> >= tau_h into per-head lists using wave-aggregated atomics.
//
// Work unit: a tile of 16 rows = four wave-wide loads (4 rows each).  Tiles [0, T_s) walk the
// compacted survivor list (16/r groups per tile), tiles [T_s, T_s + T_b) walk the buffer.
// The survivor count is read from device memory, so the grid is fixed and waves stride over
// the tiles; a wave whose first tile is past the end exits at once.
#include "lvr_internal.h"

namespace {

template <typename KT, int G>
__global__ void __launch_bounds__(256)
filter_kernel(const void *__restrict__ K, const int32_t *__restrict__ slot_pos, const float *__restrict__ q,
              const float *__restrict__ tau, const int32_t *__restrict__ surv_list,
              const int32_t *__restrict__ surv_count, int32_t *__restrict__ out_idx, int32_t *__restrict__ out_count,
              int32_t *__restrict__ emit_count, int32_t *__restrict__ overflow, int64_t cap_rows, int64_t max_groups,
              int64_t n_indexed, int64_t n_total, int log2r, int64_t cap, int n_q_heads, int n_kv_heads,
              int buffer_dense) {
    const int bh = blockIdx.y;
    const int b = bh / n_kv_heads, kvh = bh % n_kv_heads;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane >> 4, li = lane & 15;
    const int64_t hq0 = (int64_t)b * n_q_heads + kvh * G;

    float qv[G][8];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        const float *qh = q + (hq0 + h) * LVR_D + li * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) qv[h][e] = qh[e];
    }
    // lane li < G reports head li
    const float my_tau = (li < G) ? lvr_effective_tau(tau[hq0 + li]) : INFINITY;

    const int64_t rows_surv = (int64_t)surv_count[bh] << log2r;
    const int64_t surv_tiles = (rows_surv + 15) >> 4;
    const int64_t buf_tiles = (n_total - n_indexed + 15) >> 4;
    const int64_t total_tiles = surv_tiles + buf_tiles;
    const char *Kb = static_cast<const char *>(K) + (int64_t)bh * cap_rows * LVR_D * sizeof(KT);
    const int32_t *list = surv_list + (int64_t)bh * max_groups;
    const int32_t *spos = slot_pos ? slot_pos + (int64_t)bh * cap_rows : nullptr;
    const int rmask = (1 << log2r) - 1;

    for (int64_t t = (int64_t)blockIdx.x * 4 + wave; t < total_tiles; t += (int64_t)gridDim.x * 4) {
        const bool in_buf = t >= surv_tiles;
        int64_t slot[4];
        bool valid[4];
        float x[4][8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int ri = i * 4 + sub;
            if (!in_buf) {
                const int64_t rowidx = t * 16 + ri;
                valid[i] = rowidx < rows_surv;
                const int32_t gid = valid[i] ? list[rowidx >> log2r] : 0;
                slot[i] = ((int64_t)gid << log2r) + (rowidx & rmask);
            } else {
                slot[i] = n_indexed + (t - surv_tiles) * 16 + ri;
                valid[i] = slot[i] < n_total;
                if (!valid[i]) slot[i] = 0;
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) lvr_load8<KT>(Kb, slot[i], li, x[i]);

#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float mine = 0.f;
#pragma unroll
            for (int h = 0; h < G; ++h) {
                float p = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) p += qv[h][e] * x[i][e];
                const float s = lvr_row16_sum(p);
                mine = (li == h) ? s : mine;
            }
            const bool pred = valid[i] && li < G && (mine >= my_tau || (in_buf && buffer_dense));
            const uint64_t any = __ballot(pred);
            if (any) {   // wave-uniform
                // lanes li, li+16, li+32, li+48 hold the four rows' results for head li
                const uint64_t mh = (li < G) ? (any & (0x0001000100010001ull << li)) : 0ull;
                const int cnt = __popcll(mh);
                const int leader = cnt ? (__ffsll((unsigned long long)mh) - 1) : lane;
                int base = 0;
                if (cnt && lane == leader) {
                    base = atomicAdd(&out_count[hq0 + li], cnt);
                    atomicAdd(&emit_count[bh], cnt);
                }
                base = __shfl(base, leader, 64);
                if (pred) {
                    const int64_t p = base + __popcll(mh & ((1ull << lane) - 1ull));
                    if (p < cap)
                        out_idx[(hq0 + li) * cap + p] = spos ? spos[slot[i]] : (int32_t)slot[i];
                    else
                        *overflow = 1;
                }
            }
        }
    }
}

template <typename KT>
hipError_t launch_filter_t(lvr_index *ix, const float *q, const float *tau, int32_t *out_idx, int32_t *out_count,
                           int64_t cap, hipStream_t st) {
    const int64_t max_tiles = (ix->n_total + 15) / 16 + 1;
    int64_t gx = (max_tiles + 15) / 16;   // 4 waves x ~4 tiles each when every group survives
    if (gx < 1) gx = 1;
    if (gx > 2048) gx = 2048;
    dim3 grid((unsigned)gx, (unsigned)lvr_n_bh(ix));
    int log2r = 0;
    while ((1 << log2r) < ix->cfg.group_size) ++log2r;
    const int dense = (ix->cfg.flags & LVR_ATTEND_BUFFER_DENSE) ? 1 : 0;
#define LVR_FILTER_CASE(GG)                                                                                        \
    case GG:                                                                                                       \
        hipLaunchKernelGGL((filter_kernel<KT, GG>), grid, dim3(256), 0, st, ix->K, ix->slot_pos, q, tau,           \
                           ix->surv_list, lvr_surv_count(ix), out_idx, out_count, lvr_emit_count(ix),              \
                           lvr_overflow_flag(ix), ix->cap_rows, ix->max_groups, ix->n_indexed, ix->n_total, log2r, \
                           cap, ix->cfg.n_q_heads, ix->cfg.n_kv_heads, dense);                                     \
        break;
    switch (ix->G) {
        LVR_FILTER_CASE(1)
        LVR_FILTER_CASE(2)
        LVR_FILTER_CASE(4)
        LVR_FILTER_CASE(8)
        default: return hipErrorInvalidValue;
    }
#undef LVR_FILTER_CASE
    return hipGetLastError();
}

}  // namespace

hipError_t lvr_launch_filter(lvr_index *ix, const float *q, const float *tau, int32_t *out_idx, int32_t *out_count,
                             int64_t cap, hipStream_t st) {
    if (ix->n_total <= 0) return hipSuccess;
    return ix->cfg.kv_dtype == LVR_BF16 ? launch_filter_t<lvr_bf16_t>(ix, q, tau, out_idx, out_count, cap, st)
                                        : launch_filter_t<lvr_f32_t>(ix, q, tau, out_idx, out_count, cap, st);
}
