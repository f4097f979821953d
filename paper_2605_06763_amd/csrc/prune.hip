// Bound-pruning kernel: scores every ball of the index against the query halfspace and
// compacts the ids of the groups that may hold a qualifying key.
//
// For a group g with centre c_g and per-subspace radii rho_{s,g} the upper bound on the score
// of any member is   UB_g(q) = <q, c_g> + sum_s rho_{s,g} |pi_s q|   (Eq. (2) applied in each
// coordinate block and summed, as in Sec. 4.2 "Query 2", where the full dot product is the sum
// of the subspace terms).  A group is kept iff UB_g(q_h) >= tau_h for at least one of the G
// query heads that share this KV head; those heads are scored in the same pass so each centre
// is read from HBM once (the GQA reuse of App. "GPU Filter Pipeline").
//
// With one grouping shared by all subspaces this per-group sum rule retains a subset of what
// the sorted depth scan of Alg. 4 would retain (a group outside the scan's live set ranks
// below the stopping depth in every subspace, so its sum is below U(d*) < tau), and it needs no
// sort: one streaming pass over the centres, a ballot per tile and a prefix sum per workgroup.
//
// Compaction without global atomics: a workgroup owns a segment of consecutive groups and writes
// the ids of its survivors to the same range of the survivor list, plus one count per segment.
// The exact filter later runs one workgroup per segment.  (Same-address atomics are served
// serially by the memory side; thousands of them per launch would cost more than the scan.)
//
// The kernel also clears the per-head counters of the query it belongs to, so no separate
// reset launch is needed while the index is non-empty.
//
// bf16 centres are scored on the matrix cores (mfma_score.h): a tile is 16 groups (4 KiB of
// centres), two tiles in flight per wave.  fp32 centres use the vector ALU.
#include "mfma_score.h"

namespace {

struct PruneArgs {
    const void *centres;
    const float *radii;
    const float *q;
    const float *tau;
    int32_t *surv_list;
    int32_t *seg_count;      // [n_bh][max_segs]
    int32_t *head_count;     // padded per-head counters, cleared here
    int64_t n_groups, max_groups, max_segs;
    int n_q_heads, n_kv_heads, G, tiles_per_wave;
};

__global__ void reset_kernel(int32_t *head_count, int n_bhq) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_bhq) head_count[(size_t)i * LVR_CNT_STRIDE] = 0;
}

__device__ __forceinline__ void clear_query_counters(const PruneArgs &a, int64_t hq0) {
    if (blockIdx.x == 0 && (int)threadIdx.x < a.G) a.head_count[(hq0 + threadIdx.x) * LVR_CNT_STRIDE] = 0;
}

// Workgroup-level compaction of per-lane survivor bit masks (bit k of lane l of wave w = group
// wave_gbase + l*W + k) into the workgroup's segment of the survivor list.
template <int W>
__device__ __forceinline__ void compact_segment(const PruneArgs &a, int bh, int lane, int wave, uint32_t mybits,
                                                int64_t wave_gbase, int64_t seg_base) {
    __shared__ int s_tot[4];
    const int cnt = __popc(mybits);
    const int incl = lvr_wave_inclusive_sum(cnt);
    if (lane == 63) s_tot[wave] = incl;
    __syncthreads();
    int before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        before += (w < wave) ? s_tot[w] : 0;
        total += s_tot[w];
    }
    if (threadIdx.x == 0) a.seg_count[(int64_t)bh * a.max_segs + blockIdx.x] = total;
    int32_t *out = a.surv_list + (int64_t)bh * a.max_groups + seg_base + before + (incl - cnt);
    // one pass per set bit of the fullest mask in the wave
    int j = 0;
    uint32_t left = mybits;
    while (__ballot(left != 0)) {   // wave-uniform
        if (left != 0) {
            out[j++] = (int32_t)(wave_gbase + (int64_t)lane * W + __builtin_ctz(left));
            left &= left - 1;
        }
    }
}

// ------------------------------------------------------------------------------------------
// bf16 centres on the matrix cores.  HB = 4-head blocks, S = subspaces (compile time so the
// radii of a group are fetched with vector loads).
// ------------------------------------------------------------------------------------------
template <int HB, int S>
__global__ void __launch_bounds__(256)
prune_mfma_kernel(const PruneArgs a) {
    __shared__ uint4 s_bq[HB][4][64];
    __shared__ float s_qn[HB * 4][16];
    const int bh = blockIdx.y;
    const int b = bh / a.n_kv_heads, kvh = bh % a.n_kv_heads;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 15, kq = lane >> 4;
    const int64_t hq0 = (int64_t)b * a.n_q_heads + kvh * a.G;
    clear_query_counters(a, hq0);

    // --- prologue shared by the four waves: the subspace norms of q and its B fragments ---
    if ((int)threadIdx.x < HB * 64) {   // 16 lanes per head: sums of squares per coordinate block
        const int h = threadIdx.x >> 4, li = threadIdx.x & 15;
        float ss = 0.f;
        if (h < a.G) {
            const float *qh = a.q + (hq0 + h) * LVR_D + li * 8;
#pragma unroll
            for (int e = 0; e < 8; ++e) ss += qh[e] * qh[e];
        }
        constexpr int lanes_per_sub = 16 / S;
#pragma unroll
        for (int off = 1; off < lanes_per_sub; off <<= 1) ss += __shfl_xor(ss, off, 64);
        // rounded up a little so the radius term is never under-estimated
        if ((li % lanes_per_sub) == 0) s_qn[h][li / lanes_per_sub] = sqrtf(ss) * (1.0f + 0x1p-20f);
    }
    lvr_bf16x8 bq[HB][4];
    lvr_build_q_frags_wg<HB>(a.q + hq0 * LVR_D, a.G, 1.0f, s_bq, bq);   // syncs: s_qn is visible after it
    float qn[HB][S], taue[HB];
    bool rep[HB];
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) {
        const int h = hb * 4 + n - 8;
        rep[hb] = n >= 8 && n < 12 && h < a.G;
#pragma unroll
        for (int s = 0; s < S; ++s) qn[hb][s] = rep[hb] ? s_qn[h][s] : 0.f;
        taue[hb] = rep[hb] ? lvr_effective_tau(a.tau[hq0 + h]) : INFINITY;
    }

    const char *Cb = static_cast<const char *>(a.centres) + (int64_t)bh * a.max_groups * LVR_D * 2;
    const float *Rb = a.radii + (int64_t)bh * a.max_groups * S;
    const int64_t n_tiles = (a.n_groups + 15) >> 4;
    // a wave owns `tiles_per_wave` consecutive tiles (<= 64, even); lane `it` keeps tile it's mask
    const int64_t tile0 = ((int64_t)blockIdx.x * 4 + wave) * a.tiles_per_wave;
    uint32_t mybits = 0;
    for (int it = 0; it < a.tiles_per_wave; it += 2) {
        if (tile0 + it >= n_tiles) break;   // wave-uniform
        constexpr int SP = (S <= 4) ? S : 1;   // radii are fetched ahead only when they are few
        uint4 av[2][4];
        float rad[2][4][SP];
        int64_t g_row[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int64_t g0 = (tile0 + it + u) * 16;
            int64_t g = g0 + n;
            if (g >= a.n_groups) g = a.n_groups - 1;
            g_row[u] = g0;
            lvr_load_a_frags(Cb, g, av[u]);
            if constexpr (S <= 4) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    int64_t gj = g0 + 4 * kq + j;
                    if (gj >= a.n_groups) gj = a.n_groups - 1;
                    const float *rp = Rb + gj * S;
                    if constexpr (S == 4) {
                        const float4 r = *reinterpret_cast<const float4 *>(rp);
                        rad[u][j][0] = r.x; rad[u][j][1] = r.y; rad[u][j][2] = r.z; rad[u][j][3] = r.w;
                    } else {
#pragma unroll
                        for (int s = 0; s < S; ++s) rad[u][j][s] = rp[s];
                    }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            uint32_t alive4 = 0;   // bit j: group 4*kq + j of the tile survives for my head
#pragma unroll
            for (int hb = 0; hb < HB; ++hb) {
                const lvr_f32x4 sc = lvr_score_tile(av[u], bq[hb]);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    float ub = sc[j];
                    if constexpr (S <= 4) {
#pragma unroll
                        for (int s = 0; s < S; ++s) ub += rad[u][j][s] * qn[hb][s];
                    } else {
                        int64_t gj = g_row[u] + 4 * kq + j;
                        if (gj >= a.n_groups) gj = a.n_groups - 1;
                        const float4 *rp = reinterpret_cast<const float4 *>(Rb + gj * S);
#pragma unroll
                        for (int s4 = 0; s4 < S / 4; ++s4) {
                            const float4 r = rp[s4];
                            ub += r.x * qn[hb][4 * s4] + r.y * qn[hb][4 * s4 + 1] + r.z * qn[hb][4 * s4 + 2] +
                                  r.w * qn[hb][4 * s4 + 3];
                        }
                    }
                    const bool ok = rep[hb] && ub >= taue[hb] && (g_row[u] + 4 * kq + j) < a.n_groups;
                    alive4 |= ok ? (1u << j) : 0u;
                }
            }
            // OR over the reporting lanes of each quarter: 16-bit tile mask, bit 4*kq + j
            uint32_t mask16 = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint64_t bal = __ballot((alive4 >> j) & 1u);
#pragma unroll
                for (int qd = 0; qd < 4; ++qd)
                    mask16 |= ((bal >> (16 * qd)) & 0xffffull) ? (1u << (4 * qd + j)) : 0u;
            }
            if (lane == it + u) mybits = mask16;
        }
    }
    compact_segment<16>(a, bh, lane, wave, mybits, tile0 * 16,
                        (int64_t)blockIdx.x * 4 * a.tiles_per_wave * 16);
}

// ------------------------------------------------------------------------------------------
// Generic centres (fp32 storage) on the vector ALU: 16 lanes per centre, 4 centres per load.
// ------------------------------------------------------------------------------------------
constexpr int VALU_ITERS = 16;   // 4 groups per iteration and wave, loads issued 4 iterations at a time

template <typename KT, int G>
__global__ void __launch_bounds__(256)
prune_valu_kernel(const PruneArgs a, int S) {
    const int bh = blockIdx.y;
    const int b = bh / a.n_kv_heads, kvh = bh % a.n_kv_heads;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane >> 4, li = lane & 15;
    const int lanes_per_sub = 16 / S;
    const int64_t hq0 = (int64_t)b * a.n_q_heads + kvh * G;
    clear_query_counters(a, hq0);

    float qv[G][8], qn[G], taue[G];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        const float *qh = a.q + (hq0 + h) * LVR_D + li * 8;
        float ss = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            qv[h][e] = qh[e];
            ss += qv[h][e] * qv[h][e];
        }
        for (int off = 1; off < lanes_per_sub; off <<= 1) ss += __shfl_xor(ss, off, 64);
        const float mine = __shfl(ss, (lane & 48) + ((li < S) ? li * lanes_per_sub : li), 64);
        qn[h] = (li < S) ? sqrtf(mine) * (1.0f + 0x1p-20f) : 0.f;
        taue[h] = lvr_effective_tau(a.tau[hq0 + h]);
    }
    const char *Cb = static_cast<const char *>(a.centres) + (int64_t)bh * a.max_groups * LVR_D * sizeof(KT);
    const float *Rb = a.radii + (int64_t)bh * a.max_groups * S;
    const int64_t gbase = ((int64_t)blockIdx.x * 4 + wave) * (4 * VALU_ITERS);

    uint32_t mybits = 0;
    for (int it0 = 0; it0 < VALU_ITERS; it0 += 4) {
        float x[4][8], rad[4];
        bool valid[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t g = gbase + (it0 + u) * 4 + sub;
            valid[u] = g < a.n_groups;
            const int64_t gc = valid[u] ? g : a.n_groups - 1;
            lvr_load8<KT>(Cb, gc, li, x[u]);
            rad[u] = Rb[gc * S + (li & (S - 1))];    // lanes li >= S multiply it by zero below
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            bool alive = false;
#pragma unroll
            for (int h = 0; h < G; ++h) {
                float p = rad[u] * qn[h];
#pragma unroll
                for (int e = 0; e < 8; ++e) p += qv[h][e] * x[u][e];
                alive |= (lvr_row16_sum(p) >= taue[h]);
            }
            const uint64_t bal = __ballot(alive && valid[u] && li == 0);
            const uint32_t mask4 = (uint32_t)(bal & 1u) | (uint32_t)((bal >> 15) & 2u) |
                                   (uint32_t)((bal >> 30) & 4u) | (uint32_t)((bal >> 45) & 8u);
            if (lane == it0 + u) mybits = mask4;
        }
    }
    compact_segment<4>(a, bh, lane, wave, mybits, gbase, (int64_t)blockIdx.x * 4 * (4 * VALU_ITERS));
}

template <int HB>
void launch_mfma_s(dim3 grid, hipStream_t st, const PruneArgs &a, int S) {
    switch (S) {
        case 1: hipLaunchKernelGGL((prune_mfma_kernel<HB, 1>), grid, dim3(256), 0, st, a); break;
        case 2: hipLaunchKernelGGL((prune_mfma_kernel<HB, 2>), grid, dim3(256), 0, st, a); break;
        case 4: hipLaunchKernelGGL((prune_mfma_kernel<HB, 4>), grid, dim3(256), 0, st, a); break;
        case 8: hipLaunchKernelGGL((prune_mfma_kernel<HB, 8>), grid, dim3(256), 0, st, a); break;
        default: hipLaunchKernelGGL((prune_mfma_kernel<HB, 16>), grid, dim3(256), 0, st, a); break;
    }
}

}  // namespace

hipError_t lvr_launch_reset(lvr_index *ix, hipStream_t st) {
    const int n_bhq = lvr_n_bhq(ix);
    hipLaunchKernelGGL(reset_kernel, dim3((n_bhq + 255) / 256), dim3(256), 0, st, lvr_head_count(ix), n_bhq);
    ix->n_segs = 0;
    return hipGetLastError();
}

hipError_t lvr_launch_prune(lvr_index *ix, const float *q, const float *tau, hipStream_t st) {
    if (ix->n_indexed <= 0) return hipErrorInvalidValue;
    PruneArgs a;
    a.centres = ix->centres;
    a.radii = ix->radii;
    a.q = q;
    a.tau = tau;
    a.surv_list = ix->surv_list;
    a.seg_count = lvr_seg_count(ix);
    a.head_count = lvr_head_count(ix);
    a.n_groups = ix->n_indexed / ix->cfg.group_size;
    a.max_groups = ix->max_groups;
    a.max_segs = lvr_max_segs(ix->max_groups);
    a.n_q_heads = ix->cfg.n_q_heads;
    a.n_kv_heads = ix->cfg.n_kv_heads;
    a.G = ix->G;
    const int n_bh = lvr_n_bh(ix);
    const int S = ix->cfg.n_subspaces;
    int seg_groups;
    if (ix->cfg.kv_dtype == LVR_BF16) {
        // segment = 4 waves x tiles_per_wave tiles x 16 groups; aim at ~1024 workgroups per launch
        int64_t want = a.n_groups * n_bh / 1024;
        int tpw = 2;
        while (tpw < 16 && (int64_t)tpw * 64 < want) tpw *= 2;
        a.tiles_per_wave = tpw;
        seg_groups = tpw * 64;
    } else {
        a.tiles_per_wave = 0;
        seg_groups = 4 * 4 * VALU_ITERS;
    }
    const int64_t n_segs = (a.n_groups + seg_groups - 1) / seg_groups;
    dim3 grid((unsigned)n_segs, (unsigned)n_bh);
    if (ix->cfg.kv_dtype == LVR_BF16) {
        if (ix->G <= 4)
            launch_mfma_s<1>(grid, st, a, S);
        else
            launch_mfma_s<2>(grid, st, a, S);
    } else {
        switch (ix->G) {
            case 1: hipLaunchKernelGGL((prune_valu_kernel<lvr_f32_t, 1>), grid, dim3(256), 0, st, a, S); break;
            case 2: hipLaunchKernelGGL((prune_valu_kernel<lvr_f32_t, 2>), grid, dim3(256), 0, st, a, S); break;
            case 4: hipLaunchKernelGGL((prune_valu_kernel<lvr_f32_t, 4>), grid, dim3(256), 0, st, a, S); break;
            case 8: hipLaunchKernelGGL((prune_valu_kernel<lvr_f32_t, 8>), grid, dim3(256), 0, st, a, S); break;
            default: return hipErrorInvalidValue;
        }
    }
    ix->seg_groups = seg_groups;
    ix->n_segs = (int)n_segs;
    return hipGetLastError();
}
