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
// sort: one streaming pass over the centres, wave-level reductions, ballot + prefix sum.
#include "lvr_internal.h"

namespace {

constexpr int PRUNE_ITERS = 16;                       // 4 groups per iteration and wave
constexpr int PRUNE_GROUPS_PER_WAVE = 4 * PRUNE_ITERS;
constexpr int PRUNE_GROUPS_PER_BLOCK = 4 * PRUNE_GROUPS_PER_WAVE;

__global__ void reset_kernel(int32_t *surv_count, int32_t *emit_count, int n_bh, int32_t *out_count, int n_bhq) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_bh) {
        surv_count[i] = 0;
        emit_count[i] = 0;
    }
    if (out_count && i < n_bhq) out_count[i] = 0;
}

template <typename KT, int G>
__global__ void __launch_bounds__(256)
prune_kernel(const void *__restrict__ centres, const float *__restrict__ radii, const float *__restrict__ q,
             const float *__restrict__ tau, int32_t *__restrict__ surv_list, int32_t *__restrict__ surv_count,
             int64_t n_groups, int64_t max_groups, int S, int n_q_heads, int n_kv_heads) {
    const int bh = blockIdx.y;
    const int b = bh / n_kv_heads, kvh = bh % n_kv_heads;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane >> 4, li = lane & 15;
    const int lanes_per_sub = 16 / S;

    // query slices, |pi_s q_h| for the subspace this lane reports (lanes li < S), thresholds
    float qv[G][8], qn[G], taue[G];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        const float *qh = q + ((int64_t)b * n_q_heads + kvh * G + h) * LVR_D + li * 8;
        float ss = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            qv[h][e] = qh[e];
            ss += qv[h][e] * qv[h][e];
        }
        for (int off = 1; off < lanes_per_sub; off <<= 1) ss += __shfl_xor(ss, off, 64);
        // lane li (< S) needs subspace li, whose lanes start at li * lanes_per_sub in this quarter
        float mine = __shfl(ss, (lane & 48) + ((li < S) ? li * lanes_per_sub : li), 64);
        // round the norm up so the radius term is never under-estimated
        qn[h] = (li < S) ? sqrtf(mine) * (1.0f + 0x1p-20f) : 0.f;
        taue[h] = lvr_effective_tau(tau[(int64_t)b * n_q_heads + kvh * G + h]);
    }

    const char *Cb = static_cast<const char *>(centres) + (int64_t)bh * max_groups * LVR_D * sizeof(KT);
    const float *Rb = radii + (int64_t)bh * max_groups * S;
    const int64_t gbase = (int64_t)blockIdx.x * PRUNE_GROUPS_PER_BLOCK + wave * PRUNE_GROUPS_PER_WAVE;

    uint32_t mybits = 0;   // lane `it` keeps the 4 survive bits of iteration `it`
#pragma unroll 4
    for (int it = 0; it < PRUNE_ITERS; ++it) {
        const int64_t g = gbase + it * 4 + sub;
        const bool valid = g < n_groups;
        const int64_t gc = valid ? g : n_groups - 1;
        float x[8];
        lvr_load8<KT>(Cb, gc, li, x);
        const float rad = (li < S) ? Rb[gc * S + li] : 0.f;
        bool alive = false;
#pragma unroll
        for (int h = 0; h < G; ++h) {
            float p = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) p += qv[h][e] * x[e];
            p += rad * qn[h];
            const float ub = lvr_row16_sum(p);
            alive |= (ub >= taue[h]);
        }
        const uint64_t bal = __ballot(alive && valid && li == 0);
        const uint32_t mask4 = (uint32_t)(bal & 1u) | (uint32_t)((bal >> 15) & 2u) | (uint32_t)((bal >> 30) & 4u) |
                               (uint32_t)((bal >> 45) & 8u);
        if (lane == it) mybits = mask4;
    }

    // wave-level compaction: prefix sum of per-lane survivor counts, one atomic per wave
    const int cnt = __popc(mybits);
    int incl = cnt;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        int t = __shfl_up(incl, off, 64);
        if (lane >= off) incl += t;
    }
    const int total = __shfl(incl, 63, 64);
    if (total == 0) return;
    int base = 0;
    if (lane == 0) base = atomicAdd(&surv_count[bh], total);
    base = __shfl(base, 0, 64);
    int32_t *out = surv_list + (int64_t)bh * max_groups + base + (incl - cnt);
    int j = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k)
        if (mybits & (1u << k)) out[j++] = (int32_t)(gbase + lane * 4 + k);
}

template <typename KT>
hipError_t launch_prune_g(lvr_index *ix, const float *q, const float *tau, hipStream_t st) {
    const int64_t n_groups = ix->n_indexed / ix->cfg.group_size;
    dim3 grid((unsigned)((n_groups + PRUNE_GROUPS_PER_BLOCK - 1) / PRUNE_GROUPS_PER_BLOCK), (unsigned)lvr_n_bh(ix));
#define LVR_PRUNE_CASE(GG)                                                                                        \
    case GG:                                                                                                      \
        hipLaunchKernelGGL((prune_kernel<KT, GG>), grid, dim3(256), 0, st, ix->centres, ix->radii, q, tau,        \
                           ix->surv_list, lvr_surv_count(ix), n_groups, ix->max_groups, ix->cfg.n_subspaces,     \
                           ix->cfg.n_q_heads, ix->cfg.n_kv_heads);                                               \
        break;
    switch (ix->G) {
        LVR_PRUNE_CASE(1)
        LVR_PRUNE_CASE(2)
        LVR_PRUNE_CASE(4)
        LVR_PRUNE_CASE(8)
        default: return hipErrorInvalidValue;
    }
#undef LVR_PRUNE_CASE
    return hipGetLastError();
}

}  // namespace

hipError_t lvr_launch_reset(lvr_index *ix, int32_t *out_count, hipStream_t st) {
    const int n_bh = lvr_n_bh(ix), n_bhq = ix->cfg.batch * ix->cfg.n_q_heads;
    const int n = n_bh > n_bhq ? n_bh : n_bhq;
    hipLaunchKernelGGL(reset_kernel, dim3((n + 255) / 256), dim3(256), 0, st, lvr_surv_count(ix), lvr_emit_count(ix),
                       n_bh, out_count, n_bhq);
    return hipGetLastError();
}

hipError_t lvr_launch_prune(lvr_index *ix, const float *q, const float *tau, hipStream_t st) {
    if (ix->n_indexed <= 0) return hipSuccess;
    return ix->cfg.kv_dtype == LVR_BF16 ? launch_prune_g<lvr_bf16_t>(ix, q, tau, st)
                                        : launch_prune_g<lvr_f32_t>(ix, q, tau, st);
}
