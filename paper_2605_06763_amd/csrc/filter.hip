// Exact-filter kernel: the dot-product check that closes both query algorithms of Sec. 4.2
// ("Candidates then undergo an exact dot-product check"; Alg. 3 / Alg. 4, the line that forms
// L*).  It streams the key rows of the groups that survived the bound test, plus the rows of
// the not-yet-indexed buffer (Sec. 4.3), computes <q_h, k> in fp32 for the G query heads that
// share the KV head (each row is read once), and emits the token positions with
// <q_h, k> >= tau_h into per-head lists.
//
// Work split: one workgroup per segment of the survivor list (the bound test left a count per
// segment, so no device-wide counter is read), one more per (sequence, KV head) for the buffer.
// A wave takes tiles of 16 rows, two tiles (8 KiB) in flight.
//
// Emission: qualifying positions go to a small per-wave queue in LDS first; a queue is flushed
// with ONE atomic per head on a counter that owns its cache line, so a launch issues a few
// thousand atomics spread over many lines instead of one per hit on a few lines (atomics on
// one line are served serially by the memory side).
//
// Two bodies: bf16 rows are scored on the matrix cores (mfma_score.h); fp32 rows (the small
// single-head workload) on the vector ALU.
#include "emitter.h"
#include "mfma_score.h"

namespace {

constexpr int QCAP = LVR_QCAP;

struct FilterArgs {
    const void *K;
    const int32_t *slot_pos;
    const float *q;
    const float *tau;
    const int32_t *surv_list;
    const int32_t *seg_count;
    lvr_emit_target emit;
    int64_t cap_rows, max_groups, max_segs, n_indexed, n_total;
    int log2r, n_q_heads, n_kv_heads, G, buffer_dense, n_segs, seg_groups;
};

struct SegWork {
    int64_t rows;        // rows of surviving groups in this segment (0 for the buffer workgroup)
    int64_t tiles;
    const int32_t *list;
    bool buffer;         // this workgroup scans the buffer rows instead
    int64_t buf_row0, buf_rows;
};

__device__ __forceinline__ SegWork seg_work(const FilterArgs &a, int bh) {
    SegWork w;
    w.buffer = (int)blockIdx.x >= a.n_segs;
    if (!w.buffer) {
        w.rows = (int64_t)a.seg_count[(int64_t)bh * a.max_segs + blockIdx.x] << a.log2r;
        w.list = a.surv_list + (int64_t)bh * a.max_groups + (int64_t)blockIdx.x * a.seg_groups;
        w.buf_row0 = w.buf_rows = 0;
    } else {
        w.rows = a.n_total - a.n_indexed;
        w.list = a.surv_list;
        w.buf_row0 = a.n_indexed;
        w.buf_rows = w.rows;
    }
    w.tiles = (w.rows + 15) >> 4;
    return w;
}

// ------------------------------------------------------------------------------------------
// bf16 rows, matrix cores.  HB = number of 4-head blocks (G <= 4: 1, G = 8: 2).
// ------------------------------------------------------------------------------------------
template <int HB>
__global__ void __launch_bounds__(256)
filter_mfma_kernel(const FilterArgs a) {
    __shared__ uint4 s_bq[HB][4][64];
    __shared__ int32_t s_queue[4][HB][4][QCAP];
    const int bh = blockIdx.y;
    const int b = bh / a.n_kv_heads, kvh = bh % a.n_kv_heads;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 15, kq = lane >> 4;
    const int64_t hq0 = (int64_t)b * a.n_q_heads + kvh * a.G;

    const SegWork w = seg_work(a, bh);
    if (w.tiles == 0) return;   // uniform over the workgroup

    lvr_bf16x8 bq[HB][4];
    lvr_build_q_frags_wg<HB>(a.q + hq0 * LVR_D, a.G, 1.0f, s_bq, bq);
    float my_tau[HB];
    bool rep[HB];
    lvr_emitter<4> em[HB];
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) {
        const int h = hb * 4 + n - 8;
        rep[hb] = n >= 8 && n < 12 && h < a.G;
        my_tau[hb] = rep[hb] ? lvr_effective_tau(a.tau[hq0 + h]) : INFINITY;
        em[hb].q = s_queue[wave][hb];
        em[hb].count = 0;
        em[hb].rep_base = 8;
        em[hb].hq_base = hq0 + hb * 4;
    }
    const char *Kb = static_cast<const char *>(a.K) + (int64_t)bh * a.cap_rows * LVR_D * 2;
    const int32_t *spos = a.slot_pos ? a.slot_pos + (int64_t)bh * a.cap_rows : nullptr;
    const int rmask = (1 << a.log2r) - 1;

    // two tiles per trip: t and t + 4 (the four waves interleave)
    for (int64_t t0 = wave; t0 < w.tiles; t0 += 8) {
        int slot[2], nvalid[2];
        int32_t gid[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int64_t t = t0 + 4 * u;
            int64_t rowidx = t * 16 + n;
            const int64_t left = w.rows - t * 16;
            nvalid[u] = left <= 0 ? 0 : (left < 16 ? (int)left : 16);
            if (rowidx >= w.rows) rowidx = 0;
            gid[u] = w.buffer ? 0 : w.list[rowidx >> a.log2r];
            slot[u] = (int)rowidx;   // finished below once gid has arrived
        }
        uint4 av[2][4];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int rowidx = slot[u];
            slot[u] = w.buffer ? (int)(w.buf_row0 + rowidx) : (int)(((int64_t)gid[u] << a.log2r) + (rowidx & rmask));
            lvr_load_a_frags(Kb, slot[u], av[u]);
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            if (nvalid[u] == 0) continue;   // wave-uniform
#pragma unroll
            for (int hb = 0; hb < HB; ++hb) {
                const lvr_f32x4 s = lvr_score_tile(av[u], bq[hb]);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int trow = 4 * kq + j;
                    const bool pred = trow < nvalid[u] && rep[hb] &&
                                      (s[j] >= my_tau[hb] || (w.buffer && a.buffer_dense));
                    em[hb].push(a.emit, lane, rep[hb], pred, slot[u], trow, spos);
                }
            }
        }
    }
#pragma unroll
    for (int hb = 0; hb < HB; ++hb)
        if (__ballot(em[hb].count > 0)) em[hb].flush(a.emit, lane, rep[hb], spos);
}

// ------------------------------------------------------------------------------------------
// Generic rows (fp32 storage), vector ALU: 16 lanes per row, four rows per wave-wide load.
// ------------------------------------------------------------------------------------------
template <typename KT, int G>
__global__ void __launch_bounds__(256)
filter_valu_kernel(const FilterArgs a) {
    __shared__ int32_t s_queue[4][G][QCAP];
    const int bh = blockIdx.y;
    const int b = bh / a.n_kv_heads, kvh = bh % a.n_kv_heads;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane >> 4, li = lane & 15;
    const int64_t hq0 = (int64_t)b * a.n_q_heads + kvh * G;

    const SegWork w = seg_work(a, bh);
    if (w.tiles == 0) return;

    float qv[G][8];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        const float *qh = a.q + (hq0 + h) * LVR_D + li * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) qv[h][e] = qh[e];
    }
    const bool rep = li < G;
    const float my_tau = rep ? lvr_effective_tau(a.tau[hq0 + li]) : INFINITY;
    lvr_emitter<G> em;
    em.q = s_queue[wave];
    em.count = 0;
    em.rep_base = 0;
    em.hq_base = hq0;
    const char *Kb = static_cast<const char *>(a.K) + (int64_t)bh * a.cap_rows * LVR_D * sizeof(KT);
    const int32_t *spos = a.slot_pos ? a.slot_pos + (int64_t)bh * a.cap_rows : nullptr;
    const int rmask = (1 << a.log2r) - 1;

    for (int64_t t = wave; t < w.tiles; t += 4) {
        int slot[4];
        bool valid[4];
        int32_t gid[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int64_t rowidx = t * 16 + i * 4 + sub;
            valid[i] = rowidx < w.rows;
            if (!valid[i]) rowidx = 0;
            gid[i] = w.buffer ? 0 : w.list[rowidx >> a.log2r];
            slot[i] = (int)rowidx;
        }
        lvr_raw8<KT> raw[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int rowidx = slot[i];
            slot[i] = w.buffer ? (int)(w.buf_row0 + rowidx) : (int)(((int64_t)gid[i] << a.log2r) + (rowidx & rmask));
            lvr_load_raw(Kb, slot[i], li, raw[i]);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float x[8];
            lvr_unpack(raw[i], x);
            float mine = 0.f;
#pragma unroll
            for (int h = 0; h < G; ++h) {
                float p = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) p += qv[h][e] * x[e];
                const float s = lvr_row16_sum(p);
                mine = (li == h) ? s : mine;
            }
            const bool pred = valid[i] && rep && (mine >= my_tau || (w.buffer && a.buffer_dense));
            em.push(a.emit, lane, rep, pred, slot[i], lane, spos);   // the reporting lane holds the row's slot itself
        }
    }
    if (__ballot(em.count > 0)) em.flush(a.emit, lane, rep, spos);
}

__global__ void publish_counts_kernel(int32_t *__restrict__ head_count, int32_t *__restrict__ head_stat,
                                      int32_t *__restrict__ out_count, int n_bhq) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_bhq) {
        const int32_t c = head_count[(size_t)i * LVR_CNT_STRIDE];
        out_count[i] = c;
        head_stat[i] = c;
        head_count[(size_t)i * LVR_CNT_STRIDE] = 0;
    }
}

}  // namespace

hipError_t lvr_launch_filter(lvr_index *ix, const float *q, const float *tau, int32_t *out_idx, int64_t cap,
                             hipStream_t st) {
    FilterArgs a;
    a.K = ix->K;
    a.slot_pos = ix->slot_pos;
    a.q = q;
    a.tau = tau;
    a.surv_list = ix->surv_list;
    a.seg_count = lvr_seg_count(ix);
    a.emit.out_idx = out_idx;
    a.emit.head_count = lvr_head_count(ix);
    a.emit.overflow = lvr_overflow_flag(ix);
    a.emit.cap = cap;
    a.emit.out_score = nullptr;
    a.emit.score_stride = 0;
    a.cap_rows = ix->cap_rows;
    a.max_groups = ix->max_groups;
    a.max_segs = lvr_max_segs(ix->max_groups);
    a.n_indexed = ix->n_indexed;
    a.n_total = ix->n_total;
    a.log2r = 0;
    while ((1 << a.log2r) < ix->cfg.group_size) ++a.log2r;
    a.n_q_heads = ix->cfg.n_q_heads;
    a.n_kv_heads = ix->cfg.n_kv_heads;
    a.G = ix->G;
    a.buffer_dense = (ix->cfg.flags & LVR_ATTEND_BUFFER_DENSE) ? 1 : 0;
    a.n_segs = ix->n_indexed > 0 ? ix->n_segs : 0;
    a.seg_groups = ix->seg_groups;
    const int has_buffer = ix->n_total > ix->n_indexed ? 1 : 0;
    if (a.n_segs + has_buffer == 0) return hipSuccess;
    dim3 grid((unsigned)(a.n_segs + has_buffer), (unsigned)lvr_n_bh(ix));
    if (ix->cfg.kv_dtype == LVR_BF16) {
        if (ix->G <= 4)
            hipLaunchKernelGGL(filter_mfma_kernel<1>, grid, dim3(256), 0, st, a);
        else
            hipLaunchKernelGGL(filter_mfma_kernel<2>, grid, dim3(256), 0, st, a);
    } else {
        switch (ix->G) {
            case 1: hipLaunchKernelGGL((filter_valu_kernel<lvr_f32_t, 1>), grid, dim3(256), 0, st, a); break;
            case 2: hipLaunchKernelGGL((filter_valu_kernel<lvr_f32_t, 2>), grid, dim3(256), 0, st, a); break;
            case 4: hipLaunchKernelGGL((filter_valu_kernel<lvr_f32_t, 4>), grid, dim3(256), 0, st, a); break;
            case 8: hipLaunchKernelGGL((filter_valu_kernel<lvr_f32_t, 8>), grid, dim3(256), 0, st, a); break;
            default: return hipErrorInvalidValue;
        }
    }
    return hipGetLastError();
}

hipError_t lvr_launch_publish_counts(lvr_index *ix, int32_t *out_count, hipStream_t st) {
    const int n_bhq = lvr_n_bhq(ix);
    hipLaunchKernelGGL(publish_counts_kernel, dim3((n_bhq + 255) / 256), dim3(256), 0, st, lvr_head_count(ix),
                       lvr_head_stat(ix), out_count, n_bhq);
    return hipGetLastError();
}
