// Attention kernels.
//
//  sparse_attention_kernel attention restricted to a per-head index list (Sec. 2 "Sparse
//                         Attention"; App. "GPU Sparse Attention Kernel"): the list is cut into
//                         P splits, each wave gathers its K and V rows (256 B each for bf16),
//                         keeps running softmax statistics (m, l) and an fp32 accumulator o.
//  dense_partial_kernel   the dense baseline (Sec. 2 "Attention"): every held key, contiguous
//                         streaming, the G query heads of a KV head served from one read.
//  combine_kernel         merges the P partial triples (m_p, l_p, o_p) into the output.
//
// Logits are kept in base-2 units (q is pre-multiplied by sigma * log2 e) so the exponentials
// are single exp2 instructions; the softmax is unchanged by the change of base.
#include <hip/hip_ext.h>

#include "mfma_score.h"

namespace {

constexpr float LOG2E = 1.4426950408889634f;

__device__ __forceinline__ float exp2_safe(float a, float b) {   // 2^(a-b) with (-inf) - (-inf) -> 0
    return (a == -INFINITY) ? 0.f : exp2f(a - b);
}

// Split geometry of the sparse attention: 16 entries per split (one gather batch) while the
// list fits in P_max splits, longer splits otherwise.  Returns the split length; *used = splits
// that hold entries.  The partial and the combine kernel derive it from the same count.
__device__ __forceinline__ int64_t split_length(int64_t cnt, int P_max, int *used) {
    int64_t L = (((cnt + P_max - 1) / P_max) + 15) & ~(int64_t)15;
    if (L < 16) L = 16;
    *used = (int)((cnt + L - 1) / L);
    return L;
}

// One wave per (query head, split).  The split's positions are fetched with one coalesced load,
// then rows are gathered 16 at a time (K and V of four row-quads in flight together).  The
// partials are merged by combine_kernel in a launch of its own: making them visible to a
// "last wave" inside this launch would take a device-scope fence per wave, which costs more
// on this multi-die part than the extra launch does.
// CARRY: the raw scores of the listed keys are given (written by the query kernel that made the
// list), so only V rows are gathered.
template <typename KT, bool CARRY>
__global__ void __launch_bounds__(64)
sparse_attention_kernel(const void *__restrict__ K, const void *__restrict__ V, const int32_t *__restrict__ pos_slot,
                        const float *__restrict__ q, const int32_t *__restrict__ idx,
                        const float *__restrict__ scores, int64_t score_stride,
                        const int32_t *__restrict__ count, int count_stride, int64_t cap,
                        float *__restrict__ part_ml, float *__restrict__ part_o, int64_t cap_rows, int64_t n_total,
                        int P, int n_q_heads, int n_kv_heads, int G, float qscale) {
    const int64_t hq = blockIdx.y;
    const int p = blockIdx.x;
    const int bh = (int)((uint32_t)hq / (uint32_t)G);   // (hq / H_q) * H_kv + (hq % H_q) / G with H_q = H_kv * G: one 32-bit division
    const int lane = threadIdx.x & 63, sub = lane >> 4, li = lane & 15;

    const int32_t *my_idx = idx + hq * cap;
    // The split geometry depends on the count, and the positions on the geometry: two dependent
    // loads before the first gather.  The common geometry (16 entries per split) is assumed for a
    // speculative load of the positions that goes out together with the count.
    const int64_t e_spec = (int64_t)p * 16 + lane;
    const int32_t pos_spec = (lane < 16 && e_spec < cap) ? my_idx[e_spec] : -1;
    const float *my_sc = CARRY ? scores + hq * score_stride : nullptr;
    float sc_spec = 0.f;
    if constexpr (CARRY) sc_spec = (lane < 16 && e_spec < cap && e_spec < score_stride) ? my_sc[e_spec] : 0.f;
    int64_t cnt = count[hq * count_stride];
    if (cnt > cap) cnt = cap;
    if (cnt < 0) cnt = 0;
    int used;
    const int64_t L = split_length(cnt, P, &used);
    if (p >= used) return;     // the combine pass reads only the `used` partials
    const int64_t start = (int64_t)p * L;
    const int64_t end = (start + L < cnt) ? start + L : cnt;

    float qv[8];
    {
        const float *qh = q + hq * LVR_D + li * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) qv[e] = qh[e] * qscale;
    }
    const char *Kb = static_cast<const char *>(K) + (int64_t)bh * cap_rows * LVR_D * sizeof(KT);
    const char *Vb = static_cast<const char *>(V) + (int64_t)bh * cap_rows * LVR_D * sizeof(KT);
    const int32_t *pslot = pos_slot ? pos_slot + (int64_t)bh * cap_rows : nullptr;

    float m = -INFINITY, l = 0.f, acc[8];
    lvr_zero8(acc);
    for (int64_t c0 = start; c0 < end; c0 += 64) {          // uniform over the wave
        // positions of up to 64 entries, validated and mapped to arena rows once
        int64_t e = c0 + lane;
        int myslot = -1;
        float myscore = 0.f;
        if (e < end) {
            const int64_t pos = (L == 16) ? (int64_t)pos_spec : (int64_t)my_idx[e];
            if constexpr (CARRY) myscore = ((L == 16) ? sc_spec : my_sc[e]) * qscale;
            if (pos >= 0 && pos < n_total) myslot = pslot ? pslot[pos] : (int)pos;
        }
        const int chunk = (int)((end - c0 < 64) ? end - c0 : 64);
        for (int b0 = 0; b0 < chunk; b0 += 16) {
            lvr_raw8<KT> kr[CARRY ? 1 : 4], vr[4];
            int slot[4];
            float given[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                slot[i] = __shfl(myslot, (b0 + i * 4 + sub) & 63, 64);
                if constexpr (CARRY) given[i] = __shfl(myscore, (b0 + i * 4 + sub) & 63, 64);
                if (b0 + i * 4 + sub >= chunk) slot[i] = -1;
                const int64_t sl = slot[i] < 0 ? 0 : slot[i];
                if constexpr (!CARRY) lvr_load_raw(Kb, sl, li, kr[i]);
                lvr_load_raw(Vb, sl, li, vr[i]);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float vx[8];
                lvr_unpack(vr[i], vx);
                float s;
                if constexpr (CARRY) {
                    s = given[i];
                } else {
                    float kx[8];
                    lvr_unpack(kr[i], kx);
                    float d = 0.f;
#pragma unroll
                    for (int c = 0; c < 8; ++c) d += qv[c] * kx[c];
                    s = lvr_row16_sum(d);
                }
                s = (slot[i] >= 0) ? s : -INFINITY;
                const float m_new = fmaxf(m, s);
                const float alpha = exp2_safe(m, m_new);
                const float w = exp2_safe(s, m_new);
                l = l * alpha + w;
#pragma unroll
                for (int c = 0; c < 8; ++c) acc[c] = acc[c] * alpha + w * vx[c];
                m = m_new;
            }
        }
    }
    // merge the four quarter rows of the wave
    float m_all = fmaxf(m, __shfl_xor(m, 16, 64));
    m_all = fmaxf(m_all, __shfl_xor(m_all, 32, 64));
    const float sc = exp2_safe(m, m_all);
    l *= sc;
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        float a = acc[c] * sc;
        a += __shfl_xor(a, 16, 64);
        a += __shfl_xor(a, 32, 64);
        acc[c] = a;
    }
    if (sub == 0) {
        float *o = part_o + (hq * P + p) * LVR_D + li * 8;
#pragma unroll
        for (int c = 0; c < 8; ++c) o[c] = acc[c];
        if (li == 0) {
            part_ml[(hq * P + p) * 2] = m_all;
            part_ml[(hq * P + p) * 2 + 1] = l;
        }
    }
}

// Sparse attention in ONE launch: a 1024-thread workgroup (16 waves) per query head.  Each wave
// takes a contiguous share of the head's index list exactly as sparse_attention_kernel does,
// then the 16 partial triples are merged through LDS, so no partials travel through HBM and no
// combine launch follows.  Thread 0 also publishes (and clears) the head's internal counter
// when asked to.
template <typename KT, bool CARRY>
__global__ void __launch_bounds__(1024)
sparse_attention_wg_kernel(const void *__restrict__ K, const void *__restrict__ V,
                           const int32_t *__restrict__ pos_slot, const float *__restrict__ q,
                           const int32_t *__restrict__ idx, const float *__restrict__ scores, int64_t score_stride,
                           const int32_t *count, int count_stride,   // may alias head_count: not restrict
                           int64_t cap, float *__restrict__ out, int64_t cap_rows, int64_t n_total, int n_q_heads,
                           int n_kv_heads, int G, float qscale, int32_t *head_count,
                           int32_t *__restrict__ head_stat, int32_t *__restrict__ publish_count) {
    constexpr int NW = 16;
    __shared__ float s_m[NW], s_l[NW];
    __shared__ float s_o[NW][LVR_D];
    const int64_t hq = blockIdx.x;
    const int bh = (int)((uint32_t)hq / (uint32_t)G);   // (hq / H_q) * H_kv + (hq % H_q) / G with H_q = H_kv * G: one 32-bit division
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, sub = lane >> 4, li = lane & 15;

    int64_t cnt = count[hq * count_stride];
    const int32_t true_cnt = (int32_t)cnt;
    if (cnt > cap) cnt = cap;
    if (cnt < 0) cnt = 0;
    const int64_t L = (((cnt + NW - 1) / NW) + 15) & ~(int64_t)15;
    const int64_t start = (int64_t)wave * L;
    const int64_t end = (start + L < cnt) ? start + L : cnt;

    float qv[8];
    {
        const float *qh = q + hq * LVR_D + li * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) qv[e] = qh[e] * qscale;
    }
    const char *Kb = static_cast<const char *>(K) + (int64_t)bh * cap_rows * LVR_D * sizeof(KT);
    const char *Vb = static_cast<const char *>(V) + (int64_t)bh * cap_rows * LVR_D * sizeof(KT);
    const int32_t *my_idx = idx + hq * cap;
    const int32_t *pslot = pos_slot ? pos_slot + (int64_t)bh * cap_rows : nullptr;

    float m = -INFINITY, l = 0.f, acc[8];
    lvr_zero8(acc);
    for (int64_t c0 = start; c0 < end; c0 += 64) {          // uniform over the wave
        int64_t e = c0 + lane;
        int myslot = -1;
        float myscore = 0.f;
        if (e < end) {
            const int64_t pos = my_idx[e];
            if constexpr (CARRY) myscore = (e < score_stride ? scores[hq * score_stride + e] : 0.f) * qscale;
            if (pos >= 0 && pos < n_total) myslot = pslot ? pslot[pos] : (int)pos;
        }
        const int chunk = (int)((end - c0 < 64) ? end - c0 : 64);
        for (int b0 = 0; b0 < chunk; b0 += 16) {
            lvr_raw8<KT> kr[CARRY ? 1 : 4], vr[4];
            int slot[4];
            float given[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                slot[i] = __shfl(myslot, (b0 + i * 4 + sub) & 63, 64);
                if constexpr (CARRY) given[i] = __shfl(myscore, (b0 + i * 4 + sub) & 63, 64);
                if (b0 + i * 4 + sub >= chunk) slot[i] = -1;
                const int64_t sl = slot[i] < 0 ? 0 : slot[i];
                if constexpr (!CARRY) lvr_load_raw(Kb, sl, li, kr[i]);
                lvr_load_raw(Vb, sl, li, vr[i]);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float vx[8];
                lvr_unpack(vr[i], vx);
                float s;
                if constexpr (CARRY) {
                    s = given[i];
                } else {
                    float kx[8];
                    lvr_unpack(kr[i], kx);
                    float d = 0.f;
#pragma unroll
                    for (int c = 0; c < 8; ++c) d += qv[c] * kx[c];
                    s = lvr_row16_sum(d);
                }
                s = (slot[i] >= 0) ? s : -INFINITY;
                const float m_new = fmaxf(m, s);
                const float alpha = exp2_safe(m, m_new);
                const float w = exp2_safe(s, m_new);
                l = l * alpha + w;
#pragma unroll
                for (int c = 0; c < 8; ++c) acc[c] = acc[c] * alpha + w * vx[c];
                m = m_new;
            }
        }
    }
    float m_all = fmaxf(m, __shfl_xor(m, 16, 64));
    m_all = fmaxf(m_all, __shfl_xor(m_all, 32, 64));
    const float sc = exp2_safe(m, m_all);
    l *= sc;
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        float a = acc[c] * sc;
        a += __shfl_xor(a, 16, 64);
        a += __shfl_xor(a, 32, 64);
        if (sub == 0) s_o[wave][li * 8 + c] = a;
    }
    if (lane == 0) {
        s_m[wave] = m_all;
        s_l[wave] = l;
    }
    __syncthreads();
    if (threadIdx.x < LVR_D) {
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < NW; ++w) M = fmaxf(M, s_m[w]);
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float wt = exp2_safe(s_m[w], M);
            den += wt * s_l[w];
            num += wt * s_o[w][threadIdx.x];
        }
        out[hq * LVR_D + threadIdx.x] = (den > 0.f && M != -INFINITY) ? num / den : 0.f;
    }
    if (publish_count && threadIdx.x == 0) {
        publish_count[hq] = true_cnt;
        head_stat[hq] = true_cnt;
        head_count[hq * LVR_CNT_STRIDE] = 0;
    }
}

// The one-launch form for lists that carry their scores (the decode step on bf16 caches): the same 1024-thread
// workgroup per head, with the dependent round trips to memory cut to two.
//   trip 1  the count AND the positions and scores of the first 1024 list entries: which entries a lane asks for
//           does not depend on the count (lane (quarter s, j) of wave w asks for entry j of batch w + 16 s, a batch
//           being 16 consecutive entries), what lies beyond the count is dropped when it arrives;
//   trip 2  the V rows of ALL the wave's batches (up to four: 16 rows per lane quarter in flight), then the
//           softmax update over them.
// sparse_attention_wg_kernel pays count -> positions -> one trip per batch: five in a row for 656 keys per head.
// Lists longer than 1024 entries take further rounds of two trips each.
template <typename KT>
__global__ void __launch_bounds__(1024)
sparse_attention_wg_carry_kernel(const void *__restrict__ V, const int32_t *__restrict__ pos_slot,
                                 const int32_t *__restrict__ idx, const float *__restrict__ scores, int64_t score_stride,
                                 const int32_t *count, int count_stride,   // may alias head_count: not restrict
                                 int64_t cap, float *__restrict__ out, int64_t cap_rows, int64_t n_total, int n_q_heads,
                                 int n_kv_heads, int G, float qscale, int32_t *head_count,
                                 int32_t *__restrict__ head_stat, int32_t *__restrict__ publish_count) {
    constexpr int NW = 16;
    __shared__ float s_m[NW], s_l[NW];
    __shared__ float s_o[NW][LVR_D];
    const int64_t hq = blockIdx.x;
    const int bh = (int)((uint32_t)hq / (uint32_t)G);   // (hq / H_q) * H_kv + (hq % H_q) / G with H_q = H_kv * G: one 32-bit division
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, sub = lane >> 4, li = lane & 15;
    const int32_t *my_idx = idx + hq * cap;
    const float *my_sc = scores + hq * score_stride;
    const char *Vb = static_cast<const char *>(V) + (int64_t)bh * cap_rows * LVR_D * sizeof(KT);
    const int32_t *pslot = pos_slot ? pos_slot + (int64_t)bh * cap_rows : nullptr;

    // trip 1 (the count first: it is read through the scalar unit, whose argument loads and the read itself form a
    // chain of their own that should start before the vector loads are set up, not after)
    int64_t cnt = count[hq * count_stride];
    const int64_t e_rel = (int64_t)(wave + NW * sub) * 16 + li;   // this lane's entry within a round of 1024
    int32_t pos = (e_rel < cap) ? my_idx[e_rel] : -1;
    float sc = (e_rel < cap && e_rel < score_stride) ? my_sc[e_rel] : 0.f;
    const int32_t true_cnt = (int32_t)cnt;
    if (cnt > cap) cnt = cap;
    if (cnt < 0) cnt = 0;

    // m and l are the same in all lanes of the wave; acc holds the partial sums of this lane quarter's rows
    float m = -INFINITY, l = 0.f, acc[8];
    lvr_zero8(acc);
    for (int64_t base = 0; base < cnt; base += NW * 64) {   // uniform over the workgroup
        const int64_t e = base + e_rel;
        if (base > 0) {
            pos = (e < cnt) ? my_idx[e] : -1;
            sc = (e < cnt && e < score_stride) ? my_sc[e] : 0.f;
        }
        int myslot = -1;
        if (e < cnt && pos >= 0 && pos < n_total) myslot = pslot ? pslot[pos] : (int)pos;
        // trip 2: batch bq of this wave is entries base + (wave + 16 bq) * 16 ..; row i * 4 + sub of it is held by lane 16 bq + i * 4 + sub
        lvr_raw8<KT> vr[16];
        bool have[4];
#pragma unroll
        for (int bq = 0; bq < 4; ++bq) {
            have[bq] = base + (int64_t)(wave + NW * bq) * 16 < cnt;   // wave-uniform
            if (have[bq]) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int sl = __shfl(myslot, 16 * bq + i * 4 + sub, 64);
                    lvr_load_raw(Vb, sl < 0 ? 0 : sl, li, vr[bq * 4 + i]);
                }
            }
        }
        if (!have[0]) continue;   // wave-uniform: none of this wave's batches holds an entry in this pass over 1024 entries
        // The scores are here already, so the softmax weights of all 64 entries are formed while the rows travel:
        // one maximum and one sum over the wave, one exponential per lane, instead of a chain of rescalings per row.
        const float s_e = (myslot >= 0) ? sc * qscale : -INFINITY;
        float mw = s_e;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) mw = fmaxf(mw, __shfl_xor(mw, off, 64));
        const float m_new = fmaxf(m, mw);
        const float w_e = exp2_safe(s_e, m_new);
        float lw = w_e;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) lw += __shfl_xor(lw, off, 64);
        const float alpha = exp2_safe(m, m_new);
        l = l * alpha + lw;
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[c] *= alpha;
        m = m_new;
#pragma unroll
        for (int bq = 0; bq < 4; ++bq) {
            if (have[bq]) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float w = __shfl(w_e, 16 * bq + i * 4 + sub, 64);   // 0 for a masked entry
                    float vx[8];
                    lvr_unpack(vr[bq * 4 + i], vx);
#pragma unroll
                    for (int c = 0; c < 8; ++c) acc[c] += w * vx[c];
                }
            }
        }
    }
    const float m_all = m;
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        float a = acc[c];
        a += __shfl_xor(a, 16, 64);
        a += __shfl_xor(a, 32, 64);
        if (sub == 0) s_o[wave][li * 8 + c] = a;
    }
    if (lane == 0) {
        s_m[wave] = m_all;
        s_l[wave] = l;
    }
    __syncthreads();
    if (threadIdx.x < LVR_D) {
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < NW; ++w) M = fmaxf(M, s_m[w]);
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float wt = exp2_safe(s_m[w], M);
            den += wt * s_l[w];
            num += wt * s_o[w][threadIdx.x];
        }
        out[hq * LVR_D + threadIdx.x] = (den > 0.f && M != -INFINITY) ? num / den : 0.f;
    }
    // every thread's read of the count lies before the barrier above, so the counter can be handed over and cleared
    if (publish_count && threadIdx.x == 0) {
        publish_count[hq] = true_cnt;
        head_stat[hq] = true_cnt;
        head_count[hq * LVR_CNT_STRIDE] = 0;
    }
}

// The same with SPLIT workgroups per head (SPLIT = 2), each responsible for one half of the channels: it reads one cache line of
// every V row (eight lanes per row instead of sixteen) and writes 64 of the 128 outputs.  Both form the same
// softmax weights from the carried scores, so nothing has to be merged between them; what one compute unit has to
// pull through its 64 bytes per clock halves.  The two take a ticket once all their threads hold the count; the
// one that draws the second ticket publishes the count and clears the head's counter when it ends.
template <typename KT, int SPLIT>
__global__ void __launch_bounds__(1024)
sparse_attention_wg_carry_split_kernel(const void *__restrict__ V, const int32_t *__restrict__ pos_slot,
                                 const int32_t *__restrict__ idx, const float *__restrict__ scores, int64_t score_stride,
                                 const int32_t *count, int count_stride,   // may alias head_count: not restrict
                                 int64_t cap, float *__restrict__ out, int64_t cap_rows, int64_t n_total, int n_q_heads,
                                 int n_kv_heads, int G, float qscale, int32_t *head_count,
                                 int32_t *__restrict__ head_stat, int32_t *__restrict__ publish_count,
                                 int32_t *__restrict__ ticket) {
    constexpr int NW = 16;
    constexpr int LPR = 16 / SPLIT;          // lanes per row (16 bytes each)
    constexpr int RPL = 64 / LPR;            // rows per load instruction of a wave
    constexpr int NLOAD = 64 / RPL;          // load instructions that cover a wave's 64 entries
    constexpr int CH = LVR_D / SPLIT;        // channels this workgroup is responsible for
    __shared__ float s_m[NW], s_l[NW];
    __shared__ float s_o[NW][CH];
    const int64_t hq = blockIdx.x / SPLIT;
    const int part = blockIdx.x % SPLIT;
    const int bh = (int)((uint32_t)hq / (uint32_t)G);   // (hq / H_q) * H_kv + (hq % H_q) / G with H_q = H_kv * G: one 32-bit division
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, sub = lane >> 4, li = lane & 15;
    const int grp = lane / LPR, lp = lane % LPR;   // this lane's row within a load, its 16-byte piece of the row part
    const int32_t *my_idx = idx + hq * cap;
    const float *my_sc = scores + hq * score_stride;
    const char *Vb = static_cast<const char *>(V) + (int64_t)bh * cap_rows * LVR_D * sizeof(KT);
    const int32_t *pslot = pos_slot ? pos_slot + (int64_t)bh * cap_rows : nullptr;

    // trip 1 (the count first: it is read through the scalar unit, whose argument loads and the read itself form a
    // chain of their own that should start before the vector loads are set up, not after)
    int64_t cnt = count[hq * count_stride];
    const int64_t e_rel = (int64_t)(wave + NW * sub) * 16 + li;   // this lane's entry within a round of 1024
    int32_t pos = (e_rel < cap) ? my_idx[e_rel] : -1;
    float sc = (e_rel < cap && e_rel < score_stride) ? my_sc[e_rel] : 0.f;
    const int32_t true_cnt = (int32_t)cnt;
    if (cnt > cap) cnt = cap;
    if (cnt < 0) cnt = 0;
    int drawn = 0;
    if constexpr (SPLIT > 1) {
        // the empty statement consumes the loaded value, so every thread waits for its copy of the count before the
        // barrier; behind the barrier the workgroup may announce that it no longer needs the counter
        asm volatile("" ::"v"(true_cnt));
        __syncthreads();
        if (threadIdx.x == 0) drawn = atomicAdd(&ticket[hq], 1);
    }

    // m and l are the same in all lanes of the wave; acc holds the partial sums of this lane group's rows
    float m = -INFINITY, l = 0.f, acc[8];
    lvr_zero8(acc);
    for (int64_t base = 0; base < cnt; base += NW * 64) {   // uniform over the workgroup
        const int64_t e = base + e_rel;
        if (base > 0) {
            pos = (e < cnt) ? my_idx[e] : -1;
            sc = (e < cnt && e < score_stride) ? my_sc[e] : 0.f;
        }
        int myslot = -1;
        if (e < cnt && pos >= 0 && pos < n_total) myslot = pslot ? pslot[pos] : (int)pos;
        // trip 2: load j of the wave fetches the rows of the entries held by lanes j * RPL .. j * RPL + RPL - 1 (row
        // grp of them is this lane's); those lanes belong to batch (j * RPL) / 16 of the wave, entries
        // base + (wave + 16 bq) * 16 ..
        lvr_raw8<KT> vr[NLOAD];
        bool have[4];
#pragma unroll
        for (int bq = 0; bq < 4; ++bq) have[bq] = base + (int64_t)(wave + NW * bq) * 16 < cnt;   // wave-uniform
#pragma unroll
        for (int j = 0; j < NLOAD; ++j) {
            if (have[(j * RPL) / 16]) {
                const int sl = __shfl(myslot, j * RPL + grp, 64);
                lvr_load_raw(Vb, sl < 0 ? 0 : sl, part * LPR + lp, vr[j]);
            }
        }
        if (!have[0]) continue;   // wave-uniform: none of this wave's batches holds an entry in this pass over 1024 entries
        // The scores are here already, so the softmax weights of all 64 entries are formed while the rows travel:
        // one maximum and one sum over the wave, one exponential per lane, instead of a chain of rescalings per row.
        const float s_e = (myslot >= 0) ? sc * qscale : -INFINITY;
        float mw = s_e;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) mw = fmaxf(mw, __shfl_xor(mw, off, 64));
        const float m_new = fmaxf(m, mw);
        const float w_e = exp2_safe(s_e, m_new);
        float lw = w_e;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) lw += __shfl_xor(lw, off, 64);
        const float alpha = exp2_safe(m, m_new);
        l = l * alpha + lw;
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[c] *= alpha;
        m = m_new;
#pragma unroll
        for (int j = 0; j < NLOAD; ++j) {
            if (have[(j * RPL) / 16]) {
                const float w = __shfl(w_e, j * RPL + grp, 64);   // 0 for a masked entry
                float vx[8];
                lvr_unpack(vr[j], vx);
#pragma unroll
                for (int c = 0; c < 8; ++c) acc[c] += w * vx[c];
            }
        }
    }
    const float m_all = m;
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        float a = acc[c];
#pragma unroll
        for (int off = LPR; off < 64; off <<= 1) a += __shfl_xor(a, off, 64);
        if (grp == 0) s_o[wave][lp * 8 + c] = a;
    }
    if (lane == 0) {
        s_m[wave] = m_all;
        s_l[wave] = l;
    }
    __syncthreads();
    if (threadIdx.x < CH) {
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < NW; ++w) M = fmaxf(M, s_m[w]);
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float wt = exp2_safe(s_m[w], M);
            den += wt * s_l[w];
            num += wt * s_o[w][threadIdx.x];
        }
        out[hq * LVR_D + part * CH + threadIdx.x] = (den > 0.f && M != -INFINITY) ? num / den : 0.f;
    }
    // every thread's read of the count lies before a barrier above (in both workgroups of a split head once the
    // second ticket has been drawn), so the counter can be handed over and cleared
    if (publish_count && threadIdx.x == 0 && (SPLIT == 1 || drawn == SPLIT - 1)) {
        publish_count[hq] = true_cnt;
        head_stat[hq] = true_cnt;
        head_count[hq * LVR_CNT_STRIDE] = 0;
        if constexpr (SPLIT > 1) ticket[hq] = 0;
    }
}

// Merge of the partial triples of one query head.  512 threads: thread (slice s, channel c) owns
// every fourth partial of channel c; its values are requested first, then the weights
// w_p = 2^(m_p - M) are computed into LDS, the slices are weighted, and the four slices are
// added through LDS.  With a count pointer the number of partials in use follows the sparse
// attention's split geometry; without one all P are merged (dense baseline).
constexpr int COMBINE_MAX_P = 256;

// `count` and `head_count` may be the same array (the decode step hands the internal counters to
// both), so neither is declared restrict, every thread reads the count BEFORE the kernel's first
// barrier and the counter is cleared only AFTER it.
__global__ void __launch_bounds__(512)
combine_kernel(const float *__restrict__ part_ml, const float *__restrict__ part_o, float *__restrict__ out, int P,
               const int32_t *count, int count_stride, int64_t cap, int32_t *head_count,
               int32_t *__restrict__ head_stat, int32_t *__restrict__ publish_count) {
    __shared__ float s_w[COMBINE_MAX_P];
    __shared__ float s_red[8];
    __shared__ float s_num[4][LVR_D];
    const int64_t hq = blockIdx.x;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int c = t & (LVR_D - 1), sl = t >> 7;
    const float *po = part_o + hq * P * LVR_D + c;
    // up to 16 partials per thread (all of them for P <= 64) and the (m, l) pairs are requested
    // first, together with the count, so that nothing waits for a second trip to memory; what
    // lies beyond the partials in use is stale and is masked once the count has arrived
    float pv[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int p = sl + 4 * i;
        pv[i] = (p < P) ? po[(int64_t)p * LVR_D] : 0.f;
    }
    const float m_raw = (t < P) ? part_ml[(hq * P + t) * 2] : -INFINITY;
    const float l_raw = (t < P) ? part_ml[(hq * P + t) * 2 + 1] : 0.f;
    int used = P;
    int32_t true_cnt = 0;
    if (count) {
        int64_t cnt = count[hq * count_stride];
        true_cnt = (int32_t)cnt;
        if (cnt > cap) cnt = cap;
        if (cnt < 0) cnt = 0;
        split_length(cnt, P, &used);
    }
    const float m = (t < used) ? m_raw : -INFINITY;
    const float l = (t < used) ? l_raw : 0.f;
    float mx = m;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
    if (lane == 0) s_red[wave] = mx;
    __syncthreads();
    // every thread's read of the count has completed (its value fed the shuffle above), so the
    // counter can be handed over and cleared for the next query
    if (count && publish_count && t == 0) {
        publish_count[hq] = true_cnt;
        head_stat[hq] = true_cnt;
        head_count[hq * LVR_CNT_STRIDE] = 0;
    }
    float M = s_red[0];
#pragma unroll
    for (int w = 1; w < 8; ++w) M = fmaxf(M, s_red[w]);
    __syncthreads();
    const float w_p = exp2_safe(m, M);
    if (t < COMBINE_MAX_P) s_w[t] = w_p;
    float dn = w_p * l;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) dn += __shfl_xor(dn, off, 64);
    if (lane == 0) s_red[wave] = dn;
    __syncthreads();
    float den = 0.f;
#pragma unroll
    for (int w = 0; w < 8; ++w) den += s_red[w];
    float num = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int p = sl + 4 * i;
        num += (p < used) ? s_w[p] * pv[i] : 0.f;
    }
#pragma unroll 4
    for (int p = sl + 64; p < used; p += 4) num += s_w[p] * po[(int64_t)p * LVR_D];
    s_num[sl][c] = num;
    __syncthreads();
    if (t < LVR_D) {
        const float tot = s_num[0][t] + s_num[1][t] + s_num[2][t] + s_num[3][t];
        out[hq * LVR_D + t] = (den > 0.f && M != -INFINITY) ? tot / den : 0.f;
    }
}

template <typename KT, int G>
__global__ void __launch_bounds__(256)
dense_partial_kernel(const void *__restrict__ K, const void *__restrict__ V, const float *__restrict__ q,
                     float *__restrict__ part_ml, float *__restrict__ part_o, int64_t cap_rows, int64_t n_total,
                     int P, int n_q_heads, int n_kv_heads, float qscale) {
    __shared__ float sm_m[4][G], sm_l[4][G];
    __shared__ float sm_o[4][G][LVR_D];
    const int bh = blockIdx.y, p = blockIdx.x;
    const int b = bh / n_kv_heads, kvh = bh % n_kv_heads;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane >> 4, li = lane & 15;
    const int64_t hq0 = (int64_t)b * n_q_heads + kvh * G;

    const int64_t R = (((n_total + P - 1) / P) + 15) & ~(int64_t)15;
    const int64_t start = (int64_t)p * R;
    const int64_t end = (start + R < n_total) ? start + R : n_total;

    float qv[G][8];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        const float *qh = q + (hq0 + h) * LVR_D + li * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) qv[h][e] = qh[e] * qscale;
    }
    const char *Kb = static_cast<const char *>(K) + (int64_t)bh * cap_rows * LVR_D * sizeof(KT);
    const char *Vb = static_cast<const char *>(V) + (int64_t)bh * cap_rows * LVR_D * sizeof(KT);

    float m[G], l[G], acc[G][8];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        m[h] = -INFINITY;
        l[h] = 0.f;
        lvr_zero8(acc[h]);
    }
    for (int64_t r0 = start + wave * 4; r0 < end; r0 += 16) {   // uniform over the wave
        const int64_t row = r0 + sub;
        const bool valid = row < end;
        const int64_t rc = valid ? row : 0;
        float kx[8], vx[8];
        lvr_load8<KT>(Kb, rc, li, kx);
        lvr_load8<KT>(Vb, rc, li, vx);
#pragma unroll
        for (int h = 0; h < G; ++h) {
            float d = 0.f;
#pragma unroll
            for (int c = 0; c < 8; ++c) d += qv[h][c] * kx[c];
            float s = lvr_row16_sum(d);
            s = valid ? s : -INFINITY;
            const float m_new = fmaxf(m[h], s);
            const float alpha = exp2_safe(m[h], m_new);
            const float w = exp2_safe(s, m_new);
            l[h] = l[h] * alpha + w;
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[h][c] = acc[h][c] * alpha + w * vx[c];
            m[h] = m_new;
        }
    }
#pragma unroll
    for (int h = 0; h < G; ++h) {
        float m_all = fmaxf(m[h], __shfl_xor(m[h], 16, 64));
        m_all = fmaxf(m_all, __shfl_xor(m_all, 32, 64));
        const float sc = exp2_safe(m[h], m_all);
        float lh = l[h] * sc;
        lh += __shfl_xor(lh, 16, 64);
        lh += __shfl_xor(lh, 32, 64);
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            float a = acc[h][c] * sc;
            a += __shfl_xor(a, 16, 64);
            a += __shfl_xor(a, 32, 64);
            if (sub == 0) sm_o[wave][h][li * 8 + c] = a;
        }
        if (lane == 0) {
            sm_m[wave][h] = m_all;
            sm_l[wave][h] = lh;
        }
    }
    __syncthreads();
    // 256 threads merge the four waves: thread -> (head pair, channel)
    for (int item = threadIdx.x; item < G * LVR_D; item += 256) {
        const int h = item / LVR_D, c = item % LVR_D;
        float M = fmaxf(fmaxf(sm_m[0][h], sm_m[1][h]), fmaxf(sm_m[2][h], sm_m[3][h]));
        float o = 0.f, lt = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float sc = exp2_safe(sm_m[w][h], M);
            o += sc * sm_o[w][h][c];
            lt += sc * sm_l[w][h];
        }
        part_o[((hq0 + h) * P + p) * LVR_D + c] = o;
        if (c == 0) {
            part_ml[((hq0 + h) * P + p) * 2] = M;
            part_ml[((hq0 + h) * P + p) * 2 + 1] = lt;
        }
    }
}

// Dense baseline for bf16 caches with the logits on the matrix cores.  A wave takes tiles of 16
// rows: K in MFMA operand layout (scores as in mfma_score.h, q pre-scaled by sigma*log2 e), V in
// row layout (lane (sub, li): row 4i+sub, channels 8li..8li+7).  The lanes that hold the scores
// keep the running maximum, turn the tile's scores into weights and hand them (and the rescale
// factor) to the V lanes through LDS; the weighted sum of V runs on the vector ALU.
template <int HB>
__global__ void __launch_bounds__(256)
dense_mfma_kernel(const void *__restrict__ K, const void *__restrict__ V, const float *__restrict__ q,
                  float *__restrict__ part_ml, float *__restrict__ part_o, int64_t cap_rows, int64_t n_total, int P,
                  int n_q_heads, int n_kv_heads, int G, float qscale) {
    constexpr int NH = HB * 4;
    __shared__ uint4 s_bq[HB][4][64];
    __shared__ float s_p[4][NH][4][4];      // [wave][head][row % 4][row / 4]
    __shared__ float s_alpha[4][NH];
    __shared__ float sm_m[4][NH], sm_l[4][NH];
    __shared__ float sm_o[4][NH][LVR_D];
    const int bh = blockIdx.y, p = blockIdx.x;
    const int b = bh / n_kv_heads, kvh = bh % n_kv_heads;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 15, kq = lane >> 4;     // MFMA roles
    const int sub = kq, li = n;                  // V roles
    const int64_t hq0 = (int64_t)b * n_q_heads + kvh * G;

    const int64_t R = (((n_total + P - 1) / P) + 15) & ~(int64_t)15;
    const int64_t start = (int64_t)p * R;
    const int64_t end = (start + R < n_total) ? start + R : n_total;

    lvr_bf16x8 bq[HB][4];
    lvr_build_q_frags_wg<HB>(q + hq0 * LVR_D, G, qscale, s_bq, bq);
    const bool rep = n >= 8 && n < 12;           // this lane holds scores of head hb*4 + n - 8
    const char *Kb = static_cast<const char *>(K) + (int64_t)bh * cap_rows * LVR_D * 2;
    const char *Vb = static_cast<const char *>(V) + (int64_t)bh * cap_rows * LVR_D * 2;

    float m_run[HB], l_run[HB], acc[NH][8];
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) {
        m_run[hb] = -INFINITY;
        l_run[hb] = 0.f;
    }
#pragma unroll
    for (int h = 0; h < NH; ++h) lvr_zero8(acc[h]);

    // the waves of the workgroups that share a compute unit take turns at the top priority (at equal priority the
    // oldest wave is served first and the workgroups dispatched last finish last), as in the sparse path's query kernel
    const int prio_phase = (int)((blockIdx.y * gridDim.x + blockIdx.x) >> 8);
    int turn = 0;
    for (int64_t r0 = start + wave * 16; r0 < end; r0 += 64) {   // uniform over the wave
        switch ((prio_phase + (turn++ >> 1)) & 3) {
            case 0: __builtin_amdgcn_s_setprio(0); break;
            case 1: __builtin_amdgcn_s_setprio(1); break;
            case 2: __builtin_amdgcn_s_setprio(2); break;
            default: __builtin_amdgcn_s_setprio(3); break;
        }
        uint4 av[4];
        lvr_raw8<lvr_bf16_t> vr[4];
        {
            int64_t row = r0 + n;
            if (row >= end) row = end - 1;
            lvr_load_a_frags(Kb, row, av);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int64_t row = r0 + 4 * i + sub;
            if (row >= end) row = end - 1;
            lvr_load_raw(Vb, row, li, vr[i]);
        }
#pragma unroll
        for (int hb = 0; hb < HB; ++hb) {
            lvr_f32x4 s = lvr_score_tile(av, bq[hb]);
            float tmax = -INFINITY;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (r0 + 4 * kq + j >= end) s[j] = -INFINITY;
                tmax = fmaxf(tmax, s[j]);
            }
            tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
            tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
            const float m_new = fmaxf(m_run[hb], tmax);
            const float alpha = exp2_safe(m_run[hb], m_new);
            float psum = 0.f;
            float pj[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                pj[j] = exp2_safe(s[j], m_new);
                psum += pj[j];
            }
            l_run[hb] = l_run[hb] * alpha + psum;
            m_run[hb] = m_new;
            if (rep) {
                const int h = hb * 4 + n - 8;
#pragma unroll
                for (int j = 0; j < 4; ++j) s_p[wave][h][j][kq] = pj[j];
                if (kq == 0) s_alpha[wave][h] = alpha;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        float vx[4][8];
#pragma unroll
        for (int i = 0; i < 4; ++i) lvr_unpack(vr[i], vx[i]);
#pragma unroll
        for (int h = 0; h < NH; ++h) {
            const float4 pw = *reinterpret_cast<const float4 *>(&s_p[wave][h][sub][0]);
            const float al = s_alpha[wave][h];
#pragma unroll
            for (int c = 0; c < 8; ++c)
                acc[h][c] = acc[h][c] * al + pw.x * vx[0][c] + pw.y * vx[1][c] + pw.z * vx[2][c] + pw.w * vx[3][c];
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
    __builtin_amdgcn_s_setprio(0);
    // per wave: add the four row subsets (same running maximum), collect l over the score lanes
#pragma unroll
    for (int h = 0; h < NH; ++h) {
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            float a = acc[h][c];
            a += __shfl_xor(a, 16, 64);
            a += __shfl_xor(a, 32, 64);
            if (sub == 0) sm_o[wave][h][li * 8 + c] = a;
        }
    }
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) {
        float lh = l_run[hb];
        lh += __shfl_xor(lh, 16, 64);
        lh += __shfl_xor(lh, 32, 64);
        if (rep && kq == 0) {
            sm_m[wave][hb * 4 + n - 8] = m_run[hb];
            sm_l[wave][hb * 4 + n - 8] = lh;
        }
    }
    __syncthreads();
    for (int item = threadIdx.x; item < G * LVR_D; item += 256) {
        const int h = item / LVR_D, c = item % LVR_D;
        const float M = fmaxf(fmaxf(sm_m[0][h], sm_m[1][h]), fmaxf(sm_m[2][h], sm_m[3][h]));
        float o = 0.f, lt = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float sc = exp2_safe(sm_m[w][h], M);
            o += sc * sm_o[w][h][c];
            lt += sc * sm_l[w][h];
        }
        part_o[((hq0 + h) * P + p) * LVR_D + c] = o;
        if (c == 0) {
            part_ml[((hq0 + h) * P + p) * 2] = M;
            part_ml[((hq0 + h) * P + p) * 2 + 1] = lt;
        }
    }
}

template <typename KT>
hipError_t launch_dense_t(lvr_index *ix, const float *q, float *out, int P, hipStream_t st) {
    dim3 grid((unsigned)P, (unsigned)lvr_n_bh(ix));
    const float qscale = ix->sigma * LOG2E;
#define LVR_DENSE_CASE(GG)                                                                                     \
    case GG:                                                                                                   \
        hipLaunchKernelGGL((dense_partial_kernel<KT, GG>), grid, dim3(256), 0, st, ix->K, ix->V, q, ix->part_ml, \
                           ix->part_o, ix->cap_rows, ix->n_total, P, ix->cfg.n_q_heads, ix->cfg.n_kv_heads,    \
                           qscale);                                                                            \
        break;
    switch (ix->G) {
        LVR_DENSE_CASE(1)
        LVR_DENSE_CASE(2)
        LVR_DENSE_CASE(4)
        LVR_DENSE_CASE(8)
        default: return hipErrorInvalidValue;
    }
#undef LVR_DENSE_CASE
    return hipGetLastError();
}

}  // namespace

hipError_t lvr_launch_sparse_attention_wg(lvr_index *ix, const float *q, const int32_t *idx, const float *scores,
                                          const int32_t *count, int count_stride, int64_t cap, float *out,
                                          int32_t *publish_count, hipStream_t st) {
    const int n_bhq = lvr_n_bhq(ix);
    const float qscale = ix->sigma * LOG2E;
    // a pair of events handed in by the caller goes into the dispatch itself (they then read the kernel's own start and end)
    hipEvent_t ev0 = ix->launch_start, ev1 = ix->launch_stop;
#define LVR_AT_LAUNCH(KERNEL, GRID, ...)                                                                    \
    do {                                                                                                    \
        if (ev0) hipExtLaunchKernelGGL(KERNEL, GRID, dim3(1024), 0, st, ev0, ev1, 0, __VA_ARGS__);           \
        else hipLaunchKernelGGL(KERNEL, GRID, dim3(1024), 0, st, __VA_ARGS__);                              \
    } while (0)
#define LVR_WG_LAUNCH(KT, CARRY)                                                                                         \
    LVR_AT_LAUNCH((sparse_attention_wg_kernel<KT, CARRY>), dim3((unsigned)n_bhq), ix->K, ix->V,                          \
                  ix->pos_slot, q, idx, scores, ix->cap_rows, count, count_stride, cap, out, ix->cap_rows,               \
                  ix->n_total, ix->cfg.n_q_heads, ix->cfg.n_kv_heads, ix->G, qscale, lvr_head_count(ix),                 \
                  lvr_head_stat(ix), publish_count)
    if (ix->cfg.kv_dtype == LVR_BF16) {
        // With more heads than compute units the workgroups queue up behind each other and the lighter kernel wins
        // (512 heads: 24.0 against 26.0 us); with one workgroup per unit the shorter chain of trips does (32 heads:
        // 8.4 against 8.7 us at 328 keys per head, 10.5 against 10.9 us at 656).
        // Up to 128 heads two workgroups can share a head (one per half of the channels) and every workgroup still
        // has a compute unit of its own.  That pays where a head's list is long (656 keys per head at 128k keys of
        // context: 9.1 against 9.7 us); short lists lose more to the extra barrier and the ticket than they gain
        // (3.6 keys per head: 7.6 against 6.9 us), and the list lengths are not known on the host, so the context
        // length stands in as it does for the launch form.
        if (scores && n_bhq > 256) LVR_WG_LAUNCH(lvr_bf16_t, true);
        else if (scores && n_bhq <= 128 && publish_count && ix->n_total > 65536)
            LVR_AT_LAUNCH((sparse_attention_wg_carry_split_kernel<lvr_bf16_t, 2>), dim3((unsigned)n_bhq * 2),
                               ix->V, ix->pos_slot, idx, scores, ix->cap_rows, count, count_stride, cap, out, ix->cap_rows,
                               ix->n_total, ix->cfg.n_q_heads, ix->cfg.n_kv_heads, ix->G, qscale, lvr_head_count(ix),
                               lvr_head_stat(ix), publish_count, lvr_head_ticket(ix));
        else if (scores)
            LVR_AT_LAUNCH((sparse_attention_wg_carry_kernel<lvr_bf16_t>), dim3((unsigned)n_bhq), ix->V,
                               ix->pos_slot, idx, scores, ix->cap_rows, count, count_stride, cap, out, ix->cap_rows,
                               ix->n_total, ix->cfg.n_q_heads, ix->cfg.n_kv_heads, ix->G, qscale, lvr_head_count(ix),
                               lvr_head_stat(ix), publish_count);
        else LVR_WG_LAUNCH(lvr_bf16_t, false);
    } else {
        if (scores) LVR_WG_LAUNCH(lvr_f32_t, true);
        else LVR_WG_LAUNCH(lvr_f32_t, false);
    }
#undef LVR_WG_LAUNCH
#undef LVR_AT_LAUNCH
    return hipGetLastError();
}

hipError_t lvr_launch_sparse_partial(lvr_index *ix, const float *q, const int32_t *idx, const float *scores,
                                     const int32_t *count, int count_stride, int64_t cap, hipStream_t st) {
    const int n_bhq = lvr_n_bhq(ix);
    const int P = ix->P;
    dim3 grid((unsigned)P, (unsigned)n_bhq);
    const float qscale = ix->sigma * LOG2E;
#define LVR_PART_LAUNCH(KT, CARRY)                                                                                       \
    hipLaunchKernelGGL((sparse_attention_kernel<KT, CARRY>), grid, dim3(64), 0, st, ix->K, ix->V, ix->pos_slot, q, idx,  \
                       scores, ix->cap_rows, count, count_stride, cap, ix->part_ml, ix->part_o, ix->cap_rows,            \
                       ix->n_total, P, ix->cfg.n_q_heads, ix->cfg.n_kv_heads, ix->G, qscale)
    if (ix->cfg.kv_dtype == LVR_BF16) {
        if (scores) LVR_PART_LAUNCH(lvr_bf16_t, true);
        else LVR_PART_LAUNCH(lvr_bf16_t, false);
    } else {
        if (scores) LVR_PART_LAUNCH(lvr_f32_t, true);
        else LVR_PART_LAUNCH(lvr_f32_t, false);
    }
#undef LVR_PART_LAUNCH
    return hipGetLastError();
}

int lvr_dense_splits(const lvr_index *ix) {
    int64_t P = (ix->n_total + 63) / 64;
    if (P > ix->P_dense) P = ix->P_dense;
    if (P < 1) P = 1;
    return (int)P;
}

hipError_t lvr_launch_dense_partial(lvr_index *ix, const float *q, hipStream_t st) {
    const int P = lvr_dense_splits(ix);
    if (ix->cfg.kv_dtype == LVR_BF16 && ix->n_total > 0) {
        dim3 grid((unsigned)P, (unsigned)lvr_n_bh(ix));
        const float qscale = ix->sigma * LOG2E;
        if (ix->G <= 4)
            hipLaunchKernelGGL(dense_mfma_kernel<1>, grid, dim3(256), 0, st, ix->K, ix->V, q, ix->part_ml, ix->part_o,
                               ix->cap_rows, ix->n_total, P, ix->cfg.n_q_heads, ix->cfg.n_kv_heads, ix->G, qscale);
        else
            hipLaunchKernelGGL(dense_mfma_kernel<2>, grid, dim3(256), 0, st, ix->K, ix->V, q, ix->part_ml, ix->part_o,
                               ix->cap_rows, ix->n_total, P, ix->cfg.n_q_heads, ix->cfg.n_kv_heads, ix->G, qscale);
        return hipGetLastError();
    }
    return ix->cfg.kv_dtype == LVR_BF16 ? launch_dense_t<lvr_bf16_t>(ix, q, nullptr, P, st)
                                        : launch_dense_t<lvr_f32_t>(ix, q, nullptr, P, st);
}

hipError_t lvr_launch_combine(lvr_index *ix, float *out, int P, const int32_t *count, int count_stride, int64_t cap,
                              int32_t *publish_count, hipStream_t st) {
    const int n_bhq = lvr_n_bhq(ix);
    hipLaunchKernelGGL(combine_kernel, dim3((unsigned)n_bhq), dim3(512), 0, st, ix->part_ml, ix->part_o, out, P, count,
                       count_stride, cap, lvr_head_count(ix), lvr_head_stat(ix), publish_count);
    return hipGetLastError();
}
