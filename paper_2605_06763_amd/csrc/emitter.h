// Per-wave emission queue shared by the exact-filter kernels.
//
// Qualifying positions go to a small per-wave queue in LDS first; a queue is flushed with ONE
// atomic per head on a counter that owns its cache line, so a launch issues a few thousand
// atomics spread over many lines instead of one per hit on a few lines (atomics that hit one
// line are served one after the other by the memory side).
#pragma once
#include "lvr_internal.h"

#ifdef __HIPCC__
constexpr int LVR_QCAP = 64;   // queue entries per (wave, head)

struct lvr_emit_target {
    int32_t *out_idx;        // [n_bhq][cap]
    int32_t *head_count;     // padded, LVR_CNT_STRIDE ints apart
    int32_t *overflow;
    int64_t cap;
    float *out_score;        // [n_bhq][score_stride] raw scores of the emitted keys (emitters that carry them), or NULL
    int64_t score_stride;
};

// The lanes with (lane % 16) in [rep_base, rep_base+NH) report head (lane % 16) - rep_base; the
// four lanes (one per quarter of the wave) that report the same head keep identical counts.
// CARRY: the raw score of every queued key travels with it, so that the attention that follows
// needs neither the key row nor the dot product again.
template <int NH, bool CARRY = false>
struct lvr_emitter {
    int32_t (*q)[LVR_QCAP];   // LDS, [NH][LVR_QCAP], private to the wave
    float (*qs)[LVR_QCAP];    // LDS, scores of the queued keys (CARRY only)
    int count;                // queued entries of my head (0 on lanes that report nothing)
    int rep_base;
    int64_t hq_base;          // flat index of head 0

    // The queue holds arena rows; `spos` (row -> token position, or NULL when rows are stored in
    // arrival order) is applied here, one gather per flush instead of one dependent load per hit.
    __device__ __forceinline__ void flush(const lvr_emit_target &a, int lane, bool reporting, const int32_t *spos) {
        const int hl = (lane & 15) - rep_base;
        int base = 0;
        if (reporting && (lane >> 4) == 0 && count > 0)
            base = atomicAdd(&a.head_count[(hq_base + hl) * LVR_CNT_STRIDE], count);
        write_out(a, lane, spos, base);
    }

    // The queued entries go to positions base .. base + count - 1 of their head's list; `base` is read from the
    // lanes of the first quarter that report a head (the caller has reserved the range).
    __device__ __forceinline__ void write_out(const lvr_emit_target &a, int lane, const int32_t *spos, int base) {
        __builtin_amdgcn_wave_barrier();
        // four heads: unrolled, the four gathers overlap; eight heads unrolled would keep all eight in
        // registers at once (182 VGPRs in the query kernel), so they go two at a time
        constexpr int kUnroll = NH <= 4 ? NH : 2;
#pragma unroll kUnroll
        for (int h = 0; h < NH; ++h) {
            // the reporting lane is the same for the whole wave: a lane read, not a shuffle through LDS
            const int b_h = __builtin_amdgcn_readlane(base, rep_base + h);
            const int c_h = __builtin_amdgcn_readlane(count, rep_base + h);
            if (lane < c_h) {
                const int64_t p = (int64_t)b_h + lane;
                if (p < a.cap) {
                    const int32_t row = q[h][lane];
                    a.out_idx[(hq_base + h) * a.cap + p] = spos ? spos[row] : row;
                    if constexpr (CARRY) {
                        if (p < a.score_stride) a.out_score[(hq_base + h) * a.score_stride + p] = qs[h][lane];
                    }
                } else
                    *a.overflow = 1;
            }
        }
        __builtin_amdgcn_wave_barrier();
        count = 0;
    }

    // pred: this lane's (row, head) qualifies; the row's arena slot is held by lane `src_lane`.
    __device__ __forceinline__ void push(const lvr_emit_target &a, int lane, bool reporting, bool pred, int my_slot,
                                         int src_lane, const int32_t *spos, float score = 0.f) {
        const uint64_t any = __ballot(pred);
        if (!any) return;   // wave-uniform
        const int slot = __shfl(my_slot, src_lane, 64);
        const uint64_t mh = reporting ? (any & (0x0001000100010001ull << (lane & 15))) : 0ull;
        if (pred) {
            const int hl = (lane & 15) - rep_base;
            const int at = count + __popcll(mh & ((1ull << lane) - 1ull));
            q[hl][at] = slot;
            if constexpr (CARRY) qs[hl][at] = score;
        }
        count += __popcll(mh);
        if (__ballot(count > LVR_QCAP - 4)) flush(a, lane, reporting, spos);
    }
};
#endif
