// Internal declarations shared by the translation units of liblouver: the index object,
// host-side launcher prototypes and the device helpers every kernel uses.
//
// Thread mapping used throughout: a 64-lane wavefront is split into four "quarter rows" of
// 16 lanes; one head_dim = 128 row (a key, a value or a centre) is spread over the 16 lanes
// of a quarter, 8 consecutive elements per lane, so one wave-wide 16-byte load covers four
// bf16 rows (1 KiB) fully coalesced.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/louver.h"

#define LVR_D 128          // head_dim this build is specialised for
#define LVR_LANES_PER_ROW 16
#define LVR_ELEMS_PER_LANE 8
#define LVR_MAX_G 8

struct lvr_index {
    lvr_config cfg;
    int device;
    int G;                 // query heads per KV head
    int box;               // 1: groups are enclosed by axis-aligned boxes (two rows per group in `centres`)
    int S_store;           // floats per group in `radii` (S for balls, 1 for boxes)
    int cf8;               // 1: centres are stored as e4m3 codes, 128 bytes per group, in matrix-operand order
    int cf6;               // 1: centres are stored as e2m3 codes with a scale per 32 coordinates, 96 bytes per group,
                           //    in matrix-operand order; `radii` holds 12 bytes per group (four bf16 radii, four scale bytes)
    int centre_bytes;      // bytes of one enclosure row in `centres` (256 / 512 in the cache's format, 128, 96)
    int chan_scaled;       // 1: the 6-bit index lives in a rescaled space, coordinate c of every key divided by 2^e_c
                           //    (e_c per (sequence, KV head), see lvr_chan_exp); the query multiplies q_c by 2^e_c
    int64_t cap_rows;      // arena rows per (sequence, KV head), multiple of 64
    int64_t max_groups;    // cap_rows / r
    int64_t n_total;       // keys held
    int64_t n_indexed;     // keys inside groups (multiple of r)
    int built;
    int attn_one_launch;   // sparse attention as one workgroup per head (default) or partials + combine
    int P;                 // attention splits of the two-launch form
    int P_dense;           // splits of the dense baseline
    float sigma;
    size_t elt;            // bytes per K/V element
    // arena (device)
    void *K;               // [batch][H_kv][cap_rows][d]  (device address; host-resident in offloaded mode)
    void *V;
    void *K_host, *V_host; // offloaded mode: the pinned host allocations behind K and V, else NULL
    void *centres;         // [batch][H_kv][max_groups][d]  (boxes: [..][max_groups][2][d], upper then lower corner)
    float *radii;          // [batch][H_kv][max_groups][S_store]
    int32_t *slot_pos;     // [batch][H_kv][cap_rows] token position of arena row (TREE grouping), else NULL
    int32_t *pos_slot;     // inverse map, or NULL
    int32_t *reservoir;    // [batch][H_kv][R] token positions kept by reservoir sampling (-1 = unused), or NULL
    // one grouping per coordinate block (LVR_GROUP_SUBSPACE_TREE): per key its group in every block, and the
    // per-query table of block bounds that the labels point into
    uint16_t *labels;      // [batch][H_kv][cap_rows][S]
    float *f_table;        // [batch][H_kv][max_groups][S][4]
    int per_subspace;      // 1: that layout
    // work space of the tree grouping (TREE grouping only)
    uint64_t *tree_keys_a, *tree_keys_b;   // [n_bh * padded entries] sort keys, ping-pong
    int32_t *tree_axis;                    // [n_bh * nodes] split axis per node of the current level
    double *tree_partial;                  // partial coordinate statistics of large nodes
    void *tree_temp;                       // rocPRIM sort storage
    size_t tree_temp_bytes;
    int64_t tree_cap_keys;                 // keys tree_keys_* can hold
    void *chunk_K, *chunk_V;               // [n_bh][B][d] staging of a buffer chunk being regrouped
    // work space (device)
    int32_t *surv_list;    // [batch][H_kv][max_groups]: segment x owns entries [x*seg_groups, (x+1)*seg_groups)
    int32_t *counters;     // see lvr_head_count / lvr_overflow_flag / lvr_seg_count
    int seg_groups;        // groups per segment used by the last bound test
    int n_segs;            // segments per (sequence, KV head) filled by the last bound test (0: none)
    int counters_dirty;    // a query was started but its counts were never published (a launch failed)
    int skip_bounds;       // lvr_set_bound_test(ix, 0): queries run the exact filter alone over every indexed key
    float *scores;         // [batch][H_q][cap_rows] raw scores of the keys the fused query emitted, or NULL
    float *part_ml;        // [batch][H_q][Pmax][2]
    float *part_o;         // [batch][H_q][Pmax][d]
    int64_t last_buffer_rows; // buffer rows scanned by the last query (host copy for stats)
    int64_t last_indexed;     // indexed rows the last query saw
    int last_skipped;         // the last query ran with the bound test off
    // concurrent update (LVR_CONCURRENT_UPDATE): a full buffer is grouped on `side` while the
    // caller's stream keeps answering queries that still see those keys as buffer keys
    hipStream_t side;
    hipEvent_t ev_fork, ev_done;
    int pending;              // a chunk's groups are being prepared / wait to be published
    int64_t pend_row0;        // first arena row of that chunk
    struct lvr_tree_perm *pend_perm;   // TREE grouping: the chunk's order, gathered at publish time
    // optional per-kernel timing (lvr_profile_enable): pairs of events around every launch
    int prof_on;
    int prof_used;            // events handed out so far
    int prof_cap;             // events allocated
    hipEvent_t *prof_events;  // [prof_cap]
    uint8_t *prof_kind;       // [prof_cap / 2] kernel kind of each pair
    hipEvent_t launch_start, launch_stop;   // non-null: the next launch of a kernel that supports it hands these two to
                                            // the dispatch itself (they then read the kernel's own start and end, as a
                                            // profiler's trace does, instead of bracketing the launch on the stream)
};

enum lvr_kernel_kind {
    LVR_K_COPY = 0, LVR_K_BUILD, LVR_K_RESET, LVR_K_PRUNE, LVR_K_FILTER, LVR_K_ATTN_PARTIAL, LVR_K_ATTN_COMBINE,
    LVR_K_DENSE_PARTIAL, LVR_K_DENSE_COMBINE, LVR_K_COUNT
};

static inline int lvr_n_bh(const lvr_index *ix) { return ix->cfg.batch * ix->cfg.n_kv_heads; }
static inline int lvr_n_bhq(const lvr_index *ix) { return ix->cfg.batch * ix->cfg.n_q_heads; }

// Device counters.  Atomics that hit one 128-byte line are served one after the other
// (about 12 ns each on this part), so every counter that takes atomics owns a whole line.
#define LVR_CNT_STRIDE 32   // ints per counter slot (128 bytes)
#define LVR_CHAN_STRIDE (LVR_D + LVR_D * 4)   // bytes of channel scaling per (sequence, KV head): 128 exponents, 128 factors
#define LVR_MIN_SEG_GROUPS 64
// per query head: size of the retrieved set of the running query (padded).  Zero between
// queries: the kernel that publishes the counts clears them.
static inline int32_t *lvr_head_count(const lvr_index *ix) { return ix->counters; }
static inline int32_t *lvr_overflow_flag(const lvr_index *ix) { return ix->counters + (size_t)lvr_n_bhq(ix) * LVR_CNT_STRIDE; }
// per query head: set size of the last finished query (kept for statistics)
static inline int32_t *lvr_head_stat(const lvr_index *ix) { return ix->counters + ((size_t)lvr_n_bhq(ix) + 1) * LVR_CNT_STRIDE; }
// per (sequence, KV head, segment): surviving groups of the segment (plain stores, no atomics)
static inline int32_t *lvr_seg_count(const lvr_index *ix) { return ix->counters + ((size_t)lvr_n_bhq(ix) + 1) * LVR_CNT_STRIDE + (size_t)lvr_n_bhq(ix); }
static inline int64_t lvr_max_segs(int64_t max_groups) { return max_groups / LVR_MIN_SEG_GROUPS + 2; }
static inline size_t lvr_counter_ints(int n_bh, int n_bhq, int64_t max_groups) {
    return ((size_t)n_bhq + 1) * LVR_CNT_STRIDE + (size_t)n_bhq + (size_t)n_bh * (size_t)lvr_max_segs(max_groups) + (size_t)n_bhq +
           (size_t)n_bh * (LVR_CHAN_STRIDE / 4) + 32;   // + room to start the channel exponents on a 128-byte boundary
}
// per query head: tickets drawn by the workgroups that share the head in the attention launch (zero between launches)
static inline int32_t *lvr_head_ticket(const lvr_index *ix) {
    return ix->counters + ((size_t)lvr_n_bhq(ix) + 1) * LVR_CNT_STRIDE + (size_t)lvr_n_bhq(ix) +
           (size_t)lvr_n_bh(ix) * (size_t)lvr_max_segs(ix->max_groups);
}

// per (sequence, KV head), LVR_CHAN_STRIDE bytes: 128 signed bytes, the channel exponents e_c of a rescaled 6-bit index
// (all zero: no rescaling), then the 128 factors 2^e_c as floats (all 1), which is the form the query kernel multiplies
// q with
static inline int8_t *lvr_chan_exp(const lvr_index *ix) {
    const uintptr_t p = reinterpret_cast<uintptr_t>(lvr_head_ticket(ix) + lvr_n_bhq(ix));
    return reinterpret_cast<int8_t *>((p + 127) & ~(uintptr_t)127);
}

// ---- launchers (each returns a hipError_t from hipGetLastError after the launch) ----
// channel exponents from the keys about to be indexed (element strides ks for (sequence, head, token))
hipError_t lvr_launch_channel_scales(lvr_index *ix, const void *K, const int64_t ks[3], int64_t n, hipStream_t st);
// copies `rows` key rows and value rows into the arena starting at arena row dst_row0 (one launch)
hipError_t lvr_launch_copy_kv(lvr_index *ix, const void *K, const int64_t ks[3], const void *V, const int64_t vs[3],
                              int64_t dst_row0, int64_t rows, hipStream_t st, int64_t k_first = 0);
hipError_t lvr_launch_build_groups(lvr_index *ix, int64_t g0, int64_t g1, hipStream_t st, const void *K_src = nullptr,
                                   const int64_t *ks = nullptr);
hipError_t lvr_launch_iota_rows(lvr_index *ix, int64_t row0, int64_t rows, hipStream_t st);
// clears the per-head counters (used when there is no index to prune)
hipError_t lvr_launch_reset(lvr_index *ix, hipStream_t st);
// bound test; clears the per-head counters; fills the per-segment survivor lists
hipError_t lvr_launch_prune(lvr_index *ix, const float *q, const float *tau, hipStream_t st);
// exact check on survivors and buffer; fills out_idx and the internal per-head counters
hipError_t lvr_launch_filter(lvr_index *ix, const float *q, const float *tau, int32_t *out_idx, int64_t cap,
                             hipStream_t st);
// bf16 caches: bound test + exact check in one launch (per-head counters must be zero on entry)
hipError_t lvr_launch_query_fused(lvr_index *ix, const float *q, const float *tau, const float *tau_s, int32_t *out_idx,
                                  int64_t cap, hipStream_t st, const void *k_new = nullptr, const void *v_new = nullptr,
                                  int64_t m_new = 0);
// internal per-head counters -> caller's array and the statistics copy; clears the counters
hipError_t lvr_launch_publish_counts(lvr_index *ix, int32_t *out_count, hipStream_t st);
// partial softmax per (head, split); count is read with the given stride (1 = caller's array)
// scores: raw <q,k> of the listed keys, [n_bhq][cap_rows] (then no key row is read), or NULL
hipError_t lvr_launch_sparse_partial(lvr_index *ix, const float *q, const int32_t *idx, const float *scores,
                                     const int32_t *count, int count_stride, int64_t cap, hipStream_t st);
// whole sparse attention of a head in one workgroup (16 splits merged through LDS), one launch
hipError_t lvr_launch_sparse_attention_wg(lvr_index *ix, const float *q, const int32_t *idx, const float *scores,
                                          const int32_t *count, int count_stride, int64_t cap, float *out,
                                          int32_t *publish_count, hipStream_t st);
hipError_t lvr_launch_dense_partial(lvr_index *ix, const float *q, hipStream_t st);
// merge the partials of every head.  count == NULL: all P (dense baseline); otherwise as many as the
// sparse split geometry uses for that count.  publish_count != NULL: also hands the internal
// per-head counters to the caller (and to the statistics copy) and clears them
hipError_t lvr_launch_combine(lvr_index *ix, float *out, int P, const int32_t *count, int count_stride, int64_t cap,
                              int32_t *publish_count, hipStream_t st);
int lvr_dense_splits(const lvr_index *ix);
// reservoir of past keys and threshold selection (threshold.hip)
hipError_t lvr_launch_reservoir_reset(lvr_index *ix, hipStream_t st);
hipError_t lvr_launch_reservoir_update(lvr_index *ix, int64_t pos0, int64_t count, hipStream_t st);
hipError_t lvr_launch_safe_tau_s(lvr_index *ix, const float *q, const float *tau, float *tau_s, hipStream_t st);
hipError_t lvr_launch_threshold(lvr_index *ix, const float *q, int mode, float param, float *tau_out, hipStream_t st);
// one grouping per coordinate block (subspace_layout.hip)
hipError_t lvr_launch_subspace_groups(lvr_index *ix, const struct lvr_tree_perm *perm, int s, int64_t row0, int64_t g_base,
                                      int64_t n_new_groups, hipStream_t st);
hipError_t lvr_launch_subspace_bounds(lvr_index *ix, const float *q, hipStream_t st);
hipError_t lvr_launch_label_filter(lvr_index *ix, const float *q, const float *tau, int32_t *out_idx, int64_t cap,
                                   hipStream_t st);
// tree grouping (tree.hip)
size_t lvr_tree_sort_temp_bytes(int64_t total_keys);
// order of the rows after the tree grouping: sorted keys whose low pos_bits give the source row
struct lvr_tree_perm {
    uint64_t *keys;
    int64_t np;
    int pos_bits;
};
bool lvr_tree_feasible(const lvr_index *ix, int64_t n_real);
// c_lo, c_hi: the split axis of every node is chosen among coordinates [c_lo, c_hi) only
hipError_t lvr_tree_order(lvr_index *ix, const void *Ksrc, const int64_t ks[3], int64_t n_real, hipStream_t st,
                          lvr_tree_perm *perm, int c_lo = 0, int c_hi = LVR_D);
hipError_t lvr_tree_gather(lvr_index *ix, const void *Ksrc, const int64_t ks[3], const void *Vsrc, const int64_t vs[3],
                           const lvr_tree_perm *perm, int64_t n_real, int64_t row0, hipStream_t st);
hipError_t lvr_tree_group(lvr_index *ix, const void *Ksrc, const int64_t ks[3], const void *Vsrc, const int64_t vs[3],
                          int64_t n_real, int64_t row0, hipStream_t st);

#ifdef __HIPCC__
// ------------------------------------------------------------------------------------------
// Device helpers
// ------------------------------------------------------------------------------------------
struct lvr_bf16_t { uint16_t bits; };   // tag types for the two storage formats
struct lvr_f32_t { float v; };

__device__ __forceinline__ float lvr_bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float lvr_bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// Round-to-nearest-even fp32 -> bf16 bit pattern (finite inputs).
// Inclusive prefix sum over the 64 lanes of a wave in six DPP steps (within rows of 16 lanes: shifts by 1, 2, 4, 8;
// then lane 15 of a row into the next row, lane 31 into the upper half): no trip through LDS, unlike six shuffles.
__device__ __forceinline__ int lvr_wave_inclusive_sum(int v) {
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1 and 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2 and 3
    return v;
}

__device__ __forceinline__ uint32_t lvr_f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// Load the 8 consecutive elements of a row that belong to this lane (lane-in-row li).
template <typename KT>
__device__ __forceinline__ void lvr_load8(const void *base, int64_t row, int li, float (&x)[8]);

template <>
__device__ __forceinline__ void lvr_load8<lvr_bf16_t>(const void *base, int64_t row, int li, float (&x)[8]) {
    const uint4 *p = reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(base) + row * LVR_D) + li;
    uint4 w = *p;
    x[0] = lvr_bf16_lo(w.x); x[1] = lvr_bf16_hi(w.x);
    x[2] = lvr_bf16_lo(w.y); x[3] = lvr_bf16_hi(w.y);
    x[4] = lvr_bf16_lo(w.z); x[5] = lvr_bf16_hi(w.z);
    x[6] = lvr_bf16_lo(w.w); x[7] = lvr_bf16_hi(w.w);
}

template <>
__device__ __forceinline__ void lvr_load8<lvr_f32_t>(const void *base, int64_t row, int li, float (&x)[8]) {
    const float4 *p = reinterpret_cast<const float4 *>(static_cast<const float *>(base) + row * LVR_D) + 2 * li;
    float4 a = p[0], b = p[1];
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
    x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
}

// Two-step form of lvr_load8: issue the load now, unpack later, so that a run of loads can be
// put in flight before the first use.
template <typename KT> struct lvr_raw8;
template <> struct lvr_raw8<lvr_bf16_t> { uint4 a; };
template <> struct lvr_raw8<lvr_f32_t> { float4 a, b; };

__device__ __forceinline__ void lvr_load_raw(const void *base, int64_t row, int li, lvr_raw8<lvr_bf16_t> &r) {
    r.a = reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(base) + row * LVR_D)[li];
}
__device__ __forceinline__ void lvr_load_raw(const void *base, int64_t row, int li, lvr_raw8<lvr_f32_t> &r) {
    const float4 *p = reinterpret_cast<const float4 *>(static_cast<const float *>(base) + row * LVR_D) + 2 * li;
    r.a = p[0];
    r.b = p[1];
}
__device__ __forceinline__ void lvr_store_raw(void *base, int64_t row, int li, const lvr_raw8<lvr_bf16_t> &r) {
    reinterpret_cast<uint4 *>(static_cast<uint16_t *>(base) + row * LVR_D)[li] = r.a;
}
__device__ __forceinline__ void lvr_store_raw(void *base, int64_t row, int li, const lvr_raw8<lvr_f32_t> &r) {
    float4 *p = reinterpret_cast<float4 *>(static_cast<float *>(base) + row * LVR_D) + 2 * li;
    p[0] = r.a;
    p[1] = r.b;
}
__device__ __forceinline__ void lvr_unpack(const lvr_raw8<lvr_bf16_t> &r, float (&x)[8]) {
    x[0] = lvr_bf16_lo(r.a.x); x[1] = lvr_bf16_hi(r.a.x);
    x[2] = lvr_bf16_lo(r.a.y); x[3] = lvr_bf16_hi(r.a.y);
    x[4] = lvr_bf16_lo(r.a.z); x[5] = lvr_bf16_hi(r.a.z);
    x[6] = lvr_bf16_lo(r.a.w); x[7] = lvr_bf16_hi(r.a.w);
}
__device__ __forceinline__ void lvr_unpack(const lvr_raw8<lvr_f32_t> &r, float (&x)[8]) {
    x[0] = r.a.x; x[1] = r.a.y; x[2] = r.a.z; x[3] = r.a.w;
    x[4] = r.b.x; x[5] = r.b.y; x[6] = r.b.z; x[7] = r.b.w;
}

__device__ __forceinline__ void lvr_zero8(float (&x)[8]) {
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = 0.f;
}

// Sum over the 16 lanes of a quarter row; every lane of the quarter gets the total.
// DPP data movement inside a row of 16 lanes: two quad permutes, then the half-row and
// full-row mirrors.
template <int CTRL>
__device__ __forceinline__ float lvr_dpp(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}

__device__ __forceinline__ float lvr_row16_sum(float v) {
    v += lvr_dpp<0xB1>(v);    // quad_perm [1,0,3,2]  : lane ^ 1
    v += lvr_dpp<0x4E>(v);    // quad_perm [2,3,0,1]  : lane ^ 2
    v += lvr_dpp<0x141>(v);   // row_half_mirror      : 7 - lane within 8
    v += lvr_dpp<0x140>(v);   // row_mirror           : 15 - lane within 16
    return v;
}

__device__ __forceinline__ int lvr_lane() { return threadIdx.x & 63; }

// Threshold the kernels compare against: tau lowered by half of the 1e-4*|tau| tolerance band,
// so that keys whose score differs from tau only by summation order are kept.
__device__ __forceinline__ float lvr_effective_tau(float tau) {
    return (tau == -INFINITY) ? tau : tau - 0.5e-4f * fabsf(tau);
}
#endif  // __HIPCC__
