// C ABI of liblouver: argument checking, arena ownership, and the order in which the kernels
// of one call are enqueued.  No kernel lives here.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <new>

#include "lvr_internal.h"

namespace {

thread_local int g_last_hip_error = 0;

inline int hip_fail(hipError_t e) {
    g_last_hip_error = (int)e;
    return LVR_E_HIP;
}

#define LVR_HIP(expr)                                   \
    do {                                                \
        hipError_t e__ = (expr);                        \
        if (e__ != hipSuccess) return hip_fail(e__);    \
    } while (0)

inline bool is_pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }

inline bool fp8_centres_supported(const lvr_config *c) {
    if (c->kv_dtype != LVR_BF16 || (c->flags & LVR_SEPARATE_KERNELS)) return false;
    if (c->grouping == LVR_GROUP_SUBSPACE_TREE) return false;   // that layout keeps its centres in the cache's format
    return c->enclosing == LVR_ENCLOSE_AABB || c->n_subspaces <= 4;   // boxes do not look at n_subspaces
}

// 6-bit centres: balls only (a box corner has to be rounded outwards per coordinate, which a shared scale makes
// coarse).  AUTO takes them wherever they are supported and K/V are in device memory: a fifth less index
// outweighed the somewhat larger balls on every workload and group size measured (128k keys, one key per
// group: 34.1 against 37.2 us per step; groups of four: 60.7 against 62.1 us, on keys with positional locality
// 24.4 against 25.5 us).  Behind the host link a surviving key row costs a hundred times more than an index
// byte, so the tighter centres in the cache's own format are kept there.
inline bool fp6_centres_supported(const lvr_config *c) {
    return fp8_centres_supported(c) && c->enclosing == LVR_ENCLOSE_BALL && c->n_subspaces <= 4;
}
inline bool fp6_centres(const lvr_config *c) {
    return c->index_dtype == LVR_INDEX_FP6 ||
           (c->index_dtype == LVR_INDEX_AUTO && fp6_centres_supported(c) && !(c->flags & LVR_KV_IN_HOST_MEMORY));
}

// 8-bit centres: asked for explicitly (AUTO's coded format is the 6-bit one, which serves every
// configuration of balls that this one serves).
inline bool fp8_centres(const lvr_config *c) { return c->index_dtype == LVR_INDEX_FP8; }

int check_config(const lvr_config *c) {
    if (!c) return LVR_E_INVALID;
    if (c->batch <= 0 || c->n_q_heads <= 0 || c->n_kv_heads <= 0 || c->capacity <= 0) return LVR_E_INVALID;
    if (c->n_q_heads % c->n_kv_heads != 0) return LVR_E_INVALID;
    if (c->kv_dtype != LVR_BF16 && c->kv_dtype != LVR_F32) return LVR_E_INVALID;
    if (c->grouping != LVR_GROUP_CONTIGUOUS && c->grouping != LVR_GROUP_TREE && c->grouping != LVR_GROUP_SUBSPACE_TREE)
        return LVR_E_INVALID;
    if (c->scale < 0.f || c->attn_splits < -1) return LVR_E_INVALID;
    if (c->head_dim != LVR_D) return LVR_E_UNSUPPORTED;
    const int G = c->n_q_heads / c->n_kv_heads;
    if (!(G == 1 || G == 2 || G == 4 || G == 8)) return LVR_E_UNSUPPORTED;
    if (!is_pow2(c->group_size) || c->group_size > 16) return LVR_E_UNSUPPORTED;
    if (!is_pow2(c->n_subspaces) || c->n_subspaces > 16) return LVR_E_UNSUPPORTED;
    if (c->buffer_size <= 0 || c->buffer_size % 16 != 0 || c->buffer_size % c->group_size != 0) return LVR_E_INVALID;
    if (c->attn_splits > 256) return LVR_E_INVALID;
    if (c->capacity > (int64_t)1 << 30) return LVR_E_UNSUPPORTED;   // positions are int32
    if (c->enclosing != LVR_ENCLOSE_BALL && c->enclosing != LVR_ENCLOSE_AABB) return LVR_E_INVALID;
    if (c->reservoir_size < 0 || c->reservoir_size > 256) return LVR_E_INVALID;
    if (c->enclosing == LVR_ENCLOSE_AABB && (c->kv_dtype != LVR_BF16 || (c->flags & LVR_SEPARATE_KERNELS)))
        return LVR_E_UNSUPPORTED;
    if (c->index_dtype != LVR_INDEX_AUTO && c->index_dtype != LVR_INDEX_SAME && c->index_dtype != LVR_INDEX_FP8 &&
        c->index_dtype != LVR_INDEX_FP6)
        return LVR_E_INVALID;
    if (c->query_workgroups < 0 || c->query_workgroups > (1 << 20)) return LVR_E_INVALID;
    if (c->flags & ~(uint32_t)(LVR_ATTEND_BUFFER_DENSE | LVR_SEPARATE_KERNELS | LVR_CONCURRENT_UPDATE | LVR_KV_IN_HOST_MEMORY))
        return LVR_E_INVALID;
    if (c->index_dtype == LVR_INDEX_FP8 && !fp8_centres_supported(c)) return LVR_E_UNSUPPORTED;
    if (c->index_dtype == LVR_INDEX_FP6 && !fp6_centres_supported(c)) return LVR_E_UNSUPPORTED;
    if (c->grouping == LVR_GROUP_SUBSPACE_TREE) {
        // one grouping per coordinate block: labels are 16 bits, one launch form, one head block
        if (c->kv_dtype != LVR_BF16 || c->enclosing != LVR_ENCLOSE_BALL || G > 4) return LVR_E_UNSUPPORTED;
        if (c->flags & (LVR_SEPARATE_KERNELS | LVR_CONCURRENT_UPDATE | LVR_KV_IN_HOST_MEMORY)) return LVR_E_UNSUPPORTED;
        if ((c->capacity + 63) / 64 * 64 / c->group_size > 65536) return LVR_E_UNSUPPORTED;
    }
    return LVR_OK;
}

struct Sizes {
    int64_t cap_rows, max_groups;
    int P, P_dense, Pmax;
    size_t kv, centres, radii, list, counters, part_ml, part_o, scores, total;
    // tree grouping only
    int64_t tree_keys;
    size_t maps, tree_keybytes, tree_axis, tree_partial, tree_temp, chunk;
    // one grouping per coordinate block only
    size_t labels, f_table;
};

Sizes sizes_of(const lvr_config *c) {
    Sizes s;
    const size_t elt = c->kv_dtype == LVR_BF16 ? 2 : 4;
    const int64_t n_bh = (int64_t)c->batch * c->n_kv_heads, n_bhq = (int64_t)c->batch * c->n_q_heads;
    s.cap_rows = (c->capacity + 63) / 64 * 64;
    s.max_groups = s.cap_rows / c->group_size;
    s.P = c->attn_splits > 0 ? c->attn_splits : 64;
    int64_t pd = 1024 / n_bh;   // ~1024 workgroups per launch of the dense baseline
    s.P_dense = (int)(pd < 4 ? 4 : (pd > 256 ? 256 : pd));
    s.Pmax = s.P > s.P_dense ? s.P : s.P_dense;
    auto al = [](size_t b) { return (b + 255) / 256 * 256; };
    s.kv = al((size_t)n_bh * s.cap_rows * LVR_D * elt);
    const bool box = c->enclosing == LVR_ENCLOSE_AABB;
    const size_t c_row = fp6_centres(c) ? LVR_D * 3 / 4 : (fp8_centres(c) ? LVR_D : LVR_D * elt);
    s.centres = al((size_t)n_bh * s.max_groups * c_row * (box ? 2 : 1));
    // boxes: one allowance; 8-bit balls: four bf16; 6-bit balls: four bf16 and four scale bytes
    s.radii = al((size_t)n_bh * s.max_groups * (box ? 1 : (fp6_centres(c) ? 3 : (fp8_centres(c) ? 2 : c->n_subspaces))) * sizeof(float));
    s.list = al((size_t)n_bh * s.max_groups * sizeof(int32_t));
    s.counters = al(lvr_counter_ints((int)n_bh, (int)n_bhq, s.max_groups) * sizeof(int32_t));
    s.part_ml = al((size_t)n_bhq * s.Pmax * 2 * sizeof(float));
    s.part_o = al((size_t)n_bhq * s.Pmax * LVR_D * sizeof(float));
    const bool fused_path = c->kv_dtype == LVR_BF16 && !(c->flags & LVR_SEPARATE_KERNELS);
    s.scores = fused_path ? al((size_t)n_bhq * s.cap_rows * sizeof(float)) : 0;
    const bool kv_on_host = (c->flags & LVR_KV_IN_HOST_MEMORY) != 0;
    s.total = s.scores + (kv_on_host ? 0 : 2 * s.kv) + s.centres + s.radii + s.list + s.counters + s.part_ml + s.part_o;
    s.tree_keys = 0;
    s.maps = s.tree_keybytes = s.tree_axis = s.tree_partial = s.tree_temp = s.chunk = 0;
    s.labels = s.f_table = 0;
    const bool per_subspace = c->grouping == LVR_GROUP_SUBSPACE_TREE;
    if (c->grouping == LVR_GROUP_TREE || per_subspace) {
        int64_t gp = 1;
        while (gp < s.max_groups) gp <<= 1;
        const int64_t np = gp * c->group_size;
        s.tree_keys = n_bh * np;
        s.maps = per_subspace ? 0 : al((size_t)n_bh * s.cap_rows * sizeof(int32_t));   // rows stay in arrival order there
        s.tree_keybytes = al((size_t)s.tree_keys * sizeof(uint64_t));
        s.tree_axis = al((size_t)n_bh * gp * sizeof(int32_t));
        s.tree_partial = al((size_t)n_bh * (np / 1024 + 1) * 258 * sizeof(double));
        s.tree_temp = 0;   // asked from the sort library at create time
        s.chunk = per_subspace ? 0 : al((size_t)n_bh * c->buffer_size * LVR_D * elt);
        s.total += 2 * s.maps + 2 * s.tree_keybytes + s.tree_axis + s.tree_partial + 2 * s.chunk;
    }
    if (per_subspace) {
        s.labels = al((size_t)n_bh * s.cap_rows * c->n_subspaces * sizeof(uint16_t));
        s.f_table = al((size_t)n_bh * s.max_groups * c->n_subspaces * 4 * sizeof(float));
        s.total += s.labels + s.f_table;
    }
    return s;
}

void free_all(lvr_index *ix) {
    if (ix->K_host || ix->V_host) {   // K and V alias pinned host memory
        if (ix->K_host) (void)hipHostFree(ix->K_host);
        if (ix->V_host) (void)hipHostFree(ix->V_host);
        ix->K = ix->V = nullptr;
    }
    void *ptrs[] = {ix->K, ix->V, ix->centres, ix->radii, ix->slot_pos, ix->pos_slot,
                    ix->surv_list, ix->counters, ix->part_ml, ix->part_o, ix->tree_keys_a, ix->tree_keys_b,
                    ix->tree_axis, ix->tree_partial, ix->tree_temp, ix->chunk_K, ix->chunk_V, ix->reservoir, ix->scores,
                    ix->labels, ix->f_table};
    for (void *p : ptrs)
        if (p) (void)hipFree(p);
    if (ix->ev_fork) (void)hipEventDestroy(ix->ev_fork);
    if (ix->ev_done) (void)hipEventDestroy(ix->ev_done);
    if (ix->side) (void)hipStreamDestroy(ix->side);
    delete ix->pend_perm;
}

// Phase 2 of the two-stream update (App. "GPU Update"): `st` waits for the side stream, then
// the prepared groups become visible to the launches that follow.
// force = false: publish only if the side stream has already finished (a host-side poll that never
// blocks), so a slow update stays hidden behind as many decode steps as it needs.
int publish_pending(lvr_index *ix, hipStream_t st, bool force) {
    if (!ix->pending) return LVR_OK;
    const int64_t B = ix->cfg.buffer_size;
    const int r = ix->cfg.group_size;
    if (!force) {
        const hipError_t qe = hipEventQuery(ix->ev_done);
        if (qe == hipErrorNotReady) {
            (void)hipGetLastError();   // "not ready" is an answer, not a failure to be reported later
            return LVR_OK;
        }
        LVR_HIP(qe);
    }
    LVR_HIP(hipStreamWaitEvent(st, ix->ev_done, 0));
    if (ix->cfg.grouping == LVR_GROUP_TREE) {
        // the chunk's order was computed on the side stream from a staged copy; moving the rows
        // and forming their bounds happens here, where no query can be reading them
        const int64_t cs[3] = {(int64_t)ix->cfg.n_kv_heads * B * LVR_D, B * LVR_D, LVR_D};
        LVR_HIP(lvr_tree_gather(ix, ix->chunk_K, cs, ix->chunk_V, cs, ix->pend_perm, B, ix->pend_row0, st));
        const int64_t g0 = ix->pend_row0 / r;
        LVR_HIP(lvr_launch_build_groups(ix, g0, g0 + B / r, st));
    }
    ix->n_indexed = ix->pend_row0 + B;
    ix->pending = 0;
    return LVR_OK;
}

// Optional event pair around one kernel launch.  in_dispatch: the launcher passes the pair to the dispatch (the events
// then hold the kernel's own start and end times); otherwise the pair is recorded on the stream before and after the
// launch, which also brackets the launch latency that back-to-back launches hide (2-3 us on a 25 us kernel).
struct Timed {
    lvr_index *ix;
    hipStream_t st;
    int slot;
    bool in_dispatch;
    Timed(lvr_index *ix_, int kind, hipStream_t st_, bool in_dispatch_ = false) : ix(ix_), st(st_), slot(-1), in_dispatch(in_dispatch_) {
        if (ix->prof_on && ix->prof_used + 2 <= ix->prof_cap) {
            slot = ix->prof_used;
            ix->prof_used += 2;
            ix->prof_kind[slot / 2] = (uint8_t)kind;
            if (in_dispatch) {
                ix->launch_start = ix->prof_events[slot];
                ix->launch_stop = ix->prof_events[slot + 1];
            } else
                (void)hipEventRecord(ix->prof_events[slot], st);
        }
    }
    ~Timed() {
        if (slot >= 0 && !in_dispatch) (void)hipEventRecord(ix->prof_events[slot + 1], st);
        if (in_dispatch) ix->launch_start = ix->launch_stop = nullptr;
    }
};

void prof_free(lvr_index *ix) {
    for (int i = 0; i < ix->prof_cap; ++i) (void)hipEventDestroy(ix->prof_events[i]);
    free(ix->prof_events);
    free(ix->prof_kind);
    ix->prof_events = nullptr;
    ix->prof_kind = nullptr;
    ix->prof_cap = ix->prof_used = ix->prof_on = 0;
}

// Sparse attention as one launch (a workgroup per head merges its splits in LDS) or as partials plus
// a combine launch.  One launch wins whenever there are many heads in the batch or few keys per head;
// with one sequence's 32 heads and several hundred retrieved keys each, 32 workgroups cannot gather
// fast enough and the two-launch form wins (measured crossover: between 32k and 128k keys of context
// at 0.5-1 % retrieved).  The set sizes are not known on the host, so the context length stands in.
inline bool one_launch_attention(const lvr_index *ix, bool carried = false) {
    if (ix->attn_one_launch >= 0) return ix->attn_one_launch != 0;
    // lists that carry their scores take the one-launch kernels with two dependent trips (two workgroups per head
    // beyond 65536 keys), which moves the crossover up: one launch against two, us per step at 0.5 % retrieved,
    // 32 heads: 39.7 / 41.3 at 196608 keys, 50.2 / 51.3 at 262144, 102.5 / 101.5 at 524288
    return lvr_n_bhq(ix) >= 128 || ix->n_total <= (carried ? 262144 : 65536);
}

// One grouping per coordinate block: groups [g0, g0 + ng) are formed from arena rows g0*r .. (g0+ng)*r - 1
// (a whole build, or one buffer chunk).  Per block: the tree order over the block's coordinates
// (Alg. 2), then the block's centres, radii and the members' labels.
int build_subspace_groups(lvr_index *ix, int64_t g0, int64_t ng, hipStream_t st) {
    if (ng <= 0) return LVR_OK;
    const int r = ix->cfg.group_size, S = ix->cfg.n_subspaces;
    const int64_t row0 = g0 * r;
    const char *src = static_cast<const char *>(ix->K) + row0 * LVR_D * (int64_t)ix->elt;
    const int64_t as[3] = {(int64_t)ix->cfg.n_kv_heads * ix->cap_rows * LVR_D, ix->cap_rows * LVR_D, LVR_D};
    for (int sb = 0; sb < S; ++sb) {
        lvr_tree_perm perm;
        hipError_t e = lvr_tree_order(ix, src, as, ng * r, st, &perm, sb * (LVR_D / S), (sb + 1) * (LVR_D / S));
        if (e == hipErrorInvalidValue) return LVR_E_UNSUPPORTED;   // sort key wider than 64 bits
        LVR_HIP(e);
        LVR_HIP(lvr_launch_subspace_groups(ix, &perm, sb, row0, g0, ng, st));
    }
    return LVR_OK;
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool aligned4(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 3u) == 0; }

// The arena belongs to the device that was current in lvr_create; a launch from another device
// would hand that device's kernels pointers it cannot read.
inline bool on_home_device(const lvr_index *ix) {
    int d = -1;
    return hipGetDevice(&d) == hipSuccess && d == ix->device;
}

}  // namespace

extern "C" {

size_t lvr_arena_bytes(const lvr_config *cfg) {
    if (check_config(cfg) != LVR_OK) return 0;
    return sizes_of(cfg).total;
}

size_t lvr_host_bytes(const lvr_config *cfg) {
    if (check_config(cfg) != LVR_OK || !(cfg->flags & LVR_KV_IN_HOST_MEMORY)) return 0;
    return 2 * sizes_of(cfg).kv;
}

int lvr_create(const lvr_config *cfg, lvr_index **out) {
    if (!out) return LVR_E_INVALID;
    int rc = check_config(cfg);
    if (rc != LVR_OK) return rc;
    lvr_index *ix = new (std::nothrow) lvr_index();
    if (!ix) return LVR_E_NOMEM;
    memset(ix, 0, sizeof(*ix));
    ix->cfg = *cfg;
    const Sizes s = sizes_of(cfg);
    ix->G = cfg->n_q_heads / cfg->n_kv_heads;
    ix->box = cfg->enclosing == LVR_ENCLOSE_AABB;
    ix->cf8 = fp8_centres(cfg);
    ix->cf6 = fp6_centres(cfg);
    // 8-bit centres: 8 bytes of radii per group (four bf16); 6-bit centres: the same and four scale bytes
    ix->S_store = ix->box ? 1 : (ix->cf6 ? 3 : (ix->cf8 ? 2 : cfg->n_subspaces));
    ix->centre_bytes = ix->cf6 ? LVR_D * 3 / 4 : (ix->cf8 ? LVR_D : LVR_D * (cfg->kv_dtype == LVR_BF16 ? 2 : 4));
    // 6-bit centres share a scale among 32 coordinates, so one large channel would drown the others: the index is
    // built in a space where every channel is divided by a power of two of its own (taken from the keys at lvr_build).
    // The query kernels carry the rescaled query (bound phase) beside the original one (key rows).
    ix->chan_scaled = ix->cf6;
    ix->cap_rows = s.cap_rows;
    ix->max_groups = s.max_groups;
    ix->P = s.P;
    ix->P_dense = s.P_dense;
    ix->attn_one_launch = cfg->attn_splits < 0 ? 1 : (cfg->attn_splits == 0 ? -1 : 0);   // -1: chosen per call
    ix->elt = cfg->kv_dtype == LVR_BF16 ? 2 : 4;
    ix->sigma = cfg->scale > 0.f ? cfg->scale : 1.0f / sqrtf((float)cfg->head_dim);
    hipError_t e = hipGetDevice(&ix->device);
    const bool kv_on_host = (cfg->flags & LVR_KV_IN_HOST_MEMORY) != 0;
    if (kv_on_host) {
        // pinned, GPU-mapped host memory: kernels read (and the build/append copies write) it in place
        if (e == hipSuccess) e = hipHostMalloc(&ix->K_host, s.kv, hipHostMallocMapped);
        if (e == hipSuccess) e = hipHostMalloc(&ix->V_host, s.kv, hipHostMallocMapped);
        if (e == hipSuccess) e = hipHostGetDevicePointer(&ix->K, ix->K_host, 0);
        if (e == hipSuccess) e = hipHostGetDevicePointer(&ix->V, ix->V_host, 0);
    }
    struct { void **p; size_t bytes; } allocs[] = {
        {&ix->K, kv_on_host ? 0 : s.kv}, {&ix->V, kv_on_host ? 0 : s.kv}, {&ix->centres, s.centres}, {(void **)&ix->radii, s.radii},
        {(void **)&ix->surv_list, s.list}, {(void **)&ix->counters, s.counters},
        {(void **)&ix->part_ml, s.part_ml}, {(void **)&ix->part_o, s.part_o}, {(void **)&ix->scores, s.scores}};
    for (auto &a : allocs) {
        if (e != hipSuccess) break;
        if (a.bytes) e = hipMalloc(a.p, a.bytes);
    }
    ix->per_subspace = cfg->grouping == LVR_GROUP_SUBSPACE_TREE;
    if (e == hipSuccess && ix->per_subspace) {
        e = hipMalloc((void **)&ix->labels, s.labels);
        if (e == hipSuccess) e = hipMalloc((void **)&ix->f_table, s.f_table);
    }
    if (e == hipSuccess && (cfg->grouping == LVR_GROUP_TREE || ix->per_subspace)) {
        ix->tree_cap_keys = s.tree_keys;
        ix->tree_temp_bytes = lvr_tree_sort_temp_bytes(s.tree_keys);
        struct { void **p; size_t bytes; } tallocs[] = {
            {(void **)&ix->slot_pos, s.maps}, {(void **)&ix->pos_slot, s.maps},
            {(void **)&ix->tree_keys_a, s.tree_keybytes}, {(void **)&ix->tree_keys_b, s.tree_keybytes},
            {(void **)&ix->tree_axis, s.tree_axis}, {(void **)&ix->tree_partial, s.tree_partial},
            {&ix->tree_temp, ix->tree_temp_bytes ? ix->tree_temp_bytes : 256}, {&ix->chunk_K, s.chunk},
            {&ix->chunk_V, s.chunk}};
        for (auto &a : tallocs) {
            if (e != hipSuccess) break;
            if (a.bytes) e = hipMalloc(a.p, a.bytes);
        }
    }
    if (e == hipSuccess && cfg->reservoir_size > 0) {
        const size_t rb = (size_t)lvr_n_bh(ix) * cfg->reservoir_size * sizeof(int32_t);
        e = hipMalloc((void **)&ix->reservoir, rb);
        if (e == hipSuccess) e = hipMemset(ix->reservoir, 0xff, rb);
    }
    if (e == hipSuccess && (cfg->flags & LVR_CONCURRENT_UPDATE)) {
        e = hipEventCreateWithFlags(&ix->ev_fork, hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&ix->ev_done, hipEventDisableTiming);
        if (e == hipSuccess) {
            ix->pend_perm = new (std::nothrow) lvr_tree_perm();
            if (!ix->pend_perm) e = hipErrorOutOfMemory;
        }
    }
    if (e == hipSuccess) e = hipMemset(ix->counters, 0, s.counters);
    if (e == hipSuccess) {   // channel scaling starts as the identity: exponents 0 (the memset), factors 1
        const size_t n_bh = (size_t)lvr_n_bh(ix);
        float *ones = static_cast<float *>(malloc(LVR_D * sizeof(float)));
        if (!ones) e = hipErrorOutOfMemory;
        for (int c = 0; ones && c < LVR_D; ++c) ones[c] = 1.0f;
        for (size_t i = 0; ones && i < n_bh && e == hipSuccess; ++i)
            e = hipMemcpy(lvr_chan_exp(ix) + i * LVR_CHAN_STRIDE + LVR_D, ones, LVR_D * sizeof(float), hipMemcpyHostToDevice);
        free(ones);
    }
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        free_all(ix);
        delete ix;
        (void)hipGetLastError();   // the failure is reported here, not by whatever HIP call comes next
        if (e == hipErrorOutOfMemory) {
            g_last_hip_error = (int)e;
            return LVR_E_NOMEM;
        }
        return hip_fail(e);
    }
    *out = ix;
    return LVR_OK;
}

int lvr_destroy(lvr_index *ix) {
    if (!ix) return LVR_E_INVALID;
    (void)hipDeviceSynchronize();
    prof_free(ix);
    free_all(ix);
    delete ix;
    return LVR_OK;
}

int lvr_build(lvr_index *ix, const void *K, const void *V, int64_t n, const int64_t ks[3], const int64_t vs[3],
              void *stream) {
    if (!ix || n < 0 || (n > 0 && (!K || !V || !ks || !vs))) return LVR_E_INVALID;
    if (n > ix->cfg.capacity) return LVR_E_CAPACITY;
    if (!on_home_device(ix)) return LVR_E_STATE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t per16 = 16 / (int64_t)ix->elt;
    if (n > 0) {
        if (!aligned16(K) || !aligned16(V)) return LVR_E_INVALID;
        for (int i = 0; i < 3; ++i)
            if (ks[i] < 0 || vs[i] < 0 || ks[i] % per16 || vs[i] % per16) return LVR_E_INVALID;
        if (ks[2] < LVR_D || vs[2] < LVR_D) return LVR_E_INVALID;
    }
    if (ix->pending) {   // an unpublished update belongs to the content being discarded
        LVR_HIP(hipStreamWaitEvent(st, ix->ev_done, 0));
        ix->pending = 0;
    }
    ix->built = 0;
    ix->n_total = 0;
    ix->n_indexed = 0;
    const int r = ix->cfg.group_size;
    const int64_t n_groups = n / r;
    LVR_HIP(lvr_launch_channel_scales(ix, K, ks, n, st));   // before any group is formed
    if (n > 0 && ix->per_subspace) {
        // rows stay in arrival order; every coordinate block gets the tree order of its own coordinates,
        // and from it the block's balls and the keys' labels (Alg. 1: one BalancedPCATree call per subspace)
        {
            Timed t(ix, LVR_K_COPY, st);
            LVR_HIP(lvr_launch_copy_kv(ix, K, ks, V, vs, 0, n, st));
        }
        Timed t(ix, LVR_K_BUILD, st);
        int rc = build_subspace_groups(ix, 0, n_groups, st);
        if (rc != LVR_OK) return rc;
    } else if (n > 0 && ix->cfg.grouping == LVR_GROUP_TREE) {
        // rows of the n_groups*r leading keys go into the arena in tree order; the tail stays in arrival order
        Timed t(ix, LVR_K_COPY, st);
        const int64_t n_tree = n_groups * r;
        hipError_t e = lvr_tree_group(ix, K, ks, V, vs, n_tree, 0, st);
        if (e == hipErrorInvalidValue) return LVR_E_UNSUPPORTED;   // sort key wider than 64 bits
        LVR_HIP(e);
        if (n > n_tree) {
            const char *Kt = static_cast<const char *>(K) + n_tree * ks[2] * (int64_t)ix->elt;
            const char *Vt = static_cast<const char *>(V) + n_tree * vs[2] * (int64_t)ix->elt;
            LVR_HIP(lvr_launch_copy_kv(ix, Kt, ks, Vt, vs, n_tree, n - n_tree, st));
            LVR_HIP(lvr_launch_iota_rows(ix, n_tree, n - n_tree, st));
        }
    } else if (n > 0) {
        // contiguous groups: V and the ungrouped tail of K are copied here, the grouped key rows by the
        // build kernel below, which reads them from the caller's K anyway
        Timed t(ix, LVR_K_COPY, st);
        LVR_HIP(lvr_launch_copy_kv(ix, K, ks, V, vs, 0, n, st, n_groups * r));
    }
    if (!ix->per_subspace) {
        Timed t(ix, LVR_K_BUILD, st);
        const bool fused_copy = n > 0 && ix->cfg.grouping != LVR_GROUP_TREE;
        LVR_HIP(lvr_launch_build_groups(ix, 0, n_groups, st, fused_copy ? K : nullptr, fused_copy ? ks : nullptr));
    }
    LVR_HIP(lvr_launch_reservoir_reset(ix, st));
    LVR_HIP(lvr_launch_reservoir_update(ix, 0, n, st));
    ix->n_total = n;
    ix->n_indexed = n_groups * r;
    ix->built = 1;
    return LVR_OK;
}

int lvr_append(lvr_index *ix, const void *k_new, const void *v_new, int64_t m, void *stream) {
    if (!ix || m < 0 || (m > 0 && (!k_new || !v_new))) return LVR_E_INVALID;
    if (!ix->built) return LVR_E_STATE;
    if (!on_home_device(ix)) return LVR_E_STATE;
    if (m == 0) return LVR_OK;
    if (ix->n_total + m > ix->cfg.capacity) return LVR_E_CAPACITY;
    if (!aligned16(k_new) || !aligned16(v_new)) return LVR_E_INVALID;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // Everything that can refuse the call is settled before a row is stored, so a call that returns
    // LVR_E_UNSUPPORTED has changed nothing and may be repeated differently: whether a chunk can be
    // grouped by the tree (the width of its sort key), and the side stream of the two-stream update.
    if ((ix->cfg.grouping == LVR_GROUP_TREE || ix->per_subspace) &&
        ix->n_total + m - ix->n_indexed >= ix->cfg.buffer_size && !lvr_tree_feasible(ix, ix->cfg.buffer_size))
        return LVR_E_UNSUPPORTED;
    if ((ix->cfg.flags & LVR_CONCURRENT_UPDATE) && !ix->side)
        LVR_HIP(hipStreamCreateWithFlags(&ix->side, hipStreamNonBlocking));
    {
        // groups prepared earlier become visible as soon as they are ready; they must be before
        // the next chunk is formed
        const int64_t unpublished = ix->pending ? ix->cfg.buffer_size : 0;
        const bool next_chunk_fills = ix->n_total + m - ix->n_indexed - unpublished >= ix->cfg.buffer_size;
        int rc = publish_pending(ix, st, next_chunk_fills);
        if (rc != LVR_OK) return rc;
    }
    const int64_t strides[3] = {(int64_t)ix->cfg.n_kv_heads * m * LVR_D, m * LVR_D, LVR_D};
    {
        Timed t(ix, LVR_K_COPY, st);
        LVR_HIP(lvr_launch_copy_kv(ix, k_new, strides, v_new, strides, ix->n_total, m, st));
        LVR_HIP(lvr_launch_iota_rows(ix, ix->n_total, m, st));   // no-op without position maps
        LVR_HIP(lvr_launch_reservoir_update(ix, ix->n_total, m, st));
    }
    ix->n_total += m;
    // every full buffer of B keys becomes B/r new groups at the tail of the index
    const int64_t B = ix->cfg.buffer_size;
    const int r = ix->cfg.group_size;
    const int64_t full = ix->pending ? 0 : (ix->n_total - ix->n_indexed) / B;   // pending: its B keys are spoken for, fewer than B more
    if (full == 1 && (ix->cfg.flags & LVR_CONCURRENT_UPDATE)) {
        // Phase 1 on the side stream: it starts once the rows copied above are in the arena and
        // writes only index slots (and staging) that no query launched before the publish reads
        const int64_t g0 = ix->n_indexed / r;
        LVR_HIP(hipEventRecord(ix->ev_fork, st));
        LVR_HIP(hipStreamWaitEvent(ix->side, ix->ev_fork, 0));
        if (ix->cfg.grouping == LVR_GROUP_TREE) {
            const size_t row_bytes = LVR_D * ix->elt;
            const int64_t cs[3] = {(int64_t)ix->cfg.n_kv_heads * B * LVR_D, B * LVR_D, LVR_D};
            LVR_HIP(hipMemcpy2DAsync(ix->chunk_K, B * row_bytes, static_cast<char *>(ix->K) + ix->n_indexed * row_bytes,
                                     ix->cap_rows * row_bytes, B * row_bytes, lvr_n_bh(ix), hipMemcpyDefault,
                                     ix->side));
            LVR_HIP(hipMemcpy2DAsync(ix->chunk_V, B * row_bytes, static_cast<char *>(ix->V) + ix->n_indexed * row_bytes,
                                     ix->cap_rows * row_bytes, B * row_bytes, lvr_n_bh(ix), hipMemcpyDefault,
                                     ix->side));
            hipError_t e = lvr_tree_order(ix, ix->chunk_K, cs, B, ix->side, ix->pend_perm);
            if (e == hipErrorInvalidValue) return LVR_E_UNSUPPORTED;
            LVR_HIP(e);
        } else {
            LVR_HIP(lvr_launch_build_groups(ix, g0, g0 + B / r, ix->side));
        }
        LVR_HIP(hipEventRecord(ix->ev_done, ix->side));
        ix->pend_row0 = ix->n_indexed;
        ix->pending = 1;
    } else if (full > 0 && ix->per_subspace) {
        // every chunk of B buffered keys is grouped on its own, block by block (Sec. 4.3)
        Timed t(ix, LVR_K_BUILD, st);
        for (int64_t c = 0; c < full; ++c) {
            int rc = build_subspace_groups(ix, ix->n_indexed / r, B / r, st);
            if (rc != LVR_OK) return rc;
            ix->n_indexed += B;
        }
    } else if (full > 0) {
        const int64_t g0 = ix->n_indexed / r, g1 = g0 + full * (B / r);
        Timed t(ix, LVR_K_BUILD, st);
        if (ix->cfg.grouping == LVR_GROUP_TREE) {
            // each chunk of B buffered keys is clustered on its own (Sec. 4.3): stage its rows, then
            // write them back in tree order
            const size_t row_bytes = LVR_D * ix->elt;
            const int64_t cs[3] = {(int64_t)ix->cfg.n_kv_heads * B * LVR_D, B * LVR_D, LVR_D};
            for (int64_t c = 0; c < full; ++c) {
                const int64_t row0 = ix->n_indexed + c * B;
                LVR_HIP(hipMemcpy2DAsync(ix->chunk_K, B * row_bytes, static_cast<char *>(ix->K) + row0 * row_bytes,
                                         ix->cap_rows * row_bytes, B * row_bytes, lvr_n_bh(ix),
                                         hipMemcpyDefault, st));
                LVR_HIP(hipMemcpy2DAsync(ix->chunk_V, B * row_bytes, static_cast<char *>(ix->V) + row0 * row_bytes,
                                         ix->cap_rows * row_bytes, B * row_bytes, lvr_n_bh(ix),
                                         hipMemcpyDefault, st));
                hipError_t e = lvr_tree_group(ix, ix->chunk_K, cs, ix->chunk_V, cs, B, row0, st);
                if (e == hipErrorInvalidValue) return LVR_E_UNSUPPORTED;
                LVR_HIP(e);
            }
        }
        LVR_HIP(lvr_launch_build_groups(ix, g0, g1, st));
        ix->n_indexed += full * B;
    }
    return LVR_OK;
}

int lvr_publish(lvr_index *ix, void *stream) {
    if (!ix) return LVR_E_INVALID;
    if (!ix->built) return LVR_E_STATE;
    if (!on_home_device(ix)) return LVR_E_STATE;
    return publish_pending(ix, static_cast<hipStream_t>(stream), true);
}

}  // extern "C"

namespace {

// bound test + exact filter; leaves the set sizes in the internal per-head counters
int enqueue_query(lvr_index *ix, const float *q, const float *tau, int32_t *out_idx, int64_t cap, hipStream_t st,
                  const float *tau_s = nullptr, const void *k_new = nullptr, const void *v_new = nullptr,
                  int64_t m_new = 0) {
    const bool fused = ix->cfg.kv_dtype == LVR_BF16 && !(ix->cfg.flags & LVR_SEPARATE_KERNELS);
    if (ix->counters_dirty) {   // an earlier query never published its counts: start from zero again
        Timed t(ix, LVR_K_RESET, st);
        LVR_HIP(lvr_launch_reset(ix, st));
    }
    ix->counters_dirty = 1;
    if (ix->per_subspace) {
        if (ix->n_indexed > 0) {
            Timed t(ix, LVR_K_PRUNE, st);
            LVR_HIP(lvr_launch_subspace_bounds(ix, q, st));
        }
        Timed t(ix, LVR_K_FILTER, st);
        LVR_HIP(lvr_launch_label_filter(ix, q, tau, out_idx, cap, st));
    } else if (fused) {
        Timed t(ix, LVR_K_FILTER, st, true);
        LVR_HIP(lvr_launch_query_fused(ix, q, tau, tau_s, out_idx, cap, st, k_new, v_new, m_new));
        ix->n_total += m_new;
    } else {
        if (ix->n_indexed > 0) {
            Timed t(ix, LVR_K_PRUNE, st);
            LVR_HIP(lvr_launch_prune(ix, q, tau, st));
        } else {
            ix->n_segs = 0;
        }
        Timed t(ix, LVR_K_FILTER, st);
        LVR_HIP(lvr_launch_filter(ix, q, tau, out_idx, cap, st));
    }
    ix->last_buffer_rows = ix->n_total - ix->n_indexed;
    ix->last_indexed = ix->n_indexed;
    ix->last_skipped = fused && ix->skip_bounds && !tau_s;
    return LVR_OK;
}

// query + attention; with k_new the query launch also appends m_new rows (see lvr_append_decode_step)
int decode_step_impl(lvr_index *ix, const float *q, const float *tau, float *out, int32_t *out_idx, int32_t *out_count,
                     int64_t cap, hipStream_t st, const void *k_new, const void *v_new, int64_t m_new) {
    int rc = enqueue_query(ix, q, tau, out_idx, cap, st, nullptr, k_new, v_new, m_new);
    if (rc != LVR_OK) return rc;
    // The fused query kernel leaves the raw score of every emitted key beside its position; an attention that
    // uses it gathers V rows only and forms its softmax weights while they travel.  (With the first fused kernels
    // the query launch that followed such an attention was measured ~3 us slower at 128k keys and groups of four:
    // it no longer found the retrieved K rows touched just before it.  On the present kernels the scores win for
    // every group size: 59.8 -> 57.1 us per step at 128k keys with r = 4 where every group survives, 24.7 -> 21.7
    // on keys with positional locality.)
    const bool fused = ix->cfg.kv_dtype == LVR_BF16 && !(ix->cfg.flags & LVR_SEPARATE_KERNELS);
    const bool one_launch = one_launch_attention(ix, fused);
    const float *carried = fused ? ix->scores : nullptr;
    if (one_launch) {   // reads the set sizes from the internal counters and hands them to the caller
        Timed t(ix, LVR_K_ATTN_PARTIAL, st, true);
        LVR_HIP(lvr_launch_sparse_attention_wg(ix, q, out_idx, carried, lvr_head_count(ix), LVR_CNT_STRIDE, cap, out, out_count, st));
        ix->counters_dirty = 0;
        return LVR_OK;
    }
    {   // the attention reads the set sizes straight from the internal counters ...
        Timed t(ix, LVR_K_ATTN_PARTIAL, st);
        LVR_HIP(lvr_launch_sparse_partial(ix, q, out_idx, carried, lvr_head_count(ix), LVR_CNT_STRIDE, cap, st));
    }
    {   // ... and the combine pass hands them to the caller
        Timed t(ix, LVR_K_ATTN_COMBINE, st);
        LVR_HIP(lvr_launch_combine(ix, out, ix->P, lvr_head_count(ix), LVR_CNT_STRIDE, cap, out_count, st));
    }
    ix->counters_dirty = 0;
    return LVR_OK;
}

}  // namespace

extern "C" {

int lvr_query(lvr_index *ix, const float *q, const float *tau, int32_t *out_idx, int32_t *out_count, int64_t cap,
              void *stream) {
    if (!ix || !q || !tau || !out_count || cap < 0 || (cap > 0 && !out_idx)) return LVR_E_INVALID;
    if (!ix->built) return LVR_E_STATE;
    if (!on_home_device(ix)) return LVR_E_STATE;
    if (!aligned4(q) || !aligned4(tau) || !aligned4(out_idx) || !aligned4(out_count)) return LVR_E_INVALID;
    hipStream_t st = static_cast<hipStream_t>(stream);
    int rc = enqueue_query(ix, q, tau, out_idx, cap, st);
    if (rc != LVR_OK) return rc;
    {
        Timed t(ix, LVR_K_RESET, st);
        LVR_HIP(lvr_launch_publish_counts(ix, out_count, st));
    }
    ix->counters_dirty = 0;
    return LVR_OK;
}

int lvr_query1(lvr_index *ix, const float *q, const float *tau_s, const float *tau, int32_t *out_idx,
               int32_t *out_count, int64_t cap, void *stream) {
    if (!ix || !q || !tau_s || !tau || !out_count || cap < 0 || (cap > 0 && !out_idx)) return LVR_E_INVALID;
    if (!ix->built) return LVR_E_STATE;
    if (!on_home_device(ix)) return LVR_E_STATE;
    if (!aligned4(q) || !aligned4(tau) || !aligned4(tau_s) || !aligned4(out_idx) || !aligned4(out_count)) return LVR_E_INVALID;
    if (ix->cfg.kv_dtype != LVR_BF16 || (ix->cfg.flags & LVR_SEPARATE_KERNELS) || (ix->box && ix->cfg.n_subspaces > 4) ||
        ix->per_subspace)
        return LVR_E_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    int rc = enqueue_query(ix, q, tau, out_idx, cap, st, tau_s);
    if (rc != LVR_OK) return rc;
    {
        Timed t(ix, LVR_K_RESET, st);
        LVR_HIP(lvr_launch_publish_counts(ix, out_count, st));
    }
    ix->counters_dirty = 0;
    return LVR_OK;
}

int lvr_subspace_thresholds(lvr_index *ix, const float *q, const float *tau, float *tau_s_out, void *stream) {
    if (!ix || !q || !tau || !tau_s_out) return LVR_E_INVALID;
    if (!ix->built || !on_home_device(ix)) return LVR_E_STATE;
    if (!aligned4(q) || !aligned4(tau) || !aligned4(tau_s_out)) return LVR_E_INVALID;
    if (ix->cfg.kv_dtype != LVR_BF16 || (ix->cfg.flags & LVR_SEPARATE_KERNELS) || (ix->box && ix->cfg.n_subspaces > 4) ||
        ix->per_subspace)
        return LVR_E_UNSUPPORTED;
    LVR_HIP(lvr_launch_safe_tau_s(ix, q, tau, tau_s_out, static_cast<hipStream_t>(stream)));
    return LVR_OK;
}

int lvr_sparse_attention(lvr_index *ix, const float *q, const int32_t *idx, const int32_t *count, int64_t cap,
                         float *out, void *stream) {
    if (!ix || !q || !count || !out || cap < 0 || (cap > 0 && !idx)) return LVR_E_INVALID;
    if (!ix->built) return LVR_E_STATE;
    if (!on_home_device(ix)) return LVR_E_STATE;
    if (!aligned4(q) || !aligned4(idx) || !aligned4(count) || !aligned4(out)) return LVR_E_INVALID;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (one_launch_attention(ix)) {
        Timed t(ix, LVR_K_ATTN_PARTIAL, st, true);
        LVR_HIP(lvr_launch_sparse_attention_wg(ix, q, idx, nullptr, count, 1, cap, out, nullptr, st));
        return LVR_OK;
    }
    {
        Timed t(ix, LVR_K_ATTN_PARTIAL, st);
        LVR_HIP(lvr_launch_sparse_partial(ix, q, idx, nullptr, count, 1, cap, st));
    }
    {
        Timed t(ix, LVR_K_ATTN_COMBINE, st);
        LVR_HIP(lvr_launch_combine(ix, out, ix->P, count, 1, cap, nullptr, st));
    }
    return LVR_OK;
}

int lvr_decode_step(lvr_index *ix, const float *q, const float *tau, float *out, int32_t *out_idx, int32_t *out_count,
                    int64_t cap, void *stream) {
    if (!ix || !q || !tau || !out || !out_count || cap < 0 || (cap > 0 && !out_idx)) return LVR_E_INVALID;
    if (!ix->built) return LVR_E_STATE;
    if (!on_home_device(ix)) return LVR_E_STATE;
    if (!aligned4(q) || !aligned4(tau) || !aligned4(out) || !aligned4(out_idx) || !aligned4(out_count)) return LVR_E_INVALID;
    return decode_step_impl(ix, q, tau, out, out_idx, out_count, cap, static_cast<hipStream_t>(stream), nullptr, nullptr, 0);
}

int lvr_append_decode_step(lvr_index *ix, const void *k_new, const void *v_new, int64_t m, const float *q,
                           const float *tau, float *out, int32_t *out_idx, int32_t *out_count, int64_t cap,
                           void *stream) {
    if (!ix || !q || !tau || !out || !out_count || cap < 0 || (cap > 0 && !out_idx)) return LVR_E_INVALID;
    if (m < 0 || (m > 0 && (!k_new || !v_new))) return LVR_E_INVALID;
    if (!ix->built) return LVR_E_STATE;
    if (!on_home_device(ix)) return LVR_E_STATE;
    if (!aligned4(q) || !aligned4(tau) || !aligned4(out) || !aligned4(out_idx) || !aligned4(out_count)) return LVR_E_INVALID;
    if (ix->n_total + m > ix->cfg.capacity) return LVR_E_CAPACITY;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // The copy rides in the query launch when that launch has a buffer workgroup to do it and the
    // append needs nothing else (no chunk becomes full, no position maps, no reservoir, no update in
    // flight); otherwise the two calls run one after the other.
    const bool rides = m > 0 && m <= 64 && ix->cfg.kv_dtype == LVR_BF16 && !(ix->cfg.flags & LVR_SEPARATE_KERNELS) &&
                       !ix->slot_pos && !ix->reservoir && !ix->pending && !ix->per_subspace && aligned16(k_new) && aligned16(v_new) &&
                       ix->n_total + m - ix->n_indexed < ix->cfg.buffer_size;
    if (!rides) {
        int rc = lvr_append(ix, k_new, v_new, m, stream);
        if (rc != LVR_OK) return rc;
        return decode_step_impl(ix, q, tau, out, out_idx, out_count, cap, st, nullptr, nullptr, 0);
    }
    return decode_step_impl(ix, q, tau, out, out_idx, out_count, cap, st, k_new, v_new, m);
}

int lvr_threshold(lvr_index *ix, const float *q, int mode, float param, float *tau_out, void *stream) {
    if (!ix || !q || !tau_out || mode < LVR_TAU_SAMPLE_MAX || mode > LVR_TAU_BUDGET) return LVR_E_INVALID;
    if (mode == LVR_TAU_BUDGET && !(param > 0.f && param <= 1.f)) return LVR_E_INVALID;
    if (mode == LVR_TAU_SAMPLE_TOPK && param < 1.f) return LVR_E_INVALID;
    if (!ix->built || !ix->reservoir || !on_home_device(ix)) return LVR_E_STATE;
    if (!aligned4(q) || !aligned4(tau_out)) return LVR_E_INVALID;
    LVR_HIP(lvr_launch_threshold(ix, q, mode, param, tau_out, static_cast<hipStream_t>(stream)));
    return LVR_OK;
}

int lvr_export_reservoir(lvr_index *ix, int32_t *positions) {
    if (!ix || !positions) return LVR_E_INVALID;
    if (!ix->reservoir) return LVR_E_STATE;
    LVR_HIP(hipDeviceSynchronize());
    LVR_HIP(hipMemcpy(positions, ix->reservoir, (size_t)lvr_n_bh(ix) * ix->cfg.reservoir_size * sizeof(int32_t),
                      hipMemcpyDeviceToHost));
    return LVR_OK;
}

int lvr_dense_attention(lvr_index *ix, const float *q, float *out, void *stream) {
    if (!ix || !q || !out) return LVR_E_INVALID;
    if (!ix->built) return LVR_E_STATE;
    if (!on_home_device(ix)) return LVR_E_STATE;
    if (!aligned4(q) || !aligned4(out)) return LVR_E_INVALID;
    hipStream_t st = static_cast<hipStream_t>(stream);
    {
        Timed t(ix, LVR_K_DENSE_PARTIAL, st);
        LVR_HIP(lvr_launch_dense_partial(ix, q, st));
    }
    {
        Timed t(ix, LVR_K_DENSE_COMBINE, st);
        LVR_HIP(lvr_launch_combine(ix, out, lvr_dense_splits(ix), nullptr, 0, 0, nullptr, st));
    }
    return LVR_OK;
}

int lvr_get_stats(lvr_index *ix, lvr_stats *out) {
    if (!ix || !out) return LVR_E_INVALID;
    LVR_HIP(hipDeviceSynchronize());
    const int n_bh = lvr_n_bh(ix), n_bhq = lvr_n_bhq(ix);
    const size_t n_ints = lvr_counter_ints(n_bh, n_bhq, ix->max_groups);
    int32_t *host = static_cast<int32_t *>(malloc(sizeof(int32_t) * n_ints));
    if (!host) return LVR_E_NOMEM;
    hipError_t e = hipMemcpy(host, ix->counters, sizeof(int32_t) * n_ints, hipMemcpyDeviceToHost);
    if (e != hipSuccess) {
        free(host);
        return hip_fail(e);
    }
    memset(out, 0, sizeof(*out));
    const int r = ix->cfg.group_size;
    int64_t surv = 0, emitted = 0;
    const int32_t *stat = host + ((size_t)n_bhq + 1) * LVR_CNT_STRIDE;
    for (int i = 0; i < n_bhq; ++i) emitted += stat[i];
    const int overflow = host[(size_t)n_bhq * LVR_CNT_STRIDE];
    const int32_t *seg = stat + n_bhq;
    const int64_t max_segs = lvr_max_segs(ix->max_groups);
    for (int i = 0; i < n_bh; ++i)
        for (int x = 0; x < ix->n_segs; ++x) surv += seg[(size_t)i * max_segs + x];
    free(host);
    const int64_t row_bytes = (int64_t)LVR_D * (int64_t)ix->elt;
    out->n_keys = ix->n_total;
    out->n_indexed = ix->n_indexed;
    out->groups_scored = ix->last_skipped ? 0 : (ix->last_indexed / r) * n_bh;   // no bound was evaluated when the test was off
    out->update_pending = ix->pending;
    out->groups_surviving = surv;   // one grouping per block: the candidate KEYS (a key has S groups, none of which is "its" group)
    out->keys_scanned = (ix->per_subspace ? surv : surv * r) + ix->last_buffer_rows * n_bh;
    out->keys_emitted = emitted;
    out->bytes_index = out->groups_scored * ((int64_t)ix->centre_bytes * (ix->box ? 2 : 1) + (int64_t)ix->S_store * 4);
    if (ix->per_subspace)   // plus the labels of every indexed key; the block-bound table is work space, not index
        out->bytes_index += ix->last_indexed * n_bh * (int64_t)ix->cfg.n_subspaces * 2;
    out->bytes_keys = out->keys_scanned * row_bytes;
    out->bytes_attention = emitted * 2 * row_bytes;
    out->overflow = overflow;
    if (overflow) {
        LVR_HIP(hipMemset(lvr_overflow_flag(ix), 0, sizeof(int32_t)));
        return LVR_E_OVERFLOW;
    }
    return LVR_OK;
}

int lvr_export_index(lvr_index *ix, void *centres, float *radii, int32_t *slot_pos, void *keys) {
    if (!ix) return LVR_E_INVALID;
    if (!ix->built) return LVR_E_STATE;
    LVR_HIP(hipDeviceSynchronize());
    const int n_bh = lvr_n_bh(ix);
    const int r = ix->cfg.group_size, S = ix->S_store;
    const int64_t ng = ix->n_indexed / r, n = ix->n_total;
    const size_t row_bytes = LVR_D * ix->elt;
    const size_t crow = row_bytes * (ix->box ? 2 : 1);   // bytes of one group's enclosure rows
    for (int bh = 0; bh < n_bh; ++bh) {
        if (centres && ng > 0 && ix->cf6) {
            // e2m3 codes (6 bits, matrix-operand order) times the scale of their block -> bf16 bit patterns in
            // coordinate order (exact: 4 significant bits).  Lane piece b of a row is its bytes 24 b .. 24 b + 23:
            // 32 codes, code 8 kk + e = coordinate 32 kk + 8 b + e; the scale of piece b is byte b of the third
            // word of the group's 12-byte record in `radii`.
            const int cb = ix->centre_bytes;
            int8_t chan[LVR_D];
            LVR_HIP(hipMemcpy(chan, lvr_chan_exp(ix) + (size_t)bh * LVR_CHAN_STRIDE, LVR_D, hipMemcpyDeviceToHost));
            uint8_t *codes = static_cast<uint8_t *>(malloc((size_t)ng * cb));
            uint32_t *rec = static_cast<uint32_t *>(malloc((size_t)ng * 12));
            if (!codes || !rec) {
                free(codes);
                free(rec);
                return LVR_E_NOMEM;
            }
            hipError_t e = hipMemcpy(codes, static_cast<char *>(ix->centres) + (size_t)bh * ix->max_groups * cb, (size_t)ng * cb,
                                     hipMemcpyDeviceToHost);
            if (e == hipSuccess)
                e = hipMemcpy(rec, ix->radii + (size_t)bh * ix->max_groups * 3, (size_t)ng * 12, hipMemcpyDeviceToHost);
            if (e != hipSuccess) {
                free(codes);
                free(rec);
                return hip_fail(e);
            }
            uint16_t *dst = static_cast<uint16_t *>(centres) + (size_t)bh * ng * LVR_D;
            for (int64_t g = 0; g < ng; ++g)
                for (int c = 0; c < LVR_D; ++c) {
                    const int kk = c / 32, b = (c % 32) / 8, j = c % 8;
                    const int bit = 6 * (8 * kk + j);
                    const uint8_t *piece = codes + g * cb + 24 * b;
                    const uint32_t two = (uint32_t)piece[bit >> 3] | ((uint32_t)piece[(bit >> 3) + 1 < 24 ? (bit >> 3) + 1 : 23] << 8);
                    const uint32_t code = (two >> (bit & 7)) & 63u;
                    const int sgn = code >> 5, ex = (code >> 3) & 3, m = code & 7;
                    const int E = (int)((rec[g * 3 + 2] >> (8 * b)) & 0xffu) - 127 + (int)chan[c];   // back to the keys' own space
                    const float v = ldexpf(ex == 0 ? (float)m / 8.f : ldexpf(1.f + (float)m / 8.f, ex - 1), E);
                    uint32_t bits;
                    const float sv = sgn ? -v : v;
                    memcpy(&bits, &sv, 4);
                    dst[g * LVR_D + c] = (uint16_t)(bits >> 16);
                }
            free(codes);
            free(rec);
        } else if (centres && ng > 0 && ix->cf8) {
            // e4m3 codes in matrix-operand order -> bf16 bit patterns in coordinate order (exact);
            // one row of codes per ball, two (upper, lower corner) per box
            const int64_t nr = ng * (ix->box ? 2 : 1), max_rows = ix->max_groups * (ix->box ? 2 : 1);
            uint8_t *codes = static_cast<uint8_t *>(malloc((size_t)nr * LVR_D));
            if (!codes) return LVR_E_NOMEM;
            hipError_t e = hipMemcpy(codes, static_cast<char *>(ix->centres) + (size_t)bh * max_rows * LVR_D,
                                     (size_t)nr * LVR_D, hipMemcpyDeviceToHost);
            if (e != hipSuccess) {
                free(codes);
                return hip_fail(e);
            }
            uint16_t *dst = static_cast<uint16_t *>(centres) + (size_t)bh * nr * LVR_D;
            for (int64_t g = 0; g < nr; ++g)
                for (int c = 0; c < LVR_D; ++c) {
                    const int kk = c / 32, kq = (c % 32) / 8, j = c % 8;
                    const uint8_t code = codes[g * LVR_D + kq * 32 + kk * 8 + j];
                    const int sgn = code >> 7, ex = (code >> 3) & 15, m = code & 7;
                    const float v = ex == 0 ? ldexpf((float)m / 8.f, -6) : ldexpf(1.f + (float)m / 8.f, ex - 7);
                    uint32_t bits;
                    const float sv = sgn ? -v : v;
                    memcpy(&bits, &sv, 4);
                    dst[g * LVR_D + c] = (uint16_t)(bits >> 16);   // 4 significant bits: exact in bf16
                }
            free(codes);
        } else if (centres && ng > 0)
            LVR_HIP(hipMemcpy(static_cast<char *>(centres) + (size_t)bh * ng * crow,
                              static_cast<char *>(ix->centres) + (size_t)bh * ix->max_groups * crow,
                              (size_t)ng * crow, hipMemcpyDeviceToHost));
        if (radii && ng > 0 && (ix->cf8 || ix->cf6) && !ix->box) {
            // four bf16 per group (slot s = rho_s) -> one float per subspace; records of 8 bytes (8-bit centres)
            // or 12 bytes (6-bit centres: the scale bytes follow the radii)
            const int Ss = ix->cfg.n_subspaces;
            const int rec16 = ix->S_store * 2;   // record length in 16-bit units
            uint16_t *blk = static_cast<uint16_t *>(malloc((size_t)ng * rec16 * 2));
            if (!blk) return LVR_E_NOMEM;
            hipError_t e = hipMemcpy(blk, ix->radii + (size_t)bh * ix->max_groups * ix->S_store, (size_t)ng * rec16 * 2, hipMemcpyDeviceToHost);
            if (e != hipSuccess) {
                free(blk);
                return hip_fail(e);
            }
            for (int64_t g = 0; g < ng; ++g)
                for (int sidx = 0; sidx < Ss; ++sidx) {
                    const uint32_t hi = (uint32_t)blk[g * rec16 + sidx] << 16;
                    float fh;
                    memcpy(&fh, &hi, 4);
                    radii[((size_t)bh * ng + g) * Ss + sidx] = fh;
                }
            free(blk);
        } else if (radii && ng > 0)
            LVR_HIP(hipMemcpy(radii + (size_t)bh * ng * S, ix->radii + (size_t)bh * ix->max_groups * S,
                              (size_t)ng * S * sizeof(float), hipMemcpyDeviceToHost));
        if (keys && n > 0)
            LVR_HIP(hipMemcpy(static_cast<char *>(keys) + (size_t)bh * n * row_bytes,
                              static_cast<char *>(ix->K) + (size_t)bh * ix->cap_rows * row_bytes, (size_t)n * row_bytes,
                              hipMemcpyDefault));
        if (slot_pos && n > 0) {
            if (ix->slot_pos) {
                LVR_HIP(hipMemcpy(slot_pos + (size_t)bh * n, ix->slot_pos + (size_t)bh * ix->cap_rows,
                                  (size_t)n * sizeof(int32_t), hipMemcpyDeviceToHost));
            } else {
                for (int64_t i = 0; i < n; ++i) slot_pos[(size_t)bh * n + i] = (int32_t)i;
            }
        }
    }
    return LVR_OK;
}

int lvr_export_channel_scales(lvr_index *ix, int8_t *exp_host) {
    if (!ix || !exp_host) return LVR_E_INVALID;
    if (!ix->built) return LVR_E_STATE;
    LVR_HIP(hipDeviceSynchronize());
    LVR_HIP(hipMemcpy2D(exp_host, LVR_D, lvr_chan_exp(ix), LVR_CHAN_STRIDE, LVR_D, (size_t)lvr_n_bh(ix), hipMemcpyDeviceToHost));
    return LVR_OK;
}

int lvr_export_labels(lvr_index *ix, int32_t *labels_host) {
    if (!ix || !labels_host) return LVR_E_INVALID;
    if (!ix->built || !ix->per_subspace) return LVR_E_STATE;
    LVR_HIP(hipDeviceSynchronize());
    const int n_bh = lvr_n_bh(ix), S = ix->cfg.n_subspaces;
    const int64_t ni = ix->n_indexed;
    if (ni == 0) return LVR_OK;
    uint16_t *tmp = static_cast<uint16_t *>(malloc((size_t)ni * S * sizeof(uint16_t)));
    if (!tmp) return LVR_E_NOMEM;
    for (int bh = 0; bh < n_bh; ++bh) {
        hipError_t e = hipMemcpy(tmp, ix->labels + (size_t)bh * ix->cap_rows * S, (size_t)ni * S * sizeof(uint16_t),
                                 hipMemcpyDeviceToHost);
        if (e != hipSuccess) {
            free(tmp);
            return hip_fail(e);
        }
        for (int sb = 0; sb < S; ++sb)
            for (int64_t j = 0; j < ni; ++j) labels_host[((size_t)bh * S + sb) * ni + j] = tmp[j * S + sb];
    }
    free(tmp);
    return LVR_OK;
}

int lvr_profile_enable(lvr_index *ix, int max_launches) {
    if (!ix || max_launches < 0 || max_launches > (1 << 20)) return LVR_E_INVALID;
    LVR_HIP(hipDeviceSynchronize());
    prof_free(ix);
    if (max_launches == 0) return LVR_OK;
    ix->prof_events = static_cast<hipEvent_t *>(calloc((size_t)2 * max_launches, sizeof(hipEvent_t)));
    ix->prof_kind = static_cast<uint8_t *>(calloc((size_t)max_launches, 1));
    if (!ix->prof_events || !ix->prof_kind) {
        prof_free(ix);
        return LVR_E_NOMEM;
    }
    for (int i = 0; i < 2 * max_launches; ++i) {
        hipError_t e = hipEventCreate(&ix->prof_events[i]);
        if (e != hipSuccess) {
            ix->prof_cap = i;
            prof_free(ix);
            return hip_fail(e);
        }
    }
    ix->prof_cap = 2 * max_launches;
    ix->prof_on = 1;
    return LVR_OK;
}

int lvr_profile_read(lvr_index *ix, lvr_profile *out) {
    if (!ix || !out) return LVR_E_INVALID;
    memset(out, 0, sizeof(*out));
    LVR_HIP(hipDeviceSynchronize());
    for (int s = 0; s + 1 < ix->prof_used; s += 2) {
        float ms = 0.f;
        LVR_HIP(hipEventElapsedTime(&ms, ix->prof_events[s], ix->prof_events[s + 1]));
        const int k = ix->prof_kind[s / 2];
        out->ms[k] += ms;
        out->launches[k] += 1;
    }
    ix->prof_used = 0;
    return LVR_OK;
}

int lvr_set_bound_test(lvr_index *ix, int enabled) {
    if (!ix) return LVR_E_INVALID;
    if (!enabled && (ix->cfg.kv_dtype != LVR_BF16 || (ix->cfg.flags & LVR_SEPARATE_KERNELS) || ix->per_subspace))
        return LVR_E_UNSUPPORTED;
    ix->skip_bounds = enabled ? 0 : 1;
    return LVR_OK;
}

int lvr_length(const lvr_index *ix, int64_t *n, int64_t *n_indexed) {
    if (!ix) return LVR_E_INVALID;
    if (n) *n = ix->n_total;
    if (n_indexed) *n_indexed = ix->n_indexed;
    return LVR_OK;
}

const char *lvr_strerror(int code) {
    switch (code) {
        case LVR_OK: return "ok";
        case LVR_E_INVALID: return "invalid argument";
        case LVR_E_UNSUPPORTED: return "unsupported configuration";
        case LVR_E_CAPACITY: return "index capacity exceeded";
        case LVR_E_OVERFLOW: return "a retrieved set exceeded the output capacity (list truncated)";
        case LVR_E_HIP: return "HIP runtime error";
        case LVR_E_NOMEM: return "out of memory";
        case LVR_E_STATE: return "call out of order (index not built)";
        default: return "unknown error";
    }
}

int lvr_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
