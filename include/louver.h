/*
 * louver.h — C ABI of the MI355X (gfx950) library for the decode-time hot path of the Louver
 * KV-cache index: build/append an index of bounding balls over the cached keys, answer the
 * halfspace range query { k : <q,k> >= tau } per query head with no false negatives, and run
 * softmax attention over only the retrieved keys and values.
 *
 * Conventions
 *   - Every pointer named *_dev is DEVICE memory on the GPU that was current at lvr_create;
 *     every pointer named *_host is HOST memory.  The caller owns all buffers it passes in;
 *     the library owns the index arena (its own copy of K and V, centres, radii, work lists).
 *     That GPU must be the current device in every later call on the index (LVR_E_STATE
 *     otherwise).  fp32 and int32 arrays must be 4-byte aligned, K and V rows 16-byte aligned
 *     (LVR_E_INVALID otherwise; the pointers themselves are not dereferenced on the host).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All device work
 *     of a call is enqueued on that stream and the hot-path calls never synchronise with the
 *     host; results are valid once the stream reaches the end of the call's work.
 *     Calls that touch the same index must be ordered by the caller (same stream, or events).
 *   - Return value: 0 on success, a negative lvr_error otherwise.  Nothing is thrown across
 *     the ABI.  lvr_strerror gives a static string for every code.
 *   - Layouts are row-major with the last index contiguous.  Head mapping for grouped-query
 *     attention: query head h reads KV head h / (n_q_heads / n_kv_heads)  (Sec. 2, "KV Cache").
 *   - tau is in RAW dot-product units (Problem 1, Sec. 2); the softmax scale sigma multiplies
 *     the logits only inside the attention (Alg. 3 / Alg. 4, input "scale sigma").
 *   - Positions reported in index lists are token positions in order of arrival
 *     (0 .. n-1 for the keys given to lvr_build, then one more per appended token).
 */
#ifndef LOUVER_H_
#define LOUVER_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lvr_index lvr_index; /* opaque, owned by the library */

enum lvr_dtype { LVR_BF16 = 0, LVR_F32 = 1 };

/* How keys are put into groups of r (Def. 2 of the appendix "Ablation on Index Design";
 * the query result does not depend on the choice, only the pruning power does).
 *   CONTIGUOUS: r consecutive token positions form a group (the appendix's best performer).
 *   TREE:       recursive median split on the coordinate axis of largest variance (Alg. 2),
 *               one tree over the full key shared by all subspaces; rows are stored regrouped.
 *   SUBSPACE_TREE: the paper's own layout (Sec. 4.1, Alg. 1): Alg. 2 is run once per subspace on that
 *               subspace's coordinates, so every subspace has a grouping of its own and a key carries one
 *               16-bit label per subspace; rows stay in arrival order.  A key is a candidate iff the
 *               bounds of its S groups add up to tau ("Query 2"'s bound, evaluated per key; a subset of
 *               what Alg. 4's depth scan keeps).  bf16 caches, balls with centres in the cache's format,
 *               at most four query heads per KV head, at most 65536 groups per (sequence, KV head),
 *               fused launch form, single-stream update, K and V in device memory; lvr_query1,
 *               lvr_subspace_thresholds and lvr_set_bound_test are not available (LVR_E_UNSUPPORTED). */
enum lvr_grouping { LVR_GROUP_CONTIGUOUS = 0, LVR_GROUP_TREE = 1, LVR_GROUP_SUBSPACE_TREE = 2 };

/* Shape that encloses a group (appendix "Ablation on Index Design", Def. 1).
 *   BALL: centre + one radius per coordinate block (Sec. 4.1, Eq. (1)); bound of Eq. (2) per block, summed.
 *   AABB: per coordinate the smallest and largest member value; bound sum_c max(q_c lo_c, q_c hi_c)
 *         (two dot products per group, usually tighter).  bf16 caches, fused query kernel only;
 *         n_subspaces is ignored. */
enum lvr_enclosing { LVR_ENCLOSE_BALL = 0, LVR_ENCLOSE_AABB = 1 };

/* Storage of the centres (Sec. 4.1; the paper does not fix their precision).  Whatever the
 * format, every radius is measured against the centre AS STORED, so a ball always encloses its
 * members and no qualifying key can be lost; a coarser centre only makes the balls larger.
 *   SAME: the cache's own format (bf16 or fp32), 2 or 4 bytes per coordinate.
 *   FP8:  OCP e4m3 codes (1 sign, 4 exponent, 3 mantissa bits), 1 byte per coordinate: the index
 *         read of a query halves.  Box corners are rounded outwards (upper corner up, lower corner
 *         down), so the stored box contains the exact one.  bf16 caches and the fused query kernel;
 *         balls with n_subspaces <= 4, or boxes (LVR_E_UNSUPPORTED otherwise).
 *   FP6:  6-bit codes with a shared power-of-two scale per 32 coordinates (the OCP microscaling
 *         element format e2m3: 1 sign, 2 exponent, 3 mantissa bits; scale = an 8-bit exponent), 96 bytes
 *         of codes and 12 bytes of radii and scales per group: a fifth less index than FP8 for balls
 *         about 1.6 times as large.  The 32 coordinates that share a scale are the ones one lane of the
 *         query kernel holds (coordinates 32 kk + 8 b + e, kk = 0..3, e = 0..7, for scale block b), so a
 *         lane decodes its share of a centre with one conversion instruction.  Balls with
 *         n_subspaces <= 4, bf16 caches, the fused query kernel (LVR_E_UNSUPPORTED otherwise).
 *         Such an index lives in a rescaled space:
 *         coordinate c of every key of a (sequence, KV head) is divided by 2^e_c (e_c in [-8, 8], taken
 *         from the keys handed to lvr_build; zero before the first build), so that one large channel does
 *         not drown the 31 that share its scale; the query kernels multiply q_c by 2^e_c, which leaves
 *         every dot product as it was.  Centres, codes and radii are formed in that space, and the balls
 *         enclose the rescaled keys (lvr_export_channel_scales hands out the exponents).
 *   AUTO: FP6 for balls where it is supported and K/V are in device memory, else SAME. */
enum lvr_index_dtype { LVR_INDEX_AUTO = 0, LVR_INDEX_SAME = 1, LVR_INDEX_FP8 = 2, LVR_INDEX_FP6 = 3 };

enum lvr_flags {
    /* Keys not yet in the index (the buffer of Sec. 4.3 "Dynamic Updates") are retrieved
     * whatever their score, as in Alg. 3 / Alg. 4's  K[L*] ∪ B.  Default (flag clear): they are
     * scored exactly and thresholded like every other key, so the result is Problem 1's set. */
    LVR_ATTEND_BUFFER_DENSE = 1u,
    /* Run the bound test and the exact check as two kernel launches (survivor list through
     * HBM) instead of the fused single launch.  Same results; lets the two stages be timed
     * apart.  fp32 caches always run this way. */
    LVR_SEPARATE_KERNELS = 2u,
    /* Two-stream update (App. "GPU Update").  When an lvr_append fills the buffer, the B buffered
     * keys are grouped on a stream the library owns, into index slots beyond the published group
     * count, while calls on the caller's stream keep answering queries with those keys still in
     * the buffer (scanned exactly, so results do not change).  The new groups are published by
     * lvr_publish, or by a later lvr_append: the first one that finds the side stream finished
     * (a host-side poll; it never blocks), at the latest the one that fills the next chunk.  To
     * publish, the caller's stream waits for the side stream's event, then the published count
     * advances.  All calls on one index must be
     * ordered on one stream. */
    LVR_CONCURRENT_UPDATE = 4u,
    /* Offloaded mode (Sec. 5 "KV Cache Offloading"): the K and V arena lives in pinned host
     * memory that the GPU reads in place; only the index (centres or boxes, radii) and the
     * work space stay in device memory.  The bound test runs on the GPU over the index; only
     * the rows of surviving groups, and later the retrieved rows, cross the host link.  Every
     * entry point works unchanged; lvr_arena_bytes then excludes the K and V arena. */
    LVR_KV_IN_HOST_MEMORY = 8u
};

enum lvr_error {
    LVR_OK = 0,
    LVR_E_INVALID = -1,     /* bad argument (NULL, misaligned, negative size, unknown flag)   */
    LVR_E_UNSUPPORTED = -2, /* valid request this build has no kernel for                      */
    LVR_E_CAPACITY = -3,    /* more keys than lvr_config.capacity                               */
    LVR_E_OVERFLOW = -4,    /* a retrieved set was larger than the caller's `cap` (sticky)      */
    LVR_E_HIP = -5,         /* a HIP runtime call failed; see lvr_last_hip_error                */
    LVR_E_NOMEM = -6,
    LVR_E_STATE = -7        /* call order wrong (e.g. query before build), or the current device
                             * is not the one the index was created on                        */
};

typedef struct lvr_config {
    int32_t batch;       /* independent sequences, each with its own cache                      */
    int32_t n_q_heads;   /* H_q                                                                  */
    int32_t n_kv_heads;  /* H_kv, divides H_q; G = H_q / H_kv in {1,2,4,8}                       */
    int32_t head_dim;    /* d; this build supports 128                                           */
    int32_t kv_dtype;    /* lvr_dtype of K, V and of the stored centres                          */
    int32_t group_size;  /* r in {1,2,4,8,16}  (Def. 2)                                          */
    int32_t n_subspaces; /* S in {1,2,4,8,16}: contiguous coordinate blocks of d/S (Sec. 4.1)    */
    int32_t buffer_size; /* B: appended keys are indexed B at a time; multiple of 16 and of r    */
    int32_t grouping;    /* lvr_grouping                                                         */
    int32_t enclosing;   /* lvr_enclosing                                                        */
    uint32_t flags;      /* lvr_flags                                                            */
    int64_t capacity;    /* max keys per (sequence, KV head): the arena is sized once (App. "GPU Update") */
    float scale;         /* sigma; 0 means 1/sqrt(head_dim)  (Sec. 2, "Attention")               */
    int32_t attn_splits; /* P > 0: up to P partial-softmax splits per head, then a combine launch;
                          * -1: one workgroup per head, 16 splits merged in LDS, a single launch;
                          * 0: chosen per call: the single launch for batches of 128 heads or more
                          *    and for contexts up to 65536 keys, else 64 splits + combine      */
    int32_t reservoir_size; /* R <= 256 past keys kept per (sequence, KV head) by reservoir sampling for
                             * lvr_threshold (appendix "Threshold Oracle Comparison"); 0 = none         */
    uint64_t seed;          /* seed of the counter-based generator behind the reservoir              */
    int32_t index_dtype;    /* lvr_index_dtype: storage of the centres                               */
    int32_t query_workgroups; /* workgroups a range-query launch aims at (its segment size follows from it);
                               * 0 = the default, 1024 (four per compute unit); a tuning knob, results do not
                               * depend on it                                                        */
} lvr_config;

/* Counters of the most recent lvr_query / lvr_decode_step, summed over batch and heads. */
typedef struct lvr_stats {
    int64_t n_keys;           /* keys per (sequence, KV head) currently held                     */
    int64_t n_indexed;        /* of which inside index groups (the rest is the buffer)           */
    int64_t groups_scored;    /* balls tested                                                    */
    int64_t groups_surviving; /* balls whose bound reached tau for at least one head of the group */
    int64_t keys_scanned;     /* keys given the exact dot product (survivors * r + buffer)       */
    int64_t keys_emitted;     /* sum of retrieved-set sizes                                      */
    int64_t bytes_index;      /* centre + radius bytes read                                      */
    int64_t bytes_keys;       /* candidate key bytes read by the exact filter                    */
    int64_t bytes_attention;  /* K and V bytes gathered by the sparse attention                  */
    int32_t overflow;         /* 1 if some retrieved set exceeded cap since the last call here   */
    int32_t update_pending;   /* 1 while groups prepared by a concurrent update await lvr_publish */
} lvr_stats;

/* Allocate an index (arena for `capacity` keys per sequence and KV head, plus work space) on
 * the current device.  *out is set only on success. */
int lvr_create(const lvr_config *cfg_host, lvr_index **out);
int lvr_destroy(lvr_index *ix);

/* Device bytes lvr_create would allocate for this configuration (0 if it is invalid). */
size_t lvr_arena_bytes(const lvr_config *cfg_host);
/* Pinned host bytes lvr_create would allocate (non-zero only with LVR_KV_IN_HOST_MEMORY). */
size_t lvr_host_bytes(const lvr_config *cfg_host);

/* Index construction (Sec. 4.1, Alg. 1; grouping per lvr_config.grouping; Eq. (1) balls).
 * K_dev, V_dev: [batch][n_kv_heads][n][head_dim] of kv_dtype, addressed with ELEMENT strides
 * k_strides_host / v_strides_host = {batch, kv head, token}; the head_dim axis is contiguous.
 * Copies K and V into the arena, forms floor(n/r) groups; a tail of n mod r keys waits in the
 * buffer and is scanned exactly.  Discards any earlier content.  n <= capacity. */
int lvr_build(lvr_index *ix, const void *K_dev, const void *V_dev, int64_t n,
              const int64_t k_strides_host[3], const int64_t v_strides_host[3], void *stream);

/* Dynamic update (Sec. 4.3; App. "GPU Update", single-stream form): m new tokens per
 * (sequence, KV head), k_new_dev / v_new_dev: [batch][n_kv_heads][m][head_dim] contiguous.
 * New keys join the buffer; whenever the buffer holds B keys they are grouped and their
 * balls appended to the index.
 * A call that returns LVR_E_INVALID, LVR_E_STATE, LVR_E_CAPACITY or LVR_E_UNSUPPORTED has stored
 * nothing (every such check precedes the first store).  After LVR_E_HIP the rows may or may not
 * have been stored: rebuild the index with lvr_build rather than repeating the append. */
int lvr_append(lvr_index *ix, const void *k_new_dev, const void *v_new_dev, int64_t m, void *stream);

/* Phase 2 of the two-stream update (App. "GPU Update"): make `stream` wait for the side stream's
 * update-done event and publish the prepared groups to later queries.  No-op when nothing is
 * pending (always, without LVR_CONCURRENT_UPDATE). */
int lvr_publish(lvr_index *ix, void *stream);

/* Range query (Problem 1; Sec. 4.2): bound test of every ball against the halfspace
 * (Eq. (2), summed over subspaces as in "Query 2"), then the exact dot product on the keys
 * of surviving groups and on the buffer.
 *   q_dev   [batch][n_q_heads][head_dim] fp32
 *   tau_dev [batch][n_q_heads] fp32, -INFINITY allowed (retrieves everything)
 *   out_idx_dev   [batch][n_q_heads][cap] int32 positions, order within a head unspecified
 *   out_count_dev [batch][n_q_heads] int32, the TRUE set size even when it exceeds cap
 * A key is emitted iff its fp32 score >= tau - 0.5e-4*|tau| (the comparison leans towards
 * inclusion so that rounding-order differences never lose a key).  The slack is relative to
 * |tau|: at tau = 0 it vanishes and the decision is the sign of the kernel's own fp32 score (bf16
 * products are exact, accumulation is fp32 in matrix-core order), which can differ from another
 * summation order by a few units of 2^-24 * sum_c |q_c k_c|; every key whose exact score exceeds
 * tau by more than head_dim * 2^-23 * sum_c |q_c k_c| is returned whatever tau is, and integer-valued
 * data (exact sums) is decided exactly.  If a set exceeds cap the
 * list is truncated and a sticky overflow flag is raised (reported by lvr_get_stats). */
int lvr_query(lvr_index *ix, const float *q_dev, const float *tau_dev, int32_t *out_idx_dev,
              int32_t *out_count_dev, int64_t cap, void *stream);

/* "Query 1" (Sec. 4.2, Eq. "ball gate" per subspace; Alg. 3): per-subspace thresholds.
 *   tau_s_dev [batch][n_q_heads][S] fp32: tau_s is a lower bound on <pi_s q, pi_s k> for every
 *             key the caller regards as relevant; a group is a candidate for a head iff in EVERY
 *             subspace its ball bound reaches that subspace's threshold
 *   tau_dev   [batch][n_q_heads]: the exact check on candidates, as in lvr_query
 * Every key with <q,k> >= tau whose subspace products all reach their tau_s is returned; keys
 * with <q,k> >= tau that miss some tau_s may or may not be (they are outside Query 1's promise).
 * Buffer keys are checked against tau only.  bf16 caches, fused launch form: balls with any
 * n_subspaces; boxes with n_subspaces <= 4 blocks (per block the box bound of that block's
 * coordinates plus the group's allowance); other configurations return LVR_E_UNSUPPORTED. */
int lvr_query1(lvr_index *ix, const float *q_dev, const float *tau_s_dev, const float *tau_dev, int32_t *out_idx_dev,
               int32_t *out_count_dev, int64_t cap, void *stream);

/* Per-subspace thresholds for lvr_query1 derived from tau alone (Sec. 4.2: Query 1 is correct
 * when tau_s is a lower bound on the subspace term of every relevant key).  For every query
 * head, tau_s = tau - (sum over the OTHER subspaces of the largest ball bound, Eq. (2), among the
 * indexed groups): every key with <q,k> >= tau then reaches tau_s in every subspace, so
 * lvr_query1 with these thresholds returns Problem 1's set.  One pass over the index.
 *   q_dev [batch][n_q_heads][head_dim], tau_dev [batch][n_q_heads] (-INFINITY gives -INFINITY),
 *   tau_s_out_dev [batch][n_q_heads][S]; all -INFINITY while no group is indexed.
 * Same configurations as lvr_query1 (LVR_E_UNSUPPORTED otherwise).  Uses the work space of the
 * attention entry points: order it with them on one stream. */
int lvr_subspace_thresholds(lvr_index *ix, const float *q_dev, const float *tau_dev, float *tau_s_out_dev,
                            void *stream);

/* Attention over given index lists (Sec. 2 "Sparse Attention"; App. "GPU Sparse Attention
 * Kernel": P splits with partial (m, l, o), then a combine pass).  Softmax is normalised over
 * the listed keys only.  idx_dev / count_dev as produced by lvr_query (count is clamped to
 * cap; positions outside [0, n) are skipped).  out_dev [batch][n_q_heads][head_dim] fp32;
 * an empty list gives zeros. */
int lvr_sparse_attention(lvr_index *ix, const float *q_dev, const int32_t *idx_dev,
                         const int32_t *count_dev, int64_t cap, float *out_dev, void *stream);

/* lvr_sparse_attention for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  No lvr_index is needed and
 * nothing is allocated or freed, by this call or by anything it uses: K_dev and V_dev are the
 * caller's own cache, contiguous [batch][n_kv_heads][n][128] of kv_dtype (rows 16-byte aligned),
 * positions in idx_dev are row numbers 0 .. n-1, and the split pass keeps its partial (m, l, o)
 * triples in a static device array inside the library (8.1 MiB per GPU, held until the process
 * ends) whose per-device address is looked up on the first call on that device.
 * Same kernels and same results as lvr_sparse_attention with attn_splits = 64 (64 splits per
 * head, then the combine pass).  scale = 0 means 1/sqrt(128).
 * Limits: batch * n_q_heads <= 256 and n <= 2^30, else LVR_E_CAPACITY.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two
 * streams, two threads) race on it and must be ordered by the caller.  The array keeps the last
 * call's partials; none of it has to start at zero, since a call reads only what its own split
 * pass has just written. */
int lvr_sparse_attention_static(const void *K_dev, const void *V_dev, int64_t n, int32_t kv_dtype, int32_t batch,
                                int32_t n_q_heads, int32_t n_kv_heads, float scale, const float *q_dev,
                                const int32_t *idx_dev, const int32_t *count_dev, int64_t cap, float *out_dev,
                                void *stream);

/* lvr_query followed by lvr_sparse_attention on its result, in one call (Alg. 3 / Alg. 4 end to
 * end: retrieve, then attend).  Launches kernels only: no allocation, no host synchronisation,
 * no memset, so the call may be recorded while `stream` is under HIP graph capture; a recorded
 * step stays valid until the next lvr_build / lvr_append / lvr_publish on the index. */
int lvr_decode_step(lvr_index *ix, const float *q_dev, const float *tau_dev, float *out_dev,
                    int32_t *out_idx_dev, int32_t *out_count_dev, int64_t cap, void *stream);

/* lvr_append of m tokens followed by lvr_decode_step, as one call (Sec. 4.3 followed by Sec. 4.2:
 * the token generated by the previous step joins the cache, then the next query is answered).
 * Same results as the two calls.  When the append only has to store rows (no buffer chunk becomes
 * full, contiguous grouping, no reservoir) the store rides in the query launch, which saves a
 * launch per decode step; otherwise the two calls run one after the other. */
int lvr_append_decode_step(lvr_index *ix, const void *k_new_dev, const void *v_new_dev, int64_t m, const float *q_dev,
                           const float *tau_dev, float *out_dev, int32_t *out_idx_dev, int32_t *out_count_dev,
                           int64_t cap, void *stream);

/* Built-in threshold selection (appendix "Threshold Oracle Comparison"): tau per query head from
 * the dot products of q with the reservoir of past keys of its KV head.
 *   SAMPLE_MAX       largest reservoir score
 *   SAMPLE_MEAN_MAX  mean of the largest and the average reservoir score
 *   SAMPLE_GAP       cut at the largest gap between consecutive sorted scores: tau = the smallest
 *                    score above the gap
 *   SAMPLE_TOPK      param = k: the k-th largest reservoir score
 *   BUDGET           param = alpha in (0, 1]: the ceil(alpha * m)-th largest of the m reservoir
 *                    scores, i.e. the (1 - alpha) quantile
 * tau_out_dev [batch][n_q_heads] fp32.  With an empty reservoir tau is -INFINITY.  Needs
 * lvr_config.reservoir_size > 0 (LVR_E_STATE otherwise). */
enum lvr_threshold_mode {
    LVR_TAU_SAMPLE_MAX = 0, LVR_TAU_SAMPLE_MEAN_MAX = 1, LVR_TAU_SAMPLE_GAP = 2, LVR_TAU_SAMPLE_TOPK = 3,
    LVR_TAU_BUDGET = 4
};
int lvr_threshold(lvr_index *ix, const float *q_dev, int mode, float param, float *tau_out_dev, void *stream);

/* Synchronises the device and copies the reservoir (token positions, [batch][n_kv_heads][R],
 * unused slots -1) to host memory. */
int lvr_export_reservoir(lvr_index *ix, int32_t *positions_host);

/* Dense attention over all held keys (Sec. 2 "Attention"): the baseline the sparse path is
 * measured against, on the same arena. */
int lvr_dense_attention(lvr_index *ix, const float *q_dev, float *out_dev, void *stream);

/* Synchronises the device, then reports counters of the last query and clears the overflow
 * flag.  Returns LVR_E_OVERFLOW (with *out_host filled) if the flag was set. */
int lvr_get_stats(lvr_index *ix, lvr_stats *out_host);

/* Synchronises the device and copies the index to host memory for inspection (tests check the
 * enclosure invariant on it).  Any pointer may be NULL to skip that part.
 *   centres_host  [batch][n_kv_heads][n_groups][head_dim] of kv_dtype, in coordinate order whatever the
 *                 storage format: coded centres (FP8, FP6) are decoded, which is exact in bf16
 *                 (AABB: [batch][n_kv_heads][n_groups][2][head_dim], upper corner then lower corner)
 *   radii_host    [batch][n_kv_heads][n_groups][n_subspaces] fp32
 *                 (AABB: [batch][n_kv_heads][n_groups][1], the rounding allowance of the bound)
 *   slot_pos_host [batch][n_kv_heads][n] int32: token position stored in arena row `slot`
 *                 (group g owns rows g*r .. g*r+r-1; rows >= n_indexed are the buffer)
 *   keys_host     [batch][n_kv_heads][n][head_dim] of kv_dtype, arena row order */
int lvr_export_index(lvr_index *ix, void *centres_host, float *radii_host, int32_t *slot_pos_host,
                     void *keys_host);

/* The channel exponents e_c of a 6-bit index in a rescaled space (enum lvr_index_dtype, FP6):
 * exp_host [batch][n_kv_heads][head_dim] signed bytes; all zero where the index is not rescaled.
 * lvr_export_index returns the centres mapped back to the keys' own space (times 2^e_c) and the
 * radii as they are stored, i.e. measured in the rescaled space: ball s of group g encloses
 * pi_s(k_j / 2^e) within radii[g][s] of pi_s(centre_g / 2^e).  Synchronises the device. */
int lvr_export_channel_scales(lvr_index *ix, int8_t *exp_host);

/* Synchronises the device and copies the per-subspace group labels of a LVR_GROUP_SUBSPACE_TREE index to
 * host memory: labels_host [batch][n_kv_heads][n_subspaces][n_indexed] int32, the group of key j in
 * subspace s (Sec. 4.1: "n assignment labels" per subspace).  LVR_E_STATE for other groupings. */
int lvr_export_labels(lvr_index *ix, int32_t *labels_host);

/* Per-kernel GPU time, for measurement (App. "Kernel Implementation Details" names the stages).
 * While enabled, every kernel launch of every call gets a pair of HIP events (from a pool
 * allocated by lvr_profile_enable, so the hot-path calls still allocate nothing).  The fused
 * query kernel and the one-launch attention kernels carry their pair in the dispatch itself
 * (the events hold the kernel's own start and end, as a profiler's trace does); the other
 * kernels are bracketed by a pair recorded on the call's stream, which also measures the launch
 * latency (2-3 us).  When the pool of `max_launches` pairs is used up further
 * launches are simply not timed.  lvr_profile_read synchronises the device, adds up the
 * elapsed time of each pair by kernel, and empties the pool. */
typedef struct lvr_profile {
    double ms[9];      /* total milliseconds per kernel, indexed by lvr_kernel                */
    int64_t launches[9];
} lvr_profile;
enum lvr_kernel {
    LVR_KERNEL_COPY = 0, LVR_KERNEL_BUILD = 1, LVR_KERNEL_RESET = 2, LVR_KERNEL_PRUNE = 3,
    LVR_KERNEL_FILTER = 4, LVR_KERNEL_ATTN_PARTIAL = 5, LVR_KERNEL_ATTN_COMBINE = 6,
    LVR_KERNEL_DENSE_PARTIAL = 7, LVR_KERNEL_DENSE_COMBINE = 8
};
int lvr_profile_enable(lvr_index *ix, int max_launches); /* 0 turns timing off and frees the pool */
int lvr_profile_read(lvr_index *ix, lvr_profile *out_host);

/* Measurement aid: the exact filter without the index (Sec. 4.2: what the bound test of Eq. (2)
 * buys is the difference to this).  enabled = 0: lvr_query / lvr_decode_step /
 * lvr_append_decode_step skip the bound test and give every indexed key the exact dot product,
 * reading no centre and no radius; enabled = 1 (the state after lvr_create) restores the test.
 * Results are the same either way (Problem 1's set).  lvr_query1 ignores the setting.  bf16
 * caches in the fused launch form; LVR_E_UNSUPPORTED otherwise.  Takes effect from the next call. */
int lvr_set_bound_test(lvr_index *ix, int enabled);

/* Measurement aid: one launch of a kernel that only READS `bytes` bytes (rounded down to a
 * multiple of 16) from src_dev, 16 bytes per lane, eight consecutive KiB per wave in flight, and
 * writes nothing (sink_dev, 4 bytes of device memory, is there so that the loads cannot be
 * dropped).  workgroups = launch size (0 = 4096).  Timed by the caller, it gives the
 * streaming-read rate this GPU reaches in practice, the ceiling the HBM-bound kernels of
 * Sec. 4.2 are read against beside the published peak. */
int lvr_stream_read(const void *src_dev, int64_t bytes, uint32_t *sink_dev, int32_t workgroups, void *stream);

/* n = keys held per (sequence, KV head); n_indexed = keys inside groups. */
int lvr_length(const lvr_index *ix, int64_t *n_host, int64_t *n_indexed_host);

const char *lvr_strerror(int code);
/* hipError_t value of the most recent failing HIP call made by this library on this thread. */
int lvr_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* LOUVER_H_ */
