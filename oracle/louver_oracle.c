/*
 * CPU oracle for the decode-time hot path: threshold range query over cached keys
 * followed by softmax attention restricted to the retrieved set.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, by-the-definition program used
 * to check the GPU library and to report a CPU baseline.  It shares no code with the
 * GPU library and the GPU library never calls it.
 *
 * What each function follows (paper sections):
 *   scores, range set      Problem 1 (Sec. 2): K* = { k : <q,k> >= tau }, raw dot product.
 *   attention on a set     Sec. 2 "Attention" / "Sparse Attention"; Alg. 3 and Alg. 4's last
 *                          step: ordinary softmax attention over the retrieved keys only,
 *                          logits scaled by sigma.
 *   ball index             Sec. 4.1 "Ball enclosing", Eq. (1): centre = mean of the group's
 *                          projected keys, radius = largest member distance.
 *   ball bound             Eq. (2) and Sec. 4.2 "Query 2": f = <pi_s q, c> + rho ||pi_s q||.
 *   box index / bound      appendix "Ablation on Index Design", Def. 1 with an axis-aligned
 *                          bounding box: per coordinate the smallest and largest member value;
 *                          the largest <q,x> over the box is sum_c max(q_c lo_c, q_c hi_c).
 *   Query 1                Sec. 4.2 "Query 1", Alg. 3: per-subspace thresholds, AND across subspaces.
 *   TA filter              Sec. 4.2 "Query 2", Alg. 4: sorted per-subspace bounds, depth scan.
 *   reservoir, thresholds  appendix "Threshold Oracle Comparison": a uniform reservoir of past
 *                          keys kept by reservoir sampling, and tau estimated from the query's
 *                          dot products with it (sample-max, sample-mean-max, sample-gap,
 *                          sample-topk(m), budget(alpha)).
 *   balanced tree          Sec. 4.1 "Grouping via balanced PCA trees", Alg. 2, with leaf ids
 *                          handed out by a running counter (the printed id formula collides
 *                          when a subtree yields more leaves than ceil(l/r)).
 *
 * Arithmetic: fp64 everywhere, except lvo_scores_f32, which is the "fp32 score" the
 * parity tolerance is phrased in: one fp32 accumulator, coordinates in ascending
 * order, multiply and add rounded separately (built with -ffp-contract=off).
 *
 * Key/value storage: either fp32 (kv_bf16 = 0) or bf16 bit patterns in uint16
 * (kv_bf16 = 1); bf16 is widened exactly (its 16 bits are the top half of an fp32).
 * GQA head mapping: query head h reads KV head h / (n_q_heads / n_kv_heads).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static inline float load_elem(const void *base, int kv_bf16, int64_t i) {
    if (kv_bf16) {
        uint32_t u = ((uint32_t)((const uint16_t *)base)[i]) << 16;
        float f;
        memcpy(&f, &u, 4);
        return f;
    }
    return ((const float *)base)[i];
}

int lvo_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void lvo_set_threads(int t) {
#ifdef _OPENMP
    if (t > 0) omp_set_num_threads(t);
#else
    (void)t;
#endif
}

/* ---------------------------------------------------------------- Problem 1: scores */

/* s[j] = sum_c q[c] * K[j][c] in fp64.  K is [n][d]. */
void lvo_scores_f64(const float *q, const void *K, int kv_bf16, int64_t n, int d, double *s) {
    for (int64_t j = 0; j < n; ++j) {
        double acc = 0.0;
        for (int c = 0; c < d; ++c) acc += (double)q[c] * (double)load_elem(K, kv_bf16, j * d + c);
        s[j] = acc;
    }
}

/* Same sum with a single fp32 accumulator, c ascending, no fused multiply-add. */
void lvo_scores_f32(const float *q, const void *K, int kv_bf16, int64_t n, int d, float *s) {
    for (int64_t j = 0; j < n; ++j) {
        float acc = 0.0f;
        for (int c = 0; c < d; ++c) {
            float p = q[c] * load_elem(K, kv_bf16, j * d + c);
            acc = acc + p;
        }
        s[j] = acc;
    }
}

/* I = { j : s_j >= tau } from fp32 scores, ascending j.  Returns |I|; writes at most cap
 * indices (the count is always the true size). */
int64_t lvo_range_query(const float *q, const void *K, int kv_bf16, int64_t n, int d, float tau,
                        int32_t *idx, int64_t cap) {
    float *s = (float *)malloc(sizeof(float) * (size_t)(n > 0 ? n : 1));
    lvo_scores_f32(q, K, kv_bf16, n, d, s);
    int64_t m = 0;
    for (int64_t j = 0; j < n; ++j) {
        if (s[j] >= tau) {
            if (m < cap) idx[m] = (int32_t)j;
            ++m;
        }
    }
    free(s);
    return m;
}

/* ---------------------------------------------------------------- attention on a set */

/* out[c] = sum_{j in idx} softmax_j(sigma <q,k_j>) v_j[c], normalised over idx only.
 * Empty idx gives zeros.  K, V are [n][d]; idx holds m row numbers. */
void lvo_attention_on_list(const float *q, const void *K, const void *V, int kv_bf16, int d,
                           const int32_t *idx, int64_t m, double sigma, float *out) {
    for (int c = 0; c < d; ++c) out[c] = 0.0f;
    if (m <= 0) return;
    double *logit = (double *)malloc(sizeof(double) * (size_t)m);
    double mx = -INFINITY;
    for (int64_t t = 0; t < m; ++t) {
        int64_t j = idx[t];
        double acc = 0.0;
        for (int c = 0; c < d; ++c) acc += (double)q[c] * (double)load_elem(K, kv_bf16, j * d + c);
        logit[t] = sigma * acc;
        if (logit[t] > mx) mx = logit[t];
    }
    double denom = 0.0;
    double *o = (double *)calloc((size_t)d, sizeof(double));
    for (int64_t t = 0; t < m; ++t) {
        double w = exp(logit[t] - mx);
        int64_t j = idx[t];
        denom += w;
        for (int c = 0; c < d; ++c) o[c] += w * (double)load_elem(V, kv_bf16, j * d + c);
    }
    for (int c = 0; c < d; ++c) out[c] = (float)(o[c] / denom);
    free(o);
    free(logit);
}

/* ---------------------------------------------------------------- one decode step, GQA layout */

/* K, V: [batch][n_kv_heads][n][d]; q: [batch][n_q_heads][d]; tau: [batch][n_q_heads].
 * idx: [batch][n_q_heads][cap] (ascending positions), count: [batch][n_q_heads] true sizes,
 * out: [batch][n_q_heads][d].  If extra_from >= 0 every position >= extra_from is retrieved
 * whatever its score (the "recent keys are always attended" behaviour of Sec. 4.3). */
void lvo_decode_step(const void *K, const void *V, int kv_bf16, int64_t batch, int n_q_heads,
                     int n_kv_heads, int64_t n, int d, const float *q, const float *tau,
                     double sigma, int64_t extra_from, int32_t *idx, int64_t cap, int64_t *count,
                     float *out) {
    int G = n_q_heads / n_kv_heads;
    int64_t units = batch * n_q_heads;
    size_t esz = kv_bf16 ? 2 : 4;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t u = 0; u < units; ++u) {
        int64_t b = u / n_q_heads;
        int h = (int)(u % n_q_heads);
        int g = h / G;
        const char *Kh = (const char *)K + (size_t)((b * n_kv_heads + g) * n * d) * esz;
        const char *Vh = (const char *)V + (size_t)((b * n_kv_heads + g) * n * d) * esz;
        const float *qh = q + u * d;
        float *s = (float *)malloc(sizeof(float) * (size_t)(n > 0 ? n : 1));
        int32_t *full = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
        lvo_scores_f32(qh, Kh, kv_bf16, n, d, s);
        int64_t m = 0;
        for (int64_t j = 0; j < n; ++j) {
            if (s[j] >= tau[u] || (extra_from >= 0 && j >= extra_from)) full[m++] = (int32_t)j;
        }
        count[u] = m;
        for (int64_t t = 0; t < m && t < cap; ++t) idx[u * cap + t] = full[t];
        lvo_attention_on_list(qh, Kh, Vh, kv_bf16, d, full, m, sigma, out + u * d);
        free(full);
        free(s);
    }
}

/* Full (dense) attention for every query head: the tau = -inf special case written out
 * on its own so that the dense GPU baseline has a direct counterpart. */
void lvo_dense_attention(const void *K, const void *V, int kv_bf16, int64_t batch, int n_q_heads,
                         int n_kv_heads, int64_t n, int d, const float *q, double sigma, float *out) {
    int G = n_q_heads / n_kv_heads;
    int64_t units = batch * n_q_heads;
    size_t esz = kv_bf16 ? 2 : 4;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t u = 0; u < units; ++u) {
        int64_t b = u / n_q_heads;
        int g = (int)(u % n_q_heads) / G;
        const char *Kh = (const char *)K + (size_t)((b * n_kv_heads + g) * n * d) * esz;
        const char *Vh = (const char *)V + (size_t)((b * n_kv_heads + g) * n * d) * esz;
        int32_t *all = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
        for (int64_t j = 0; j < n; ++j) all[j] = (int32_t)j;
        lvo_attention_on_list(q + u * d, Kh, Vh, kv_bf16, d, all, n, sigma, out + u * d);
        free(all);
    }
}

/* ---------------------------------------------------------------- Eq. (1): ball index */

/* Subspace s covers coordinates [lo, hi): contiguous blocks whose widths differ by at most
 * one (Alg. 1, first line). */
void lvo_subspace_range(int d, int S, int s, int *lo, int *hi) {
    int base = d / S, rem = d % S;
    *lo = s * base + (s < rem ? s : rem);
    *hi = *lo + base + (s < rem ? 1 : 0);
}

/* Given group labels label[j] in [0, n_groups) for the keys K [n][d]:
 * centre[i][c] = mean over members; radius[i][s] = max member distance inside subspace s,
 * both fp64.  A group with no member gets centre 0 and radius 0. */
void lvo_ball_index(const void *K, int kv_bf16, int64_t n, int d, int S, const int32_t *label,
                    int64_t n_groups, double *centre, double *radius) {
    int64_t *size = (int64_t *)calloc((size_t)(n_groups > 0 ? n_groups : 1), sizeof(int64_t));
    for (int64_t i = 0; i < n_groups * d; ++i) centre[i] = 0.0;
    for (int64_t i = 0; i < n_groups * S; ++i) radius[i] = 0.0;
    for (int64_t j = 0; j < n; ++j) {
        int64_t g = label[j];
        size[g] += 1;
        for (int c = 0; c < d; ++c) centre[g * d + c] += (double)load_elem(K, kv_bf16, j * d + c);
    }
    for (int64_t g = 0; g < n_groups; ++g)
        if (size[g] > 0)
            for (int c = 0; c < d; ++c) centre[g * d + c] /= (double)size[g];
    for (int64_t j = 0; j < n; ++j) {
        int64_t g = label[j];
        for (int s = 0; s < S; ++s) {
            int lo, hi;
            lvo_subspace_range(d, S, s, &lo, &hi);
            double acc = 0.0;
            for (int c = lo; c < hi; ++c) {
                double diff = (double)load_elem(K, kv_bf16, j * d + c) - centre[g * d + c];
                acc += diff * diff;
            }
            double dist = sqrt(acc);
            if (dist > radius[g * S + s]) radius[g * S + s] = dist;
        }
    }
    free(size);
}

/* Radii of the given (already stored, possibly rounded) centres: radius[i][s] = max member
 * distance to centre[i] inside subspace s.  Used to check an index whose centres are kept
 * in reduced precision: the enclosure has to hold for the centres as stored. */
void lvo_ball_radii_for_centres(const void *K, int kv_bf16, int64_t n, int d, int S,
                                const int32_t *label, int64_t n_groups, const double *centre,
                                double *radius) {
    for (int64_t i = 0; i < n_groups * S; ++i) radius[i] = 0.0;
    for (int64_t j = 0; j < n; ++j) {
        int64_t g = label[j];
        for (int s = 0; s < S; ++s) {
            int lo, hi;
            lvo_subspace_range(d, S, s, &lo, &hi);
            double acc = 0.0;
            for (int c = lo; c < hi; ++c) {
                double diff = (double)load_elem(K, kv_bf16, j * d + c) - centre[g * d + c];
                acc += diff * diff;
            }
            double dist = sqrt(acc);
            if (dist > radius[g * S + s]) radius[g * S + s] = dist;
        }
    }
}

/* Eq. (2): f[s][i] = <pi_s q, c_{s,i}> + rho_{s,i} ||pi_s q||_2, fp64.
 * centre is [n_groups][d] (subspace s uses its coordinate block), radius [n_groups][S];
 * f is [S][n_groups]. */
void lvo_ball_bounds(const float *q, int d, int S, const double *centre, const double *radius,
                     int64_t n_groups, double *f) {
    for (int s = 0; s < S; ++s) {
        int lo, hi;
        lvo_subspace_range(d, S, s, &lo, &hi);
        double qn = 0.0;
        for (int c = lo; c < hi; ++c) qn += (double)q[c] * (double)q[c];
        qn = sqrt(qn);
        for (int64_t i = 0; i < n_groups; ++i) {
            double dot = 0.0;
            for (int c = lo; c < hi; ++c) dot += (double)q[c] * centre[i * d + c];
            f[(int64_t)s * n_groups + i] = dot + radius[i * S + s] * qn;
        }
    }
}

/* ---------------------------------------------------------------- Def. 1 with boxes */

/* lo[i][c] / hi[i][c] = smallest / largest coordinate c over the members of group i.
 * A group with no member gets lo = +inf, hi = -inf. */
void lvo_aabb_index(const void *K, int kv_bf16, int64_t n, int d, const int32_t *label, int64_t n_groups,
                    double *lo, double *hi) {
    for (int64_t i = 0; i < n_groups * d; ++i) {
        lo[i] = INFINITY;
        hi[i] = -INFINITY;
    }
    for (int64_t j = 0; j < n; ++j) {
        int64_t g = label[j];
        for (int c = 0; c < d; ++c) {
            double x = (double)load_elem(K, kv_bf16, j * d + c);
            if (x < lo[g * d + c]) lo[g * d + c] = x;
            if (x > hi[g * d + c]) hi[g * d + c] = x;
        }
    }
}

/* ub[i] = max over the box [lo_i, hi_i] of <q, x> = sum_c max(q_c lo_ic, q_c hi_ic). */
void lvo_aabb_bounds(const float *q, int d, const double *lo, const double *hi, int64_t n_groups, double *ub) {
    for (int64_t i = 0; i < n_groups; ++i) {
        double acc = 0.0;
        for (int c = 0; c < d; ++c) {
            double a = (double)q[c] * lo[i * d + c], b = (double)q[c] * hi[i * d + c];
            acc += a > b ? a : b;
        }
        ub[i] = acc;
    }
}

/* ---------------------------------------------------------------- Alg. 3: Query 1 */

/* f: [S][n_groups] ball bounds, label: [S][n], tau_s: [S].  A key is a candidate iff in every
 * subspace the ball of its cluster reaches that subspace's threshold. */
void lvo_query1_filter(const double *f, const int32_t *label, int S, int64_t n_groups, int64_t n,
                       const double *tau_s, uint8_t *alive) {
    for (int64_t j = 0; j < n; ++j) {
        uint8_t a = 1;
        for (int s = 0; s < S; ++s)
            if (f[(int64_t)s * n_groups + label[(int64_t)s * n + j]] < tau_s[s]) a = 0;
        alive[j] = a;
    }
}

/* Per-subspace thresholds that are valid for EVERY key with <q,k> >= tau (Sec. 4.2: Query 1 is
 * correct when tau_s is a lower bound on the subspace term of every relevant key).  The dot
 * product is the sum of its subspace terms and the term of subspace t never exceeds the largest
 * ball bound M_t = max_i f[t][i], hence a key with <q,k> >= tau has term_s >= tau - sum_{t != s} M_t.
 * f: [S][n_groups]; no groups: nothing can be pruned, tau_s = -inf. */
void lvo_safe_subspace_thresholds(const double *f, int S, int64_t n_groups, double tau, double *tau_s) {
    for (int s = 0; s < S; ++s) {
        if (n_groups <= 0) {
            tau_s[s] = -INFINITY;
            continue;
        }
        double others = 0.0;
        for (int t = 0; t < S; ++t) {
            if (t == s) continue;
            double m = f[(int64_t)t * n_groups];
            for (int64_t i = 1; i < n_groups; ++i)
                if (f[(int64_t)t * n_groups + i] > m) m = f[(int64_t)t * n_groups + i];
            others += m;
        }
        tau_s[s] = tau - others;
    }
}

/* ---------------------------------------------------------------- Alg. 4: TA filter */

typedef struct {
    double f;
    int64_t i;
} lvo_pair;

static int cmp_desc(const void *a, const void *b) {
    const lvo_pair *x = (const lvo_pair *)a, *y = (const lvo_pair *)b;
    if (x->f > y->f) return -1;
    if (x->f < y->f) return 1;
    return (x->i > y->i) - (x->i < y->i); /* equal bounds: lower cluster id first */
}

/* f: [S][n_groups] bounds; label: [S][n] cluster of key j in subspace s.
 * Rounds d = 1, 2, ...: add the members of the d-th ranked cluster of every subspace to the
 * live set, then U = sum_s f[s][sigma_s(d)]; stop when U < tau or every cluster is visited.
 * alive[j] = 1 iff key j is in the live set.  Returns the stopping depth. */
int64_t lvo_ta_filter(const double *f, const int32_t *label, int S, int64_t n_groups, int64_t n,
                      double tau, uint8_t *alive) {
    lvo_pair *sorted = (lvo_pair *)malloc(sizeof(lvo_pair) * (size_t)(S * n_groups > 0 ? S * n_groups : 1));
    uint8_t *cl_alive = (uint8_t *)calloc((size_t)(S * n_groups > 0 ? S * n_groups : 1), 1);
    for (int s = 0; s < S; ++s) {
        for (int64_t i = 0; i < n_groups; ++i) {
            sorted[(int64_t)s * n_groups + i].f = f[(int64_t)s * n_groups + i];
            sorted[(int64_t)s * n_groups + i].i = i;
        }
        qsort(sorted + (int64_t)s * n_groups, (size_t)n_groups, sizeof(lvo_pair), cmp_desc);
    }
    int64_t depth = 0;
    while (depth < n_groups) {
        double U = 0.0;
        for (int s = 0; s < S; ++s) {
            lvo_pair p = sorted[(int64_t)s * n_groups + depth];
            cl_alive[(int64_t)s * n_groups + p.i] = 1;
            U += p.f;
        }
        ++depth;
        if (U < tau) break;
    }
    for (int64_t j = 0; j < n; ++j) {
        uint8_t a = 0;
        for (int s = 0; s < S; ++s) a |= cl_alive[(int64_t)s * n_groups + label[(int64_t)s * n + j]];
        alive[j] = a;
    }
    free(cl_alive);
    free(sorted);
    return depth;
}

/* ---------------------------------------------------------------- Alg. 2: balanced tree */

typedef struct {
    double key;
    int64_t j;
} lvo_sortrec;

static int cmp_asc(const void *a, const void *b) {
    const lvo_sortrec *x = (const lvo_sortrec *)a, *y = (const lvo_sortrec *)b;
    if (x->key < y->key) return -1;
    if (x->key > y->key) return 1;
    return (x->j > y->j) - (x->j < y->j); /* equal projections: lower key index first */
}

static void tree_rec(const void *K, int kv_bf16, int d, int lo, int hi, int r, int64_t *members,
                     int64_t m, int32_t *label, int64_t *next_id) {
    if (m <= r) {
        for (int64_t t = 0; t < m; ++t) label[members[t]] = (int32_t)(*next_id);
        *next_id += 1;
        return;
    }
    /* coordinate axis of largest variance among the subspace's axes (first wins a tie) */
    int best = lo;
    double best_var = -1.0;
    for (int c = lo; c < hi; ++c) {
        double mean = 0.0;
        for (int64_t t = 0; t < m; ++t) mean += (double)load_elem(K, kv_bf16, members[t] * d + c);
        mean /= (double)m;
        double var = 0.0;
        for (int64_t t = 0; t < m; ++t) {
            double diff = (double)load_elem(K, kv_bf16, members[t] * d + c) - mean;
            var += diff * diff;
        }
        var /= (double)m;
        if (var > best_var) {
            best_var = var;
            best = c;
        }
    }
    lvo_sortrec *rec = (lvo_sortrec *)malloc(sizeof(lvo_sortrec) * (size_t)m);
    for (int64_t t = 0; t < m; ++t) {
        rec[t].key = (double)load_elem(K, kv_bf16, members[t] * d + best);
        rec[t].j = members[t];
    }
    qsort(rec, (size_t)m, sizeof(lvo_sortrec), cmp_asc);
    for (int64_t t = 0; t < m; ++t) members[t] = rec[t].j;
    free(rec);
    int64_t left = m / 2;
    tree_rec(K, kv_bf16, d, lo, hi, r, members, left, label, next_id);
    tree_rec(K, kv_bf16, d, lo, hi, r, members + left, m - left, label, next_id);
}

/* Recursive median split of the keys K [n][d], looking only at coordinates [lo, hi), until a
 * node holds at most r keys.  label[j] = leaf id, ids numbered left to right from 0.
 * order[t] (may be NULL) = key index at position t of the left-to-right leaf sequence.
 * Returns the number of leaves. */
int64_t lvo_balanced_tree(const void *K, int kv_bf16, int64_t n, int d, int lo, int hi, int r,
                          int32_t *label, int64_t *order) {
    int64_t *members = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n > 0 ? n : 1));
    for (int64_t j = 0; j < n; ++j) members[j] = j;
    int64_t next_id = 0;
    if (n > 0) tree_rec(K, kv_bf16, d, lo, hi, r, members, n, label, &next_id);
    if (order)
        for (int64_t j = 0; j < n; ++j) order[j] = members[j];
    free(members);
    return next_id;
}

/* ---------------------------------------------------------------- threshold oracles */

/* Counter-based generator shared (as a published algorithm, re-implemented on each side) with
 * the GPU library: the splitmix64 finaliser of seed + stream * C1 + counter * C2, top 32 bits. */
uint32_t lvo_hash32(uint64_t seed, uint64_t stream, uint64_t counter) {
    uint64_t z = seed + stream * 0xD1B54A32D192ED03ull + counter * 0x9E3779B97F4A7C15ull;
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    z ^= z >> 31;
    return (uint32_t)(z >> 32);
}

/* Reservoir sampling over positions 0..n-1 in arrival order (classic algorithm R): the first R
 * positions fill the reservoir; position i >= R draws j uniform in [0, i] and replaces slot j if
 * j < R.  j = floor(hash32 * (i+1) / 2^32).  res[0..min(n,R)) holds positions. */
void lvo_reservoir(uint64_t seed, uint64_t stream, int64_t n, int R, int32_t *res) {
    for (int64_t i = 0; i < n; ++i) {
        if (i < R) {
            res[i] = (int32_t)i;
        } else {
            uint64_t j = ((uint64_t)lvo_hash32(seed, stream, (uint64_t)i) * (uint64_t)(i + 1)) >> 32;
            if (j < (uint64_t)R) res[j] = (int32_t)i;
        }
    }
}

static int cmp_float_desc(const void *a, const void *b) {
    float x = *(const float *)a, y = *(const float *)b;
    return (x < y) - (x > y);
}

/* tau from m reservoir scores.  mode: 0 sample-max, 1 sample-mean-max (mean of the maximum and
 * the mean score), 2 sample-gap (largest gap between consecutive sorted scores; tau is the
 * smaller score of the upper side, so everything above the gap qualifies), 3 sample-topk
 * (param = k: the k-th largest), 4 budget (param = alpha: the ceil(alpha * m)-th largest, the
 * (1 - alpha) quantile).  m = 0 gives -inf (nothing is known: retrieve everything). */
float lvo_threshold(const float *scores, int m, int mode, double param) {
    if (m <= 0) return -INFINITY;
    float *s = (float *)malloc(sizeof(float) * (size_t)m);
    memcpy(s, scores, sizeof(float) * (size_t)m);
    qsort(s, (size_t)m, sizeof(float), cmp_float_desc);
    float tau = s[0];
    if (mode == 1) {
        double mean = 0.0;
        for (int i = 0; i < m; ++i) mean += (double)s[i];
        mean /= (double)m;
        tau = (float)(0.5 * ((double)s[0] + mean));
    } else if (mode == 2) {
        int best = 0;
        float gap = -1.0f;
        for (int i = 0; i + 1 < m; ++i) {
            float g = s[i] - s[i + 1];
            if (g > gap) {
                gap = g;
                best = i;
            }
        }
        tau = s[best];
    } else if (mode == 3) {
        int k = (int)param;
        if (k < 1) k = 1;
        if (k > m) k = m;
        tau = s[k - 1];
    } else if (mode == 4) {
        int k = (int)ceil(param * (double)m);
        if (k < 1) k = 1;
        if (k > m) k = m;
        tau = s[k - 1];
    }
    free(s);
    return tau;
}
