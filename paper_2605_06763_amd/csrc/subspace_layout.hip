// The index layout as the paper states it (Sec. 4.1 "Index Construction", Alg. 1): every coordinate
// block ("subspace") s has a grouping OF ITS OWN — Alg. 2 run on the block's coordinates — so a key
// belongs to S different groups, one per block, and carries S labels a_{s,j}.  Per block and group
// the index keeps the centre (mean of the members' block coordinates) and the radius (Eq. (1)).
//
// Storage: K and V stay in arrival order.  centres[g] is one 128-coordinate row whose block s holds
// the centre of block s's group g (the groups of different blocks share nothing but the number g);
// radii[g][s] likewise; labels[j][s] (16 bits) name key j's group in block s.
//
// Query (Sec. 4.2 "Query 2"): f_{s,g} = <pi_s q, c_{s,g}> + rho_{s,g} |pi_s q| for every block and
// group (subspace_bounds_kernel), then key j is a candidate iff  sum_s f_{s, a_{s,j}} >= tau
// (label_filter_kernel).  That sum bounds <q, k_j> from above because every term bounds the
// block's share of the product; a key outside the live set of Alg. 4's depth scan ranks below the
// stopping depth in every block, so its sum is below the stopping sum U(d) < tau: the rule keeps a
// subset of what the depth scan keeps, needs no sort, and loses no qualifying key.  Candidates
// then get the exact dot product (the last step of Alg. 4) in the same launch.
#include <type_traits>

#include "emitter.h"
#include "mfma_score.h"

namespace {

// ------------------------------------------------------------------------------------------------
// Build: balls of block s from that block's tree order
// ------------------------------------------------------------------------------------------------
// perm: sorted tree keys of lvr_tree_order (low pos_bits = position relative to row0); entries
// [g*r, (g+1)*r) are group g's members.  One quarter wave per group; a lane holds 8 coordinates of a
// row, the lanes of block s are li in [s*16/S, (s+1)*16/S).
__global__ void __launch_bounds__(256)
subspace_groups_kernel(const void *__restrict__ K, void *__restrict__ centres, float *__restrict__ radii,
                       uint16_t *__restrict__ labels, const uint64_t *__restrict__ perm, int64_t np, int pos_bits,
                       int64_t cap_rows, int64_t max_groups, int64_t row0, int64_t g_base, int64_t n_new_groups, int r,
                       int S, int s) {
    const int bh = blockIdx.y;
    const int li = threadIdx.x & 15;
    int64_t gl = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);   // group within this build
    const bool valid = gl < n_new_groups;
    if (!valid) gl = 0;   // keep every lane busy so the shuffles below see defined data
    const char *Kb = static_cast<const char *>(K) + (int64_t)bh * cap_rows * LVR_D * 2;
    const uint64_t *pp = perm + (int64_t)bh * np + gl * r;
    const uint64_t pos_mask = (1ull << pos_bits) - 1ull;
    const int lanes_per_sub = 16 / S;
    const bool mine = li / lanes_per_sub == s;   // this lane's coordinates belong to block s

    float c[8];
    lvr_zero8(c);
    for (int m = 0; m < r; ++m) {
        const int64_t row = row0 + (int64_t)(pp[m] & pos_mask);
        float x[8];
        lvr_load8<lvr_bf16_t>(Kb, row, li, x);
#pragma unroll
        for (int e = 0; e < 8; ++e) c[e] += x[e];
    }
    const float inv = 1.0f / (float)r;
    uint32_t b[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        b[e] = lvr_f32_to_bf16_bits(c[e] * inv);
        c[e] = __uint_as_float(b[e] << 16);   // from here on: the centre as stored
    }
    const int64_t g = g_base + gl;
    if (valid && mine)
        reinterpret_cast<uint4 *>(static_cast<char *>(centres) + ((int64_t)bh * max_groups + g) * LVR_D * 2)[li] =
            make_uint4(b[0] | (b[1] << 16), b[2] | (b[3] << 16), b[4] | (b[5] << 16), b[6] | (b[7] << 16));
    float cn2 = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) cn2 += c[e] * c[e];
    for (int off = 1; off < lanes_per_sub; off <<= 1) cn2 += __shfl_xor(cn2, off, 64);
    float max_d2 = 0.f;
    for (int m = 0; m < r; ++m) {
        const int64_t pos = (int64_t)(pp[m] & pos_mask);
        float x[8];
        lvr_load8<lvr_bf16_t>(Kb, row0 + pos, li, x);
        float d2 = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float t = x[e] - c[e];
            d2 += t * t;
        }
        for (int off = 1; off < lanes_per_sub; off <<= 1) d2 += __shfl_xor(d2, off, 64);
        max_d2 = fmaxf(max_d2, d2);
        if (valid && li == 0) labels[((int64_t)bh * cap_rows + row0 + pos) * S + s] = (uint16_t)g;
    }
    // the radius is measured against the centre as stored and widened so that no fp32 rounding of the
    // bound at query time can push it below a member's exact block product (same rule as the shared layout)
    float rho = sqrtf(max_d2) * (1.0f + 0x1p-12f) + sqrtf(cn2) * 0x1p-12f;
    rho = __uint_as_float(__float_as_uint(rho) + 1u);
    if (valid && mine && (li % lanes_per_sub) == 0) radii[((int64_t)bh * max_groups + g) * S + s] = rho;
}

// ------------------------------------------------------------------------------------------------
// Query, step 1: the table f[group][block][head] of Eq. (2)
// ------------------------------------------------------------------------------------------------
struct BoundsArgs {
    const void *centres;
    const float *radii;
    const float *q;
    float *f;   // [n_bh][max_groups][S][4]
    int64_t n_groups, max_groups;
    int n_q_heads, n_kv_heads, G, tiles_per_wave;
};

template <int S>
__global__ void __launch_bounds__(256)
subspace_bounds_kernel(const BoundsArgs a) {
    __shared__ uint4 s_bq[1][4][64];
    __shared__ float s_qn[4][16];
    const int bh = blockIdx.y;
    const int b = bh / a.n_kv_heads, kvh = bh % a.n_kv_heads;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 15, kq = lane >> 4;
    const int64_t hq0 = (int64_t)b * a.n_q_heads + kvh * a.G;
    if ((int)threadIdx.x < 64) {   // |pi_s q_h|, rounded up
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
        if ((li % lanes_per_sub) == 0) s_qn[h][li / lanes_per_sub] = sqrtf(ss) * (1.0f + 0x1p-20f);
    }
    lvr_bf16x8 bq[1][4];
    lvr_build_q_frags_wg<1>(a.q + hq0 * LVR_D, a.G, 1.0f, s_bq, bq);   // syncs
    const bool rep = n >= 8 && n < 12 && (n - 8) < a.G;
    const int h = n - 8;
    float qn[S];
#pragma unroll
    for (int s = 0; s < S; ++s) qn[s] = rep ? s_qn[h][s] : 0.f;
    const char *Cb = static_cast<const char *>(a.centres) + (int64_t)bh * a.max_groups * LVR_D * 2;
    const float *Rb = a.radii + (int64_t)bh * a.max_groups * S;
    float *Fb = a.f + (int64_t)bh * a.max_groups * S * 4;
    const int64_t n_tiles = (a.n_groups + 15) >> 4;
    const int64_t tile0 = ((int64_t)blockIdx.x * 4 + wave) * a.tiles_per_wave;
    for (int it = 0; it < a.tiles_per_wave && tile0 + it < n_tiles; ++it) {   // wave-uniform
        const int64_t g0 = (tile0 + it) * 16;
        int64_t g = g0 + n;
        if (g >= a.n_groups) g = a.n_groups - 1;
        uint4 ac[4];
        lvr_load_a_frags(Cb, g, ac);
        auto emit = [&](auto s_c, const lvr_f32x4 &sc) {
            constexpr int s = decltype(s_c)::value;
            if (n >= 8 && n < 12) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int64_t gj = g0 + 4 * kq + j;
                    if (gj < a.n_groups) Fb[(gj * S + s) * 4 + h] = rep ? sc[j] + Rb[gj * S + s] * qn[s] : 0.f;
                }
            }
        };
        if constexpr (S <= 4) {
            constexpr int KPS = 4 / S;   // 32-coordinate steps per block
            auto block = [&](auto s_c) {
                constexpr int s = decltype(s_c)::value;
                emit(s_c, lvr_score_tile_block<s * KPS, (s + 1) * KPS>(ac, bq[0]));
            };
            block(std::integral_constant<int, 0>{});
            if constexpr (S >= 2) block(std::integral_constant<int, 1>{});
            if constexpr (S >= 4) {
                block(std::integral_constant<int, 2>{});
                block(std::integral_constant<int, 3>{});
            }
        } else {
            // a block is a half (S = 8) or a quarter (S = 16) of a 32-coordinate step: the step is issued
            // once per block with the query operand masked to the block's lanes
            constexpr int BPS = S / 4, QPB = 4 / BPS;
            auto step = [&](auto kk_c) {
                constexpr int kk = decltype(kk_c)::value;
                auto sub = [&](auto t_c) {
                    constexpr int t = decltype(t_c)::value;
                    emit(std::integral_constant<int, kk * BPS + t>{},
                         lvr_score_tile_subblock<kk, t * QPB, (t + 1) * QPB>(ac, bq[0], kq));
                };
                sub(std::integral_constant<int, 0>{});
                sub(std::integral_constant<int, 1>{});
                if constexpr (BPS == 4) {
                    sub(std::integral_constant<int, 2>{});
                    sub(std::integral_constant<int, 3>{});
                }
            };
            step(std::integral_constant<int, 0>{});
            step(std::integral_constant<int, 1>{});
            step(std::integral_constant<int, 2>{});
            step(std::integral_constant<int, 3>{});
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Query, step 2: candidates by the labels' summed bounds, then the exact check
// ------------------------------------------------------------------------------------------------
constexpr int SEG_MAX_KEYS = 4096;

struct LabelArgs {
    const uint16_t *labels;   // [n_bh][cap_rows][S]
    const float *f;           // [n_bh][max_groups][S][4]
    const void *K;
    const float *q;
    const float *tau;
    int32_t *seg_count;       // candidates per segment, for statistics
    lvr_emit_target emit;
    int64_t max_groups, max_segs, cap_rows, n_indexed, n_total;
    int n_q_heads, n_kv_heads, G, buffer_dense, n_segs, seg_keys;
};

template <int S>
__global__ void __launch_bounds__(256)
label_filter_kernel(const LabelArgs a) {
    __shared__ union {
        uint4 bq[1][4][64];
        float qscore[4][1][4][LVR_QCAP];
    } s_u;
    static_assert(sizeof(s_u.bq) == sizeof(s_u.qscore), "aliasing assumes equal sizes");
    __shared__ int32_t s_queue[4][1][4][LVR_QCAP];
    __shared__ int32_t s_cand[4][SEG_MAX_KEYS / 4];   // candidate rows, one list per wave
    __shared__ int s_tot[4];
    const int bh = blockIdx.y;
    const int b = bh / a.n_kv_heads, kvh = bh % a.n_kv_heads;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 15, kq = lane >> 4;
    const int64_t hq0 = (int64_t)b * a.n_q_heads + kvh * a.G;
    const bool buffer_wg = (int)blockIdx.x >= a.n_segs;

    float tau4[4];
#pragma unroll
    for (int h = 0; h < 4; ++h) tau4[h] = h < a.G ? lvr_effective_tau(a.tau[hq0 + h]) : INFINITY;
    lvr_bf16x8 bq[1][4];
    lvr_build_q_frags_wg<1>(a.q + hq0 * LVR_D, a.G, 1.0f, s_u.bq, bq);   // syncs
    const bool rep = n >= 8 && n < 12 && (n - 8) < a.G;
    const float taue = rep ? tau4[(n - 8) & 3] : INFINITY;

    int64_t rows;            // rows this wave checks exactly
    int64_t row_base = 0;    // buffer workgroup: first row of the wave-interleaved run
    if (!buffer_wg) {
        const int64_t j0 = (int64_t)blockIdx.x * a.seg_keys;
        const uint16_t *Lb = a.labels + (int64_t)bh * a.cap_rows * S;
        const float4 *Fb = reinterpret_cast<const float4 *>(a.f) + (int64_t)bh * a.max_groups * S;
        int mine = 0;
        for (int it = 0; it < a.seg_keys; it += 256) {   // uniform
            const int64_t j = j0 + it + threadIdx.x;
            const bool in = j < a.n_indexed;
            const int64_t jc = in ? j : a.n_indexed - 1;
            uint16_t lab[S];
            if constexpr (S == 1) {
                lab[0] = Lb[jc];
            } else if constexpr (S == 2) {
                const uint32_t w = reinterpret_cast<const uint32_t *>(Lb)[jc];
                lab[0] = (uint16_t)w; lab[1] = (uint16_t)(w >> 16);
            } else if constexpr (S == 4) {
                const uint2 w = reinterpret_cast<const uint2 *>(Lb)[jc];
                lab[0] = (uint16_t)w.x; lab[1] = (uint16_t)(w.x >> 16); lab[2] = (uint16_t)w.y; lab[3] = (uint16_t)(w.y >> 16);
            } else {
#pragma unroll
                for (int v = 0; v < S / 8; ++v) {
                    const uint4 w = reinterpret_cast<const uint4 *>(Lb)[jc * (S / 8) + v];
                    const uint32_t ws[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        lab[8 * v + 2 * e] = (uint16_t)ws[e];
                        lab[8 * v + 2 * e + 1] = (uint16_t)(ws[e] >> 16);
                    }
                }
            }
            float4 fv[S];
#pragma unroll
            for (int s = 0; s < S; ++s) fv[s] = Fb[(int64_t)lab[s] * S + s];   // all S gathers in flight together
            float u0 = 0.f, u1 = 0.f, u2 = 0.f, u3 = 0.f;
#pragma unroll
            for (int s = 0; s < S; ++s) {
                u0 += fv[s].x; u1 += fv[s].y; u2 += fv[s].z; u3 += fv[s].w;
            }
            const bool alive = in && (u0 >= tau4[0] || u1 >= tau4[1] || u2 >= tau4[2] || u3 >= tau4[3]);
            const uint64_t m = __ballot(alive);
            if (alive) s_cand[wave][mine + __popcll(m & ((1ull << lane) - 1ull))] = (int32_t)j;
            mine += __popcll(m);
        }
        if (lane == 0) s_tot[wave] = mine;
        rows = mine;
    } else {
        // buffer rows (not yet in any group) are dealt to the waves in runs of 16
        rows = 0;
        row_base = a.n_indexed;
    }
    // every wave holds its operand pieces: the staging bytes become the score queues
    __syncthreads();
    if (!buffer_wg && threadIdx.x == 0)
        a.seg_count[(int64_t)bh * a.max_segs + blockIdx.x] = s_tot[0] + s_tot[1] + s_tot[2] + s_tot[3];

    lvr_emitter<4, true> em;
    em.q = s_queue[wave][0];
    em.qs = s_u.qscore[wave][0];
    em.count = 0;
    em.rep_base = 8;
    em.hq_base = hq0;
    const char *Kb = static_cast<const char *>(a.K) + (int64_t)bh * a.cap_rows * LVR_D * 2;
    const int64_t buf_rows = a.n_total - a.n_indexed;
    // candidate workgroup: tiles 0, 1, 2, ... of the wave's own list; buffer workgroup: tiles wave, wave+4, ... of the buffer
    const int64_t total = buffer_wg ? buf_rows : rows;
    const int64_t tiles = (total + 15) >> 4;
    const int64_t t_first = buffer_wg ? wave : 0, t_step = buffer_wg ? 4 : 1;
    for (int64_t t = t_first; t < tiles; t += 2 * t_step) {   // two tiles in flight
        int slot[2], nvalid[2];
        uint4 av[2][4];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int64_t tt = t + u * t_step;
            int64_t rowidx = tt * 16 + n;
            const int64_t left = total - tt * 16;
            nvalid[u] = tt >= tiles ? 0 : (left < 16 ? (int)left : 16);
            if (rowidx >= total) rowidx = 0;
            slot[u] = buffer_wg ? (int)(row_base + rowidx) : s_cand[wave][rowidx];
            if (total > 0) lvr_load_a_frags(Kb, slot[u], av[u]);
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            if (nvalid[u] == 0) continue;   // wave-uniform
            const lvr_f32x4 sc = lvr_score_tile(av[u], bq[0]);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int trow = 4 * kq + j;
                const bool pred = trow < nvalid[u] && rep && (sc[j] >= taue || (buffer_wg && a.buffer_dense));
                em.push(a.emit, lane, rep, pred, slot[u], trow, nullptr, sc[j]);
            }
        }
    }
    if (__ballot(em.count > 0)) em.flush(a.emit, lane, rep, nullptr);
}

}  // namespace

hipError_t lvr_launch_subspace_groups(lvr_index *ix, const lvr_tree_perm *perm, int s, int64_t row0, int64_t g_base,
                                      int64_t n_new_groups, hipStream_t st) {
    if (n_new_groups <= 0 || !perm->keys) return hipSuccess;
    dim3 grid((unsigned)((n_new_groups + 15) / 16), (unsigned)lvr_n_bh(ix));
    hipLaunchKernelGGL(subspace_groups_kernel, grid, dim3(256), 0, st, ix->K, ix->centres, ix->radii, ix->labels, perm->keys,
                       perm->np, perm->pos_bits, ix->cap_rows, ix->max_groups, row0, g_base, n_new_groups,
                       ix->cfg.group_size, ix->cfg.n_subspaces, s);
    return hipGetLastError();
}

hipError_t lvr_launch_subspace_bounds(lvr_index *ix, const float *q, hipStream_t st) {
    BoundsArgs a;
    a.centres = ix->centres;
    a.radii = ix->radii;
    a.q = q;
    a.f = ix->f_table;
    a.n_groups = ix->n_indexed / ix->cfg.group_size;
    a.max_groups = ix->max_groups;
    a.n_q_heads = ix->cfg.n_q_heads;
    a.n_kv_heads = ix->cfg.n_kv_heads;
    a.G = ix->G;
    if (a.n_groups <= 0) return hipSuccess;
    const int n_bh = lvr_n_bh(ix);
    const int64_t n_tiles = (a.n_groups + 15) / 16;
    int tpw = 1;
    while (tpw < 16 && n_tiles * n_bh / (4 * tpw) > 2048) tpw *= 2;
    a.tiles_per_wave = tpw;
    dim3 grid((unsigned)((n_tiles + 4 * tpw - 1) / (4 * tpw)), (unsigned)n_bh);
    switch (ix->cfg.n_subspaces) {
        case 1: hipLaunchKernelGGL(subspace_bounds_kernel<1>, grid, dim3(256), 0, st, a); break;
        case 2: hipLaunchKernelGGL(subspace_bounds_kernel<2>, grid, dim3(256), 0, st, a); break;
        case 4: hipLaunchKernelGGL(subspace_bounds_kernel<4>, grid, dim3(256), 0, st, a); break;
        case 8: hipLaunchKernelGGL(subspace_bounds_kernel<8>, grid, dim3(256), 0, st, a); break;
        default: hipLaunchKernelGGL(subspace_bounds_kernel<16>, grid, dim3(256), 0, st, a); break;
    }
    return hipGetLastError();
}

hipError_t lvr_launch_label_filter(lvr_index *ix, const float *q, const float *tau, int32_t *out_idx, int64_t cap,
                                   hipStream_t st) {
    LabelArgs a;
    a.labels = ix->labels;
    a.f = ix->f_table;
    a.K = ix->K;
    a.q = q;
    a.tau = tau;
    a.seg_count = lvr_seg_count(ix);
    a.emit.out_idx = out_idx;
    a.emit.head_count = lvr_head_count(ix);
    a.emit.overflow = lvr_overflow_flag(ix);
    a.emit.cap = cap;
    a.emit.out_score = ix->scores;
    a.emit.score_stride = ix->cap_rows;
    a.max_groups = ix->max_groups;
    a.max_segs = lvr_max_segs(ix->max_groups);
    a.cap_rows = ix->cap_rows;
    a.n_indexed = ix->n_indexed;
    a.n_total = ix->n_total;
    a.n_q_heads = ix->cfg.n_q_heads;
    a.n_kv_heads = ix->cfg.n_kv_heads;
    a.G = ix->G;
    a.buffer_dense = (ix->cfg.flags & LVR_ATTEND_BUFFER_DENSE) ? 1 : 0;
    const int n_bh = lvr_n_bh(ix);
    // segments of 256 .. 4096 keys, about 1024 workgroups per launch
    int seg = 256;
    while (seg < SEG_MAX_KEYS && ix->n_indexed * n_bh / seg > 1024) seg *= 2;
    // the per-segment counters were sized for segments of LVR_MIN_SEG_GROUPS groups
    while (seg < SEG_MAX_KEYS && (ix->n_indexed + seg - 1) / seg > a.max_segs) seg *= 2;
    a.seg_keys = seg;
    a.n_segs = (int)((ix->n_indexed + seg - 1) / seg);
    if (a.n_segs > a.max_segs) return hipErrorInvalidValue;
    const int has_buffer = a.n_total > ix->n_indexed ? 1 : 0;
    ix->seg_groups = seg;
    ix->n_segs = a.n_segs;
    if (a.n_segs + has_buffer == 0) return hipSuccess;
    dim3 grid((unsigned)(a.n_segs + has_buffer), (unsigned)n_bh);
    switch (ix->cfg.n_subspaces) {
        case 1: hipLaunchKernelGGL(label_filter_kernel<1>, grid, dim3(256), 0, st, a); break;
        case 2: hipLaunchKernelGGL(label_filter_kernel<2>, grid, dim3(256), 0, st, a); break;
        case 4: hipLaunchKernelGGL(label_filter_kernel<4>, grid, dim3(256), 0, st, a); break;
        case 8: hipLaunchKernelGGL(label_filter_kernel<8>, grid, dim3(256), 0, st, a); break;
        default: hipLaunchKernelGGL(label_filter_kernel<16>, grid, dim3(256), 0, st, a); break;
    }
    return hipGetLastError();
}
