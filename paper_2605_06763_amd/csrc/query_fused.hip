// Fused range-query kernel for bf16 caches: bound test and exact check in one launch.
//
// A workgroup owns a segment of consecutive groups of one (sequence, KV head):
//   phase A  (Sec. 4.2 "Query 2" bound, Eq. (2) per coordinate block, summed; or "Query 1":
//            Eq. (2) per coordinate block against that block's own threshold): every wave
//            scores its tiles of 16 centres on the matrix cores, adds the radius terms and
//            keeps a bit per group; the four waves compact the surviving group ids into LDS
//            (ballot + prefix sum, no global traffic).
//   phase B  (the exact dot-product check of Alg. 3 / Alg. 4): the waves walk the surviving
//            groups' key rows in tiles of 16 rows, two tiles in flight, score them for the G
//            heads of the KV head and queue the qualifying positions (emitter.h).
// One extra workgroup per (sequence, KV head) scans the not-yet-indexed buffer rows (Sec. 4.3).
//
// Compared with two launches this keeps the survivor list on chip, builds the query operand
// once per segment instead of twice, and removes one kernel tail from the step.
// The per-head counters must be zero when the kernel starts; the kernels that publish the
// counts (publish_counts_kernel, combine_kernel) clear them for the next query.
#include <type_traits>

#include <hip/hip_ext.h>

#include "emitter.h"
#include "mfma_score.h"

namespace {

constexpr int SEG_MAX_TILES = 64;                          // tiles per wave (at most 64: lane `it` of a wave keeps the mask of its tile `it`)
constexpr int SEG_MAX_GROUPS = 4 * SEG_MAX_TILES * 16;     // 4 waves x 64 tiles x 16 groups; the survivor list holds 16-bit offsets into the segment

struct FusedArgs {
    const void *centres;
    const float *radii;
    const void *K;
    const int32_t *slot_pos;
    const float *q;
    const float *tau;
    const float *tau_s;      // Query 1: [batch][H_q][S] per-block thresholds; NULL: Query 2
    const int8_t *chan_exp;  // per (sequence, KV head) LVR_CHAN_STRIDE bytes: channel exponents of a 6-bit index in a rescaled
                             // space (else all zero), then the factors 2^e_c as floats (else all 1)
    const void *k_new, *v_new;   // rows appended by this launch ([batch][H_kv][m_new][d]), or NULL
    void *V;
    int m_new;               // n_total already counts them
    int32_t *seg_count;      // survivors per segment, for statistics only
    lvr_emit_target emit;
    int64_t n_groups, max_groups, max_segs, cap_rows, n_indexed, n_total;
    int log2r, n_q_heads, n_kv_heads, G, buffer_dense, n_segs, tiles_per_wave;
    int skip_bounds;         // 1: no bound test, every group of the segment goes to the exact check
};

// UA = centre tiles per phase-A trip; ENC = 1: boxes instead of balls; Q1 = 1: per-block thresholds (S <= 4);
// CF = 1: centres (balls, S <= 4) or box corners stored as e4m3 codes; CF = 2: centres of balls (S <= 4) stored as
//     e2m3 codes with a power-of-two scale per lane piece (96 bytes per group, 12-byte records of radii and scales)
// W = heads per head block: 4 (three exact bf16 terms of four heads in the 16 operand columns; HB blocks) or
//     8 (two terms of eight heads fill the columns, the rarely non-zero third term has an operand of its own:
//     one pass per tile for up to eight heads; balls with one threshold per head, HB = 1)
// Four waves per SIMD (four workgroups per compute unit) are asked for wherever the kernel fits 128 registers: one
// head block of balls with at most four coordinate blocks, and the eight-head operand.  Left to itself the compiler
// has filled 128 vector registers and then needed four accumulator registers more, which costs a quarter of the waves.
// And no more than four: the launches aim at 1024 workgroups (four per compute unit) and larger batches run as whole
// rounds of 1024; a fifth resident workgroup makes the rounds uneven (1280 + 768 for 2048 workgroups: 1.2 % slower at
// 16 sequences of 32k keys).  The launcher sees to that with unused dynamic LDS (a fifth of a compute unit's LDS and a
// little more per workgroup) whenever a launch has more workgroups than fit at once; a launch that fits takes whatever
// residency the registers allow, which is where the few workgroups beyond 1024 (the buffer's) find room.
template <int HB, int S, int UA, int ENC, int Q1 = 0, int CF = 0, int W = 4>
__global__ void __launch_bounds__(256, ((HB == 1 && !ENC && S <= 4) || W == 8) ? 4 : 1)
query_fused_kernel(const FusedArgs a) {
    static_assert(!(Q1 && ENC) || S <= 4, "Query 1 on boxes: blocks of whole MFMA steps");
    static_assert(!CF || S <= 4, "coded centres: at most four coordinate blocks");
    static_assert(CF != 2 || !ENC, "6-bit codes: balls only");
    constexpr bool C6 = CF == 2;
    static_assert(W == 4 || (W == 8 && HB == 1 && !ENC && !Q1), "the eight-head operand serves balls with one threshold per head");
    // RP: the radii of 8-bit balls are stored as bf16 in the radius step's operand form; boxes keep one fp32 allowance per group
    constexpr bool RP = CF && !ENC;
    // the staging area of the query operand is dead once every wave holds its fragments; the score
    // queues of the emitters live in the same bytes afterwards
    __shared__ union {
        uint4 bq[HB][4][64];
        float qscore[4][HB][4][LVR_QCAP];
    } s_u;
    static_assert(sizeof(s_u.bq) == sizeof(s_u.qscore), "aliasing assumes equal sizes");
    // W = 8: main operand and the operand of the third terms (q itself).  With a rescaled 6-bit index (CS8) the bound
    // phase needs the same pair for q_c * 2^e_c: that pair lives in the bytes of the emission queues, which are idle
    // until the key-row phase (with both pairs held for good the workgroup's LDS goes past a quarter of a compute unit's).
    constexpr bool CS8 = CF == 2 && W == 8;
    __shared__ uint4 s_bq8[W == 8 ? 2 : 1][4][64];
    // BL: with eight heads per KV head the query operand (two head blocks, 32 registers) stays in LDS
    // and a lane fetches its pieces right before the matrix instructions that use them; that brings
    // the kernel back under the register budget of four waves per SIMD.  The staging area then keeps
    // its content, so the score queues get bytes of their own.
    constexpr bool BL = (HB == 2 && !Q1) || W == 8;
    __shared__ float s_qs2[BL ? 4 : 1][BL ? HB : 1][W][BL ? LVR_QCAP : 1];
    __shared__ uint4 s_bq2[ENC ? HB : 1][4][64];
    __shared__ __align__(16) float s_qn[HB * W][16];
    __shared__ float s_qpart[HB * 4][4];   // squared norm of q_h over the 32 coordinates of MFMA step kk (NQ only)
    // the emission queues belong to the key-row phase; until then their bytes keep the query operand of that phase
    // when the bound phase works with a rescaled one (see CS below)
    __shared__ union {
        int32_t queue[4][HB][W][LVR_QCAP];
        uint4 stash[HB][4][64];
        uint4 bq8s[CS8 ? 2 : 1][CS8 ? 4 : 1][CS8 ? 64 : 1];   // CS8: the bound phase's operands
    } s_qu;
    static_assert(!CS8 || sizeof(s_qu.bq8s) <= sizeof(s_qu.queue), "the rescaled operands fit the queues' bytes");
    auto &s_queue = s_qu.queue;
    __shared__ uint16_t s_list[SEG_MAX_GROUPS];   // surviving groups, as offsets from the segment's first group
    __shared__ int s_tot[4];
    __shared__ int s_wcnt[4][HB * W], s_wbase[HB * W];
    const int bh = blockIdx.y;
    // the wave's number is the same in all its lanes: said so, what depends on it alone is computed on the scalar unit
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 15, kq = lane >> 4;
    // first query head of this (sequence, KV head): (bh / H_kv) * H_q + (bh % H_kv) * G with H_q = H_kv * G
    const int64_t hq0 = (int64_t)bh * a.G;
    const bool buffer_wg = (int)blockIdx.x >= a.n_segs;

    // ---- phase A, first trip: the centre and radius loads do not depend on q, so they are put
    // in flight before the prologue builds the query operand ----
    constexpr int SP = (S <= 4) ? S : 1;      // radii are fetched ahead only when they are few
    // balls: one row per group (the centre); boxes: two rows per group (upper corner, lower corner)
    const char *Cb = static_cast<const char *>(a.centres) + (int64_t)bh * a.max_groups * (C6 ? LVR_D * 3 / 4 : LVR_D * (CF ? 1 : 2)) * (ENC ? 2 : 1);
    // boxes: one allowance per group, whatever S; 8-bit centres: 8 bytes of radii per group (four bf16); 6-bit centres:
    // 12 bytes (the radii, then the four scale bytes)
    constexpr int RW = C6 ? 3 : (RP ? 2 : (ENC ? 1 : S));   // 32-bit words per group in the radii array
    const float *Rb = a.radii + (int64_t)bh * a.max_groups * RW;
    const int64_t n_tiles = (a.n_groups + 15) >> 4;
    const int64_t tile0 = ((int64_t)blockIdx.x * 4 + wave) * a.tiles_per_wave;
    // RM: the radius term rides on the matrix cores as a fifth step (S <= 4, one threshold per head);
    // a lane then needs only its own row's radii.  Otherwise the lanes that hold the scores fetch
    // the radii of their four rows and add the terms on the vector ALU.
    constexpr bool RM = !Q1 && S <= 4;
    // operands of one trip (UA tiles of 16 groups) as they arrive from HBM
    struct Trip {
        uint4 av[C6 ? 1 : UA][CF ? 2 : 4], av2[ENC ? UA : 1][CF ? 2 : 4];
        lvr_codes6 c6[C6 ? UA : 1];
        uint32_t sc[C6 ? UA : 1];   // 6-bit centres: the exponent bytes of the row's four pieces
        float rad[RM ? 1 : UA][4][SP];
        float rrow[(RM && !RP) ? UA : 1][SP];
        uint2 rblk[(RM && RP) ? UA : 1];
    };
    // 8-bit centres leave room for two trips in registers: the next trip's loads are issued before
    // the current trip is scored, so the memory pipe does not drain between trips
    constexpr bool DB = CF && !Q1;
    Trip t0, t1;
    auto issueA = [&](Trip &T, int it) {
        auto &av = T.av; auto &av2 = T.av2; auto &rad = T.rad; auto &rrow = T.rrow; auto &rblk = T.rblk;
        auto &c6 = T.c6; auto &sc = T.sc;
        (void)av; (void)av2; (void)rad; (void)rrow; (void)rblk; (void)c6; (void)sc;
#pragma unroll
        for (int u = 0; u < UA; ++u) {
            const int64_t g0 = (tile0 + it + u) * 16;
            int64_t g = g0 + n;
            if (g >= a.n_groups) g = a.n_groups - 1;
            if (g < 0) g = 0;   // an empty index: the first trip is requested all the same (see below), from row 0
            if constexpr (C6) {
                lvr_load_a_codes6(Cb, g, c6[u]);
                sc[u] = reinterpret_cast<const uint32_t *>(Rb)[g * 3 + 2];
            } else if constexpr (ENC && CF) {
                lvr_load_a_codes(Cb, 2 * g, av[u]);
                lvr_load_a_codes(Cb, 2 * g + 1, av2[u]);
            } else if constexpr (ENC) {
                lvr_load_a_frags(Cb, 2 * g, av[u]);
                lvr_load_a_frags(Cb, 2 * g + 1, av2[u]);
            } else if constexpr (CF) {
                lvr_load_a_codes(Cb, g, av[u]);
            } else {
                lvr_load_a_frags(Cb, g, av[u]);
            }
            if constexpr (RM && RP) {
                if constexpr (C6) {
                    const uint32_t *rec = reinterpret_cast<const uint32_t *>(Rb) + g * 3;
                    rblk[u] = make_uint2(rec[0], rec[1]);
                } else rblk[u] = reinterpret_cast<const uint2 *>(Rb)[g];
            } else if constexpr (RM) {
                const float *rp = Rb + g * S;
                if constexpr (S == 4) {
                    const float4 r = *reinterpret_cast<const float4 *>(rp);
                    rrow[u][0] = r.x; rrow[u][1] = r.y; rrow[u][2] = r.z; rrow[u][3] = r.w;
                } else {
#pragma unroll
                    for (int s = 0; s < S; ++s) rrow[u][s] = rp[s];
                }
            } else if constexpr (S <= 4) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    int64_t gj = g0 + 4 * kq + j;
                    if (gj >= a.n_groups) gj = a.n_groups - 1;
                    if (gj < 0) gj = 0;
                    const float *rp = Rb + gj * (ENC ? 1 : S);
                    if constexpr (ENC) {   // the box's allowance; S only counts the blocks of Query 1
                        rad[u][j][0] = rp[0];
                    } else if constexpr (RP) {   // four bf16 per group: slot s = rho_s
                        const uint32_t *rec = reinterpret_cast<const uint32_t *>(Rb) + gj * RW;
                        const uint32_t w[2] = {rec[0], rec[1]};
#pragma unroll
                        for (int s = 0; s < S; ++s) rad[u][j][s] = __uint_as_float((w[s / 2] >> (16 * (s & 1))) << 16);
                    } else if constexpr (S == 4) {
                        const float4 r = *reinterpret_cast<const float4 *>(rp);
                        rad[u][j][0] = r.x; rad[u][j][1] = r.y; rad[u][j][2] = r.z; rad[u][j][3] = r.w;
                    } else {
#pragma unroll
                        for (int s = 0; s < S; ++s) rad[u][j][s] = rp[s];
                    }
                }
            }
        }
    };
    // Order of the first requests.  Vector memory loads return in order, so what the prologue needs (q for the
    // operand and the norms, the thresholds: a few KB that sit in the caches) is requested FIRST and the first
    // trip of centres right behind it: the prologue's arithmetic and its barrier then run while the centres
    // are still on their way, instead of waiting behind them.
    float qraw[W == 4 ? HB : 1][8];   // this lane's share of q for the operand pieces it builds
    float qnv[8];                     // and for the norms
    (void)qraw; (void)qnv;
    // CS: the 6-bit index describes the keys with coordinate c divided by 2^e_c (one exponent per channel of this
    // (sequence, KV head)); the bound phase therefore works with q_c * 2^e_c, which leaves every product <q,k> as it
    // was, and the key-row phase with q itself.  Both operands are built here; the second waits in LDS.
    // No branch on whether the exponents are all zero: a branch here would make the wait for q a wait for the first
    // trip's centres as well.
    constexpr bool CSP = CF == 2 && W == 4 && !ENC && sizeof(s_qu.stash) <= sizeof(s_qu.queue);
    float4 cfac[2];   // 2^e_c of this lane's eight coordinates
    (void)cfac;
    if constexpr (W == 4) {
#pragma unroll
        for (int hb = 0; hb < HB; ++hb) lvr_q_frag_load(a.q + hq0 * LVR_D, a.G, hb, wave, qraw[hb]);
        if constexpr (CSP) {
            const float4 *cf = reinterpret_cast<const float4 *>(a.chan_exp + (int64_t)bh * LVR_CHAN_STRIDE + LVR_D) + wave * 8 + kq * 2;
            cfac[0] = cf[0];
            cfac[1] = cf[1];
        }
    }
    // NQ: with at most four coordinate blocks every block is a whole number of MFMA steps, and wave kk has just asked
    // for the 32 coordinates of step kk of every head: the norms come out of those values, and q is read once per
    // workgroup instead of twice (a thousand workgroups ask for the same few lines at the same moment; measured
    // with per-workgroup timestamps, the operand was ready 1.7 to 4.9 us after entry)
    constexpr bool NQ = W == 4 && S <= 4;
    const bool norm_thread = !NQ && !buffer_wg && (int)threadIdx.x < HB * W * 16 && (int)(threadIdx.x >> 4) < a.G;
    if constexpr (!NQ) {
        const float *qh = a.q + (hq0 + (norm_thread ? (threadIdx.x >> 4) : 0)) * LVR_D + (threadIdx.x & 15) * 8;
        const float4 x = *reinterpret_cast<const float4 *>(qh), y = *reinterpret_cast<const float4 *>(qh + 4);
        qnv[0] = x.x; qnv[1] = x.y; qnv[2] = x.z; qnv[3] = x.w;
        qnv[4] = y.x; qnv[5] = y.y; qnv[6] = y.z; qnv[7] = y.w;
        if constexpr (CS8) {   // the norms that meet the radii are those of the rescaled query
            const float4 *cf = reinterpret_cast<const float4 *>(a.chan_exp + (int64_t)bh * LVR_CHAN_STRIDE + LVR_D) + (threadIdx.x & 15) * 2;
            const float4 f0 = cf[0], f1 = cf[1];
            qnv[0] *= f0.x; qnv[1] *= f0.y; qnv[2] *= f0.z; qnv[3] *= f0.w;
            qnv[4] *= f1.x; qnv[5] *= f1.y; qnv[6] *= f1.z; qnv[7] *= f1.w;
        }
    }
    float tau_raw[HB];
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) {
        const int h = hb * W + n - 8;
        const bool mine = n >= 8 && n < 8 + W && h < a.G;
        const float tv = a.tau[hq0 + (mine ? h : 0)];
        tau_raw[hb] = mine ? tv : INFINITY;
    }
    __builtin_amdgcn_sched_barrier(0);
    // Every wave requests a first trip, also one that has no tile to test (its rows are clamped into the arena and
    // never looked at), and every lane a threshold: with no branch around any of these loads the compiler can count
    // them, and the prologue waits for q alone instead of for everything in flight.
    issueA(t0, 0);
    __builtin_amdgcn_sched_barrier(0);

    // ---- prologue: subspace norms of q (phase A only) and the B operand of q ----
    if constexpr (CSP) {
        lvr_stash_q_frags<HB>(qraw, a.G, 1.0f, s_qu.stash);   // q itself, for the key-row phase
        const float f[8] = {cfac[0].x, cfac[0].y, cfac[0].z, cfac[0].w, cfac[1].x, cfac[1].y, cfac[1].z, cfac[1].w};
#pragma unroll
        for (int e = 0; e < 8; ++e)
#pragma unroll
            for (int hb = 0; hb < HB; ++hb) qraw[hb][e] *= f[e];
    }
    if constexpr (NQ) {
        // the lanes that build the leading terms (columns 0..3) hold q itself: 8 values per lane, 32 per head over
        // the four lane quarters
#pragma unroll
        for (int hb = 0; hb < HB; ++hb) {
            float ss = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) ss += qraw[hb][e] * qraw[hb][e];
            ss += __shfl_xor(ss, 16, 64);
            ss += __shfl_xor(ss, 32, 64);
            if (lane < 4 && hb * 4 + lane < a.G) s_qpart[hb * 4 + lane][wave] = ss;
        }
    } else if (!buffer_wg && (int)threadIdx.x < HB * W * 16) {
        const int h = threadIdx.x >> 4, li = threadIdx.x & 15;
        float ss = 0.f;
        if (h < a.G) {
#pragma unroll
            for (int e = 0; e < 8; ++e) ss += qnv[e] * qnv[e];
        }
        constexpr int lanes_per_sub = 16 / S;
#pragma unroll
        for (int off = 1; off < lanes_per_sub; off <<= 1) ss += __shfl_xor(ss, off, 64);
        if ((li % lanes_per_sub) == 0) s_qn[h][li / lanes_per_sub] = sqrtf(ss) * (1.0f + 0x1p-20f);   // rounded up
    }
    // B operands: q itself for balls; for boxes its positive part (meets the upper corners) and its
    // negative part (meets the lower corners); q = q+ + q- serves the exact check of phase B
    lvr_bf16x8 bq[HB][4], bq2[ENC ? HB : 1][4];
    bool third = false;   // W = 8: some head's query has more than 16 significant bits (the same in every thread)
    if constexpr (CS8) {   // both sync; a third term is there for q exactly when it is there for q times powers of two
        lvr_build_q_frags8_wg(a.q + hq0 * LVR_D, a.G, 1.0f, s_bq8);
        third = lvr_build_q_frags8_wg(a.q + hq0 * LVR_D, a.G, 1.0f, s_qu.bq8s, 0,
                                      reinterpret_cast<const float *>(a.chan_exp + (int64_t)bh * LVR_CHAN_STRIDE + LVR_D));
    } else if constexpr (W == 8) third = lvr_build_q_frags8_wg(a.q + hq0 * LVR_D, a.G, 1.0f, s_bq8);   // syncs
    else lvr_exchange_q_frags_wg<HB>(qraw, a.G, 1.0f, s_u.bq, bq, ENC ? 1 : 0);   // syncs
    if constexpr (ENC) lvr_exchange_q_frags_wg<HB>(qraw, a.G, 1.0f, s_bq2, bq2, -1);
    if constexpr (NQ) {
        // after the barrier of the exchange: every wave forms the block norms it is about to read and stores them
        // (four waves store the same values; a wave's own stores precede its own loads)
        if (lane < HB * 4 * S && lane / S < a.G) {
            const int h = lane / S, sb = lane % S;
            constexpr int SPB = 4 / S;   // steps per block
            float ss = 0.f;
#pragma unroll
            for (int k = 0; k < SPB; ++k) ss += s_qpart[h][sb * SPB + k];
            // rounded up: the hardware's square root is good to an ulp, and where the sum of squares left the normal
            // range (a norm below 2^-62) the constant alone is an upper bound
            s_qn[h][sb] = __builtin_amdgcn_sqrtf(ss) * (1.0f + 0x1p-20f) + 0x1p-62f;
        }
        __builtin_amdgcn_wave_barrier();
    }
    // BL: the pieces of head block hb, fetched anew at every use (the index register comes out of an
    // opaque instruction so that the loads are not hoisted out of the loops and kept in registers)
    auto fetch_bq = [&](int hb, lvr_bf16x8 (&b)[4]) {
        int z;
        asm volatile("v_mov_b32 %0, 0" : "=v"(z));
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) b[kk] = __builtin_bit_cast(lvr_bf16x8, s_u.bq[hb][kk][lane + z]);
    };
    auto fetch_bq2 = [&](int hb, lvr_bf16x8 (&b)[4]) {   // boxes: the negative part of q
        int z;
        asm volatile("v_mov_b32 %0, 0" : "=v"(z));
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) b[kk] = __builtin_bit_cast(lvr_bf16x8, s_bq2[ENC ? hb : 0][kk][lane + z]);
    };
    auto fetch_bq8 = [&](int which, lvr_bf16x8 (&b)[4]) {   // W = 8: 0 the main operand, 1 the third terms
        int z;
        asm volatile("v_mov_b32 %0, 0" : "=v"(z));
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) b[kk] = __builtin_bit_cast(lvr_bf16x8, s_bq8[W == 8 ? which : 0][kk][lane + z]);
    };
    (void)fetch_bq;
    (void)fetch_bq2;
    auto fetch_bq8s = [&](int which, lvr_bf16x8 (&b)[4]) {   // the bound phase's operands (CS8: the rescaled ones)
        if constexpr (CS8) {
            int z;
            asm volatile("v_mov_b32 %0, 0" : "=v"(z));
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) b[kk] = __builtin_bit_cast(lvr_bf16x8, s_qu.bq8s[which][kk][lane + z]);
        } else fetch_bq8(which, b);
    };
    (void)fetch_bq8;
    (void)fetch_bq8s;
    (void)third;
    lvr_bf16x8 rbq[RM ? HB : 1];
    if constexpr (RM) {
        if (!buffer_wg) {
#pragma unroll
            for (int hb = 0; hb < HB; ++hb) {
                if constexpr (W == 8) rbq[hb] = lvr_radius_b_frag8<S, RP ? 1 : 3>(s_qn, a.G);
                else rbq[hb] = lvr_radius_b_frag<S, RP ? 1 : 3>(s_qn, a.G, hb);
            }
        }
    }
    float taue[HB];
    bool rep[HB];
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) {
        const int h = hb * W + n - 8;
        rep[hb] = n >= 8 && n < 8 + W && h < a.G;
        taue[hb] = rep[hb] ? lvr_effective_tau(tau_raw[hb]) : INFINITY;
    }
    float taus[HB][Q1 ? S : 1];
    if constexpr (Q1) {
#pragma unroll
        for (int hb = 0; hb < HB; ++hb)
#pragma unroll
            for (int s = 0; s < S; ++s)
                taus[hb][s] = rep[hb] ? lvr_effective_tau(a.tau_s[(hq0 + hb * 4 + n - 8) * S + s]) : INFINITY;
    }

    // Fair shares of a SIMD.  Its four resident waves belong to four workgroups, and at equal priority the
    // arbiter serves the OLDEST first: measured with per-workgroup timestamps, the workgroups dispatched first
    // finished the bound loop in 9.2 us and those dispatched last in 12.7 us (with the priorities set the other way
    // round the order flips), so the launch waited for the youngest quarter.  Every wave therefore changes its
    // priority with every pair of trips (bound phase) or of row tiles (key-row phase), starting from its workgroup's place in the dispatch order
    // (workgroups 256 apart share a compute unit): each of the four is on top a quarter of the time.
    const int prio_phase = (int)((blockIdx.y * gridDim.x + blockIdx.x) >> 8);
    auto take_turn = [&](int turn) {
        switch ((prio_phase + turn) & 3) {
            case 0: __builtin_amdgcn_s_setprio(0); break;
            case 1: __builtin_amdgcn_s_setprio(1); break;
            case 2: __builtin_amdgcn_s_setprio(2); break;
            default: __builtin_amdgcn_s_setprio(3); break;
        }
    };

    int64_t rows;          // key rows phase B has to check
    int64_t buf_row0 = 0;
    const bool direct = buffer_wg || a.skip_bounds;   // phase B walks a run of consecutive rows, not a survivor list
    if (!buffer_wg && a.skip_bounds) {
        // the exact filter alone: the segment's groups all count as survivors
        const int64_t seg_groups = (int64_t)a.tiles_per_wave * 64;
        const int64_t g0 = (int64_t)blockIdx.x * seg_groups;
        int64_t total = a.n_groups - g0;
        if (total > seg_groups) total = seg_groups;
        if (total < 0) total = 0;
        if (threadIdx.x == 0) a.seg_count[(int64_t)bh * a.max_segs + blockIdx.x] = (int32_t)total;
        rows = total << a.log2r;
        buf_row0 = g0 << a.log2r;
        if constexpr (CSP) lvr_fetch_q_frags<HB>(s_qu.stash, bq);   // the key-row phase scores with q itself
        __syncthreads();   // no wave still reads the operand staging area that the score queues reuse
    } else if (!buffer_wg) {
        // ---------------- phase A: bound test over this segment's centres ----------------
        float qn[HB][S];
#pragma unroll
        for (int hb = 0; hb < HB; ++hb)
#pragma unroll
            for (int s = 0; s < S; ++s) qn[hb][s] = rep[hb] ? s_qn[hb * W + n - 8][s] : 0.f;
        uint32_t mybits = 0;   // lane `it` keeps the 16-bit survivor mask of the wave's tile `it`
        auto scoreA = [&](Trip &T, int it) {
            auto &av = T.av; auto &av2 = T.av2; auto &rad = T.rad; auto &rrow = T.rrow; auto &rblk = T.rblk;
            auto &c6 = T.c6; auto &sc = T.sc;
            (void)av; (void)av2; (void)rad; (void)rrow; (void)rblk; (void)c6; (void)sc;
#pragma unroll
            for (int u = 0; u < UA; ++u) {
                const int64_t g_row = (tile0 + it + u) * 16;
                uint32_t alive4 = 0;
                uint4 ac[4];   // the tile's operand pieces (decoded from the 8-bit codes if that is how they are stored)
                uint4 ac2[ENC ? 4 : 1];   // boxes: the lower corners
                (void)ac2;
                if constexpr (C6) {
                    lvr_codes6_to_a_frags(c6[u], sc[u], ac);
                } else if constexpr (CF) {
                    lvr_codes_to_a_frags(av[u], ac);
                    if constexpr (ENC) lvr_codes_to_a_frags(av2[u], ac2);
                } else {
#pragma unroll
                    for (int kk = 0; kk < 4; ++kk) {
                        ac[kk] = av[u][kk];
                        if constexpr (ENC) ac2[kk] = av2[u][kk];
                    }
                }
#pragma unroll
                for (int hb = 0; hb < HB; ++hb) {
                    if constexpr (Q1) {
                        // a group survives for a head iff every block's bound reaches that block's threshold
                        bool okb[4] = {true, true, true, true};
                        if constexpr (S <= 4) {
                            float qnw = 0.f;   // boxes: the allowance multiplies the norm of the whole query
                            if constexpr (ENC) {
#pragma unroll
                                for (int s = 0; s < S; ++s) qnw += qn[hb][s] * qn[hb][s];
                                qnw = sqrtf(qnw) * (1.0f + 0x1p-20f);
                            }
                            auto block = [&](auto s_c) {
                                constexpr int s = decltype(s_c)::value;
                                constexpr int KPS = 4 / S;
                                lvr_f32x4 sc;
                                if constexpr (ENC) sc = lvr_score_tile_block2<s * KPS, (s + 1) * KPS>(ac, bq[hb], ac2, bq2[hb]);
                                else sc = lvr_score_tile_block<s * KPS, (s + 1) * KPS>(ac, bq[hb]);
#pragma unroll
                                for (int j = 0; j < 4; ++j) {
                                    const float slack = ENC ? rad[u][j][0] * qnw : rad[u][j][s] * qn[hb][s];
                                    okb[j] = okb[j] && (sc[j] + slack >= taus[hb][s]);
                                }
                            };
                            block(std::integral_constant<int, 0>{});
                            if constexpr (S >= 2) block(std::integral_constant<int, 1>{});
                            if constexpr (S >= 4) {
                                block(std::integral_constant<int, 2>{});
                                block(std::integral_constant<int, 3>{});
                            }
                        } else {
                            // a block is a half (S = 8) or a quarter (S = 16) of a 32-coordinate step: the step is
                            // issued once per block with the query operand masked to the block's lanes
                            constexpr int BPS = S / 4;      // blocks per step
                            constexpr int QPB = 4 / BPS;    // operand quarters per block
                            const float *rp[4];
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                int64_t gj = g_row + 4 * kq + j;
                                if (gj >= a.n_groups) gj = a.n_groups - 1;
                                rp[j] = Rb + gj * S;
                            }
                            auto step = [&](auto kk_c) {
                                constexpr int kk = decltype(kk_c)::value;
                                float4 r4[4][BPS / 4 ? BPS / 4 : 1];
                                float r2[4][2];
                                (void)r4; (void)r2;
#pragma unroll
                                for (int j = 0; j < 4; ++j) {
                                    if constexpr (BPS == 4) r4[j][0] = *reinterpret_cast<const float4 *>(rp[j] + kk * 4);
                                    else { const float2 t2 = *reinterpret_cast<const float2 *>(rp[j] + kk * 2); r2[j][0] = t2.x; r2[j][1] = t2.y; }
                                }
                                auto sub = [&](auto t_c) {
                                    constexpr int t = decltype(t_c)::value;
                                    constexpr int s = kk * BPS + t;
                                    const lvr_f32x4 sc = lvr_score_tile_subblock<kk, t * QPB, (t + 1) * QPB>(ac, bq[hb], kq);
#pragma unroll
                                    for (int j = 0; j < 4; ++j) {
                                        float rho;
                                        if constexpr (BPS == 4) rho = t == 0 ? r4[j][0].x : (t == 1 ? r4[j][0].y : (t == 2 ? r4[j][0].z : r4[j][0].w));
                                        else rho = r2[j][t];
                                        okb[j] = okb[j] && (sc[j] + rho * qn[hb][s] >= taus[hb][s]);
                                    }
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
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            alive4 |= okb[j] ? (1u << j) : 0u;   // lanes that report no head compare against +inf
                        }
                        continue;
                    }
                    lvr_f32x4 sc;
                    if constexpr (RM) {
                        lvr_bf16x8 ra;
                        if constexpr (RP) ra = lvr_radius_a_stored(rblk[u]);
                        else ra = lvr_radius_a_frag<S>(rrow[u]);
                        if constexpr (ENC && BL) {
                            lvr_bf16x8 b[4], b2[4];
                            fetch_bq(hb, b);
                            fetch_bq2(hb, b2);
                            sc = lvr_bound_tile2(ac, b, ac2, b2, ra, rbq[hb]);
                        } else if constexpr (ENC) sc = lvr_bound_tile2(ac, bq[hb], ac2, bq2[hb], ra, rbq[hb]);
                        else if constexpr (W == 8) {
                            lvr_bf16x8 b[4], b3[4];
                            fetch_bq8s(0, b);
                            if (third) fetch_bq8s(1, b3);
                            sc = lvr_bound_tile8(ac, b, b3, third, ra, rbq[hb]);
                        } else if constexpr (BL) {
                            lvr_bf16x8 b[4];
                            fetch_bq(hb, b);
                            sc = lvr_bound_tile(ac, b, ra, rbq[hb]);
                        } else sc = lvr_bound_tile(ac, bq[hb], ra, rbq[hb]);
                    } else {
                        if constexpr (ENC && BL) {
                            lvr_bf16x8 b[4], b2[4];
                            fetch_bq(hb, b);
                            fetch_bq2(hb, b2);
                            sc = lvr_score_tile2(ac, b, ac2, b2);
                        } else if constexpr (ENC) sc = lvr_score_tile2(ac, bq[hb], ac2, bq2[hb]);
                        else if constexpr (W == 8) {
                            lvr_bf16x8 b[4], b3[4];
                            fetch_bq8s(0, b);
                            if (third) fetch_bq8s(1, b3);
                            sc = lvr_score_tile8(ac, b, b3, third);
                        } else if constexpr (BL) {
                            lvr_bf16x8 b[4];
                            fetch_bq(hb, b);
                            sc = lvr_score_tile(ac, b);
                        } else sc = lvr_score_tile(ac, bq[hb]);
                    }
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        float ub = sc[j];
                        if constexpr (RM) {
                            // the radius terms are already in the sum
                        } else if constexpr (S <= 4) {
#pragma unroll
                            for (int s = 0; s < S; ++s) ub += rad[u][j][s] * qn[hb][s];
                        } else {
                            int64_t gj = g_row + 4 * kq + j;
                            if (gj >= a.n_groups) gj = a.n_groups - 1;
                            const float4 *rp = reinterpret_cast<const float4 *>(Rb + gj * S);
#pragma unroll
                            for (int s4 = 0; s4 < S / 4; ++s4) {
                                const float4 r = rp[s4];
                                ub += r.x * qn[hb][4 * s4] + r.y * qn[hb][4 * s4 + 1] + r.z * qn[hb][4 * s4 + 2] +
                                      r.w * qn[hb][4 * s4 + 3];
                            }
                        }
                        alive4 |= (ub >= taue[hb]) ? (1u << j) : 0u;   // lanes that report no head compare against +inf
                    }
                }
                // "some head keeps the group": OR over the four lanes of a quarter that hold the heads' bits
                // (lanes 8..11 of each row of 16; the other lanes hold zero), then the four quarters' nibbles
                // are read off lane 11 of each row into one 16-bit mask (bit 4*kq + j = group 4*kq + j of the tile)
                uint32_t v = alive4;
                v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, true);   // row_shr:1
                v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, true);   // row_shr:2
                if constexpr (W == 8) v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, true);   // row_shr:4
                constexpr int L0 = 7 + W;   // last lane of a row that holds a head's bits: 11 (four heads) or 15 (eight)
                const uint32_t mask16 = (uint32_t)__builtin_amdgcn_readlane((int)v, L0) |
                                        ((uint32_t)__builtin_amdgcn_readlane((int)v, L0 + 16) << 4) |
                                        ((uint32_t)__builtin_amdgcn_readlane((int)v, L0 + 32) << 8) |
                                        ((uint32_t)__builtin_amdgcn_readlane((int)v, L0 + 48) << 12);
                // groups past the end of the index, tiles past the wave's share: a wave-uniform mask
                const int64_t left = a.n_groups - g_row;
                const uint32_t valid16 = (it + u) >= a.tiles_per_wave || left <= 0 ? 0u
                                         : (left >= 16 ? 0xffffu : ((1u << (int)left) - 1u));
                if (lane == it + u) mybits = mask16 & valid16;
            }
        };
        auto more = [&](int it) { return it < a.tiles_per_wave && tile0 + it < n_tiles; };   // wave-uniform
        if constexpr (DB) {
            for (int it = 0; more(it); it += 2 * UA) {
                take_turn(it / (2 * UA));
                const bool m1 = more(it + UA);
                if (m1) issueA(t1, it + UA);
                scoreA(t0, it);
                if (!m1) break;
                const bool m2 = more(it + 2 * UA);
                if (m2) issueA(t0, it + 2 * UA);
                scoreA(t1, it + UA);
                if (!m2) break;
            }
        } else {
            for (int it = 0; more(it); it += UA) {
                if (it > 0) issueA(t0, it);
                scoreA(t0, it);
            }
        }
        if constexpr (DB) __builtin_amdgcn_s_setprio(0);
        // compaction of the four waves' masks into the LDS list
        const int cnt = __popc(mybits);
        const int incl = lvr_wave_inclusive_sum(cnt);
        if (lane == 63) s_tot[wave] = incl;
        __syncthreads();
        if constexpr (CSP) {
            // every wave takes the key-row phase's operand out of the bytes that become the emission queues
            // behind the next barrier
            lvr_fetch_q_frags<HB>(s_qu.stash, bq);
        }
        int before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            before += (w < wave) ? s_tot[w] : 0;
            total += s_tot[w];
        }
        {
            // one pass per set bit of the fullest mask in the wave (a few when most groups are pruned) instead
            // of sixteen tests in every lane
            int o = before + (incl - cnt);
            uint32_t left = mybits;
            while (__ballot(left != 0)) {   // wave-uniform
                if (left != 0) {
                    const int k = __builtin_ctz(left);
                    s_list[o++] = (uint16_t)((wave * a.tiles_per_wave + lane) * 16 + k);
                    left &= left - 1;
                }
            }
        }
        if (threadIdx.x == 0) a.seg_count[(int64_t)bh * a.max_segs + blockIdx.x] = total;
        __syncthreads();
        rows = (int64_t)total << a.log2r;
    } else {
        rows = a.n_total - a.n_indexed;
        buf_row0 = a.n_indexed;
        if (a.m_new > 0) {
            // append fused into the step (Sec. 4.3): this workgroup owns the buffer of its (sequence, KV
            // head), so it stores the new K and V rows at the arena tail before it scans the buffer;
            // the attention launch that follows finds the V rows in place
            const int64_t pieces = (int64_t)a.m_new * 16;   // 16-byte pieces per matrix
            const uint4 *ks = static_cast<const uint4 *>(a.k_new) + (int64_t)bh * pieces;
            const uint4 *vs = static_cast<const uint4 *>(a.v_new) + (int64_t)bh * pieces;
            const int64_t row0 = (int64_t)bh * a.cap_rows + (a.n_total - a.m_new);
            uint4 *kd = static_cast<uint4 *>(const_cast<void *>(a.K)) + row0 * 16;
            uint4 *vd = static_cast<uint4 *>(a.V) + row0 * 16;
            for (int64_t i = threadIdx.x; i < 2 * pieces; i += 256) {
                if (i < pieces) kd[i] = ks[i];
                else vd[i - pieces] = vs[i - pieces];
            }
        }
        if constexpr (CSP) lvr_fetch_q_frags<HB>(s_qu.stash, bq);
        // the new rows are in place for every wave of this workgroup, and no wave still reads the
        // operand staging area that the score queues are about to reuse
        __syncthreads();
    }

    // ---------------- phase B: exact check of the surviving rows ----------------
    lvr_emitter<W, true> em[HB];
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) {
        em[hb].q = s_queue[wave][hb];
        if constexpr (BL) em[hb].qs = s_qs2[wave][hb];
        else em[hb].qs = s_u.qscore[wave][hb];
        em[hb].count = 0;
        em[hb].rep_base = 8;
        em[hb].hq_base = hq0 + hb * W;
    }
    const char *Kb = static_cast<const char *>(a.K) + (int64_t)bh * a.cap_rows * LVR_D * 2;
    const int32_t *spos = a.slot_pos ? a.slot_pos + (int64_t)bh * a.cap_rows : nullptr;
    const int rmask = (1 << a.log2r) - 1;
    const int64_t seg_g0 = (int64_t)blockIdx.x * a.tiles_per_wave * 64;   // first group of this workgroup's segment
    const int64_t tiles = (rows + 15) >> 4;
    // This wave checks tiles wave, wave + 4, wave + 8, ...: m of them, two at a time in two register sets.
    // Rotated form: as soon as a set has been scored the wave's next tile but one is requested into it, so
    // loads stay outstanding while the other set is scored.  Past the end the request repeats the wave's
    // last tile (a cache hit, never scored): every trip issues the same loads and the waits stay exact.
    const int64_t m = tiles > wave ? (tiles - wave + 3) >> 2 : 0;
    int slot[2], nvalid[2];
    uint4 av[2][4];
    auto request = [&](auto u_c, int64_t k) {
        constexpr int u = decltype(u_c)::value;
        const int64_t t = wave + 4 * (k < m ? k : m - 1);
        int64_t rowidx = t * 16 + n;
        const int64_t left = rows - t * 16;
        nvalid[u] = k >= m ? 0 : (left < 16 ? (int)left : 16);
        if (rowidx >= rows) rowidx = 0;
        slot[u] = direct ? (int)(buf_row0 + rowidx)
                         : (int)(((seg_g0 + s_list[rowidx >> a.log2r]) << a.log2r) + (rowidx & rmask));
        lvr_load_a_frags(Kb, slot[u], av[u]);
    };
    auto check = [&](auto u_c) {
        constexpr int u = decltype(u_c)::value;
#pragma unroll
        for (int hb = 0; hb < HB; ++hb) {
            lvr_f32x4 s;
            if constexpr (ENC && BL) {
                lvr_bf16x8 b[4], b2[4];
                fetch_bq(hb, b);
                fetch_bq2(hb, b2);
                s = lvr_score_tile2(av[u], b, av[u], b2);
            } else if constexpr (ENC) s = lvr_score_tile2(av[u], bq[hb], av[u], bq2[hb]);
            else if constexpr (W == 8) {
                lvr_bf16x8 b[4], b3[4];
                fetch_bq8(0, b);
                if (third) fetch_bq8(1, b3);
                s = lvr_score_tile8(av[u], b, b3, third);
            } else if constexpr (BL) {
                lvr_bf16x8 b[4];
                fetch_bq(hb, b);
                s = lvr_score_tile(av[u], b);
            } else s = lvr_score_tile(av[u], bq[hb]);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int trow = 4 * kq + j;
                const bool pred = trow < nvalid[u] && rep[hb] &&
                                  (s[j] >= taue[hb] || (buffer_wg && a.buffer_dense));
                em[hb].push(a.emit, lane, rep[hb], pred, slot[u], trow, spos, s[j]);
            }
        }
    };
    // The rotation pays where scoring a tile takes long against the memory latency (two head blocks:
    // 62.2 -> 60.1 us per launch at 128k keys); with one head block the launch is at the streaming
    // ceiling either way and the repeated requests of short segments cost more than they hide.
    if ((HB == 2 || W == 8) && m >= 4) {   // wave-uniform
        request(std::integral_constant<int, 0>{}, 0);
        request(std::integral_constant<int, 1>{}, 1);
        for (int64_t k = 0; k < m; k += 2) {
            take_turn((int)(k >> 1));
            check(std::integral_constant<int, 0>{});
            request(std::integral_constant<int, 0>{}, k + 2);
            if (nvalid[1] > 0) check(std::integral_constant<int, 1>{});   // wave-uniform
            request(std::integral_constant<int, 1>{}, k + 3);
        }
    } else {
        for (int64_t k = 0; k < m; k += 2) {   // both sets requested, then both scored
            take_turn((int)(k >> 1));
            request(std::integral_constant<int, 0>{}, k);
            request(std::integral_constant<int, 1>{}, k + 1);   // past the end: a repeat of the last tile, not scored
            check(std::integral_constant<int, 0>{});
            if (nvalid[1] > 0) check(std::integral_constant<int, 1>{});
        }
    }
    __builtin_amdgcn_s_setprio(0);
    // Last flush, once per workgroup instead of once per wave: the four waves add up what they still hold, ONE lane
    // per head reserves the workgroup's range in the head's list, and every wave writes behind the waves before
    // it.  Atomics on one counter are served one after the other, and at the end of a launch every wave of the
    // device arrives at the same few counters at once: a quarter of the atomics is a quarter of that queue.
    // (Flushes of a full queue in mid-flight stay per wave; they are rare and spread over time.)
#pragma unroll
    for (int hb = 0; hb < HB; ++hb)
        if (rep[hb] && kq == 0) s_wcnt[wave][hb * W + n - 8] = em[hb].count;
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int hb = 0; hb < HB; ++hb) {
            if (rep[hb] && kq == 0) {
                const int h = hb * W + n - 8;
                const int tot = s_wcnt[0][h] + s_wcnt[1][h] + s_wcnt[2][h] + s_wcnt[3][h];
                s_wbase[h] = tot > 0 ? atomicAdd(&a.emit.head_count[(hq0 + h) * LVR_CNT_STRIDE], tot) : 0;
            }
        }
    }
    __syncthreads();
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) {
        int base = 0;
        if (rep[hb] && kq == 0) {
            const int h = hb * W + n - 8;
            // all three reads at once (a loop up to `wave` would take them one LDS trip after the other)
            const int c0 = s_wcnt[0][h], c1 = s_wcnt[1][h], c2 = s_wcnt[2][h];
            base = s_wbase[h] + (wave > 0 ? c0 : 0) + (wave > 1 ? c1 : 0) + (wave > 2 ? c2 : 0);
        }
        if (__ballot(em[hb].count > 0)) em[hb].write_out(a.emit, lane, spos, base);
    }
}

// One launch of an instantiation.  With a pair of events in `ev` the dispatch itself carries them (they read the kernel's
// own start and end); without, a plain launch.
struct LaunchEvents {
    hipEvent_t start, stop;
};
#define LVR_QF_LAUNCH(KERNEL)                                                                                        \
    do {                                                                                                             \
        if (ev.start) hipExtLaunchKernelGGL(KERNEL, grid, dim3(256), dyn_lds, st, ev.start, ev.stop, 0, a);           \
        else hipLaunchKernelGGL(KERNEL, grid, dim3(256), dyn_lds, st, a);                                            \
    } while (0)

template <int UA, int W>
void launch_s(dim3 grid, unsigned dyn_lds, hipStream_t st, const FusedArgs &a, int S, const LaunchEvents &ev) {
    switch (S) {
        case 1: LVR_QF_LAUNCH((query_fused_kernel<1, 1, UA, 0, 0, 0, W>)); break;
        case 2: LVR_QF_LAUNCH((query_fused_kernel<1, 2, UA, 0, 0, 0, W>)); break;
        case 4: LVR_QF_LAUNCH((query_fused_kernel<1, 4, UA, 0, 0, 0, W>)); break;
        case 8: LVR_QF_LAUNCH((query_fused_kernel<1, 8, UA, 0, 0, 0, W>)); break;
        default: LVR_QF_LAUNCH((query_fused_kernel<1, 16, UA, 0, 0, 0, W>)); break;
    }
}

}  // namespace

hipError_t lvr_launch_query_fused(lvr_index *ix, const float *q, const float *tau, const float *tau_s,
                                  int32_t *out_idx, int64_t cap, hipStream_t st, const void *k_new, const void *v_new,
                                  int64_t m_new) {
    if (ix->cfg.kv_dtype != LVR_BF16) return hipErrorInvalidValue;
    if (tau_s && ((ix->box || ix->cf8 || ix->cf6) && ix->cfg.n_subspaces > 4)) return hipErrorInvalidValue;
    FusedArgs a;
    a.tau_s = tau_s;
    a.chan_exp = lvr_chan_exp(ix);   // exponents 0 and factors 1 unless the index is a rescaled one
    a.k_new = k_new;
    a.v_new = v_new;
    a.V = ix->V;
    a.m_new = (int)m_new;
    a.centres = ix->centres;
    a.radii = ix->radii;
    a.K = ix->K;
    a.slot_pos = ix->slot_pos;
    a.q = q;
    a.tau = tau;
    a.seg_count = lvr_seg_count(ix);
    a.emit.out_idx = out_idx;
    a.emit.head_count = lvr_head_count(ix);
    a.emit.overflow = lvr_overflow_flag(ix);
    a.emit.cap = cap;
    a.emit.out_score = ix->scores;
    a.emit.score_stride = ix->cap_rows;
    a.n_groups = ix->n_indexed / ix->cfg.group_size;
    a.max_groups = ix->max_groups;
    a.max_segs = lvr_max_segs(ix->max_groups);
    a.cap_rows = ix->cap_rows;
    a.n_indexed = ix->n_indexed;
    a.n_total = ix->n_total + m_new;
    a.log2r = 0;
    while ((1 << a.log2r) < ix->cfg.group_size) ++a.log2r;
    a.n_q_heads = ix->cfg.n_q_heads;
    a.n_kv_heads = ix->cfg.n_kv_heads;
    a.G = ix->G;
    a.buffer_dense = (ix->cfg.flags & LVR_ATTEND_BUFFER_DENSE) ? 1 : 0;
    a.skip_bounds = (ix->skip_bounds && !tau_s) ? 1 : 0;
    const int n_bh = lvr_n_bh(ix);
    // segment = 4 waves x tiles_per_wave tiles x 16 groups; aim at a fixed number of workgroups per launch
    const int64_t target_wgs = ix->cfg.query_workgroups > 0 ? ix->cfg.query_workgroups : 1024;
    const int64_t want = a.n_groups * n_bh / target_wgs;
    int tpw = 1;
    while (tpw < SEG_MAX_TILES && (int64_t)tpw * 64 < want) tpw *= 2;
    a.tiles_per_wave = tpw;
    const int seg_groups = tpw * 64;
    a.n_segs = (int)((a.n_groups + seg_groups - 1) / seg_groups);
    const int has_buffer = a.n_total > ix->n_indexed ? 1 : 0;
    ix->seg_groups = seg_groups;
    ix->n_segs = a.n_segs;
    if (a.n_segs + has_buffer == 0) return hipSuccess;
    dim3 grid((unsigned)(a.n_segs + has_buffer), (unsigned)n_bh);
    // more workgroups than 5 x 256: hold the residency at four per compute unit, so that the rounds are whole
    const unsigned dyn_lds = (int64_t)grid.x * grid.y > 1280 ? 20480u : 0u;
    const LaunchEvents ev = {ix->launch_start, ix->launch_stop};
    // one centre tile per trip for the small segments of short contexts, two per trip for long ones
    // (measured crossover between 32k and 128k keys); four per trip costs a wave per SIMD and 12 us
    const bool one = tpw == 1;
    if (tau_s && ix->box) {   // Query 1 on boxes: per-block box bounds, blocks of whole MFMA steps
        const int S = ix->cfg.n_subspaces;
#define LVR_Q1B_LAUNCH(HB, CF)                                                                                 \
    do {                                                                                                        \
        if (S == 1) LVR_QF_LAUNCH((query_fused_kernel<HB, 1, 1, 1, 1, CF>));   \
        else if (S == 2) LVR_QF_LAUNCH((query_fused_kernel<HB, 2, 1, 1, 1, CF>)); \
        else LVR_QF_LAUNCH((query_fused_kernel<HB, 4, 1, 1, 1, CF>));          \
    } while (0)
        if (ix->G <= 4) {
            if (ix->cf8) LVR_Q1B_LAUNCH(1, 1);
            else LVR_Q1B_LAUNCH(1, 0);
        } else {
            if (ix->cf8) LVR_Q1B_LAUNCH(2, 1);
            else LVR_Q1B_LAUNCH(2, 0);
        }
#undef LVR_Q1B_LAUNCH
        return hipGetLastError();
    }
    if (tau_s) {   // Query 1: per-block thresholds
        const int S = ix->cfg.n_subspaces;
#define LVR_Q1_LAUNCH(HB, CF)                                                                                  \
    do {                                                                                                        \
        if (S == 1) LVR_QF_LAUNCH((query_fused_kernel<HB, 1, 1, 0, 1, CF>));   \
        else if (S == 2) LVR_QF_LAUNCH((query_fused_kernel<HB, 2, 1, 0, 1, CF>)); \
        else if (S == 4) LVR_QF_LAUNCH((query_fused_kernel<HB, 4, 1, 0, 1, CF>)); \
        else if constexpr (!CF) {                                                                              \
            if (S == 8) LVR_QF_LAUNCH((query_fused_kernel<HB, 8, 1, 0, 1, 0>)); \
            else LVR_QF_LAUNCH((query_fused_kernel<HB, 16, 1, 0, 1, 0>));       \
        }                                                                                                       \
    } while (0)
        if (ix->G <= 4) {
            if (ix->cf6) LVR_Q1_LAUNCH(1, 2);
            else if (ix->cf8) LVR_Q1_LAUNCH(1, 1);
            else LVR_Q1_LAUNCH(1, 0);
        } else {
            if (ix->cf6) LVR_Q1_LAUNCH(2, 2);
            else if (ix->cf8) LVR_Q1_LAUNCH(2, 1);
            else LVR_Q1_LAUNCH(2, 0);
        }
#undef LVR_Q1_LAUNCH
        return hipGetLastError();
    }
    if (ix->box && ix->cf8) {   // boxes with 8-bit corners
        if (ix->G <= 4) LVR_QF_LAUNCH((query_fused_kernel<1, 1, 1, 1, 0, 1>));
        else LVR_QF_LAUNCH((query_fused_kernel<2, 1, 1, 1, 0, 1>));
        return hipGetLastError();
    }
    if (ix->cf8 || ix->cf6) {   // 8-bit or 6-bit centres
        const int S = ix->cfg.n_subspaces;
#define LVR_CODED_LAUNCH(UA, W, CF)                                                                               \
    do {                                                                                                      \
        if (S == 1) LVR_QF_LAUNCH((query_fused_kernel<1, 1, UA, 0, 0, CF, W>));  \
        else if (S == 2) LVR_QF_LAUNCH((query_fused_kernel<1, 2, UA, 0, 0, CF, W>)); \
        else LVR_QF_LAUNCH((query_fused_kernel<1, 4, UA, 0, 0, CF, W>));         \
    } while (0)
#define LVR_CODED_ANY_LAUNCH(UA, W)            \
    do {                                 \
        if (ix->cf6) LVR_CODED_LAUNCH(UA, W, 2); \
        else LVR_CODED_LAUNCH(UA, W, 1);    \
    } while (0)
        if (ix->G <= 4) {
            if (one) LVR_CODED_ANY_LAUNCH(1, 4);
            else LVR_CODED_ANY_LAUNCH(2, 4);
        } else {   // up to eight heads in one operand
            if (one) LVR_CODED_ANY_LAUNCH(1, 8);
            else LVR_CODED_ANY_LAUNCH(2, 8);
        }
#undef LVR_CODED_ANY_LAUNCH
#undef LVR_CODED_LAUNCH
        return hipGetLastError();
    }
    if (ix->box) {   // boxes: one allowance per group, one tile (two rows per group) per trip
        if (ix->G <= 4) LVR_QF_LAUNCH((query_fused_kernel<1, 1, 1, 1>));
        else LVR_QF_LAUNCH((query_fused_kernel<2, 1, 1, 1>));
        return hipGetLastError();
    }
    if (ix->G <= 4) {
        if (one) launch_s<1, 4>(grid, dyn_lds, st, a, ix->cfg.n_subspaces, ev);
        else launch_s<2, 4>(grid, dyn_lds, st, a, ix->cfg.n_subspaces, ev);
    } else {   // up to eight heads in one operand
        if (one) launch_s<1, 8>(grid, dyn_lds, st, a, ix->cfg.n_subspaces, ev);
        else launch_s<2, 8>(grid, dyn_lds, st, a, ix->cfg.n_subspaces, ev);
    }
    return hipGetLastError();
}
