// Scoring a tile of 16 bf16 rows (keys or centres) against the query heads of one KV head on
// the matrix cores.
//
// The scores S[row][head] = <q_head, row> of the G query heads that share a KV head form a
// skinny dense contraction  [16 rows x 128] . [128 x heads].  On the vector ALU this costs a
// multiply-add per element and head plus a 16-lane reduction per row and head, which at HBM
// rate would take most of the ALU issue slots; one v_mfma_f32_16x16x32_bf16 per 32 coordinates
// does the same work in a handful of cycles.
//
// Full fp32 query precision on a bf16 matrix core: each fp32 q value is split exactly into
// three bf16 terms  q = hi + mid + lo  (8 + 8 + 8 significant bits).  The three terms of four
// heads fill 12 of the 16 columns of the B operand: column n = part * 4 + head.  Products of
// two bf16 numbers are exact in fp32 and the unit accumulates in fp32, so summing the three
// columns of a head gives <q, row> to fp32 accuracy.
//
// Operand layout of v_mfma_f32_16x16x32_bf16 (lane l of the wave, j = 0..7):
//   A[i = l % 16][k = 8 * (l / 16) + j]      one 16-byte load per lane straight from a row
//   B[k = 8 * (l / 16) + j][n = l % 16]      built once per wave from q
//   D[i = 4 * (l / 16) + j'][n = l % 16]     j' = 0..3
// After  d + row_shr:4(d) + row_shr:8(d)  the lanes with n in [8, 12) hold the finished score of
// head n - 8 for rows 4 * (l / 16) + j'.
#pragma once
#include "lvr_internal.h"

#ifdef __HIPCC__
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 lvr_bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float lvr_f32x4;

// Exact three-way split of an fp32 value into bf16 bit patterns (part 0 = leading term): each term is the remainder
// cut off after its eight leading significant bits, so the three of them hold all 24 bits of x and add up to x exactly.
// (Cutting instead of rounding to nearest costs a third of the instructions; every workgroup of a query launch does
// this 8 times per lane before its first matrix instruction.)
__device__ __forceinline__ uint32_t lvr_split_part(float x, int part) {
    const uint32_t hi = __float_as_uint(x) & 0xffff0000u;
    const float r1 = x - __uint_as_float(hi);
    const uint32_t mid = __float_as_uint(r1) & 0xffff0000u;
    const float r2 = r1 - __uint_as_float(mid);   // at most eight significant bits are left: its low half is zero
    // picked with masks: written as nested selects this becomes two levels of divergent branches per value
    const uint32_t m0 = part == 0 ? 0xffffffffu : 0u, m1 = part == 1 ? 0xffffffffu : 0u, m2 = part == 2 ? 0xffffffffu : 0u;
    return ((hi & m0) | (mid & m1) | (__float_as_uint(r2) & m2)) >> 16;
}

// One B fragment: head block hb (heads hb*4 .. hb*4+3 of the KV group, those >= G are zero),
// coordinates kk*32 .. kk*32+31.  `scale` multiplies q first (1 for the range query;
// sigma*log2(e) for attention logits).
// sign: 0 takes q as it is, +1 its positive part max(q, 0), -1 its negative part min(q, 0).
__device__ __forceinline__ void lvr_build_q_frag_one(const float *__restrict__ q_group, int G, int hb, int kk,
                                                     float scale, lvr_bf16x8 &out, int sign = 0) {
    const int lane = threadIdx.x & 63;
    const int n = lane & 15, kq = lane >> 4;
    const int part = n >> 2, h = hb * 4 + (n & 3);
    const bool live = part < 3 && h < G;
    uint32_t w[8];
    const float *src = q_group + (int64_t)(live ? h : 0) * LVR_D + kk * 32 + kq * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        float x = live ? src[e] * scale : 0.f;
        if (sign > 0) x = fmaxf(x, 0.f);
        if (sign < 0) x = fminf(x, 0.f);
        w[e] = live ? lvr_split_part(x, part) : 0u;
    }
    uint4 packed = make_uint4(w[0] | (w[1] << 16), w[2] | (w[3] << 16), w[4] | (w[5] << 16), w[6] | (w[7] << 16));
    out = __builtin_bit_cast(lvr_bf16x8, packed);
}

// The same in two steps, so that the loads of q can be put in flight ahead of other loads
// (vector memory loads return in order: whatever is requested first is usable first).
__device__ __forceinline__ void lvr_q_frag_load(const float *__restrict__ q_group, int G, int hb, int kk, float (&raw)[8]) {
    const int lane = threadIdx.x & 63;
    const int n = lane & 15, kq = lane >> 4;
    const int part = n >> 2, h = hb * 4 + (n & 3);
    const bool live = part < 3 && h < G;
    const float *src = q_group + (int64_t)(live ? h : 0) * LVR_D + kk * 32 + kq * 8;
    const float4 a = *reinterpret_cast<const float4 *>(src), b = *reinterpret_cast<const float4 *>(src + 4);
    raw[0] = a.x; raw[1] = a.y; raw[2] = a.z; raw[3] = a.w;
    raw[4] = b.x; raw[5] = b.y; raw[6] = b.z; raw[7] = b.w;
}

__device__ __forceinline__ void lvr_q_frag_make(const float (&raw)[8], int G, int hb, float scale, lvr_bf16x8 &out, int sign = 0) {
    const int lane = threadIdx.x & 63;
    const int n = lane & 15;
    const int part = n >> 2, h = hb * 4 + (n & 3);
    const bool live = part < 3 && h < G;
    // The term this lane needs is what is left of x after `part` cuts (see lvr_split_part), cut once more: a lane that
    // needs the leading term subtracts zero twice.  Four instructions per value, and the last cut is the packing.
    const uint32_t cut1 = part >= 1 ? 0xffff0000u : 0u, cut2 = part >= 2 ? 0xffff0000u : 0u;
    uint32_t y[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        float x = raw[e] * scale;
        if (sign > 0) x = fmaxf(x, 0.f);
        if (sign < 0) x = fminf(x, 0.f);
        x -= __uint_as_float(__float_as_uint(x) & cut1);
        x -= __uint_as_float(__float_as_uint(x) & cut2);
        y[e] = __float_as_uint(x);
    }
    // upper halves of two words side by side
    uint4 packed = make_uint4(__builtin_amdgcn_perm(y[1], y[0], 0x07060302u), __builtin_amdgcn_perm(y[3], y[2], 0x07060302u),
                              __builtin_amdgcn_perm(y[5], y[4], 0x07060302u), __builtin_amdgcn_perm(y[7], y[6], 0x07060302u));
    if (!live) packed = make_uint4(0u, 0u, 0u, 0u);
    out = __builtin_bit_cast(lvr_bf16x8, packed);
}

// The exchange step of lvr_build_q_frags_wg for fragments made from values loaded earlier.
// Contains a __syncthreads(): every thread of the workgroup must call it.
template <int HB>
__device__ __forceinline__ void lvr_exchange_q_frags_wg(const float (&raw)[HB][8], int G, float scale, uint4 (&s_bq)[HB][4][64],
                                                        lvr_bf16x8 (&bq)[HB][4], int sign = 0) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) {
        lvr_bf16x8 f;
        lvr_q_frag_make(raw[hb], G, hb, scale, f, sign);
        s_bq[hb][wave][lane] = __builtin_bit_cast(uint4, f);
    }
    __syncthreads();
#pragma unroll
    for (int hb = 0; hb < HB; ++hb)
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) bq[hb][kk] = __builtin_bit_cast(lvr_bf16x8, s_bq[hb][kk][lane]);
}

// A second operand set put aside in LDS (no barrier here: the caller's next barrier publishes it) and fetched later.
template <int HB>
__device__ __forceinline__ void lvr_stash_q_frags(const float (&raw)[HB][8], int G, float scale, uint4 (&s_bq)[HB][4][64]) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) {
        lvr_bf16x8 f;
        lvr_q_frag_make(raw[hb], G, hb, scale, f, 0);
        s_bq[hb][wave][lane] = __builtin_bit_cast(uint4, f);
    }
}
template <int HB>
__device__ __forceinline__ void lvr_fetch_q_frags(const uint4 (&s_bq)[HB][4][64], lvr_bf16x8 (&bq)[HB][4]) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int hb = 0; hb < HB; ++hb)
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) bq[hb][kk] = __builtin_bit_cast(lvr_bf16x8, s_bq[hb][kk][lane]);
}

// All B fragments of a KV group, built once per 256-thread workgroup: wave w builds the
// fragment of coordinates w*32 .. w*32+31 for every head block, the four waves exchange them
// through LDS.  Contains a __syncthreads(): every thread of the workgroup must call it.
template <int HB>
__device__ __forceinline__ void lvr_build_q_frags_wg(const float *__restrict__ q_group, int G, float scale,
                                                     uint4 (&s_bq)[HB][4][64], lvr_bf16x8 (&bq)[HB][4], int sign = 0) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int hb = 0; hb < HB; ++hb) {
        lvr_bf16x8 f;
        lvr_build_q_frag_one(q_group, G, hb, wave, scale, f, sign);
        s_bq[hb][wave][lane] = __builtin_bit_cast(uint4, f);
    }
    __syncthreads();
#pragma unroll
    for (int hb = 0; hb < HB; ++hb)
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) bq[hb][kk] = __builtin_bit_cast(lvr_bf16x8, s_bq[hb][kk][lane]);
}

// ---- eight heads per KV head in ONE operand ----
// Column n = part * 8 + head: the two leading bf16 terms of eight heads fill all 16 columns of the
// main operand; the third term (zero for every query with at most 16 significant bits, bf16 queries
// among them) goes into columns 8..15 of a second operand that is contracted into the same
// accumulator only when some head needs it.  After  d + row_shr:8(d)  the lanes with n in [8, 16)
// hold the finished score of head n - 8.
// third = false: the main operand; third = true: the operand of the third terms.
// fac (may be NULL): 128 factors, one per coordinate, applied to q first (powers of two: a rescaled index).
// Returns true if this lane put a non-zero third term into its piece.
__device__ __forceinline__ bool lvr_build_q_frag8_one(const float *__restrict__ q_group, int G, int kk, float scale,
                                                      bool third, lvr_bf16x8 &out, const float *__restrict__ fac = nullptr) {
    const int lane = threadIdx.x & 63;
    const int n = lane & 15, kq = lane >> 4;
    const int h = n & 7;
    const int part = third ? 2 : (n >> 3);
    const bool live = h < G && (!third || n >= 8);
    uint32_t w[8];
    uint32_t any = 0;
    const float *src = q_group + (int64_t)(live ? h : 0) * LVR_D + kk * 32 + kq * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        float x = src[e] * scale;
        if (fac) x *= fac[kk * 32 + kq * 8 + e];
        w[e] = live ? lvr_split_part(x, part) : 0u;
        any |= w[e] & 0x7fffu;   // a signed zero contributes nothing either
    }
    uint4 packed = make_uint4(w[0] | (w[1] << 16), w[2] | (w[3] << 16), w[4] | (w[5] << 16), w[6] | (w[7] << 16));
    out = __builtin_bit_cast(lvr_bf16x8, packed);
    return third && any != 0;
}

// Both operands of a KV group of up to eight heads, built once per 256-thread workgroup into LDS
// (s_bq[base] = main, s_bq[base + 1] = third terms); wave w builds the pieces of coordinates w*32 .. w*32+31.
// Contains a barrier: every thread of the workgroup must call it.  Returns whether the second
// operand holds anything (the same answer in every thread).
template <int NB>
__device__ __forceinline__ bool lvr_build_q_frags8_wg(const float *__restrict__ q_group, int G, float scale,
                                                      uint4 (&s_bq)[NB][4][64], int base = 0, const float *__restrict__ fac = nullptr) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    lvr_bf16x8 f;
    lvr_build_q_frag8_one(q_group, G, wave, scale, false, f, fac);
    s_bq[base][wave][lane] = __builtin_bit_cast(uint4, f);
    const bool nz = lvr_build_q_frag8_one(q_group, G, wave, scale, true, f, fac);
    s_bq[base + 1][wave][lane] = __builtin_bit_cast(uint4, f);
    return __syncthreads_or(nz ? 1 : 0) != 0;
}

// Sum over the parts' columns for the eight-head layout.
__device__ __forceinline__ lvr_f32x4 lvr_sum_parts8(const lvr_f32x4 &acc) {
    lvr_f32x4 s;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float v = acc[j];
        s[j] = v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x118, 0xf, 0xf, true));   // row_shr:8
    }
    return s;
}

// Scores of a tile for eight heads: result valid in lanes with (lane % 16) in [8, 16).
__device__ __forceinline__ lvr_f32x4 lvr_score_tile8(const uint4 (&a)[4], const lvr_bf16x8 (&b)[4],
                                                     const lvr_bf16x8 (&b3)[4], bool third) {
    lvr_f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(lvr_bf16x8, a[kk]), b[kk], acc, 0, 0, 0);
    if (third) {   // wave-uniform
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(lvr_bf16x8, a[kk]), b3[kk], acc, 0, 0, 0);
    }
    return lvr_sum_parts8(acc);
}

// Bound of a tile of 16 balls for eight heads: centre product plus the radius step.
__device__ __forceinline__ lvr_f32x4 lvr_bound_tile8(const uint4 (&a)[4], const lvr_bf16x8 (&b)[4],
                                                     const lvr_bf16x8 (&b3)[4], bool third, lvr_bf16x8 ra, lvr_bf16x8 rb) {
    lvr_f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(lvr_bf16x8, a[kk]), b[kk], acc, 0, 0, 0);
    if (third) {   // wave-uniform
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(lvr_bf16x8, a[kk]), b3[kk], acc, 0, 0, 0);
    }
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ra, rb, acc, 0, 0, 0);
    return lvr_sum_parts8(acc);
}

// Radius step, B side, eight heads: column n = part * 8 + head with TWO terms per norm, the leading
// eight bits and the rest rounded UP to eight bits (the sum is at least the norm; a bound may be loose,
// never tight).  k-slots as in lvr_radius_b_frag.  qn_group: [heads][16] floats, |pi_s q_h| >= 0.
template <int S, int NP>
__device__ __forceinline__ lvr_bf16x8 lvr_radius_b_frag8(const float (*qn_group)[16], int G) {
    const int lane = threadIdx.x & 63;
    const int n = lane & 15, kq = lane >> 4;
    const int p = n >> 3, h = n & 7;
    const bool live = h < G;
    uint32_t val[S];
#pragma unroll
    for (int s = 0; s < S; ++s) {
        const float x = qn_group[live ? h : 0][s];
        const uint32_t hi = __float_as_uint(x) & 0xffff0000u;
        uint32_t rest = __float_as_uint(x - __uint_as_float(hi));
        if (rest & 0xffffu) rest = (rest & 0xffff0000u) + 0x10000u;
        val[s] = live ? ((p == 0 ? hi : rest) >> 16) : 0u;
    }
    uint32_t w[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        uint32_t v = 0;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            const int k = 8 * q4 + j;
            if (k < NP * S) v = (kq == q4) ? val[k % S] : v;
        }
        w[j] = v;
    }
    uint4 packed = make_uint4(w[0] | (w[1] << 16), w[2] | (w[3] << 16), w[4] | (w[5] << 16), w[6] | (w[7] << 16));
    return __builtin_bit_cast(lvr_bf16x8, packed);
}

// The four 16-byte pieces of the A operand for row `row` (lane's row = lane % 16):
// coordinates kk*32 + 8*(lane/16) .. +7 for kk = 0..3.
__device__ __forceinline__ void lvr_load_a_frags(const char *__restrict__ base, int64_t row, uint4 (&a)[4]) {
    const int kq = (threadIdx.x & 63) >> 4;
    const uint4 *p = reinterpret_cast<const uint4 *>(base + row * (LVR_D * 2)) + kq;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) a[kk] = p[kk * 4];
}

// Centres stored as e4m3 codes in operand order: a lane's 32 bytes of a row are its four pieces of
// 8 coordinates (kk = 0..3).  Two 16-byte loads instead of four ...
__device__ __forceinline__ void lvr_load_a_codes(const char *__restrict__ base, int64_t row, uint4 (&raw)[2]) {
    const int kq = (threadIdx.x & 63) >> 4;
    const uint4 *p = reinterpret_cast<const uint4 *>(base + row * LVR_D + kq * 32);
    raw[0] = p[0];
    raw[1] = p[1];
}

// ... and one conversion instruction per two codes (exact: an e4m3 value has 4 significant bits)
// turns them into the bf16 operand pieces.
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 lvr_bf16x2;
__device__ __forceinline__ void lvr_codes_to_a_frags(const uint4 (&raw)[2], uint4 (&a)[4]) {
    const uint32_t w[8] = {raw[0].x, raw[0].y, raw[0].z, raw[0].w, raw[1].x, raw[1].y, raw[1].z, raw[1].w};
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        const uint32_t d0 = w[2 * kk], d1 = w[2 * kk + 1];
        a[kk].x = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((int)d0, 1.0f, false));
        a[kk].y = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((int)d0, 1.0f, true));
        a[kk].z = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((int)d1, 1.0f, false));
        a[kk].w = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((int)d1, 1.0f, true));
    }
}

// Centres stored as e2m3 codes (6 bits) in operand order with one power-of-two scale per lane piece:
// a lane's 24 bytes of a row are its 32 codes (code 8 kk + e = coordinate 32 kk + 8 kq + e).  The
// rows are 96 bytes long, so a piece starts on an 8-byte boundary.
struct alignas(8) lvr_codes6 {
    uint32_t w[6];
};
__device__ __forceinline__ void lvr_load_a_codes6(const char *__restrict__ base, int64_t row, lvr_codes6 &raw) {
    const int kq = (threadIdx.x & 63) >> 4;
    raw = *reinterpret_cast<const lvr_codes6 *>(base + row * (LVR_D * 3 / 4) + kq * 24);
}

// One conversion instruction turns the 32 codes into the four bf16 operand pieces (exact: a code has 4
// significant bits); `scales` holds the exponent bytes of the row's four pieces, this lane uses byte kq.
typedef __attribute__((__vector_size__(6 * sizeof(uint32_t)))) uint32_t lvr_u32x6;
typedef __attribute__((__vector_size__(32 * sizeof(__bf16)))) __bf16 lvr_bf16x32;
typedef __attribute__((__vector_size__(16 * sizeof(uint32_t)))) uint32_t lvr_u32x16;
__device__ __forceinline__ void lvr_codes6_to_a_frags(const lvr_codes6 &raw, uint32_t scales, uint4 (&a)[4]) {
    const int kq = (threadIdx.x & 63) >> 4;
    const float scale = __uint_as_float(((scales >> (8 * kq)) & 0xffu) << 23);
    const lvr_u32x6 src = {raw.w[0], raw.w[1], raw.w[2], raw.w[3], raw.w[4], raw.w[5]};
    const lvr_u32x16 d = __builtin_bit_cast(lvr_u32x16, __builtin_amdgcn_cvt_scalef32_pk32_bf16_fp6(src, scale));
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) a[kk] = make_uint4(d[4 * kk], d[4 * kk + 1], d[4 * kk + 2], d[4 * kk + 3]);
}

// D = A . B over the 128 coordinates, then the three query parts are added up.
// Result valid in lanes with (lane % 16) in [8, 12): score of head hb*4 + lane%16 - 8 for rows
// 4*(lane/16) + j, j = 0..3.
__device__ __forceinline__ lvr_f32x4 lvr_score_tile(const uint4 (&a)[4], const lvr_bf16x8 (&bq)[4]) {
    lvr_f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(lvr_bf16x8, a[kk]), bq[kk], acc, 0, 0, 0);
    lvr_f32x4 s;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float v = acc[j];
        float t = v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x114, 0xf, 0xf, true));
        t += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x118, 0xf, 0xf, true));
        s[j] = t;
    }
    return s;
}

// Partial score over coordinates kk0*32 .. kk1*32-1 only (one coordinate block of "Query 1").
template <int KK0, int KK1>
__device__ __forceinline__ lvr_f32x4 lvr_score_tile_block(const uint4 (&a)[4], const lvr_bf16x8 (&bq)[4]) {
    lvr_f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = KK0; kk < KK1; ++kk)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(lvr_bf16x8, a[kk]), bq[kk], acc, 0, 0, 0);
    lvr_f32x4 s;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float v = acc[j];
        float t = v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x114, 0xf, 0xf, true));
        t += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x118, 0xf, 0xf, true));
        s[j] = t;
    }
    return s;
}

// The same for boxes: upper corners against the positive part of q, lower corners against the
// negative part, both restricted to the block, in one accumulator.
template <int KK0, int KK1>
__device__ __forceinline__ lvr_f32x4 lvr_score_tile_block2(const uint4 (&a1)[4], const lvr_bf16x8 (&b1)[4],
                                                           const uint4 (&a2)[4], const lvr_bf16x8 (&b2)[4]) {
    lvr_f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = KK0; kk < KK1; ++kk) {
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(lvr_bf16x8, a1[kk]), b1[kk], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(lvr_bf16x8, a2[kk]), b2[kk], acc, 0, 0, 0);
    }
    lvr_f32x4 s;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float v = acc[j];
        float t = v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x114, 0xf, 0xf, true));
        t += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x118, 0xf, 0xf, true));
        s[j] = t;
    }
    return s;
}

// Partial score over a coordinate block that is a FRACTION of one MFMA step: coordinates
// KK*32 + KQ0*8 .. KK*32 + KQ1*8 - 1.  A lane's B fragment holds the eight query coordinates
// KK*32 + kq*8 .. +7 of its column, so zeroing the fragment on the lanes whose kq lies outside
// [KQ0, KQ1) leaves exactly the block's products in the sum.
template <int KK, int KQ0, int KQ1>
__device__ __forceinline__ lvr_f32x4 lvr_score_tile_subblock(const uint4 (&a)[4], const lvr_bf16x8 (&bq)[4], int kq) {
    const bool in = kq >= KQ0 && kq < KQ1;
    const uint4 full = __builtin_bit_cast(uint4, bq[KK]);
    const uint4 masked = make_uint4(in ? full.x : 0u, in ? full.y : 0u, in ? full.z : 0u, in ? full.w : 0u);
    lvr_f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(lvr_bf16x8, a[KK]), __builtin_bit_cast(lvr_bf16x8, masked),
                                                  acc, 0, 0, 0);
    lvr_f32x4 s;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float v = acc[j];
        float t = v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x114, 0xf, 0xf, true));
        t += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x118, 0xf, 0xf, true));
        s[j] = t;
    }
    return s;
}

// The radius term of the bound, sum_s rho_s * |pi_s q|, as one more MFMA step.
// k-slot of the step: k = part' * S + s for k < 3S (S <= 8), zero beyond.
//   A[i = row][k]      = part' of rho_{row,s}   (three bf16 terms that add up to rho exactly;
//                        rho >= 0, so truncation gives them: top 8 bits, next 8, last 8)
//   B[k][n = (p, h)]   = part p of |pi_s q_h|   (the same three-term split as q itself)
// Summed over k this is (rho_hi + rho_mid + rho_lo) * |pi_s q|_p per subspace, and the three
// columns p of a head are added up with those of the centre product.
template <int S>
__device__ __forceinline__ lvr_bf16x8 lvr_radius_a_frag(const float (&rho)[S]) {
    static_assert(3 * S <= 32, "the radius terms must fit one MFMA step");
    const int kq = (threadIdx.x & 63) >> 4;
    uint32_t part[3][S];
#pragma unroll
    for (int s = 0; s < S; ++s) {
        const uint32_t u0 = __float_as_uint(rho[s]) & 0xffff0000u;
        const float r1 = rho[s] - __uint_as_float(u0);
        const uint32_t u1 = __float_as_uint(r1) & 0xffff0000u;
        const float r2 = r1 - __uint_as_float(u1);
        part[0][s] = u0 >> 16;
        part[1][s] = u1 >> 16;
        part[2][s] = __float_as_uint(r2) >> 16;
    }
    uint32_t w[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        uint32_t v = 0;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            const int k = 8 * q4 + j;   // compile-time
            if (k < 3 * S) v = (kq == q4) ? part[k / S][k % S] : v;
        }
        w[j] = v;
    }
    uint4 packed = make_uint4(w[0] | (w[1] << 16), w[2] | (w[3] << 16), w[4] | (w[5] << 16), w[6] | (w[7] << 16));
    return __builtin_bit_cast(lvr_bf16x8, packed);
}

// qn_group: [heads][16] floats, |pi_s q_h| for s < S (already rounded up); head block hb.
// NP = bf16 terms per radius on the A side (3: split on the fly; 1: stored as one bf16 rounded up).
template <int S, int NP = 3>
__device__ __forceinline__ lvr_bf16x8 lvr_radius_b_frag(const float (*qn_group)[16], int G, int hb) {
    const int lane = threadIdx.x & 63;
    const int n = lane & 15, kq = lane >> 4;
    const int p = n >> 2, h = hb * 4 + (n & 3);
    const bool live = p < 3 && h < G;
    // every lane reads a row (a dead lane the first one) in as few LDS reads as the row allows, and cuts its own term out
    // of each value as lvr_q_frag_make does; the terms stay in the upper halves until they are packed
    const float *row = qn_group[live ? h : 0];
    float v[S];
    if constexpr (S == 4) {
        const float4 r = *reinterpret_cast<const float4 *>(row);
        v[0] = r.x; v[1] = r.y; v[2] = r.z; v[3] = r.w;
    } else if constexpr (S == 2) {
        const float2 r = *reinterpret_cast<const float2 *>(row);
        v[0] = r.x; v[1] = r.y;
    } else {
#pragma unroll
        for (int s = 0; s < S; ++s) v[s] = row[s];
    }
    const uint32_t cut1 = p >= 1 ? 0xffff0000u : 0u, cut2 = p >= 2 ? 0xffff0000u : 0u;
    uint32_t val[S];
#pragma unroll
    for (int s = 0; s < S; ++s) {
        float x = v[s];
        x -= __uint_as_float(__float_as_uint(x) & cut1);
        x -= __uint_as_float(__float_as_uint(x) & cut2);
        val[s] = live ? __float_as_uint(x) : 0u;
    }
    uint32_t w[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        uint32_t t = 0;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            const int k = 8 * q4 + j;
            if (k < NP * S) t = (kq == q4) ? val[k % S] : t;
        }
        w[j] = t;
    }
    const uint4 packed = make_uint4(__builtin_amdgcn_perm(w[1], w[0], 0x07060302u), __builtin_amdgcn_perm(w[3], w[2], 0x07060302u),
                                    __builtin_amdgcn_perm(w[5], w[4], 0x07060302u), __builtin_amdgcn_perm(w[7], w[6], 0x07060302u));
    return __builtin_bit_cast(lvr_bf16x8, packed);
}

// Radii stored as four bf16 per group (slot s = rho_s rounded up, one part): the block IS the first
// half of the operand piece of the lanes with kq = 0 (k-slots 0..3); everything else is zero.
__device__ __forceinline__ lvr_bf16x8 lvr_radius_a_stored(const uint2 &block) {
    const bool first = ((threadIdx.x & 63) >> 4) == 0;
    uint4 r;
    r.x = first ? block.x : 0u;
    r.y = first ? block.y : 0u;
    r.z = 0u;
    r.w = 0u;
    return __builtin_bit_cast(lvr_bf16x8, r);
}

// Bound of a tile of 16 balls: centre product plus the radius step.
__device__ __forceinline__ lvr_f32x4 lvr_bound_tile(const uint4 (&a)[4], const lvr_bf16x8 (&bq)[4], lvr_bf16x8 ra,
                                                    lvr_bf16x8 rb) {
    lvr_f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(lvr_bf16x8, a[kk]), bq[kk], acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ra, rb, acc, 0, 0, 0);
    lvr_f32x4 s;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float v = acc[j];
        float t = v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x114, 0xf, 0xf, true));
        t += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x118, 0xf, 0xf, true));
        s[j] = t;
    }
    return s;
}

// Bound of a tile of 16 boxes: upper corners against q+, lower corners against q-, plus the
// allowance step.
__device__ __forceinline__ lvr_f32x4 lvr_bound_tile2(const uint4 (&a1)[4], const lvr_bf16x8 (&b1)[4],
                                                     const uint4 (&a2)[4], const lvr_bf16x8 (&b2)[4], lvr_bf16x8 ra,
                                                     lvr_bf16x8 rb) {
    lvr_f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(lvr_bf16x8, a1[kk]), b1[kk], acc, 0, 0, 0);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(lvr_bf16x8, a2[kk]), b2[kk], acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ra, rb, acc, 0, 0, 0);
    lvr_f32x4 s;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float v = acc[j];
        float t = v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x114, 0xf, 0xf, true));
        t += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x118, 0xf, 0xf, true));
        s[j] = t;
    }
    return s;
}

// Two chains into one accumulator:  D = A1 . B1 + A2 . B2  (box bound: upper corners against the
// positive part of q, lower corners against the negative part; exact check of a row against
// q = q+ + q-: the same A twice).
__device__ __forceinline__ lvr_f32x4 lvr_score_tile2(const uint4 (&a1)[4], const lvr_bf16x8 (&b1)[4],
                                                     const uint4 (&a2)[4], const lvr_bf16x8 (&b2)[4]) {
    lvr_f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(lvr_bf16x8, a1[kk]), b1[kk], acc, 0, 0, 0);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(lvr_bf16x8, a2[kk]), b2[kk], acc, 0, 0, 0);
    lvr_f32x4 s;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float v = acc[j];
        float t = v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x114, 0xf, 0xf, true));
        t += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x118, 0xf, 0xf, true));
        s[j] = t;
    }
    return s;
}
#endif
