// Index construction kernels: copy K/V rows into the arena and compute, for every group of r
// consecutive arena rows, the ball of Sec. 4.1 "Ball enclosing" / Eq. (1) in each of the S
// coordinate blocks: centre = mean of the members, radius = largest member distance.
//
// Zero false negatives under rounding: the centre is stored in the cache's own format
// (bf16 or fp32), the radius is measured against the centre AS STORED, in fp32, and then
// widened to  rho * (1 + 2^-12) + 2^-12 * |centre_s|  (+1 ulp).  The widening exceeds every
// fp32 rounding error of the bound <q,c> + sum_s rho_s |pi_s q| evaluated at query time
// (at most ~(d+S) 2^-24 of the sum of term magnitudes), so a computed bound never falls
// below the exact score of a member.
#include <type_traits>

#include "lvr_internal.h"

namespace {

// 16 bytes per thread, arbitrary source strides (in elements) for (batch, head, token).
// blockIdx.z = 0 copies keys, 1 copies values, so an append is one launch.
struct CopySide {
    const char *src;
    char *dst;
    int64_t sb, sh, st;
    int64_t first;   // rows below this one are left alone (someone else writes them)
};

// Where a build kernel takes the member rows from: the arena (base == NULL), or the caller's K with
// its element strides, in which case the kernel also writes the rows into the arena (the copy of K
// and the pass over the groups are then one read of K instead of two).
struct BuildSrc {
    const char *base;
    int64_t sb, sh, st;
    int n_kv_heads;
};

__global__ void copy_rows_kernel(CopySide k, CopySide v, int n_kv_heads, int64_t cap_rows, int64_t dst_row0,
                                 int64_t rows, int row_bytes, int elt) {
    const CopySide c = blockIdx.z == 0 ? k : v;
    const int chunks = row_bytes / 16;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= rows * chunks) return;
    int bh = blockIdx.y;
    int b = bh / n_kv_heads, h = bh % n_kv_heads;
    int64_t row = i / chunks;
    if (row < c.first) return;
    int ch = (int)(i % chunks);
    const uint4 *s = reinterpret_cast<const uint4 *>(c.src + (b * c.sb + h * c.sh + row * c.st) * elt) + ch;
    uint4 *d = reinterpret_cast<uint4 *>(c.dst + ((int64_t)bh * cap_rows + dst_row0 + row) * row_bytes) + ch;
    *d = *s;
}

__device__ __forceinline__ float seg_sum(float v, int lanes_per_sub) {
    for (int off = 1; off < lanes_per_sub; off <<= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// fp32 -> OCP e4m3 code (1 sign, 4 exponent bits of bias 7, 3 mantissa bits; subnormals below 2^-6),
// round to nearest even, magnitudes above the largest finite value (448) saturate to it.
__device__ __forceinline__ uint32_t f32_to_e4m3(float x) {
    const uint32_t sign = (__float_as_uint(x) >> 24) & 0x80u;
    float a = fabsf(x);
    if (!(a < 448.f)) a = 448.f;
    if (a < 0x1p-6f) return sign | (uint32_t)(int)rintf(a * 512.f);   // 0..8; 8 is the smallest normal
    uint32_t u = __float_as_uint(a);
    u += 0x7ffffu + ((u >> 20) & 1u);
    uint32_t code = (((u >> 23) - 120u) << 3) | ((u >> 20) & 7u);
    if (code > 0x7eu) code = 0x7eu;
    return sign | code;
}

typedef __attribute__((__vector_size__(2 * sizeof(float)))) float lvr_f32x2;

// Value of one e4m3 code (never the NaN code: the encoder above does not produce it).
__device__ __forceinline__ float e4m3_value(uint32_t code) {
    const lvr_f32x2 d = __builtin_amdgcn_cvt_pk_f32_fp8((int)(code & 0xffu), false);
    return d[0];
}

// fp32 -> e4m3 code rounded towards +inf (up = true) or -inf (up = false): the nearest code, moved one
// step in the wanted direction when it fell on the wrong side.  Codes are sign-magnitude, so a step
// up is magnitude + 1 for positive and magnitude - 1 for negative values, with -0 -> smallest positive.
// At the ends (+-448) the code stays; the caller accounts for what it cannot enclose.
__device__ __forceinline__ uint32_t f32_to_e4m3_directed(float x, bool up) {
    uint32_t c = f32_to_e4m3(x);
    const float d = e4m3_value(c);
    const uint32_t mag = c & 0x7fu;
    const bool neg = (c & 0x80u) != 0;
    if (up && d < x) {
        if (neg) c = mag == 0 ? 0x01u : (0x80u | (mag - 1u));
        else if (mag < 0x7eu) c = mag + 1u;
    } else if (!up && d > x) {
        if (!neg) c = mag == 0 ? 0x81u : (mag - 1u);
        else if (mag < 0x7eu) c = 0x80u | (mag + 1u);
    }
    return c;
}

// fp32 -> e2m3 code (1 sign, 2 exponent bits of bias 1, 3 mantissa bits: magnitudes 0, 1/8, ..., 15/8, 2, 2.25, ...,
// 3.75, 4, 4.5, ..., 7.5) of x * inv_scale, round to nearest (ties to the even code), saturating at 7.5.
__device__ __forceinline__ uint32_t f32_to_e2m3(float x, float inv_scale) {
    const uint32_t sign = (__float_as_uint(x) >> 26) & 0x20u;
    const float a = fabsf(x) * inv_scale;
    uint32_t code;
    if (a < 2.f) code = (uint32_t)(int)rintf(a * 8.f);                       // 0..16 (16 = the first code of the next binade)
    else if (a < 4.f) code = 16u + (uint32_t)(int)rintf((a - 2.f) * 4.f);    // 16..24
    else code = 24u + (uint32_t)(int)rintf((fminf(a, 7.5f) - 4.f) * 2.f);    // 24..31
    return sign | code;
}

typedef __attribute__((__vector_size__(6 * sizeof(uint32_t)))) uint32_t lvr_u32x6;
typedef __attribute__((__vector_size__(32 * sizeof(float)))) float lvr_f32x32;

// CF = 1: the centre is stored as 128 e4m3 codes in the order the matrix-core operand wants them
// (byte kq*32 + kk*8 + j holds coordinate kk*32 + kq*8 + j); only for bf16 caches.
// CF = 2: as 128 e2m3 codes of 6 bits in the same order (bits 6 (kk*8 + j) .. of the 24 bytes at kq*24), times
// one power-of-two scale per kq: the 32 coordinates of a scale block are the ones a lane of the query
// kernel holds.  The scale is the smallest power of two that brings the block's largest magnitude to
// at most 7.5; its biased exponent byte goes into the group's record in `radii` (byte kq of the third word).
// chan_exp (CF = 2 only, may be NULL): 128 signed bytes at the start of every LVR_CHAN_STRIDE bytes, one set per
// (sequence, KV head); the index then describes the keys
// with coordinate c divided by 2^e_c: centre, codes and radii are all formed in that space (an exact rescaling: powers
// of two), and the query multiplies q_c by 2^e_c, which leaves every dot product as it was.
template <typename KT, int CF = 0>
__global__ void __launch_bounds__(256)
build_groups_kernel(void *__restrict__ K, void *__restrict__ centres, float *__restrict__ radii,
                    int64_t cap_rows, int64_t max_groups, int64_t g0, int64_t g1, int r, int S, const BuildSrc src,
                    const int8_t *__restrict__ chan_exp = nullptr) {
    const int bh = blockIdx.y;
    const int li = threadIdx.x & 15;
    int64_t g = g0 + (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
    const bool valid = g < g1;
    if (!valid) g = g0;   // keep every lane busy so the shuffles below see defined data
    char *Kb = static_cast<char *>(K) + (int64_t)bh * cap_rows * LVR_D * sizeof(KT);
    const bool from_src = src.base != nullptr;   // uniform
    const char *Sb = from_src ? src.base + ((int64_t)(bh / src.n_kv_heads) * src.sb + (int64_t)(bh % src.n_kv_heads) * src.sh) * (int64_t)sizeof(KT)
                              : Kb;
    const int64_t row_stride = from_src ? src.st * (int64_t)sizeof(KT) : (int64_t)LVR_D * (int64_t)sizeof(KT);

    float c[8];
    lvr_zero8(c);
    // groups of up to four rows stay in registers between the two passes over the members
    lvr_raw8<KT> keep[4];
    const bool kept = r <= 4;   // uniform
    if (kept) {
#pragma unroll
        for (int m = 0; m < 4; ++m)
            if (m < r) lvr_load_raw(Sb + (g * r + m) * row_stride, 0, li, keep[m]);
#pragma unroll
        for (int m = 0; m < 4; ++m) {       // members in ascending row order
            if (m < r) {
                float x[8];
                if (from_src && valid) lvr_store_raw(Kb, g * r + m, li, keep[m]);   // the arena's copy of the row
                lvr_unpack(keep[m], x);
#pragma unroll
                for (int e = 0; e < 8; ++e) c[e] += x[e];
            }
        }
    } else {
        for (int m = 0; m < r; ++m) {
            float x[8];
            lvr_raw8<KT> raw;
            lvr_load_raw(Sb + (g * r + m) * row_stride, 0, li, raw);
            if (from_src && valid) lvr_store_raw(Kb, g * r + m, li, raw);
            lvr_unpack(raw, x);
#pragma unroll
            for (int e = 0; e < 8; ++e) c[e] += x[e];
        }
    }
    const float inv = 1.0f / (float)r;
#pragma unroll
    for (int e = 0; e < 8; ++e) c[e] *= inv;
    float chs[8];   // 2^-e_c of this lane's eight coordinates
#pragma unroll
    for (int e = 0; e < 8; ++e) chs[e] = 1.0f;
    if constexpr (CF == 2) {
        if (chan_exp) {
            const int8_t *ce = chan_exp + (int64_t)bh * LVR_CHAN_STRIDE + li * 8;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                chs[e] = __uint_as_float((uint32_t)(127 - (int)ce[e]) << 23);
                c[e] *= chs[e];
            }
        }
    }

    constexpr bool CF8 = CF == 1;
    char *Cb = static_cast<char *>(centres) + ((int64_t)bh * max_groups + g) * (CF == 2 ? LVR_D * 3 / 4 : LVR_D * (CF8 ? 1 : sizeof(KT)));
    uint32_t scale_bytes = 0;   // CF = 2: the four blocks' exponent bytes (the same in all 16 lanes of the group)
    (void)scale_bytes;
    if constexpr (CF == 2) {
        float amax = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf(c[e]));
        amax = fmaxf(amax, __shfl_xor(amax, 4, 64));    // the lanes of a block: same li & 3
        amax = fmaxf(amax, __shfl_xor(amax, 8, 64));
        // smallest E with amax <= 7.5 * 2^E; held to [-100, 120] so that scale, its inverse and every decoded
        // value are normal numbers (a block beyond that saturates or rounds to zero; the radius measures it)
        int p;
        const float f = frexpf(amax, &p);   // amax = f * 2^p, f in [0.5, 1)
        int E = (amax > 0.f) ? (f <= 0.9375f ? p - 3 : p - 2) : -100;
        E = E < -100 ? -100 : (E > 120 ? 120 : E);
        const float scale = __uint_as_float((uint32_t)(E + 127) << 23), inv_scale = __uint_as_float((uint32_t)(127 - E) << 23);
        uint32_t code[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) code[e] = f32_to_e2m3(c[e], inv_scale);
        const uint32_t lo = code[0] | (code[1] << 6) | (code[2] << 12) | (code[3] << 18) | (code[4] << 24) | (code[5] << 30);
        const uint32_t hi = (code[5] >> 2) | (code[6] << 4) | (code[7] << 10);   // 16 bits
        // from here on: the centre as stored (decoded by the conversion the query kernel uses, in its fp32 form)
        const lvr_u32x6 src = {lo, hi, 0u, 0u, 0u, 0u};
        const lvr_f32x32 dec = __builtin_amdgcn_cvt_scalef32_pk32_f32_fp6(src, scale);
        c[0] = dec[0]; c[1] = dec[1]; c[2] = dec[2]; c[3] = dec[3];
        c[4] = dec[4]; c[5] = dec[5]; c[6] = dec[6]; c[7] = dec[7];
        if (valid) {
            uint16_t *dst = reinterpret_cast<uint16_t *>(Cb + (li & 3) * 24 + (li >> 2) * 6);
            dst[0] = (uint16_t)lo;
            dst[1] = (uint16_t)(lo >> 16);
            dst[2] = (uint16_t)hi;
        }
        const int lane = threadIdx.x & 63, base = lane & ~15;
#pragma unroll
        for (int b = 0; b < 4; ++b) scale_bytes |= (uint32_t)(__shfl(E, base + b, 64) + 127) << (8 * b);
    } else if constexpr (CF8) {
        uint32_t code[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) code[e] = f32_to_e4m3(c[e]);
        const uint32_t w0 = code[0] | (code[1] << 8) | (code[2] << 16) | (code[3] << 24);
        const uint32_t w1 = code[4] | (code[5] << 8) | (code[6] << 16) | (code[7] << 24);
        // from here on: the centre as stored (decoded by the same instruction the query kernel uses)
        const lvr_f32x2 d0 = __builtin_amdgcn_cvt_pk_f32_fp8((int)w0, false), d1 = __builtin_amdgcn_cvt_pk_f32_fp8((int)w0, true);
        const lvr_f32x2 d2 = __builtin_amdgcn_cvt_pk_f32_fp8((int)w1, false), d3 = __builtin_amdgcn_cvt_pk_f32_fp8((int)w1, true);
        c[0] = d0[0]; c[1] = d0[1]; c[2] = d1[0]; c[3] = d1[1];
        c[4] = d2[0]; c[5] = d2[1]; c[6] = d3[0]; c[7] = d3[1];
        if (valid) *reinterpret_cast<uint2 *>(Cb + (li & 3) * 32 + (li >> 2) * 8) = make_uint2(w0, w1);
    } else if constexpr (std::is_same<KT, lvr_bf16_t>::value) {
        uint32_t b[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            b[e] = lvr_f32_to_bf16_bits(c[e]);
            c[e] = __uint_as_float(b[e] << 16);   // from here on: the centre as stored
        }
        if (valid)
            reinterpret_cast<uint4 *>(Cb)[li] =
                make_uint4(b[0] | (b[1] << 16), b[2] | (b[3] << 16), b[4] | (b[5] << 16), b[6] | (b[7] << 16));
    } else {
        if (valid) {
            reinterpret_cast<float4 *>(Cb)[2 * li] = make_float4(c[0], c[1], c[2], c[3]);
            reinterpret_cast<float4 *>(Cb)[2 * li + 1] = make_float4(c[4], c[5], c[6], c[7]);
        }
    }

    const int lanes_per_sub = 16 / S;
    float cn2 = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) cn2 += c[e] * c[e];
    cn2 = seg_sum(cn2, lanes_per_sub);

    float max_d2 = 0.f;
    auto distance = [&](const float (&x)[8]) {
        float d2 = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float t = x[e] * chs[e] - c[e];
            d2 += t * t;
        }
        d2 = seg_sum(d2, lanes_per_sub);
        max_d2 = fmaxf(max_d2, d2);
    };
    if (kept) {
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            if (m < r) {            // uniform: every lane takes part in the reduction
                float x[8];
                lvr_unpack(keep[m], x);
                distance(x);
            }
        }
    } else {
        for (int m = 0; m < r; ++m) {
            float x[8];
            lvr_load8<KT>(Sb + (g * r + m) * row_stride, 0, li, x);
            distance(x);
        }
    }
    float rho = sqrtf(max_d2) * (1.0f + 0x1p-12f) + sqrtf(cn2) * 0x1p-12f;
    rho = __uint_as_float(__float_as_uint(rho) + 1u);    // one ulp up (rho >= 0)
    if constexpr (CF != 0) {
        // The radii go out in the form the query's radius step reads them: four bf16 per group (8 bytes),
        // slot s = rho_s rounded UP to bf16's eight significant bits (looser by at most 2^-7 rho_s, never
        // tighter), slots S..3 zero.
        uint32_t slot[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) slot[k] = 0;
        const int lane = threadIdx.x & 63, base = lane & ~15;
        for (int sidx = 0; sidx < S; ++sidx) {   // S <= 4
            const float rs = __shfl(rho, base + sidx * lanes_per_sub, 64);
            uint32_t up = __float_as_uint(rs);
            if (up & 0xffffu) up = (up & 0xffff0000u) + 0x10000u;
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (k == sidx) slot[k] = up >> 16;
        }
        if constexpr (CF == 2) {   // 12-byte record: the radii, then the scale bytes
            if (valid && li == 0) {
                uint32_t *rec = reinterpret_cast<uint32_t *>(radii) + ((int64_t)bh * max_groups + g) * 3;
                rec[0] = slot[0] | (slot[1] << 16);
                rec[1] = slot[2] | (slot[3] << 16);
                rec[2] = scale_bytes;
            }
        } else if (valid && li == 0)
            reinterpret_cast<uint2 *>(radii)[(int64_t)bh * max_groups + g] =
                make_uint2(slot[0] | (slot[1] << 16), slot[2] | (slot[3] << 16));
    } else {
        if (valid && (li % lanes_per_sub) == 0) radii[((int64_t)bh * max_groups + g) * S + li / lanes_per_sub] = rho;
    }
}

// Axis-aligned box of every group (appendix "Ablation on Index Design", Def. 1): per coordinate the
// largest and the smallest member value, stored as two rows (upper corner, lower corner).  The
// corners are member values, so bf16 storage is exact.  The one float per group in `radii` is a
// rounding allowance for the bound  sum_c (q+_c hi_c + q-_c lo_c)  evaluated in fp32 over 256
// terms: 2^-15 * |a|_2 with a_c = max(|lo_c|, |hi_c|); times |q|_2 it exceeds the rounding error
// by Cauchy-Schwarz, so a computed bound never falls below a member's exact score.
// CF8: the corners are stored as e4m3 codes in matrix-operand order, the upper corner rounded up and
// the lower corner rounded down, so the stored box contains the exact one.  A member beyond +-448
// cannot be enclosed by a code; what sticks out (e_c per coordinate) is added to the allowance as
// |e|_2, which times |q|_2 exceeds sum_c |q_c| e_c.
template <bool CF8>
__global__ void __launch_bounds__(256)
build_boxes_kernel(void *__restrict__ K, void *__restrict__ corners, float *__restrict__ allowance,
                   int64_t cap_rows, int64_t max_groups, int64_t g0, int64_t g1, int r, const BuildSrc src) {
    const int bh = blockIdx.y;
    const int li = threadIdx.x & 15;
    int64_t g = g0 + (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
    const bool valid = g < g1;
    if (!valid) g = g0;
    char *Kb = static_cast<char *>(K) + (int64_t)bh * cap_rows * LVR_D * 2;
    const bool from_src = src.base != nullptr;   // uniform
    const char *Sb = from_src ? src.base + ((int64_t)(bh / src.n_kv_heads) * src.sb + (int64_t)(bh % src.n_kv_heads) * src.sh) * 2 : Kb;
    const int64_t row_stride = from_src ? src.st * 2 : (int64_t)LVR_D * 2;
    float lo[8], hi[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        lo[e] = INFINITY;
        hi[e] = -INFINITY;
    }
    for (int m = 0; m < r; ++m) {
        float x[8];
        lvr_raw8<lvr_bf16_t> raw;
        lvr_load_raw(Sb + (g * r + m) * row_stride, 0, li, raw);
        if (from_src && valid) lvr_store_raw(Kb, g * r + m, li, raw);   // the arena's copy of the row
        lvr_unpack(raw, x);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            lo[e] = fminf(lo[e], x[e]);
            hi[e] = fmaxf(hi[e], x[e]);
        }
    }
    float a2 = 0.f;
    if constexpr (CF8) {
        uint32_t ch[8], cl[8];
        float e2 = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            ch[e] = f32_to_e4m3_directed(hi[e], true);
            cl[e] = f32_to_e4m3_directed(lo[e], false);
            const float hd = e4m3_value(ch[e]), ld = e4m3_value(cl[e]);
            const float out = fmaxf(fmaxf(hi[e] - hd, ld - lo[e]), 0.f);   // non-zero only beyond +-448
            e2 += out * out;
            const float a = fmaxf(fabsf(ld), fabsf(hd));
            a2 += a * a;
        }
        a2 = seg_sum(a2, 16);
        e2 = seg_sum(e2, 16);
        if (valid) {
            char *dst = static_cast<char *>(corners) + ((int64_t)bh * max_groups + g) * 2 * LVR_D;
            const int at = (li & 3) * 32 + (li >> 2) * 8;
            *reinterpret_cast<uint2 *>(dst + at) = make_uint2(ch[0] | (ch[1] << 8) | (ch[2] << 16) | (ch[3] << 24),
                                                              ch[4] | (ch[5] << 8) | (ch[6] << 16) | (ch[7] << 24));
            *reinterpret_cast<uint2 *>(dst + LVR_D + at) = make_uint2(cl[0] | (cl[1] << 8) | (cl[2] << 16) | (cl[3] << 24),
                                                                      cl[4] | (cl[5] << 8) | (cl[6] << 16) | (cl[7] << 24));
            if (li == 0) {
                float al = sqrtf(a2) * 0x1p-15f + sqrtf(e2) * (1.0f + 0x1p-20f);
                allowance[(int64_t)bh * max_groups + g] = __uint_as_float(__float_as_uint(al) + 1u);
            }
        }
        return;
    }
    uint32_t bh_[8], bl_[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float a = fmaxf(fabsf(lo[e]), fabsf(hi[e]));
        a2 += a * a;
        bh_[e] = __float_as_uint(hi[e]) >> 16;   // exact: the values are bf16 already
        bl_[e] = __float_as_uint(lo[e]) >> 16;
    }
    a2 = seg_sum(a2, 16);
    if (valid) {
        uint4 *dst = reinterpret_cast<uint4 *>(static_cast<char *>(corners) +
                                               ((int64_t)bh * max_groups + g) * 2 * LVR_D * 2);
        dst[li] = make_uint4(bh_[0] | (bh_[1] << 16), bh_[2] | (bh_[3] << 16), bh_[4] | (bh_[5] << 16),
                             bh_[6] | (bh_[7] << 16));
        dst[16 + li] = make_uint4(bl_[0] | (bl_[1] << 16), bl_[2] | (bl_[3] << 16), bl_[4] | (bl_[5] << 16),
                                  bl_[6] | (bl_[7] << 16));
        if (li == 0) {
            float al = sqrtf(a2) * 0x1p-15f;
            allowance[(int64_t)bh * max_groups + g] = __uint_as_float(__float_as_uint(al) + 1u);
        }
    }
}

// Identity position map for rows [row0, row0+rows) (used when rows are stored in arrival order
// but a map is kept, i.e. the buffer of a regrouped arena).
__global__ void iota_rows_kernel(int32_t *slot_pos, int32_t *pos_slot, int64_t cap_rows, int64_t row0, int64_t rows) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= rows) return;
    int64_t o = (int64_t)blockIdx.y * cap_rows + row0 + i;
    slot_pos[o] = (int32_t)(row0 + i);
    pos_slot[o] = (int32_t)(row0 + i);
}

}  // namespace

hipError_t lvr_launch_copy_kv(lvr_index *ix, const void *K, const int64_t ks[3], const void *V, const int64_t vs[3],
                              int64_t dst_row0, int64_t rows, hipStream_t st, int64_t k_first) {
    if (rows <= 0) return hipSuccess;
    const int row_bytes = (int)(LVR_D * ix->elt);
    const int64_t total = rows * (row_bytes / 16);
    dim3 grid((unsigned)((total + 255) / 256), (unsigned)lvr_n_bh(ix), 2);
    // k_first > 0: the leading key rows are written by the build kernel that reads them from the caller's K
    CopySide k{static_cast<const char *>(K), static_cast<char *>(ix->K), ks[0], ks[1], ks[2], k_first};
    CopySide v{static_cast<const char *>(V), static_cast<char *>(ix->V), vs[0], vs[1], vs[2], 0};
    hipLaunchKernelGGL(copy_rows_kernel, grid, dim3(256), 0, st, k, v, ix->cfg.n_kv_heads, ix->cap_rows, dst_row0, rows,
                       row_bytes, (int)ix->elt);
    return hipGetLastError();
}

hipError_t lvr_launch_build_groups(lvr_index *ix, int64_t g0, int64_t g1, hipStream_t st, const void *K_src,
                                   const int64_t *ks) {
    if (g1 <= g0) return hipSuccess;
    dim3 grid((unsigned)((g1 - g0 + 15) / 16), (unsigned)lvr_n_bh(ix));
    // K_src: the groups' rows come from the caller's K (element strides ks) and are copied into the arena on the way
    BuildSrc src{static_cast<const char *>(K_src), K_src ? ks[0] : 0, K_src ? ks[1] : 0, K_src ? ks[2] : 0, ix->cfg.n_kv_heads};
    if (ix->box) {
        if (ix->cf8)
            hipLaunchKernelGGL(build_boxes_kernel<true>, grid, dim3(256), 0, st, ix->K, ix->centres, ix->radii, ix->cap_rows,
                               ix->max_groups, g0, g1, ix->cfg.group_size, src);
        else
            hipLaunchKernelGGL(build_boxes_kernel<false>, grid, dim3(256), 0, st, ix->K, ix->centres, ix->radii, ix->cap_rows,
                               ix->max_groups, g0, g1, ix->cfg.group_size, src);
        return hipGetLastError();
    }
    if (ix->cf6)
        hipLaunchKernelGGL((build_groups_kernel<lvr_bf16_t, 2>), grid, dim3(256), 0, st, ix->K, ix->centres, ix->radii,
                           ix->cap_rows, ix->max_groups, g0, g1, ix->cfg.group_size, ix->cfg.n_subspaces, src,
                           ix->chan_scaled ? lvr_chan_exp(ix) : nullptr);
    else if (ix->cf8)
        hipLaunchKernelGGL((build_groups_kernel<lvr_bf16_t, 1>), grid, dim3(256), 0, st, ix->K, ix->centres, ix->radii,
                           ix->cap_rows, ix->max_groups, g0, g1, ix->cfg.group_size, ix->cfg.n_subspaces, src);
    else if (ix->cfg.kv_dtype == LVR_BF16)
        hipLaunchKernelGGL(build_groups_kernel<lvr_bf16_t>, grid, dim3(256), 0, st, ix->K, ix->centres, ix->radii,
                           ix->cap_rows, ix->max_groups, g0, g1, ix->cfg.group_size, ix->cfg.n_subspaces, src);
    else
        hipLaunchKernelGGL(build_groups_kernel<lvr_f32_t>, grid, dim3(256), 0, st, ix->K, ix->centres, ix->radii,
                           ix->cap_rows, ix->max_groups, g0, g1, ix->cfg.group_size, ix->cfg.n_subspaces, src);
    return hipGetLastError();
}

// Channel exponents of a (sequence, KV head): with L_c = log2(rms of coordinate c) over a sample of the rows,
// e_c = round(L_c - o), held to [-8, 8]; a coordinate that is zero throughout keeps e_c = 0.  The offset o (the same for
// all 128 channels, so it only moves the block scales) is the circular mean of the fractional parts of L_c: channels of
// about the same size then sit in the middle of one rounding interval and get the same exponent, instead of being split
// by a boundary that happens to fall among them.  One workgroup per (sequence, KV head), thread t takes coordinate
// t % 128 of every second sampled row.  Any exponents give a correct index (the radii are measured in the rescaled space
// against the centres as stored there); these make the coordinates of a key comparable in size, so that the 32
// coordinates that share a scale in the 6-bit code are not drowned by one large channel.
__global__ void __launch_bounds__(256)
channel_scale_kernel(const char *__restrict__ K, int64_t sb, int64_t sh, int64_t stt, int n_kv_heads, int64_t n, int64_t step,
                     int8_t *__restrict__ chan_exp) {
    __shared__ float s_sum[2][LVR_D];
    const int bh = blockIdx.x;
    const int c = threadIdx.x & (LVR_D - 1), half = threadIdx.x >> 7;
    const uint16_t *base = reinterpret_cast<const uint16_t *>(K) + (int64_t)(bh / n_kv_heads) * sb + (int64_t)(bh % n_kv_heads) * sh;
    float ss = 0.f;
    for (int64_t row = half * step; row < n; row += 2 * step) {
        const float x = __uint_as_float((uint32_t)base[row * stt + c] << 16);
        ss += x * x;
    }
    s_sum[half][c] = ss;
    __syncthreads();
    const int64_t rows = (n + step - 1) / step;
    const float ms = (s_sum[0][c] + s_sum[1][c]) / (float)(rows > 0 ? rows : 1);
    const bool live = ms > 0.f && ms < INFINITY;
    const float L = live ? 0.5f * log2f(ms) : 0.f;
    __syncthreads();
    constexpr float kTwoPi = 6.283185307179586f;
    if (half == 0) {
        s_sum[0][c] = live ? cosf(kTwoPi * L) : 0.f;
        s_sum[1][c] = live ? sinf(kTwoPi * L) : 0.f;
    }
    __syncthreads();
    if (half == 0) {
        float sc = 0.f, sn = 0.f;
        for (int i = 0; i < LVR_D; ++i) {   // the same order in every thread: one offset for the head
            sc += s_sum[0][i];
            sn += s_sum[1][i];
        }
        const float o = (sc != 0.f || sn != 0.f) ? atan2f(sn, sc) / kTwoPi : 0.f;
        int e = 0;
        if (live) {
            e = (int)rintf(L - o);
            e = e < -8 ? -8 : (e > 8 ? 8 : e);
        }
        int8_t *mine = chan_exp + (int64_t)bh * LVR_CHAN_STRIDE;
        mine[c] = (int8_t)e;
        reinterpret_cast<float *>(mine + LVR_D)[c] = __uint_as_float((uint32_t)(127 + e) << 23);
    }
}

hipError_t lvr_launch_channel_scales(lvr_index *ix, const void *K, const int64_t ks[3], int64_t n, hipStream_t st) {
    if (!ix->chan_scaled || n <= 0) return hipSuccess;
    const int64_t step = (n + 4095) / 4096;   // at most 4096 rows are looked at
    hipLaunchKernelGGL(channel_scale_kernel, dim3((unsigned)lvr_n_bh(ix)), dim3(256), 0, st, static_cast<const char *>(K), ks[0],
                       ks[1], ks[2], ix->cfg.n_kv_heads, n, step, lvr_chan_exp(ix));
    return hipGetLastError();
}

hipError_t lvr_launch_iota_rows(lvr_index *ix, int64_t row0, int64_t rows, hipStream_t st) {
    if (rows <= 0 || !ix->slot_pos) return hipSuccess;
    dim3 grid((unsigned)((rows + 255) / 256), (unsigned)lvr_n_bh(ix));
    hipLaunchKernelGGL(iota_rows_kernel, grid, dim3(256), 0, st, ix->slot_pos, ix->pos_slot, ix->cap_rows, row0, rows);
    return hipGetLastError();
}
