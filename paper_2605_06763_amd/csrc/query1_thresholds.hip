// Per-subspace thresholds for "Query 1" (Sec. 4.2, Alg. 3) derived from tau alone.
//
// Query 1 is correct when tau_s is a lower bound on <pi_s q, pi_s k> for every relevant key.  With
// only tau given, the relevant keys are those with <q,k> >= tau.  The dot product is the sum of its
// subspace terms, and the term of subspace t never exceeds M_t = max over groups of the ball bound
// f_{t,g} = <pi_t q, c_{t,g}> + rho_{t,g} |pi_t q| (Eq. (2)); so every such key has
//     <pi_s q, pi_s k>  >=  tau - sum_{t != s} M_t  =: tau_s.
// One pass over the index finds M (two launches: per-workgroup maxima, then the thresholds).
// The radii are stored widened by more than the rounding error of this fp32 evaluation, so a
// computed f never falls below a member's exact subspace term.
#include "lvr_internal.h"

namespace {

typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;

__device__ __forceinline__ float seg_sum16(float v, int lanes_per_sub) {
    for (int off = 1; off < lanes_per_sub; off <<= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// grid (NB, batch * n_kv_heads), 256 threads: 16 quarter waves, one group per quarter per trip.
// Lane li of a quarter holds coordinates 8 li .. 8 li + 7, all inside subspace li / (16 / S).
// part: [batch * n_kv_heads][NB][G][S] maxima of this workgroup's groups.
// BOX: two rows per group (upper corner, lower corner); the block's bound is sum_c max(q_c lo_c, q_c hi_c)
// over the block's coordinates plus the group's allowance times the norm of the whole query.
// CF: 0 centres in the cache's format, 1 e4m3 codes, 2 e2m3 codes with a scale per lane piece (balls only)
template <int G, int CF, bool BOX = false>
__global__ void __launch_bounds__(256)
subspace_max_kernel(const void *__restrict__ centres, const float *__restrict__ radii, const float *__restrict__ q,
                    float *__restrict__ part, int64_t max_groups, int64_t n_groups, int S, int n_kv_heads, int n_q_heads,
                    const int8_t *__restrict__ chan_exp = nullptr) {
    __shared__ float s_m[16][G][16];
    const int bh = blockIdx.y, b = bh / n_kv_heads, hkv = bh % n_kv_heads;
    const int quarter = threadIdx.x >> 4, li = threadIdx.x & 15;
    const int lanes_per_sub = 16 / S, s_l = li / lanes_per_sub;
    float qv[G][8], qn[G], m[G];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        const float *qh = q + ((int64_t)b * n_q_heads + hkv * G + h) * LVR_D + li * 8;
        float n2 = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            qv[h][e] = qh[e];
            // a 6-bit index in a rescaled space (coordinate c of the keys divided by 2^e_c): q_c times 2^e_c
            if (CF == 2 && chan_exp) qv[h][e] *= __uint_as_float((uint32_t)(127 + (int)chan_exp[(int64_t)bh * LVR_CHAN_STRIDE + li * 8 + e]) << 23);
            n2 += qv[h][e] * qv[h][e];
        }
        // rounded up a little: the norm multiplies a non-negative radius in an upper bound
        qn[h] = sqrtf(seg_sum16(n2, BOX ? 16 : lanes_per_sub)) * (1.0f + 0x1p-20f);
        m[h] = -INFINITY;
    }
    constexpr bool CF8 = CF == 1;
    const char *Cb = static_cast<const char *>(centres) + (int64_t)bh * max_groups * (CF == 2 ? LVR_D * 3 / 4 : LVR_D * (CF8 ? 1 : 2)) * (BOX ? 2 : 1);
    auto load_row = [&](int64_t row, float (&x)[8]) {
        if constexpr (CF == 2) {
            // 96 bytes per row: coordinates 8 li .. 8 li + 7 are the 48 bits at (li & 3) * 24 + (li >> 2) * 6, six
            // bits per code; their scale is byte li & 3 of the third word of the group's record in `radii`
            const uint16_t *p = reinterpret_cast<const uint16_t *>(Cb + row * (LVR_D * 3 / 4) + (li & 3) * 24 + (li >> 2) * 6);
            const uint64_t bits = (uint64_t)p[0] | ((uint64_t)p[1] << 16) | ((uint64_t)p[2] << 32);
            const uint32_t sb = (reinterpret_cast<const uint32_t *>(radii)[((int64_t)bh * max_groups + row) * 3 + 2] >> (8 * (li & 3))) & 0xffu;
            const float scale = __uint_as_float(sb << 23);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t code = (uint32_t)(bits >> (6 * e)) & 63u;
                const uint32_t ex = (code >> 3) & 3u, m = code & 7u;
                // magnitudes m/8 (ex = 0) or (1 + m/8) 2^(ex-1): all exact in fp32, and so is the product with the scale
                const float mag = ex == 0 ? (float)m * 0.125f : (1.0f + (float)m * 0.125f) * (float)(1u << (ex - 1));
                x[e] = (code & 32u) ? -mag * scale : mag * scale;
            }
        } else if constexpr (CF8) {
            // 128 e4m3 codes per row in matrix-operand order: coordinates 8 li .. 8 li + 7 are the
            // eight bytes at (li & 3) * 32 + (li >> 2) * 8
            const uint2 w = *reinterpret_cast<const uint2 *>(Cb + row * LVR_D + (li & 3) * 32 + (li >> 2) * 8);
            const f32x2 d0 = __builtin_amdgcn_cvt_pk_f32_fp8((int)w.x, false), d1 = __builtin_amdgcn_cvt_pk_f32_fp8((int)w.x, true);
            const f32x2 d2 = __builtin_amdgcn_cvt_pk_f32_fp8((int)w.y, false), d3 = __builtin_amdgcn_cvt_pk_f32_fp8((int)w.y, true);
            x[0] = d0[0]; x[1] = d0[1]; x[2] = d1[0]; x[3] = d1[1];
            x[4] = d2[0]; x[5] = d2[1]; x[6] = d3[0]; x[7] = d3[1];
        } else {
            lvr_load8<lvr_bf16_t>(Cb, row, li, x);
        }
    };
    const int64_t trips = (n_groups + 16 * (int64_t)gridDim.x - 1) / (16 * (int64_t)gridDim.x);
    for (int64_t it = 0; it < trips; ++it) {        // the same trip count for every lane: the shuffles stay convergent
        int64_t g = (it * gridDim.x + blockIdx.x) * 16 + quarter;
        const bool valid = g < n_groups;
        if (!valid) g = 0;
        float x[8], x2[8], rho;
        (void)x2;
        if constexpr (BOX) {
            load_row(2 * g, x);        // upper corner
            load_row(2 * g + 1, x2);   // lower corner
            rho = radii[(int64_t)bh * max_groups + g];
        } else if constexpr (CF != 0) {
            load_row(g, x);
            // radii as four bf16 per group: slot s = rho_s (records of 8 bytes, or 12 with the scale bytes of 6-bit centres)
            const uint16_t *rb = reinterpret_cast<const uint16_t *>(radii) + ((int64_t)bh * max_groups + g) * (CF == 2 ? 6 : 4);
            rho = __uint_as_float((uint32_t)rb[s_l] << 16);
        } else {
            load_row(g, x);
            rho = radii[((int64_t)bh * max_groups + g) * S + s_l];
        }
#pragma unroll
        for (int h = 0; h < G; ++h) {
            float p = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                if constexpr (BOX) p += fmaxf(qv[h][e] * x[e], qv[h][e] * x2[e]);
                else p += qv[h][e] * x[e];
            }
            const float f = seg_sum16(p, lanes_per_sub) + rho * qn[h];
            if (valid) m[h] = fmaxf(m[h], f);
        }
    }
#pragma unroll
    for (int h = 0; h < G; ++h) s_m[quarter][h][li] = m[h];
    __syncthreads();
    if (threadIdx.x < G * 16) {
        const int h = threadIdx.x >> 4;
        float v = s_m[0][h][li];
        for (int k = 1; k < 16; ++k) v = fmaxf(v, s_m[k][h][li]);
        if (li % lanes_per_sub == 0) part[(((int64_t)bh * gridDim.x + blockIdx.x) * G + h) * S + s_l] = v;
    }
}

// One thread per (query head, subspace).
__global__ void safe_tau_s_kernel(const float *__restrict__ part, const float *__restrict__ tau, float *__restrict__ tau_s,
                                  int NB, int G, int S, int n_kv_heads, int n_q_heads, int64_t total) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int s = (int)(i % S);
    const int64_t hq = i / S;
    if (NB == 0) {           // no groups: nothing to prune
        tau_s[i] = -INFINITY;
        return;
    }
    const int b = (int)(hq / n_q_heads), h = (int)(hq % n_q_heads);
    const int bh = b * n_kv_heads + h / G, hg = h % G;
    const float t = tau[hq];
    float others = 0.f, mag = fabsf(t);
    for (int u = 0; u < S; ++u) {
        if (u == s) continue;
        float mx = -INFINITY;
        for (int k = 0; k < NB; ++k) mx = fmaxf(mx, part[(((int64_t)bh * NB + k) * G + hg) * S + u]);
        others += mx;
        mag += fabsf(mx);
    }
    // the two roundings of this subtraction stay far inside the allowance
    tau_s[i] = (t == -INFINITY) ? t : (t - others) - 0x1p-20f * mag;
}

template <int G>
void launch_max(lvr_index *ix, const float *q, float *part, int NB, int64_t n_groups, hipStream_t st) {
    dim3 grid((unsigned)NB, (unsigned)lvr_n_bh(ix));
    if (ix->cf6)
        hipLaunchKernelGGL((subspace_max_kernel<G, 2>), grid, dim3(256), 0, st, ix->centres, ix->radii, q, part,
                           ix->max_groups, n_groups, ix->cfg.n_subspaces, ix->cfg.n_kv_heads, ix->cfg.n_q_heads,
                           ix->chan_scaled ? lvr_chan_exp(ix) : nullptr);
    else if (ix->box && ix->cf8)
        hipLaunchKernelGGL((subspace_max_kernel<G, 1, true>), grid, dim3(256), 0, st, ix->centres, ix->radii, q, part,
                           ix->max_groups, n_groups, ix->cfg.n_subspaces, ix->cfg.n_kv_heads, ix->cfg.n_q_heads);
    else if (ix->box)
        hipLaunchKernelGGL((subspace_max_kernel<G, 0, true>), grid, dim3(256), 0, st, ix->centres, ix->radii, q, part,
                           ix->max_groups, n_groups, ix->cfg.n_subspaces, ix->cfg.n_kv_heads, ix->cfg.n_q_heads);
    else if (ix->cf8)
        hipLaunchKernelGGL((subspace_max_kernel<G, 1>), grid, dim3(256), 0, st, ix->centres, ix->radii, q, part,
                           ix->max_groups, n_groups, ix->cfg.n_subspaces, ix->cfg.n_kv_heads, ix->cfg.n_q_heads);
    else
        hipLaunchKernelGGL((subspace_max_kernel<G, 0>), grid, dim3(256), 0, st, ix->centres, ix->radii, q, part,
                           ix->max_groups, n_groups, ix->cfg.n_subspaces, ix->cfg.n_kv_heads, ix->cfg.n_q_heads);
}

}  // namespace

// Callers guarantee: bf16 cache; 8-bit index rows and boxes only with S <= 4.  The per-workgroup maxima go through the
// attention's partial-output buffer (at least 512 floats per query head), which no launch in flight
// on the same stream still needs once this one runs.
hipError_t lvr_launch_safe_tau_s(lvr_index *ix, const float *q, const float *tau, float *tau_s, hipStream_t st) {
    const int S = ix->cfg.n_subspaces, G = ix->G;
    const int64_t n_groups = ix->n_indexed / ix->cfg.group_size;
    int64_t nb = (n_groups + 15) / 16;
    if (nb > 512 / S) nb = 512 / S;  // NB * G * S floats per KV head must fit G * 512
    const int NB = (int)nb;
    if (NB > 0) {
        switch (G) {
            case 1: launch_max<1>(ix, q, ix->part_o, NB, n_groups, st); break;
            case 2: launch_max<2>(ix, q, ix->part_o, NB, n_groups, st); break;
            case 4: launch_max<4>(ix, q, ix->part_o, NB, n_groups, st); break;
            default: launch_max<8>(ix, q, ix->part_o, NB, n_groups, st); break;
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    const int64_t total = (int64_t)lvr_n_bhq(ix) * S;
    hipLaunchKernelGGL(safe_tau_s_kernel, dim3((unsigned)((total + 63) / 64)), dim3(64), 0, st, ix->part_o, tau, tau_s, NB,
                       G, S, ix->cfg.n_kv_heads, ix->cfg.n_q_heads, total);
    return hipGetLastError();
}
