// Grouping by a balanced axis-median tree (Sec. 4.1 "Grouping via balanced PCA trees", Alg. 2):
// starting from all keys, a node is split at the median of the coordinate axis of largest
// variance until a node holds r keys.  One tree over the full key is shared by all coordinate
// blocks, and the rows are stored regrouped, so the query kernels see the same layout as with
// contiguous grouping: group g = arena rows g*r .. g*r+r-1, plus a map slot -> token position.
//
// Level-synchronous construction.  The number of groups is padded to a power of two with
// virtual keys that compare greater than every real key; they drift to the right end, so the
// real keys always fill a prefix of full groups (for a power-of-two number of groups, which
// is what every workload here has, there is no padding and the splits are exactly Alg. 2's
// floor(m/2) medians).  At level L every node is an aligned run of n'/2^L entries of the
// current order; per level:
//   1. per node, variance of each of the 128 coordinates over its real keys -> axis of the
//      largest variance (first axis wins a tie);
//   2. one 64-bit key per entry:  [ node | coordinate on the node's axis | position ]  with the
//      coordinate mapped to an order-preserving unsigned code; because the position is part of
//      the key, equal coordinates are ordered by position (Alg. 2 is silent; this is the rule
//      the CPU reference uses) and the sort needs no values;
//   3. a device-wide radix sort of the keys (rocPRIM: a plain library sort).
// After the last level the low bits of the sorted keys are the slot -> position map.
// Only the levels whose nodes exceed 1024 entries go through steps 1-3; the levels below are finished
// by tree_small_kernel in one launch, a workgroup per node with the node's order in LDS.
#include <rocprim/device/device_radix_sort.hpp>

#include "lvr_internal.h"

namespace {

constexpr int PIECE = 1024;   // rows per partial-statistics piece for nodes larger than this

struct TreeSrc {
    const char *K;             // source key rows
    int64_t sb, sh, st;        // element strides (batch, head, token)
    int elt, n_kv_heads;
    __device__ __forceinline__ const char *row(int bh, int64_t pos) const {
        const int b = bh / n_kv_heads, h = bh % n_kv_heads;
        return K + (b * sb + h * sh + pos * st) * elt;
    }
};

// entry i of (bh): low `pos_bits` bits of keys[bh*np + i] hold the position; >= n_real is padding
__device__ __forceinline__ int64_t key_pos(uint64_t k, int pos_bits) { return (int64_t)(k & ((1ull << pos_bits) - 1ull)); }

__global__ void tree_init_kernel(uint64_t *keys, int64_t np) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < np) keys[(int64_t)blockIdx.y * np + i] = (uint64_t)i;
}

// lane owns channels 2*lane, 2*lane+1 of a row
__device__ __forceinline__ void lane_pair(const char *row, int lane, int elt, float &x0, float &x1) {
    if (elt == 2) {
        const uint32_t w = reinterpret_cast<const uint32_t *>(row)[lane];
        x0 = __uint_as_float(w << 16);
        x1 = __uint_as_float(w & 0xffff0000u);
    } else {
        const float2 v = reinterpret_cast<const float2 *>(row)[lane];
        x0 = v.x;
        x1 = v.y;
    }
}

// argmax over 128 channel variances held as (v0, v1) per lane; lowest channel wins ties
// [c_lo, c_hi): the coordinates that may be chosen (a tree over one coordinate block looks at that block only)
__device__ __forceinline__ int wave_argmax(double v0, double v1, int lane, int c_lo, int c_hi) {
    if (2 * lane < c_lo || 2 * lane >= c_hi) v0 = -1.0;           // variances are >= 0
    if (2 * lane + 1 < c_lo || 2 * lane + 1 >= c_hi) v1 = -1.0;
    double best = v0;
    int arg = 2 * lane;
    if (v1 > best) { best = v1; arg = 2 * lane + 1; }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const double ob = __shfl_xor(best, off, 64);
        const int oa = __shfl_xor(arg, off, 64);
        if (ob > best || (ob == best && oa < arg)) { best = ob; arg = oa; }
    }
    return arg;
}

// Nodes of at most PIECE entries: one wave per node, sums taken relative to the node's first
// real key (the variance does not depend on the shift; the shift removes the cancellation).
__global__ void __launch_bounds__(256)
tree_stats_small_kernel(TreeSrc src, const uint64_t *__restrict__ keys, int32_t *__restrict__ axis, int64_t np,
                        int64_t n_real, int64_t m, int pos_bits, int64_t n_nodes, int c_lo, int c_hi) {
    const int lane = threadIdx.x & 63;
    const int64_t node = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int bh = blockIdx.y;
    if (node >= n_nodes) return;
    const uint64_t *kk = keys + (int64_t)bh * np + node * m;
    double s0 = 0., s1 = 0., q0 = 0., q1 = 0.;
    float p0 = 0.f, p1 = 0.f;
    int cnt = 0;
    for (int64_t i = 0; i < m; ++i) {
        const int64_t pos = key_pos(kk[i], pos_bits);
        if (pos >= n_real) continue;   // uniform over the wave
        float x0, x1;
        lane_pair(src.row(bh, pos), lane, src.elt, x0, x1);
        if (cnt == 0) { p0 = x0; p1 = x1; }
        const double d0 = (double)x0 - (double)p0, d1 = (double)x1 - (double)p1;
        s0 += d0; s1 += d1; q0 += d0 * d0; q1 += d1 * d1;
        ++cnt;
    }
    const double inv = cnt > 0 ? 1.0 / (double)cnt : 0.;
    const double v0 = (q0 - s0 * s0 * inv) * inv, v1 = (q1 - s1 * s1 * inv) * inv;
    const int arg = wave_argmax(v0, v1, lane, c_lo, c_hi);
    if (lane == 0) axis[(int64_t)bh * n_nodes + node] = arg;
}

// Nodes larger than PIECE: partial sums per piece of PIECE entries (shifted by the node's first
// key), then one 128-thread block per node adds the pieces in fp64.
__global__ void __launch_bounds__(256)
tree_stats_piece_kernel(TreeSrc src, const uint64_t *__restrict__ keys, double *__restrict__ partial, int64_t np,
                        int64_t n_real, int64_t m, int pos_bits) {
    __shared__ double sm[4][2][128];
    __shared__ int sc[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int bh = blockIdx.y;
    const int64_t piece = blockIdx.x;
    const int64_t first = piece * PIECE;
    const int64_t node0 = (first / m) * m;
    const uint64_t *kk = keys + (int64_t)bh * np;
    float p0 = 0.f, p1 = 0.f;
    {
        const int64_t ppos = key_pos(kk[node0], pos_bits);   // first entry of the node; real unless the node is all padding
        if (ppos < n_real) lane_pair(src.row(bh, ppos), lane, src.elt, p0, p1);
    }
    double s0 = 0., s1 = 0., q0 = 0., q1 = 0.;
    int cnt = 0;
    for (int64_t i = first + wave; i < first + PIECE; i += 4) {
        const int64_t pos = key_pos(kk[i], pos_bits);
        if (pos >= n_real) continue;
        float x0, x1;
        lane_pair(src.row(bh, pos), lane, src.elt, x0, x1);
        const double d0 = (double)x0 - (double)p0, d1 = (double)x1 - (double)p1;
        s0 += d0; s1 += d1; q0 += d0 * d0; q1 += d1 * d1;
        ++cnt;
    }
    sm[wave][0][2 * lane] = s0; sm[wave][0][2 * lane + 1] = s1;
    sm[wave][1][2 * lane] = q0; sm[wave][1][2 * lane + 1] = q1;
    if (lane == 0) sc[wave] = cnt;
    __syncthreads();
    const int t = threadIdx.x;
    double *out = partial + ((int64_t)bh * (np / PIECE) + piece) * 258;
    if (t < 128) {
        out[t] = sm[0][0][t] + sm[1][0][t] + sm[2][0][t] + sm[3][0][t];
        out[128 + t] = sm[0][1][t] + sm[1][1][t] + sm[2][1][t] + sm[3][1][t];
    }
    if (t == 0) out[256] = (double)(sc[0] + sc[1] + sc[2] + sc[3]);
}

__global__ void __launch_bounds__(128)
tree_stats_merge_kernel(const double *__restrict__ partial, int32_t *__restrict__ axis, int64_t np, int64_t m,
                        int64_t n_nodes, int c_lo, int c_hi) {
    __shared__ double sv[128];
    __shared__ int sa[128];
    const int bh = blockIdx.y, t = threadIdx.x;
    const int64_t node = blockIdx.x;
    const int64_t pieces = m / PIECE;
    const double *pp = partial + ((int64_t)bh * (np / PIECE) + node * pieces) * 258;
    double s = 0.0, q = 0.0, cnt = 0.0;
    for (int64_t p = 0; p < pieces; ++p) {
        s += pp[p * 258 + t];
        q += pp[p * 258 + 128 + t];
        cnt += pp[p * 258 + 256];
    }
    const double var = cnt > 0 ? (q - s * s / cnt) / cnt : 0.0;
    sv[t] = (t >= c_lo && t < c_hi) ? var : -1.0;   // coordinates outside the block are never chosen
    sa[t] = t;
    __syncthreads();
    for (int off = 64; off >= 1; off >>= 1) {
        if (t < off) {
            if (sv[t + off] > sv[t] || (sv[t + off] == sv[t] && sa[t + off] < sa[t])) {
                sv[t] = sv[t + off];
                sa[t] = sa[t + off];
            }
        }
        __syncthreads();
    }
    if (t == 0) axis[(int64_t)bh * n_nodes + node] = sa[0];
}

// key = [ global node | order-preserving code of the coordinate | position ]
__global__ void tree_keys_kernel(TreeSrc src, uint64_t *__restrict__ keys, const int32_t *__restrict__ axis,
                                 int64_t np, int64_t n_real, int64_t m, int pos_bits, int coord_bits,
                                 int64_t n_nodes) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= np) return;
    const int bh = blockIdx.y;
    uint64_t *kk = keys + (int64_t)bh * np;
    const int64_t pos = key_pos(kk[i], pos_bits);
    const int64_t node = i / m;
    uint64_t code;
    if (pos >= n_real) {
        code = (1ull << coord_bits) - 1ull;   // padding: after every real key
    } else {
        const int c = axis[(int64_t)bh * n_nodes + node];
        const char *row = src.row(bh, pos);
        if (src.elt == 2) {
            uint32_t u = static_cast<const uint16_t *>(static_cast<const void *>(row))[c];
            if (u == 0x8000u) u = 0;   // -0 and +0 are the same coordinate
            code = (u & 0x8000u) ? (~u & 0xffffu) : (u | 0x8000u);
        } else {
            uint32_t u = __float_as_uint(static_cast<const float *>(static_cast<const void *>(row))[c]);
            if (u == 0x80000000u) u = 0;
            code = (u & 0x80000000u) ? (uint64_t)(~u) : (uint64_t)(u | 0x80000000u);
        }
    }
    const uint64_t gnode = (uint64_t)bh * (uint64_t)n_nodes + (uint64_t)node;
    kk[i] = (gnode << (coord_bits + pos_bits)) | (code << pos_bits) | (uint64_t)pos;
}

// Rows into the arena in tree order, and the two position maps.  pos_base is added to the
// positions (a chunk's positions are relative to its first row).
__global__ void tree_gather_kernel(TreeSrc ksrc, TreeSrc vsrc, const uint64_t *__restrict__ keys, char *Kdst,
                                   char *Vdst, int32_t *slot_pos, int32_t *pos_slot, int64_t np, int64_t n_real,
                                   int pos_bits, int64_t cap_rows, int64_t row0, int row_bytes) {
    const int chunks = row_bytes / 16;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_real * chunks) return;
    const int bh = blockIdx.y;
    const int64_t slot = i / chunks;
    const int ch = (int)(i % chunks);
    const int64_t pos = key_pos(keys[(int64_t)bh * np + slot], pos_bits);
    const TreeSrc &s = blockIdx.z == 0 ? ksrc : vsrc;
    char *dst = blockIdx.z == 0 ? Kdst : Vdst;
    reinterpret_cast<uint4 *>(dst + ((int64_t)bh * cap_rows + row0 + slot) * row_bytes)[ch] =
        reinterpret_cast<const uint4 *>(s.row(bh, pos))[ch];
    if (blockIdx.z == 0 && ch == 0) {
        slot_pos[(int64_t)bh * cap_rows + row0 + slot] = (int32_t)(row0 + pos);
        pos_slot[(int64_t)bh * cap_rows + row0 + pos] = (int32_t)(row0 + slot);
    }
}

// Subtrees of at most TREE_WG_MAX padded entries: ALL their remaining levels in ONE launch, one
// 256-thread workgroup per subtree.  Either the whole tree of a small input (a buffer chunk of B
// keys: keys_in == NULL, one workgroup per (sequence, KV head)), or every node of the level at which
// the level-synchronous kernels above have brought the nodes down to TREE_WG_MAX entries (keys_in =
// the order so far; the node's entries are np consecutive ones).  Same steps as the level-synchronous
// kernels (same statistics in the same order, same keys), with the order kept in LDS and a bitonic
// sort in place of the device-wide radix sort; keys are unique, so any sort gives the same order.
// The node index inside the key is local to the subtree (only the position bits are read later).
constexpr int TREE_WG_MAX = 1024;

__global__ void __launch_bounds__(256)
tree_small_kernel(TreeSrc src, const uint64_t *__restrict__ keys_in, uint64_t *__restrict__ keys_out, int64_t np_total,
                  int np, int64_t n_real, int levels, int pos_bits, int coord_bits, int c_lo, int c_hi) {
    __shared__ uint64_t s_keys[TREE_WG_MAX];
    __shared__ int32_t s_axis[TREE_WG_MAX / 2];
    __shared__ double s_part[4][256];   // per run: 128 sums, 128 sums of squares
    __shared__ int s_cnt[4];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int bh = blockIdx.y;
    const int64_t base = (int64_t)bh * np_total + (int64_t)blockIdx.x * np;   // this subtree's entries
    for (int i = t; i < np; i += 256) s_keys[i] = keys_in ? (uint64_t)key_pos(keys_in[base + i], pos_bits) : (uint64_t)i;
    __syncthreads();
    for (int L = 0; L < levels; ++L) {
        const int n_nodes = 1 << L;
        const int m = np >> L;
        // 1. split axis of every node.  The entries of the level are dealt to the four waves in
        // runs of `run` consecutive entries (a whole node, or a quarter of a big one); each wave
        // sums its run relative to the node's first key, eight rows in flight at a time, and the
        // runs of a node are added in order.
        {
            const int run = (m >= 4 * 8) ? ((n_nodes >= 4) ? m : m / (4 / n_nodes)) : m;   // entries per run
            const int runs_per_node = m / run;
            const int n_runs = n_nodes * runs_per_node;
            for (int rix = wave; rix < n_runs; rix += 4) {
                const int node = rix / runs_per_node;
                const uint64_t *kk = s_keys + node * m;
                const int i_begin = (rix % runs_per_node) * run;
                const int64_t ppos = key_pos(kk[0], pos_bits);   // padding sorts last: entry 0 is real unless all are padding
                float p0 = 0.f, p1 = 0.f;
                if (ppos < n_real) lane_pair(src.row(bh, ppos), lane, src.elt, p0, p1);
                double s0 = 0., s1 = 0., q0 = 0., q1 = 0.;
                int cnt = 0;
                for (int i0 = i_begin; i0 < i_begin + run; i0 += 8) {
                    float x0[8], x1[8];
                    bool real[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const int64_t pos = (i0 + u < i_begin + run) ? key_pos(kk[i0 + u], pos_bits) : n_real;
                        real[u] = pos < n_real;
                        lane_pair(src.row(bh, real[u] ? pos : (ppos < n_real ? ppos : 0)), lane, src.elt, x0[u], x1[u]);
                    }
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const double d0 = real[u] ? (double)x0[u] - (double)p0 : 0.;
                        const double d1 = real[u] ? (double)x1[u] - (double)p1 : 0.;
                        s0 += d0; s1 += d1; q0 += d0 * d0; q1 += d1 * d1;
                        cnt += real[u] ? 1 : 0;
                    }
                }
                double *o = s_part[rix & 3];
                o[2 * lane] = s0; o[2 * lane + 1] = s1;
                o[128 + 2 * lane] = q0; o[128 + 2 * lane + 1] = q1;
                if (lane == 0) s_cnt[rix & 3] = cnt;
                if (runs_per_node == 1) {
                    const double inv = cnt > 0 ? 1.0 / (double)cnt : 0.;
                    const double v0 = (q0 - s0 * s0 * inv) * inv, v1 = (q1 - s1 * s1 * inv) * inv;
                    const int arg = wave_argmax(v0, v1, lane, c_lo, c_hi);
                    if (lane == 0) s_axis[node] = arg;
                }
            }
            if (runs_per_node > 1) {   // 1 or 2 nodes, each summed by 4 or 2 waves: add the runs in order
                __syncthreads();
                if (wave < n_nodes) {
                    double s0 = 0., s1 = 0., q0 = 0., q1 = 0.;
                    int cnt = 0;
                    for (int k = 0; k < runs_per_node; ++k) {
                        const double *o = s_part[wave * runs_per_node + k];
                        s0 += o[2 * lane]; s1 += o[2 * lane + 1];
                        q0 += o[128 + 2 * lane]; q1 += o[128 + 2 * lane + 1];
                        cnt += s_cnt[wave * runs_per_node + k];
                    }
                    const double inv = cnt > 0 ? 1.0 / (double)cnt : 0.;
                    const double v0 = (q0 - s0 * s0 * inv) * inv, v1 = (q1 - s1 * s1 * inv) * inv;
                    const int arg = wave_argmax(v0, v1, lane, c_lo, c_hi);
                    if (lane == 0) s_axis[wave] = arg;
                }
            }
        }
        __syncthreads();
        // 2. keys [ node | coordinate code | position ]
        for (int i = t; i < np; i += 256) {
            const int64_t pos = key_pos(s_keys[i], pos_bits);
            const int node = i / m;
            uint64_t code;
            if (pos >= n_real) {
                code = (1ull << coord_bits) - 1ull;
            } else {
                const int c = s_axis[node];
                const char *row = src.row(bh, pos);
                if (src.elt == 2) {
                    uint32_t u = static_cast<const uint16_t *>(static_cast<const void *>(row))[c];
                    if (u == 0x8000u) u = 0;
                    code = (u & 0x8000u) ? (~u & 0xffffu) : (u | 0x8000u);
                } else {
                    uint32_t u = __float_as_uint(static_cast<const float *>(static_cast<const void *>(row))[c]);
                    if (u == 0x80000000u) u = 0;
                    code = (u & 0x80000000u) ? (uint64_t)(~u) : (uint64_t)(u | 0x80000000u);
                }
            }
            s_keys[i] = ((uint64_t)node << (coord_bits + pos_bits)) | (code << pos_bits) | (uint64_t)pos;
        }
        __syncthreads();
        // 3. ascending bitonic sort inside every node (nodes are aligned runs of m = 2^x entries and
        // the node index leads the key, so sorting the runs sorts the array)
        for (int k = 2; k <= m; k <<= 1) {
            for (int j = k >> 1; j > 0; j >>= 1) {
                for (int i = t; i < np; i += 256) {
                    const int partner = i ^ j;
                    if (partner > i) {
                        const uint64_t a = s_keys[i], b = s_keys[partner];
                        const bool up = k == m || (i & k) == 0;   // the last merge of every node ascends
                        if (up ? (a > b) : (a < b)) {
                            s_keys[i] = b;
                            s_keys[partner] = a;
                        }
                    }
                }
                __syncthreads();
            }
        }
    }
    for (int i = t; i < np; i += 256) keys_out[base + i] = s_keys[i];
}

int bits_for(int64_t v) {   // bits needed to hold values 0 .. v-1
    int b = 0;
    while (((int64_t)1 << b) < v) ++b;
    return b;
}

}  // namespace

size_t lvr_tree_sort_temp_bytes(int64_t total_keys) {
    size_t bytes = 0;
    uint64_t *nullk = nullptr;
    (void)rocprim::radix_sort_keys(nullptr, bytes, nullk, nullk, (size_t)total_keys, 0, 64, (hipStream_t)0);
    return bytes;
}

// Whether lvr_tree_order can handle n_real keys per (sequence, KV head): the sort key
// [node | coordinate | position] has to fit 64 bits and the work space the padded entries.
bool lvr_tree_feasible(const lvr_index *ix, int64_t n_real) {
    if (n_real <= 0) return true;
    const int r = ix->cfg.group_size;
    const int n_bh = lvr_n_bh(ix);
    int64_t groups = n_real / r, gp = 1;
    while (gp < groups) gp <<= 1;
    const int64_t np = gp * r;
    const int pos_bits = bits_for(np);
    const int coord_bits = ix->elt == 2 ? 16 : 32;
    int levels = 0;
    while (((int64_t)1 << levels) < gp) ++levels;
    const int node_bits = bits_for((int64_t)n_bh << (levels > 0 ? levels - 1 : 0));
    return pos_bits + coord_bits + node_bits <= 64 && (int64_t)n_bh * np <= ix->tree_cap_keys;
}

// Orders n_real = groups*r keys (positions 0..n_real-1 of the given source rows) by the tree and
// writes them, regrouped, to arena rows row0 .. row0+n_real-1 together with the position maps.
// Returns hipErrorInvalidValue if the sort key would not fit in 64 bits.
hipError_t lvr_tree_order(lvr_index *ix, const void *Ksrc, const int64_t ks[3], int64_t n_real, hipStream_t st,
                          lvr_tree_perm *perm, int c_lo, int c_hi) {
    perm->keys = nullptr;
    if (n_real <= 0) return hipSuccess;
    const int r = ix->cfg.group_size;
    const int n_bh = lvr_n_bh(ix);
    int64_t groups = n_real / r, gp = 1;
    while (gp < groups) gp <<= 1;
    const int64_t np = gp * r;                         // padded entries per (sequence, KV head)
    const int pos_bits = bits_for(np);
    const int coord_bits = ix->elt == 2 ? 16 : 32;
    int levels = 0;
    while (((int64_t)1 << levels) < gp) ++levels;       // nodes of r entries after `levels` splits
    const int node_bits = bits_for((int64_t)n_bh << (levels > 0 ? levels - 1 : 0));
    if (pos_bits + coord_bits + node_bits > 64) return hipErrorInvalidValue;
    if ((int64_t)n_bh * np > ix->tree_cap_keys) return hipErrorInvalidValue;

    TreeSrc ksrc{static_cast<const char *>(Ksrc), ks[0], ks[1], ks[2], (int)ix->elt, ix->cfg.n_kv_heads};
    uint64_t *cur = ix->tree_keys_a, *alt = ix->tree_keys_b;
    if (np <= TREE_WG_MAX && pos_bits + coord_bits + levels <= 64) {
        // small input (a buffer chunk): the whole tree in one launch
        hipLaunchKernelGGL(tree_small_kernel, dim3(1, (unsigned)n_bh), dim3(256), 0, st, ksrc, (const uint64_t *)nullptr, cur, np,
                           (int)np, n_real, levels, pos_bits, coord_bits, c_lo, c_hi);
        perm->keys = cur;
        perm->np = np;
        perm->pos_bits = pos_bits;
        return hipGetLastError();
    }
    // the upper levels one by one (device-wide sort per level) until a node has at most TREE_WG_MAX
    // entries; all the levels below that in one launch, a workgroup per node, sorted in LDS
    int top_levels = levels;
    for (int L = 0; L < levels; ++L)
        if ((np >> L) <= TREE_WG_MAX && pos_bits + coord_bits + (levels - L) <= 64) {
            top_levels = L;
            break;
        }
    hipLaunchKernelGGL(tree_init_kernel, dim3((unsigned)((np + 255) / 256), (unsigned)n_bh), dim3(256), 0, st, cur, np);
    for (int L = 0; L < top_levels; ++L) {
        const int64_t n_nodes = (int64_t)1 << L;
        const int64_t m = np >> L;                      // entries per node at this level (>= 2r)
        if (m <= PIECE) {
            hipLaunchKernelGGL(tree_stats_small_kernel, dim3((unsigned)((n_nodes + 3) / 4), (unsigned)n_bh), dim3(256), 0,
                               st, ksrc, cur, ix->tree_axis, np, n_real, m, pos_bits, n_nodes, c_lo, c_hi);
        } else {
            hipLaunchKernelGGL(tree_stats_piece_kernel, dim3((unsigned)(np / PIECE), (unsigned)n_bh), dim3(256), 0, st,
                               ksrc, cur, ix->tree_partial, np, n_real, m, pos_bits);
            hipLaunchKernelGGL(tree_stats_merge_kernel, dim3((unsigned)n_nodes, (unsigned)n_bh), dim3(128), 0, st,
                               ix->tree_partial, ix->tree_axis, np, m, n_nodes, c_lo, c_hi);
        }
        hipLaunchKernelGGL(tree_keys_kernel, dim3((unsigned)((np + 255) / 256), (unsigned)n_bh), dim3(256), 0, st, ksrc,
                           cur, ix->tree_axis, np, n_real, m, pos_bits, coord_bits, n_nodes);
        size_t temp = ix->tree_temp_bytes;
        const int end_bit = pos_bits + coord_bits + bits_for((int64_t)n_bh * n_nodes);
        hipError_t e = rocprim::radix_sort_keys(ix->tree_temp, temp, cur, alt, (size_t)((int64_t)n_bh * np), 0,
                                                (unsigned)end_bit, st);
        if (e != hipSuccess) return e;
        uint64_t *t = cur;
        cur = alt;
        alt = t;
    }
    if (top_levels < levels) {
        const int64_t m0 = np >> top_levels;   // entries of a node at that level
        hipLaunchKernelGGL(tree_small_kernel, dim3((unsigned)(np / m0), (unsigned)n_bh), dim3(256), 0, st, ksrc,
                           (const uint64_t *)cur, alt, np, (int)m0, n_real, levels - top_levels, pos_bits, coord_bits, c_lo, c_hi);
        cur = alt;
    }
    perm->keys = cur;
    perm->np = np;
    perm->pos_bits = pos_bits;
    return hipGetLastError();
}

hipError_t lvr_tree_gather(lvr_index *ix, const void *Ksrc, const int64_t ks[3], const void *Vsrc, const int64_t vs[3],
                           const lvr_tree_perm *perm, int64_t n_real, int64_t row0, hipStream_t st) {
    if (n_real <= 0 || !perm->keys) return hipSuccess;
    const int n_bh = lvr_n_bh(ix);
    TreeSrc ksrc{static_cast<const char *>(Ksrc), ks[0], ks[1], ks[2], (int)ix->elt, ix->cfg.n_kv_heads};
    TreeSrc vsrc{static_cast<const char *>(Vsrc), vs[0], vs[1], vs[2], (int)ix->elt, ix->cfg.n_kv_heads};
    const int row_bytes = (int)(LVR_D * ix->elt);
    const int64_t total = n_real * (row_bytes / 16);
    hipLaunchKernelGGL(tree_gather_kernel, dim3((unsigned)((total + 255) / 256), (unsigned)n_bh, 2), dim3(256), 0, st,
                       ksrc, vsrc, perm->keys, static_cast<char *>(ix->K), static_cast<char *>(ix->V), ix->slot_pos,
                       ix->pos_slot, perm->np, n_real, perm->pos_bits, ix->cap_rows, row0, row_bytes);
    return hipGetLastError();
}

hipError_t lvr_tree_group(lvr_index *ix, const void *Ksrc, const int64_t ks[3], const void *Vsrc, const int64_t vs[3],
                          int64_t n_real, int64_t row0, hipStream_t st) {
    lvr_tree_perm perm;
    hipError_t e = lvr_tree_order(ix, Ksrc, ks, n_real, st, &perm);
    if (e != hipSuccess) return e;
    return lvr_tree_gather(ix, Ksrc, ks, Vsrc, vs, &perm, n_real, row0, st);
}
