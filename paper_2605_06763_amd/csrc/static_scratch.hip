// lvr_sparse_attention_static: the sparse attention of lvr_sparse_attention for callers that
// cannot allocate (HIP graph capture, serving loops, harnesses that forbid hipMalloc).
//
// It needs no index object: K and V are the caller's own contiguous cache, and the partial
// softmax triples of the split pass (the only device memory the attention kernels use beyond
// their inputs and outputs) live in a file-scope device array instead of an arena that
// lvr_create would have allocated.  The kernels are the ones lvr_sparse_attention launches in its
// two-launch form (64 splits per head, then the combine pass); they take the array's device
// address as an argument exactly as they take the arena's.
//
// Every GPU holds its own copy of the array at its own address.  That address is looked up once
// per device (hipGetSymbolAddress with that device current) and cached; host code never passes
// the array's name to a kernel.
#include <mutex>

#include "lvr_internal.h"

namespace {

constexpr int STATIC_MAX_HEADS = 256;   // batch * n_q_heads
constexpr int STATIC_SPLITS = 64;       // P of the two-launch form
constexpr int STATIC_MAX_DEVICES = 64;
constexpr size_t ML_FLOATS = (size_t)STATIC_MAX_HEADS * STATIC_SPLITS * 2;
constexpr size_t O_FLOATS = (size_t)STATIC_MAX_HEADS * STATIC_SPLITS * LVR_D;

// (m, l) pairs first, then the o vectors: 64 KiB + 8 MiB per GPU, held until the process ends.
// Contents are whatever the last call left; nothing here has to start at zero, because a call
// reads only the partials its own split pass has just written.
static __device__ __align__(256) float scratch[ML_FLOATS + O_FLOATS];

std::mutex g_mu;
float *g_scratch_ptr[STATIC_MAX_DEVICES];   // device address of `scratch` on each GPU, once known

// Device address of this GPU's copy of the array (looked up on the first call on a device).
hipError_t scratch_on_current_device(float **out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= STATIC_MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = static_cast<float *>(p);
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool aligned4(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 3u) == 0; }

}  // namespace

extern "C" int lvr_sparse_attention_static(const void *K, const void *V, int64_t n, int32_t kv_dtype, int32_t batch,
                                           int32_t n_q_heads, int32_t n_kv_heads, float scale, const float *q,
                                           const int32_t *idx, const int32_t *count, int64_t cap, float *out,
                                           void *stream) {
    if (!q || !count || !out || cap < 0 || (cap > 0 && !idx) || n < 0 || (n > 0 && (!K || !V))) return LVR_E_INVALID;
    if (batch <= 0 || n_q_heads <= 0 || n_kv_heads <= 0 || n_q_heads % n_kv_heads != 0 || scale < 0.f) return LVR_E_INVALID;
    if (kv_dtype != LVR_BF16 && kv_dtype != LVR_F32) return LVR_E_INVALID;
    if (!aligned16(K) || !aligned16(V) || !aligned4(q) || !aligned4(idx) || !aligned4(count) || !aligned4(out))
        return LVR_E_INVALID;
    if ((int64_t)batch * n_q_heads > STATIC_MAX_HEADS || n > ((int64_t)1 << 30)) return LVR_E_CAPACITY;
    float *base = nullptr;
    if (scratch_on_current_device(&base) != hipSuccess) {
        (void)hipGetLastError();
        return LVR_E_HIP;
    }
    // A view for the launchers: the caller's cache stands where the arena would, the static
    // array where the arena's partials would.  Nothing in it is owned, nothing is allocated.
    lvr_index view = {};
    view.cfg.batch = batch;
    view.cfg.n_q_heads = n_q_heads;
    view.cfg.n_kv_heads = n_kv_heads;
    view.cfg.head_dim = LVR_D;
    view.cfg.kv_dtype = kv_dtype;
    view.G = n_q_heads / n_kv_heads;
    view.elt = kv_dtype == LVR_BF16 ? 2 : 4;
    view.sigma = scale > 0.f ? scale : 0.08838834764831845f;   // 1 / sqrt(128)
    view.K = const_cast<void *>(K);
    view.V = const_cast<void *>(V);
    view.cap_rows = n;        // contiguous [batch][n_kv_heads][n][128]
    view.n_total = n;
    view.P = STATIC_SPLITS;
    view.part_ml = base;
    view.part_o = base + ML_FLOATS;
    view.counters = reinterpret_cast<int32_t *>(base);   // handed to the combine pass, which never touches it here
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (lvr_launch_sparse_partial(&view, q, idx, nullptr, count, 1, cap, st) != hipSuccess) return LVR_E_HIP;
    if (lvr_launch_combine(&view, out, STATIC_SPLITS, count, 1, cap, nullptr, st) != hipSuccess) return LVR_E_HIP;
    return LVR_OK;
}
