"""ctypes binding of liblouver: one Python function per C entry point, same names.

Only argument marshalling happens here (tensor -> device pointer, strides, stream handle);
every step of the path runs in the library's kernels.  There is no CPU fallback: if the
library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

from .build import LIB_PATH

LVR_BF16, LVR_F32 = 0, 1
LVR_GROUP_CONTIGUOUS, LVR_GROUP_TREE, LVR_GROUP_SUBSPACE_TREE = 0, 1, 2
LVR_ENCLOSE_BALL, LVR_ENCLOSE_AABB = 0, 1
LVR_ATTEND_BUFFER_DENSE = 1
LVR_SEPARATE_KERNELS = 2
LVR_CONCURRENT_UPDATE = 4
LVR_KV_IN_HOST_MEMORY = 8
LVR_INDEX_AUTO, LVR_INDEX_SAME, LVR_INDEX_FP8, LVR_INDEX_FP6 = 0, 1, 2, 3
LVR_OK, LVR_E_INVALID, LVR_E_UNSUPPORTED, LVR_E_CAPACITY = 0, -1, -2, -3
LVR_E_OVERFLOW, LVR_E_HIP, LVR_E_NOMEM, LVR_E_STATE = -4, -5, -6, -7


class lvr_config(C.Structure):
    _fields_ = [
        ("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("kv_dtype", C.c_int32), ("group_size", C.c_int32), ("n_subspaces", C.c_int32),
        ("buffer_size", C.c_int32), ("grouping", C.c_int32), ("enclosing", C.c_int32), ("flags", C.c_uint32),
        ("capacity", C.c_int64), ("scale", C.c_float), ("attn_splits", C.c_int32),
        ("reservoir_size", C.c_int32), ("seed", C.c_uint64), ("index_dtype", C.c_int32), ("query_workgroups", C.c_int32),
    ]


class lvr_stats(C.Structure):
    _fields_ = [
        ("n_keys", C.c_int64), ("n_indexed", C.c_int64), ("groups_scored", C.c_int64),
        ("groups_surviving", C.c_int64), ("keys_scanned", C.c_int64), ("keys_emitted", C.c_int64),
        ("bytes_index", C.c_int64), ("bytes_keys", C.c_int64), ("bytes_attention", C.c_int64),
        ("overflow", C.c_int32), ("update_pending", C.c_int32),
    ]

    def as_dict(self):
        return {k: int(getattr(self, k)) for k, _ in self._fields_}


class lvr_profile(C.Structure):
    _fields_ = [("ms", C.c_double * 9), ("launches", C.c_int64 * 9)]


KERNEL_NAMES = ["copy", "build", "reset", "prune", "filter", "attn_partial", "attn_combine",
                "dense_partial", "dense_combine"]

EXPORTS = [
    "lvr_create", "lvr_destroy", "lvr_arena_bytes", "lvr_build", "lvr_append", "lvr_query",
    "lvr_sparse_attention", "lvr_decode_step", "lvr_dense_attention", "lvr_get_stats",
    "lvr_export_index", "lvr_length", "lvr_strerror", "lvr_last_hip_error",
    "lvr_profile_enable", "lvr_profile_read", "lvr_threshold", "lvr_export_reservoir", "lvr_publish", "lvr_query1", "lvr_append_decode_step", "lvr_host_bytes",
    "lvr_subspace_thresholds", "lvr_sparse_attention_static",
    "lvr_set_bound_test", "lvr_stream_read", "lvr_export_labels", "lvr_export_channel_scales",
]

_lib = None


class LouverError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = lib().lvr_strerror(code).decode()
        if code == LVR_E_HIP:
            msg += f" (hipError {lib().lvr_last_hip_error()})"
        super().__init__(f"{where}: {msg} [{code}]")


def lib():
    """The loaded shared library.  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it first (python -m paper_2605_06763_amd.build "
                           "or __graft_entry__.build()); there is no fallback path")
    L = C.CDLL(LIB_PATH)
    vp, i64 = C.c_void_p, C.c_int64
    L.lvr_create.argtypes = [C.POINTER(lvr_config), C.POINTER(vp)]
    L.lvr_destroy.argtypes = [vp]
    L.lvr_arena_bytes.argtypes = [C.POINTER(lvr_config)]
    L.lvr_arena_bytes.restype = C.c_size_t
    L.lvr_build.argtypes = [vp, vp, vp, i64, C.POINTER(i64), C.POINTER(i64), vp]
    L.lvr_append.argtypes = [vp, vp, vp, i64, vp]
    L.lvr_query.argtypes = [vp, vp, vp, vp, vp, i64, vp]
    L.lvr_sparse_attention.argtypes = [vp, vp, vp, vp, i64, vp, vp]
    L.lvr_decode_step.argtypes = [vp, vp, vp, vp, vp, vp, i64, vp]
    L.lvr_dense_attention.argtypes = [vp, vp, vp, vp]
    L.lvr_get_stats.argtypes = [vp, C.POINTER(lvr_stats)]
    L.lvr_export_index.argtypes = [vp, vp, vp, vp, vp]
    L.lvr_length.argtypes = [vp, C.POINTER(i64), C.POINTER(i64)]
    L.lvr_profile_enable.argtypes = [vp, C.c_int]
    L.lvr_profile_read.argtypes = [vp, C.POINTER(lvr_profile)]
    L.lvr_publish.argtypes = [vp, vp]
    L.lvr_append_decode_step.argtypes = [vp, vp, vp, i64, vp, vp, vp, vp, vp, i64, vp]
    L.lvr_host_bytes.argtypes = [C.POINTER(lvr_config)]
    L.lvr_host_bytes.restype = C.c_size_t
    L.lvr_query1.argtypes = [vp, vp, vp, vp, vp, vp, i64, vp]
    L.lvr_subspace_thresholds.argtypes = [vp, vp, vp, vp, vp]
    L.lvr_sparse_attention_static.argtypes = [vp, vp, i64, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_float,
                                              vp, vp, vp, i64, vp, vp]
    L.lvr_set_bound_test.argtypes = [vp, C.c_int]
    L.lvr_export_labels.argtypes = [vp, vp]
    L.lvr_export_channel_scales.argtypes = [vp, vp]
    L.lvr_stream_read.argtypes = [vp, i64, vp, C.c_int32, vp]
    L.lvr_threshold.argtypes = [vp, vp, C.c_int, C.c_float, vp, vp]
    L.lvr_export_reservoir.argtypes = [vp, vp]
    L.lvr_strerror.argtypes = [C.c_int]
    L.lvr_strerror.restype = C.c_char_p
    L.lvr_last_hip_error.restype = C.c_int
    _lib = L
    return L


def _check(code: int, where: str):
    if code != LVR_OK:
        raise LouverError(code, where)


def _stream(stream=None):
    if type(stream) is C.c_void_p:      # already marshalled (stream_arg)
        return stream
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def stream_arg(stream=None) -> C.c_void_p:
    """The stream argument marshalled once, for callers that issue many calls on one stream."""
    return _stream(stream)


class DeviceArg:
    """A device tensor checked and marshalled once (tensor_arg); the tensor is kept alive."""
    __slots__ = ("tensor", "ptr", "dtype", "shape")

    def __init__(self, t: torch.Tensor):
        if not t.is_cuda:
            raise ValueError("tensor must be a device tensor")
        if not t.is_contiguous():
            raise ValueError("tensor must be contiguous")
        self.tensor, self.ptr, self.dtype, self.shape = t, C.c_void_p(t.data_ptr()), t.dtype, tuple(t.shape)


def tensor_arg(t: torch.Tensor) -> DeviceArg:
    """Check and marshal a device tensor once; every entry point accepts the result in place
    of the tensor (saves the per-call checks in tight decode loops)."""
    return DeviceArg(t)


def _dev(t, dtype=None, name="tensor"):
    if type(t) is DeviceArg:
        if dtype is not None and t.dtype != dtype:
            raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
        return t.ptr
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return C.c_void_p(t.data_ptr())


def make_config(*, batch, n_q_heads, n_kv_heads, head_dim=128, kv_dtype=LVR_BF16, group_size=4,
                n_subspaces=4, buffer_size=256, grouping=LVR_GROUP_CONTIGUOUS, enclosing=LVR_ENCLOSE_BALL, flags=0, capacity,
                scale=0.0, attn_splits=0, reservoir_size=0, seed=0, index_dtype=0, query_workgroups=0) -> lvr_config:
    return lvr_config(batch, n_q_heads, n_kv_heads, head_dim, kv_dtype, group_size, n_subspaces,
                      buffer_size, grouping, enclosing, flags, capacity, scale, attn_splits, reservoir_size, seed, index_dtype, query_workgroups)


def lvr_arena_bytes(cfg: lvr_config) -> int:
    return int(lib().lvr_arena_bytes(C.byref(cfg)))


def lvr_host_bytes(cfg: lvr_config) -> int:
    return int(lib().lvr_host_bytes(C.byref(cfg)))


def lvr_create(cfg: lvr_config) -> C.c_void_p:
    h = C.c_void_p()
    _check(lib().lvr_create(C.byref(cfg), C.byref(h)), "lvr_create")
    return h


def lvr_destroy(h) -> None:
    _check(lib().lvr_destroy(h), "lvr_destroy")


def lvr_build(h, K: torch.Tensor, V: torch.Tensor, stream=None) -> None:
    """K, V: device tensors [batch][n_kv_heads][n][head_dim] (bf16 or fp32), last axis contiguous."""
    if K.dim() != 4 or V.shape != K.shape or (K.numel() > 0 and (K.stride(3) != 1 or V.stride(3) != 1)):
        raise ValueError("K and V must be [batch][n_kv_heads][n][head_dim] with a contiguous last axis")
    if not (K.is_cuda and V.is_cuda):
        raise ValueError("K and V must be device tensors")
    ks = (C.c_int64 * 3)(*K.stride()[:3])
    vs = (C.c_int64 * 3)(*V.stride()[:3])
    _check(lib().lvr_build(h, C.c_void_p(K.data_ptr()), C.c_void_p(V.data_ptr()), K.shape[2], ks, vs,
                           _stream(stream)), "lvr_build")


def lvr_append(h, k_new: torch.Tensor, v_new: torch.Tensor, stream=None) -> None:
    """k_new, v_new: contiguous device tensors [batch][n_kv_heads][m][head_dim]."""
    _check(lib().lvr_append(h, _dev(k_new, name="k_new"), _dev(v_new, name="v_new"), k_new.shape[2],
                            _stream(stream)), "lvr_append")


def lvr_query(h, q, tau, out_idx, out_count, stream=None) -> None:
    cap = out_idx.shape[-1]
    _check(lib().lvr_query(h, _dev(q, torch.float32, "q"), _dev(tau, torch.float32, "tau"),
                           _dev(out_idx, torch.int32, "out_idx"), _dev(out_count, torch.int32, "out_count"),
                           cap, _stream(stream)), "lvr_query")


def lvr_query1(h, q, tau_s, tau, out_idx, out_count, stream=None) -> None:
    cap = out_idx.shape[-1]
    _check(lib().lvr_query1(h, _dev(q, torch.float32, "q"), _dev(tau_s, torch.float32, "tau_s"),
                            _dev(tau, torch.float32, "tau"), _dev(out_idx, torch.int32, "out_idx"),
                            _dev(out_count, torch.int32, "out_count"), cap, _stream(stream)), "lvr_query1")


def lvr_subspace_thresholds(h, q, tau, tau_s_out, stream=None) -> None:
    _check(lib().lvr_subspace_thresholds(h, _dev(q, torch.float32, "q"), _dev(tau, torch.float32, "tau"),
                                         _dev(tau_s_out, torch.float32, "tau_s_out"), _stream(stream)),
           "lvr_subspace_thresholds")


def lvr_sparse_attention(h, q, idx, count, out, stream=None) -> None:
    cap = idx.shape[-1]
    _check(lib().lvr_sparse_attention(h, _dev(q, torch.float32, "q"), _dev(idx, torch.int32, "idx"),
                                      _dev(count, torch.int32, "count"), cap, _dev(out, torch.float32, "out"),
                                      _stream(stream)), "lvr_sparse_attention")


def lvr_sparse_attention_static(K, V, q, idx, count, out, scale=0.0, stream=None) -> None:
    """K, V: contiguous device tensors [batch][n_kv_heads][n][128] (bf16 or fp32); no index object."""
    if K.dim() != 4 or V.shape != K.shape or K.dtype != V.dtype:
        raise ValueError("K and V must be [batch][n_kv_heads][n][head_dim] of one dtype")
    if K.dtype not in (torch.bfloat16, torch.float32):
        raise ValueError("K and V must be bf16 or fp32")
    cap = idx.shape[-1]
    _check(lib().lvr_sparse_attention_static(_dev(K, name="K"), _dev(V, name="V"), K.shape[2],
                                             LVR_BF16 if K.dtype == torch.bfloat16 else LVR_F32, K.shape[0],
                                             q.shape[1], K.shape[1], float(scale), _dev(q, torch.float32, "q"),
                                             _dev(idx, torch.int32, "idx"), _dev(count, torch.int32, "count"), cap,
                                             _dev(out, torch.float32, "out"), _stream(stream)),
           "lvr_sparse_attention_static")


def lvr_decode_step(h, q, tau, out, out_idx, out_count, stream=None) -> None:
    cap = out_idx.shape[-1]
    _check(lib().lvr_decode_step(h, _dev(q, torch.float32, "q"), _dev(tau, torch.float32, "tau"),
                                 _dev(out, torch.float32, "out"), _dev(out_idx, torch.int32, "out_idx"),
                                 _dev(out_count, torch.int32, "out_count"), cap, _stream(stream)),
           "lvr_decode_step")


def lvr_append_decode_step(h, k_new, v_new, q, tau, out, out_idx, out_count, stream=None) -> None:
    cap = out_idx.shape[-1]
    _check(lib().lvr_append_decode_step(h, _dev(k_new, name="k_new"), _dev(v_new, name="v_new"), k_new.shape[2],
                                        _dev(q, torch.float32, "q"), _dev(tau, torch.float32, "tau"),
                                        _dev(out, torch.float32, "out"), _dev(out_idx, torch.int32, "out_idx"),
                                        _dev(out_count, torch.int32, "out_count"), cap, _stream(stream)),
           "lvr_append_decode_step")


def lvr_dense_attention(h, q, out, stream=None) -> None:
    _check(lib().lvr_dense_attention(h, _dev(q, torch.float32, "q"), _dev(out, torch.float32, "out"),
                                     _stream(stream)), "lvr_dense_attention")


def lvr_get_stats(h, raise_on_overflow: bool = True) -> dict:
    st = lvr_stats()
    rc = lib().lvr_get_stats(h, C.byref(st))
    if rc == LVR_E_OVERFLOW and not raise_on_overflow:
        return st.as_dict()
    _check(rc, "lvr_get_stats")
    return st.as_dict()


def lvr_profile_enable(h, max_launches: int) -> None:
    _check(lib().lvr_profile_enable(h, int(max_launches)), "lvr_profile_enable")


def lvr_profile_read(h) -> dict:
    """{kernel name: (total ms, launches)} since the last read."""
    p = lvr_profile()
    _check(lib().lvr_profile_read(h, C.byref(p)), "lvr_profile_read")
    return {KERNEL_NAMES[i]: (float(p.ms[i]), int(p.launches[i])) for i in range(9)}


TAU_MODES = {"sample-max": 0, "sample-mean-max": 1, "sample-gap": 2, "sample-topk": 3, "budget": 4}


def lvr_threshold(h, q, mode, param, tau_out, stream=None) -> None:
    m = TAU_MODES[mode] if isinstance(mode, str) else int(mode)
    _check(lib().lvr_threshold(h, _dev(q, torch.float32, "q"), m, float(param), _dev(tau_out, torch.float32, "tau_out"),
                               _stream(stream)), "lvr_threshold")


def lvr_export_reservoir(h, cfg: lvr_config):
    import numpy as np
    res = np.full((cfg.batch, cfg.n_kv_heads, max(cfg.reservoir_size, 1)), -1, dtype=np.int32)
    _check(lib().lvr_export_reservoir(h, res.ctypes.data_as(C.c_void_p)), "lvr_export_reservoir")
    return res


def lvr_publish(h, stream=None) -> None:
    _check(lib().lvr_publish(h, _stream(stream)), "lvr_publish")


def lvr_export_channel_scales(h, cfg: lvr_config):
    """[batch][n_kv_heads][head_dim] int8: the channel exponents of a rescaled 6-bit index (zeros otherwise)."""
    import numpy as np
    e = np.zeros((cfg.batch, cfg.n_kv_heads, cfg.head_dim), dtype=np.int8)
    _check(lib().lvr_export_channel_scales(h, e.ctypes.data_as(C.c_void_p)), "lvr_export_channel_scales")
    return e


def lvr_export_labels(h, cfg: lvr_config):
    """Per-subspace group labels [batch][n_kv_heads][S][n_indexed] int32 (LVR_GROUP_SUBSPACE_TREE only)."""
    import numpy as np
    _, ni = lvr_length(h)
    lab = np.zeros((cfg.batch, cfg.n_kv_heads, cfg.n_subspaces, ni), dtype=np.int32)
    _check(lib().lvr_export_labels(h, lab.ctypes.data_as(C.c_void_p)), "lvr_export_labels")
    return lab


def lvr_set_bound_test(h, enabled: bool) -> None:
    _check(lib().lvr_set_bound_test(h, 1 if enabled else 0), "lvr_set_bound_test")


def lvr_stream_read(src, sink, workgroups=0, stream=None) -> None:
    """One read-only pass over the bytes of `src` (any contiguous device tensor); sink: int32 tensor of >= 1 element."""
    t = src.tensor if type(src) is DeviceArg else src
    _check(lib().lvr_stream_read(_dev(src, name="src"), t.numel() * t.element_size(), _dev(sink, torch.int32, "sink"),
                                 int(workgroups), _stream(stream)), "lvr_stream_read")


def lvr_length(h):
    n, ni = C.c_int64(), C.c_int64()
    _check(lib().lvr_length(h, C.byref(n), C.byref(ni)), "lvr_length")
    return n.value, ni.value


def lvr_export_index(h, cfg: lvr_config):
    """Host copies (numpy) of centres [b][h][groups][d], radii [b][h][groups][S],
    slot_pos [b][h][n], keys [b][h][n][d].  bf16 data comes back as uint16 bit patterns."""
    import numpy as np
    n, ni = lvr_length(h)
    ng = ni // cfg.group_size
    dt = np.uint16 if cfg.kv_dtype == LVR_BF16 else np.float32
    box = cfg.enclosing == LVR_ENCLOSE_AABB
    centres = np.zeros((cfg.batch, cfg.n_kv_heads, ng) + ((2,) if box else ()) + (cfg.head_dim,), dtype=dt)
    radii = np.zeros((cfg.batch, cfg.n_kv_heads, ng, 1 if box else cfg.n_subspaces), dtype=np.float32)
    slot_pos = np.zeros((cfg.batch, cfg.n_kv_heads, n), dtype=np.int32)
    keys = np.zeros((cfg.batch, cfg.n_kv_heads, n, cfg.head_dim), dtype=dt)
    _check(lib().lvr_export_index(h, centres.ctypes.data_as(C.c_void_p), radii.ctypes.data_as(C.c_void_p),
                                  slot_pos.ctypes.data_as(C.c_void_p), keys.ctypes.data_as(C.c_void_p)),
           "lvr_export_index")
    return centres, radii, slot_pos, keys
