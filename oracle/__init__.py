"""ctypes front end of the CPU oracle (oracle/louver_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the bench's
cpu_baseline leg.  The GPU package never imports this module.

Every function takes and returns numpy arrays; key/value matrices are fp32 arrays
(values exact in the workload's storage type) or uint16 bf16 bit patterns.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "louver_oracle.c")
_LIB = os.path.join(_HERE, "liblouver_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction, OpenMP for the
    outer per-head loops)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-fno-fast-math", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    lib = C.CDLL(_LIB)
    vp, i32, i64, f32, f64 = C.c_void_p, C.c_int, C.c_int64, C.c_float, C.c_double
    lib.lvo_max_threads.restype = i32
    lib.lvo_set_threads.argtypes = [i32]
    lib.lvo_scores_f64.argtypes = [vp, vp, i32, i64, i32, vp]
    lib.lvo_scores_f32.argtypes = [vp, vp, i32, i64, i32, vp]
    lib.lvo_range_query.argtypes = [vp, vp, i32, i64, i32, f32, vp, i64]
    lib.lvo_range_query.restype = i64
    lib.lvo_attention_on_list.argtypes = [vp, vp, vp, i32, i32, vp, i64, f64, vp]
    lib.lvo_decode_step.argtypes = [vp, vp, i32, i64, i32, i32, i64, i32, vp, vp, f64, i64, vp, i64, vp, vp]
    lib.lvo_dense_attention.argtypes = [vp, vp, i32, i64, i32, i32, i64, i32, vp, f64, vp]
    lib.lvo_subspace_range.argtypes = [i32, i32, i32, vp, vp]
    lib.lvo_ball_index.argtypes = [vp, i32, i64, i32, i32, vp, i64, vp, vp]
    lib.lvo_ball_radii_for_centres.argtypes = [vp, i32, i64, i32, i32, vp, i64, vp, vp]
    lib.lvo_ball_bounds.argtypes = [vp, i32, i32, vp, vp, i64, vp]
    lib.lvo_aabb_index.argtypes = [vp, i32, i64, i32, vp, i64, vp, vp]
    lib.lvo_aabb_bounds.argtypes = [vp, i32, vp, vp, i64, vp]
    lib.lvo_query1_filter.argtypes = [vp, vp, i32, i64, i64, vp, vp]
    lib.lvo_ta_filter.argtypes = [vp, vp, i32, i64, i64, f64, vp]
    lib.lvo_safe_subspace_thresholds.argtypes = [vp, i32, i64, f64, vp]
    lib.lvo_safe_subspace_thresholds.restype = None
    lib.lvo_hash32.argtypes = [C.c_uint64, C.c_uint64, C.c_uint64]
    lib.lvo_hash32.restype = C.c_uint32
    lib.lvo_reservoir.argtypes = [C.c_uint64, C.c_uint64, i64, i32, vp]
    lib.lvo_threshold.argtypes = [vp, i32, i32, f64]
    lib.lvo_threshold.restype = f32
    lib.lvo_ta_filter.restype = i64
    lib.lvo_balanced_tree.argtypes = [vp, i32, i64, i32, i32, i32, i32, vp, vp]
    lib.lvo_balanced_tree.restype = i64
    _lib = lib
    return lib


def _kv(a):
    """(contiguous array, is_bf16 flag) for a key/value matrix given as fp32 or uint16."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return np.ascontiguousarray(a), 1
    return np.ascontiguousarray(a, dtype=np.float32), 0


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def max_threads() -> int:
    return int(_load().lvo_max_threads())


def set_threads(t: int) -> None:
    _load().lvo_set_threads(int(t))


def scores_f64(q, K):
    K, bf = _kv(K)
    n, d = K.shape
    q = np.ascontiguousarray(q, dtype=np.float32)
    s = np.empty(n, dtype=np.float64)
    _load().lvo_scores_f64(_p(q), _p(K), bf, n, d, _p(s))
    return s


def scores_f32(q, K):
    K, bf = _kv(K)
    n, d = K.shape
    q = np.ascontiguousarray(q, dtype=np.float32)
    s = np.empty(n, dtype=np.float32)
    _load().lvo_scores_f32(_p(q), _p(K), bf, n, d, _p(s))
    return s


def range_query(q, K, tau):
    """Ascending indices of { j : <q, k_j> >= tau } (fp32 scores)."""
    K, bf = _kv(K)
    n, d = K.shape
    q = np.ascontiguousarray(q, dtype=np.float32)
    idx = np.empty(max(n, 1), dtype=np.int32)
    m = _load().lvo_range_query(_p(q), _p(K), bf, n, d, float(tau), _p(idx), n)
    return idx[:m].copy()


def attention_on_list(q, K, V, idx, sigma):
    K, bf = _kv(K)
    V, bfv = _kv(V)
    assert bf == bfv
    d = K.shape[1]
    q = np.ascontiguousarray(q, dtype=np.float32)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    out = np.empty(d, dtype=np.float32)
    _load().lvo_attention_on_list(_p(q), _p(K), _p(V), bf, d, _p(idx), idx.size, float(sigma), _p(out))
    return out


def decode_step(K, V, q, tau, sigma, n_q_heads, *, extra_from=-1, cap=None):
    """K, V [batch][n_kv_heads][n][d]; q [batch][n_q_heads][d]; tau [batch][n_q_heads].
    Returns (list of index arrays per (batch, head), counts [batch][n_q_heads], out)."""
    K, bf = _kv(K)
    V, _ = _kv(V)
    batch, hkv, n, d = K.shape
    q = np.ascontiguousarray(q, dtype=np.float32).reshape(batch, n_q_heads, d)
    tau = np.ascontiguousarray(tau, dtype=np.float32).reshape(batch, n_q_heads)
    cap = n if cap is None else int(cap)
    idx = np.zeros((batch, n_q_heads, max(cap, 1)), dtype=np.int32)
    count = np.zeros((batch, n_q_heads), dtype=np.int64)
    out = np.zeros((batch, n_q_heads, d), dtype=np.float32)
    _load().lvo_decode_step(_p(K), _p(V), bf, batch, n_q_heads, hkv, n, d, _p(q), _p(tau),
                            float(sigma), int(extra_from), _p(idx), cap, _p(count), _p(out))
    sets = [[idx[b, h, :min(count[b, h], cap)].copy() for h in range(n_q_heads)] for b in range(batch)]
    return sets, count, out


def dense_attention(K, V, q, sigma, n_q_heads):
    K, bf = _kv(K)
    V, _ = _kv(V)
    batch, hkv, n, d = K.shape
    q = np.ascontiguousarray(q, dtype=np.float32).reshape(batch, n_q_heads, d)
    out = np.zeros((batch, n_q_heads, d), dtype=np.float32)
    _load().lvo_dense_attention(_p(K), _p(V), bf, batch, n_q_heads, hkv, n, d, _p(q), float(sigma), _p(out))
    return out


def subspace_range(d, S, s):
    lo, hi = C.c_int(0), C.c_int(0)
    _load().lvo_subspace_range(d, S, s, C.byref(lo), C.byref(hi))
    return lo.value, hi.value


def ball_index(K, label, n_groups, S):
    """Centres [n_groups][d] and radii [n_groups][S] (fp64) of the groups given by label."""
    K, bf = _kv(K)
    n, d = K.shape
    label = np.ascontiguousarray(label, dtype=np.int32)
    centre = np.empty((n_groups, d), dtype=np.float64)
    radius = np.empty((n_groups, S), dtype=np.float64)
    _load().lvo_ball_index(_p(K), bf, n, d, S, _p(label), n_groups, _p(centre), _p(radius))
    return centre, radius


def ball_radii_for_centres(K, label, centre, S):
    K, bf = _kv(K)
    n, d = K.shape
    label = np.ascontiguousarray(label, dtype=np.int32)
    centre = np.ascontiguousarray(centre, dtype=np.float64)
    n_groups = centre.shape[0]
    radius = np.empty((n_groups, S), dtype=np.float64)
    _load().lvo_ball_radii_for_centres(_p(K), bf, n, d, S, _p(label), n_groups, _p(centre), _p(radius))
    return radius


def ball_bounds(q, centre, radius):
    """f [S][n_groups] of Eq. (2)."""
    centre = np.ascontiguousarray(centre, dtype=np.float64)
    radius = np.ascontiguousarray(radius, dtype=np.float64)
    n_groups, d = centre.shape
    S = radius.shape[1]
    q = np.ascontiguousarray(q, dtype=np.float32)
    f = np.empty((S, n_groups), dtype=np.float64)
    _load().lvo_ball_bounds(_p(q), d, S, _p(centre), _p(radius), n_groups, _p(f))
    return f


def aabb_index(K, label, n_groups):
    """Per-group coordinate-wise minimum and maximum: (lo, hi), each [n_groups][d] fp64."""
    K, bf = _kv(K)
    n, d = K.shape
    label = np.ascontiguousarray(label, dtype=np.int32)
    lo = np.empty((n_groups, d), dtype=np.float64)
    hi = np.empty((n_groups, d), dtype=np.float64)
    _load().lvo_aabb_index(_p(K), bf, n, d, _p(label), n_groups, _p(lo), _p(hi))
    return lo, hi


def aabb_bounds(q, lo, hi):
    """Largest <q, x> over each box: [n_groups] fp64."""
    lo = np.ascontiguousarray(lo, dtype=np.float64)
    hi = np.ascontiguousarray(hi, dtype=np.float64)
    q = np.ascontiguousarray(q, dtype=np.float32)
    ub = np.empty(lo.shape[0], dtype=np.float64)
    _load().lvo_aabb_bounds(_p(q), lo.shape[1], _p(lo), _p(hi), lo.shape[0], _p(ub))
    return ub


def query1_filter(f, label, tau_s):
    """Alg. 3's candidate mask: f [S][n_groups], label [S][n], tau_s [S] -> bool [n]."""
    f = np.ascontiguousarray(f, dtype=np.float64)
    label = np.ascontiguousarray(label, dtype=np.int32)
    tau_s = np.ascontiguousarray(tau_s, dtype=np.float64)
    S, n_groups = f.shape
    n = label.shape[1]
    alive = np.zeros(n, dtype=np.uint8)
    _load().lvo_query1_filter(_p(f), _p(label), S, n_groups, n, _p(tau_s), _p(alive))
    return alive.astype(bool)


def safe_subspace_thresholds(f, tau: float):
    """Thresholds tau_s [S] valid for every key with <q,k> >= tau: tau minus the largest ball
    bounds of the other subspaces (f [S][n_groups])."""
    f = np.ascontiguousarray(f, dtype=np.float64)
    S, n_groups = f.shape
    out = np.empty(S, dtype=np.float64)
    _load().lvo_safe_subspace_thresholds(_p(f), S, n_groups, float(tau), _p(out))
    return out


def ta_filter(f, label, tau):
    """f [S][n_groups], label [S][n] -> (alive mask [n] bool, stopping depth)."""
    f = np.ascontiguousarray(f, dtype=np.float64)
    label = np.ascontiguousarray(label, dtype=np.int32)
    S, n_groups = f.shape
    n = label.shape[1]
    alive = np.zeros(n, dtype=np.uint8)
    depth = _load().lvo_ta_filter(_p(f), _p(label), S, n_groups, n, float(tau), _p(alive))
    return alive.astype(bool), int(depth)


def balanced_tree(K, r, lo=0, hi=None):
    """Leaf labels [n] (int32), left-to-right key order [n] (int64), number of leaves."""
    K, bf = _kv(K)
    n, d = K.shape
    hi = d if hi is None else hi
    label = np.zeros(max(n, 1), dtype=np.int32)
    order = np.zeros(max(n, 1), dtype=np.int64)
    leaves = _load().lvo_balanced_tree(_p(K), bf, n, d, lo, hi, r, _p(label), _p(order))
    return label[:n], order[:n], int(leaves)


def predicted_speedup(g: float, r: int, f_scan: float) -> float:
    """Cost model of the index family (appendix "Ablation on Index Design", paragraph
    "Achieving high pruning"): query cost is proportional to g/r + f_scan, so the speed-up
    over brute force is its reciprocal."""
    return 1.0 / (g / r + f_scan)


THRESHOLD_MODES = {"sample-max": 0, "sample-mean-max": 1, "sample-gap": 2, "sample-topk": 3, "budget": 4}


def hash32(seed: int, stream: int, counter: int) -> int:
    return int(_load().lvo_hash32(seed, stream, counter))


def reservoir(seed: int, stream: int, n: int, R: int = 256):
    """Positions held by the reservoir after the first n keys (appendix "Threshold Oracle Comparison")."""
    res = np.full(max(min(n, R), 1), -1, dtype=np.int32)
    _load().lvo_reservoir(seed, stream, n, R, _p(res))
    return res[:min(n, R)]


def threshold(scores, mode: str, param: float = 0.0) -> float:
    s = np.ascontiguousarray(scores, dtype=np.float32)
    return float(_load().lvo_threshold(_p(s), s.size, THRESHOLD_MODES[mode], float(param)))
