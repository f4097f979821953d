"""Helpers shared by the GPU parity tests: upload seeded inputs, run the library through its
binding, and compare with the CPU oracle by the stated parity rule."""
from __future__ import annotations

import math
import sys

import numpy as np
import torch

import paper_2605_06763_amd as L
import workloads as W

REL_BAND = 1e-4          # keys with |score - tau| < REL_BAND * |tau| may go either way
ATTN_TOL = 2e-3          # max_c |out - ref| / max_c |ref| per head


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def to_device(x: np.ndarray, dtype: str) -> torch.Tensor:
    """fp32 numpy array (values exact in `dtype`) -> device tensor of that dtype."""
    if dtype == "bf16":
        bits = W.f32_to_bf16_bits(x).reshape(x.shape)
        return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()


class Index:
    """A library index plus the host copy of what it holds (for the oracle)."""

    def __init__(self, K: np.ndarray, V: np.ndarray, dtype: str, n_q_heads: int, *, capacity=None,
                 group_size=4, n_subspaces=4, buffer_size=256, flags=0, grouping=L.LVR_GROUP_CONTIGUOUS,
                 enclosing=L.LVR_ENCLOSE_BALL, scale=0.0, attn_splits=0, reservoir_size=0, seed=0, index_dtype=0,
                 query_workgroups=0):
        batch, hkv, n, d = K.shape
        self.dtype = dtype
        self.K, self.V = K.copy(), V.copy()
        self.hq, self.hkv, self.batch, self.d = n_q_heads, hkv, batch, d
        self.G = n_q_heads // hkv
        self.sigma = scale if scale > 0 else 1.0 / math.sqrt(d)
        self.cfg = L.make_config(batch=batch, n_q_heads=n_q_heads, n_kv_heads=hkv, head_dim=d,
                                 kv_dtype=L.LVR_BF16 if dtype == "bf16" else L.LVR_F32,
                                 group_size=group_size, n_subspaces=n_subspaces, buffer_size=buffer_size,
                                 grouping=grouping, enclosing=enclosing, flags=flags, capacity=capacity or max(n, 1), scale=scale,
                                 attn_splits=attn_splits, reservoir_size=reservoir_size, seed=seed,
                                 index_dtype=index_dtype, query_workgroups=query_workgroups)
        self.h = L.lvr_create(self.cfg)
        self.Kd, self.Vd = to_device(K, dtype), to_device(V, dtype)
        L.lvr_build(self.h, self.Kd, self.Vd)

    def close(self):
        if self.h is not None:
            L.lvr_destroy(self.h)
            self.h = None

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    @property
    def n(self):
        return self.K.shape[2]

    def append(self, k_new: np.ndarray, v_new: np.ndarray):
        """k_new, v_new: [batch][hkv][m][d] fp32 (exact in dtype)."""
        L.lvr_append(self.h, to_device(k_new, self.dtype), to_device(v_new, self.dtype))
        self.K = np.concatenate([self.K, k_new], axis=2)
        self.V = np.concatenate([self.V, v_new], axis=2)

    def query(self, q: np.ndarray, tau: np.ndarray, cap=None, fused=False):
        cap = self.n if cap is None else cap
        qd = torch.from_numpy(np.ascontiguousarray(q, dtype=np.float32)).cuda()
        td = torch.from_numpy(np.ascontiguousarray(tau, dtype=np.float32)).cuda()
        idx = torch.full((self.batch, self.hq, max(cap, 1)), -7, dtype=torch.int32, device="cuda")
        cnt = torch.full((self.batch, self.hq), -7, dtype=torch.int32, device="cuda")
        out = torch.full((self.batch, self.hq, self.d), float("nan"), dtype=torch.float32, device="cuda")
        if fused:
            L.lvr_decode_step(self.h, qd, td, out, idx, cnt)
        else:
            L.lvr_query(self.h, qd, td, idx, cnt)
            L.lvr_sparse_attention(self.h, qd, idx, cnt, out)
        torch.cuda.synchronize()
        return idx.cpu().numpy(), cnt.cpu().numpy(), out.cpu().numpy()

    def dense(self, q: np.ndarray):
        qd = torch.from_numpy(np.ascontiguousarray(q, dtype=np.float32)).cuda()
        out = torch.full((self.batch, self.hq, self.d), float("nan"), dtype=torch.float32, device="cuda")
        L.lvr_dense_attention(self.h, qd, out)
        torch.cuda.synchronize()
        return out.cpu().numpy()

    def threshold(self, q: np.ndarray, mode: str, param: float = 0.0):
        qd = torch.from_numpy(np.ascontiguousarray(q, dtype=np.float32)).cuda()
        tau = torch.full((self.batch, self.hq), float("nan"), dtype=torch.float32, device="cuda")
        L.lvr_threshold(self.h, qd, mode, param, tau)
        torch.cuda.synchronize()
        return tau.cpu().numpy()

    def reservoir(self):
        return L.lvr_export_reservoir(self.h, self.cfg)

    def stats(self, **kw):
        return L.lvr_get_stats(self.h, **kw)

    def export(self):
        return L.lvr_export_index(self.h, self.cfg)

    def channel_factors(self):
        """[batch][hkv][128] float64: 2^e_c of the space the index is stored in (ones unless it is a rescaled 6-bit
        index).  The stored balls enclose K / factors around centres / factors, and bound <q * factors, .>."""
        return 2.0 ** L.lvr_export_channel_scales(self.h, self.cfg).astype(np.float64)


def check_head(oracle, q, Kh, Vh, tau, got_idx, got_count, got_out, sigma, *, extra_from=-1, where=""):
    """Parity of one (sequence, head): retrieved set by the band rule, attention against the
    oracle run on the GPU's own list (and on the oracle's list when the sets agree)."""
    s = oracle.scores_f32(q, Kh)
    n = s.shape[0]
    assert got_count >= 0, where
    got = got_idx[:got_count]
    assert got.size == np.unique(got).size, f"{where}: duplicate positions"
    assert got.size == 0 or (got.min() >= 0 and got.max() < n), f"{where}: position out of range"
    gset = np.zeros(n, dtype=bool)
    gset[got] = True
    band = REL_BAND * abs(float(tau)) if np.isfinite(tau) else 0.0
    extra = np.zeros(n, dtype=bool)
    if extra_from >= 0:
        extra[extra_from:] = True
    oracle_set = (s >= tau) | extra
    must = (s >= tau + band) | extra
    may = np.abs(s - tau) < band if band > 0 else np.zeros(n, dtype=bool)
    missing = oracle_set & ~gset
    assert not missing.any(), f"{where}: FALSE NEGATIVES at {np.nonzero(missing)[0][:8]} tau={tau}"
    spurious = gset & ~(must | may)
    assert not spurious.any(), f"{where}: keys below the band at {np.nonzero(spurious)[0][:8]} s={s[spurious][:4]} tau={tau}"
    ref = oracle.attention_on_list(q, Kh, Vh, np.sort(got), sigma)
    denom = max(float(np.abs(ref).max()), 1e-30)
    err = float(np.abs(got_out - ref).max()) / denom if got.size else float(np.abs(got_out).max())
    assert err <= ATTN_TOL, f"{where}: attention error {err:.3e} on {got.size} keys"
    return dict(size=int(got.size), borderline=int((gset != oracle_set).sum()), attn_err=err)


def check_step(oracle, ix: Index, q, tau, idx, cnt, out, *, heads=None, extra_from=-1, tag=""):
    """All (or the given) heads of one decode step."""
    worst, sizes, border = 0.0, 0, 0
    for b in range(ix.batch):
        for h in (range(ix.hq) if heads is None else heads):
            g = h // ix.G
            r = check_head(oracle, q[b, h], ix.K[b, g], ix.V[b, g], tau[b, h], idx[b, h], int(cnt[b, h]),
                           out[b, h], ix.sigma, extra_from=extra_from, where=f"{tag} b={b} h={h}")
            worst = max(worst, r["attn_err"])
            sizes += r["size"]
            border += r["borderline"]
    return dict(attn_err=worst, retrieved=sizes, borderline=border)


def oracle_taus(oracle, ix: Index, q, k_count=None, frac=None):
    """Per-head thresholds from the oracle's fp32 scores: midpoint so that exactly k keys qualify."""
    tau = np.zeros((ix.batch, ix.hq), dtype=np.float32)
    for b in range(ix.batch):
        for h in range(ix.hq):
            s = oracle.scores_f32(q[b, h], ix.K[b, h // ix.G])
            k = k_count if k_count is not None else int(math.ceil(frac * s.shape[0]))
            tau[b, h] = W.tau_for_count(s, k)
    return tau


def subspace_thresholds(ix: Index, q: np.ndarray, tau: np.ndarray) -> np.ndarray:
    """lvr_subspace_thresholds -> [batch][hq][S] fp32."""
    qd = torch.from_numpy(np.ascontiguousarray(q, dtype=np.float32)).cuda()
    td = torch.from_numpy(np.ascontiguousarray(tau, dtype=np.float32)).cuda()
    out = torch.full((ix.batch, ix.hq, ix.cfg.n_subspaces), float("nan"), dtype=torch.float32, device="cuda")
    L.lvr_subspace_thresholds(ix.h, qd, td, out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def query1(ix: Index, q: np.ndarray, tau_s: np.ndarray, tau: np.ndarray, cap=None):
    """lvr_query1 followed by lvr_sparse_attention; tau_s [batch][hq][S]."""
    cap = ix.n if cap is None else cap
    qd = torch.from_numpy(np.ascontiguousarray(q, dtype=np.float32)).cuda()
    td = torch.from_numpy(np.ascontiguousarray(tau, dtype=np.float32)).cuda()
    tsd = torch.from_numpy(np.ascontiguousarray(tau_s, dtype=np.float32)).cuda()
    idx = torch.full((ix.batch, ix.hq, max(cap, 1)), -7, dtype=torch.int32, device="cuda")
    cnt = torch.full((ix.batch, ix.hq), -7, dtype=torch.int32, device="cuda")
    out = torch.full((ix.batch, ix.hq, ix.d), float("nan"), dtype=torch.float32, device="cuda")
    L.lvr_query1(ix.h, qd, tsd, td, idx, cnt)
    L.lvr_sparse_attention(ix.h, qd, idx, cnt, out)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), cnt.cpu().numpy(), out.cpu().numpy()
