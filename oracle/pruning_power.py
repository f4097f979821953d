"""Pruning power of the index family on the synthetic workloads, computed on the CPU with the
oracle alone (test infrastructure, like everything under oracle/; nothing in the product path
uses it).  For one KV head of a workload and a few queries it builds, for every (grouping, S, r),
the balls of Eq. (1) exactly as the oracle defines them and reports the share of keys that

  - the summed-bound rule keeps (key j iff sum_s f_{s,a(s,j)} >= tau; "Query 2"'s bound per key),
  - Alg. 4's depth scan keeps (its live set: union over subspaces of the first d* clusters),

per query head.  Groupings: contiguous (r consecutive positions, the same in every subspace), one
axis-median tree over the full key shared by all subspaces, one tree per subspace (Alg. 1 as printed).

    python -m oracle.pruning_power <config id> <n keys> <r,r,...> [<S,S,...>]
    python -m oracle.pruning_power codings <config id> <n keys>       (groups of one key, coded centres)

The design notes quote its output for configs 2 and 3.
"""
from __future__ import annotations

import sys

import numpy as np

import oracle
import workloads as W


def balls(K, labels, S, ng):
    """Per subspace: centres [ng][d_s] (means) and radii [ng] (largest member distance), fp64."""
    n, d = K.shape
    ds = d // S
    cen, rad = np.zeros((S, ng, ds)), np.zeros((S, ng))
    for s in range(S):
        P = K[:, s * ds:(s + 1) * ds].astype(np.float64)
        lab = labels[s]
        cnt = np.bincount(lab, minlength=ng).astype(np.float64)
        c = np.zeros((ng, ds))
        np.add.at(c, lab, P)
        c /= np.maximum(cnt, 1)[:, None]
        r = np.zeros(ng)
        np.maximum.at(r, lab, np.sqrt(((P - c[lab]) ** 2).sum(1)))
        cen[s], rad[s] = c, r
    return cen, rad


def bounds(q, cen, rad):
    """f [S][ng] of Eq. (2)."""
    S, ng, ds = cen.shape
    f = np.empty((S, ng))
    for s in range(S):
        qs = q[s * ds:(s + 1) * ds].astype(np.float64)
        f[s] = cen[s] @ qs + rad[s] * np.linalg.norm(qs)
    return f


def run(cid, n, r_list, S_list, n_queries=3, kv_head=0):
    oracle.build()
    c = W.CONFIGS[cid]
    K = W.make_cache(cid, n=n, n_kv_heads=kv_head + 1).K[0, kv_head]
    qs = [W.make_queries(cid, n_q_heads=4, step=t)[0, 0] for t in range(n_queries)]
    frac = c.get("qualify_frac", 0.005)
    for r in r_list:
        ng = n // r
        for S in S_list:
            ds = 128 // S
            shared, _, leaves = oracle.balanced_tree(K, r)
            assert leaves == ng
            per = np.stack([oracle.balanced_tree(K, r, s * ds, (s + 1) * ds)[0] for s in range(S)])
            groupings = {"contiguous": np.tile((np.arange(n) // r).astype(np.int32), (S, 1)),
                         "shared tree": np.tile(shared, (S, 1)), "tree per subspace": per}
            for name, labels in groupings.items():
                cen, rad = balls(K, labels, S, ng)
                keep_sum, keep_ta = [], []
                for q in qs:
                    sc = K.astype(np.float64) @ q.astype(np.float64)
                    tau = float(W.tau_for_fraction(sc.astype(np.float32), frac))
                    f = bounds(q, cen, rad)
                    ub = sum(f[s][labels[s]] for s in range(S))
                    assert (ub >= sc - 1e-6).all(), "a summed bound below a key's score"
                    keep_sum.append(float((ub >= tau).mean()))
                    keep_ta.append(float(oracle.ta_filter(f, labels, tau)[0].mean()))
                print(f"config {cid} n={n} r={r} S={S:2d} {name:18s} summed bounds keep {np.mean(keep_sum):.4f}   "
                      f"depth scan keeps {np.mean(keep_ta):.4f}", flush=True)


def _grid(exp_bits, man_bits, bias, top=None):
    """Non-negative values of a small float format (subnormals included), ascending."""
    v = {0.0}
    for e in range(1 << exp_bits):
        for m in range(1 << man_bits):
            x = (m / (1 << man_bits)) * 2.0 ** (1 - bias) if e == 0 else (1 + m / (1 << man_bits)) * 2.0 ** (e - bias)
            if top is None or x <= top:
                v.add(x)
    return np.array(sorted(v))


E4M3 = _grid(4, 3, 7, top=448.0)     # one byte per coordinate
E2M3 = _grid(2, 3, 1)                # six bits per coordinate, largest value 7.5


def _nearest(a, grid):
    i = np.searchsorted(grid, a).clip(1, len(grid) - 1)
    lo, hi = grid[i - 1], grid[i]
    return np.where(a - lo <= hi - a, lo, hi)


def code_keys(K, coding):
    """Every key rounded to a coded centre of its own (groups of one key): 'bf16' (the key itself), 'e4m3'
    (one byte per coordinate), 'e2m3' (six bits per coordinate times one power-of-two scale per block of 32
    coordinates; block b holds coordinates 32 kk + 8 b + e, kk = 0..3, e = 0..7: the smallest scale that brings
    the block's largest magnitude to at most 7.5)."""
    K = K.astype(np.float64)
    if coding == "bf16":
        return K.copy()
    if coding == "e4m3":
        return np.sign(K) * _nearest(np.minimum(np.abs(K), 448.0), E4M3)
    n = K.shape[0]
    B = np.moveaxis(K.reshape(n, 4, 4, 8), 2, 1).reshape(n, 4, 32)
    amax = np.abs(B).max(-1, keepdims=True)
    scale = 2.0 ** np.ceil(np.log2(np.maximum(amax, 1e-300) / 7.5))
    C = np.sign(B) * _nearest(np.minimum(np.abs(B) / scale, 7.5), E2M3) * scale
    return np.moveaxis(C.reshape(n, 4, 4, 8), 1, 2).reshape(n, 128)


def channel_factors(K):
    """One power of two per coordinate, 2^round(L_c - o) with L_c = log2 of the coordinate's root mean square over the
    keys and o the circular mean of the fractional parts of L (coordinates of about the same size then get the same
    factor instead of being split by a rounding boundary that falls among them); exponents held to [-8, 8]."""
    ms = (K.astype(np.float64) ** 2).mean(axis=0)
    live = ms > 0
    L = np.where(live, 0.5 * np.log2(np.where(live, ms, 1.0)), 0.0)
    z = np.exp(2j * np.pi * L[live]).sum() if live.any() else 0.0
    o = float(np.angle(z)) / (2 * np.pi) if z != 0 else 0.0
    return 2.0 ** np.where(live, np.clip(np.rint(L - o), -8, 8), 0.0)


def coded_keep(cid, n, coding, S=4, n_queries=3, kv_head=0):
    """Share of keys whose ball (coded centre, exact radius per coordinate block) reaches tau: per head and for
    the four heads of a KV head together (a key row is read if any head keeps it); also the mean radius relative
    to the key's norm.  Every bound is checked to lie above the key's score.  A coding 'x/chan' codes the keys
    divided coordinate by coordinate by channel_factors and meets them with q times the factors: every product
    <q,k> is unchanged, the balls (centres, radii, the blocks' scales) live in the rescaled space."""
    c = W.CONFIGS[cid]
    K0 = W.make_cache(cid, n=n, n_kv_heads=kv_head + 1).K[0, kv_head].astype(np.float64)
    a = channel_factors(K0) if coding.endswith("/chan") else np.ones(K0.shape[1])
    K = K0 / a
    C = code_keys(K, coding.split("/")[0])
    ds = 128 // S
    rad = np.stack([np.sqrt((((K - C)[:, s * ds:(s + 1) * ds]) ** 2).sum(1)) for s in range(S)])
    frac = c.get("qualify_frac", 0.005)
    per, union = [], []
    drift = W.drift_queries(3, 256, n_q_heads=32) if cid == 3 else None   # config 3's queries drift, as in the bench
    for t in range(n_queries):
        Q = drift[(t * 85) % 256][0][:4] if drift is not None else W.make_queries(cid, n_q_heads=4, step=t)[0]
        any_keep = np.zeros(n, dtype=bool)
        for hq in range(4):
            q = Q[hq].astype(np.float64) * a
            sc = K @ q
            tau = float(W.tau_for_fraction(sc.astype(np.float32), frac))
            ub = C @ q + sum(rad[s] * np.linalg.norm(q[s * ds:(s + 1) * ds]) for s in range(S))
            assert (ub >= sc - 1e-9 * np.abs(sc).max()).all(), "a bound below a key's score"
            keep = ub >= tau
            per.append(float(keep.mean()))
            any_keep |= keep
        union.append(float(any_keep.mean()))
    rel = float(np.sqrt((rad ** 2).sum(0)).mean() / np.linalg.norm(K, axis=1).mean())
    return dict(per_head=float(np.mean(per)), per_kv_head=float(np.mean(union)), relative_radius=rel)


if __name__ == "__main__":
    if sys.argv[1] == "codings":   # python -m oracle.pruning_power codings <config id> <n keys>
        for coding in ("bf16", "e4m3", "e2m3", "e2m3/chan"):
            r = coded_keep(int(sys.argv[2]), int(sys.argv[3]), coding)
            print(f"config {sys.argv[2]} n={sys.argv[3]} r=1 S=4 centres {coding:9s} keep per head {r['per_head']:.4f}  "
                  f"per KV head {r['per_kv_head']:.4f}  radius / |k| {r['relative_radius']:.4f}", flush=True)
        sys.exit(0)
    cid, n = int(sys.argv[1]), int(sys.argv[2])
    r_list = [int(x) for x in sys.argv[3].split(",")]
    S_list = [int(x) for x in sys.argv[4].split(",")] if len(sys.argv) > 4 else [4, 8, 16]
    run(cid, n, r_list, S_list)
