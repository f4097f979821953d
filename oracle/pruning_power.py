"""Pruning power of the index family on the synthetic workloads, computed on the CPU with the
oracle alone (test infrastructure, like everything under oracle/; nothing in the product path
uses it).  For one KV head of a workload and a few queries it builds, for every (grouping, S, r),
the balls of Eq. (1) exactly as the oracle defines them and reports the share of keys that

  - the summed-bound rule keeps (key j iff sum_s f_{s,a(s,j)} >= tau; "Query 2"'s bound per key),
  - Alg. 4's depth scan keeps (its live set: union over subspaces of the first d* clusters),

per query head.  Groupings: contiguous (r consecutive positions, the same in every subspace), one
axis-median tree over the full key shared by all subspaces, one tree per subspace (Alg. 1 as printed).

    python -m oracle.pruning_power <config id> <n keys> <r,r,...> [<S,S,...>]

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


if __name__ == "__main__":
    cid, n = int(sys.argv[1]), int(sys.argv[2])
    r_list = [int(x) for x in sys.argv[3].split(",")]
    S_list = [int(x) for x in sys.argv[4].split(",")] if len(sys.argv) > 4 else [4, 8, 16]
    run(cid, n, r_list, S_list)
