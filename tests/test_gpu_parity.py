"""GPU parity tests at sizes the oracle finishes in seconds: every entry point goes through the
C ABI (ctypes binding) and is compared element by element with the CPU oracle."""
import math
import ctypes as C

import numpy as np
import pytest
import torch

import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import gpu_util
    assert torch.cuda.is_available(), "these tests need the GPU"
    return gpu_util


def _small_cache(config_id, n, hkv=2, batch=1):
    c = W.make_cache(config_id, n=n, n_kv_heads=hkv, batch=batch)
    return c


# ------------------------------------------------------------------ config 1 (fp32, whole size)
def test_config1_fp32_single_head(G, oracle):
    """Single head, d=128, n=4096, fp32, about 2 % qualify, 8 planted keys."""
    G.say("config1: build inputs")
    cache = W.make_cache(1)
    q = W.make_queries(1)
    K = cache.K[0, 0]
    s = oracle.scores_f32(q[0, 0], K)
    tau = float(W.tau_for_fraction(s, 0.02))
    rows = W.planted_positions(1, K.shape[0], 8)
    W.plant_rows(K, rows, (tau + 0.25) / s[rows], "f32")
    with G.Index(cache.K, cache.V, "f32", 1) as ix:
        taus = np.full((1, 1), tau, dtype=np.float32)
        for fused in (False, True):
            idx, cnt, out = ix.query(q, taus, fused=fused)
            r = G.check_step(oracle, ix, q, taus, idx, cnt, out, tag=f"config1 fused={fused}")
            assert set(rows.tolist()) <= set(idx[0, 0, :cnt[0, 0]].tolist())
            assert 82 <= cnt[0, 0] <= 82 + 8
            G.say("config1", r, ix.stats())


# ------------------------------------------------------------------ bf16 GQA, ragged sizes
@pytest.mark.parametrize("separate", [0, 2], ids=["fused", "two_kernels"])
@pytest.mark.parametrize("n", [1, 3, 64, 1000, 2051, 4096])
def test_gqa_bf16_sets_and_attention(G, oracle, n, separate):
    G.say(f"gqa bf16 n={n} flags={separate}")
    cache = _small_cache(2, n)
    q = W.make_queries(2, n_q_heads=8)
    with G.Index(cache.K, cache.V, "bf16", 8, flags=separate) as ix:
        for frac in (0.01, 0.2):
            tau = G.oracle_taus(oracle, ix, q, frac=frac)
            idx, cnt, out = ix.query(q, tau)
            r = G.check_step(oracle, ix, q, tau, idx, cnt, out, tag=f"n={n} frac={frac}")
            st = ix.stats()
            assert st["keys_emitted"] == int(cnt.sum())
            assert st["n_keys"] == n and st["n_indexed"] == n // 4 * 4
            G.say(f"  frac={frac}", r, {k: st[k] for k in ("groups_scored", "groups_surviving", "keys_scanned")})
        # dense baseline against the oracle's dense attention
        ref = oracle.dense_attention(ix.K, ix.V, q, ix.sigma, 8)
        got = ix.dense(q)
        err = np.abs(got - ref).max(axis=-1) / np.abs(ref).max(axis=-1)
        assert err.max() <= G.ATTN_TOL, err


def test_tau_extremes(G, oracle):
    """tau = -inf retrieves every key and reproduces dense attention; tau above every score
    retrieves nothing and returns zeros."""
    n = 777
    cache = _small_cache(2, n)
    q = W.make_queries(2, n_q_heads=8)
    with G.Index(cache.K, cache.V, "bf16", 8) as ix:
        tau = np.full((1, 8), -np.inf, dtype=np.float32)
        idx, cnt, out = ix.query(q, tau)
        assert (cnt == n).all()
        for h in range(8):
            assert sorted(idx[0, h, :n].tolist()) == list(range(n))
        ref = oracle.dense_attention(ix.K, ix.V, q, ix.sigma, 8)
        assert (np.abs(out - ref).max(axis=-1) / np.abs(ref).max(axis=-1)).max() <= G.ATTN_TOL
        assert (np.abs(ix.dense(q) - ref).max(axis=-1) / np.abs(ref).max(axis=-1)).max() <= G.ATTN_TOL
        tau = np.full((1, 8), np.inf, dtype=np.float32)
        idx, cnt, out = ix.query(q, tau)
        assert (cnt == 0).all() and (out == 0).all()
        assert ix.stats()["groups_surviving"] == 0
        # mixed: one head takes everything, its neighbours nothing
        tau = np.full((1, 8), np.inf, dtype=np.float32)
        tau[0, 5] = -np.inf
        idx, cnt, out = ix.query(q, tau)
        assert cnt[0].tolist() == [0, 0, 0, 0, 0, n, 0, 0]
        assert np.abs(out[0, 5] - ref[0, 5]).max() / np.abs(ref[0, 5]).max() <= G.ATTN_TOL


@pytest.mark.parametrize("r", [1, 4])
def test_tau_zero_and_tiny(G, oracle, r):
    """tau = 0 ("every key with a non-negative product") and |tau| tiny: the relative slack of the
    comparison vanishes there, so the promise is the absolute one of the header.  Integer-valued
    data (every sum exact) is decided exactly, zeros included; on real-valued data every key whose
    exact score clears tau by more than d * 2^-23 * sum|q_c k_c| comes back and nothing that far below does."""
    g = np.random.default_rng(77)
    n, hq, hkv = 3000, 8, 2
    Ki = g.integers(-3, 4, size=(1, hkv, n, 128)).astype(np.float32)
    Vi = W.round_to_bf16(g.standard_normal((1, hkv, n, 128)).astype(np.float32))
    qi = g.integers(-2, 3, size=(1, hq, 128)).astype(np.float32)
    with G.Index(Ki, Vi, "bf16", hq, group_size=r) as ix:
        for t in (0.0, 1.0, -1.0):
            tau = np.full((1, hq), t, dtype=np.float32)
            idx, cnt, out = ix.query(qi, tau, fused=True)
            for h in range(hq):
                s = oracle.scores_f64(qi[0, h], Ki[0, h // 4])
                want = set(np.nonzero(s >= t - 0.5e-4 * abs(t))[0].tolist())    # exact scores: exactly the kernel's rule
                assert set(idx[0, h, :cnt[0, h]].tolist()) == want, (t, h)
                assert (s == 0).sum() > 0                                        # the tie at zero is really there
    cache = _small_cache(2, n)
    q = W.make_queries(2, n_q_heads=hq)
    with G.Index(cache.K, cache.V, "bf16", hq, group_size=r) as ix:
        for t in (0.0, 1e-6, -1e-6):
            tau = np.full((1, hq), t, dtype=np.float32)
            idx, cnt, out = ix.query(q, tau, fused=True)
            for h in range(hq):
                Kh = cache.K[0, h // 4].astype(np.float64)
                s = Kh @ q[0, h].astype(np.float64)
                slack = 128 * 2.0 ** -23 * (np.abs(Kh) @ np.abs(q[0, h].astype(np.float64)))
                got = np.zeros(n, dtype=bool)
                got[idx[0, h, :cnt[0, h]]] = True
                assert not np.any((s >= t + slack) & ~got), (t, h, "a key clearly above tau is missing")
                assert not np.any((s <= t - slack) & got), (t, h, "a key clearly below tau came back")
                assert abs(int(got.sum()) - int((s >= t).sum())) <= 2


def test_empty_index(G, oracle):
    cache = _small_cache(2, 0)
    q = W.make_queries(2, n_q_heads=8)
    with G.Index(cache.K, cache.V, "bf16", 8, capacity=64) as ix:
        idx, cnt, out = ix.query(q, np.zeros((1, 8), np.float32), cap=4)
        assert (cnt == 0).all() and (out == 0).all()
        assert (ix.dense(q) == 0).all()


def test_exact_ties_integer_data(G, oracle):
    """Integer-valued keys and queries: fp32 dot products are exact in any summation order, so
    the sets must equal the oracle's exactly, ties at tau included (>=, not >)."""
    g = np.random.default_rng(5)
    n = 1024
    K = g.integers(-4, 5, size=(1, 2, n, 128)).astype(np.float32)
    V = g.integers(-4, 5, size=(1, 2, n, 128)).astype(np.float32)
    q = g.integers(-3, 4, size=(1, 4, 128)).astype(np.float32)
    for dtype in ("bf16", "f32"):
        with G.Index(K, V, dtype, 4) as ix:
            for quant in (0.99, 0.9):
                tau = np.zeros((1, 4), dtype=np.float32)
                for h in range(4):
                    s = oracle.scores_f32(q[0, h], K[0, h // 2])
                    # a value that occurs among the scores; scaled so tau - 0.5e-4|tau| stays above the next integer
                    tau[0, h] = np.sort(s)[int(quant * n)]
                idx, cnt, out = ix.query(q, tau)
                for h in range(4):
                    want = oracle.range_query(q[0, h], K[0, h // 2], tau[0, h])
                    assert sorted(idx[0, h, :cnt[0, h]].tolist()) == want.tolist(), (dtype, quant, h)


@pytest.mark.parametrize("separate", [0, 2], ids=["fused", "two_kernels"])
@pytest.mark.parametrize("r,S", [(1, 4), (2, 1), (8, 16), (16, 2), (4, 8)])
def test_group_size_and_subspaces(G, oracle, r, S, separate):
    n = 1500
    cache = _small_cache(2, n)
    q = W.make_queries(2, n_q_heads=8)
    with G.Index(cache.K, cache.V, "bf16", 8, group_size=r, n_subspaces=S, buffer_size=64, flags=separate) as ix:
        tau = G.oracle_taus(oracle, ix, q, frac=0.03)
        idx, cnt, out = ix.query(q, tau)
        G.check_step(oracle, ix, q, tau, idx, cnt, out, tag=f"r={r} S={S}")
        st = ix.stats()
        assert st["n_indexed"] == n // r * r


@pytest.mark.parametrize("separate", [0, 2], ids=["fused", "two_kernels"])
@pytest.mark.parametrize("hq,hkv", [(2, 2), (4, 2), (16, 2), (8, 1)])
def test_head_group_sizes(G, oracle, hq, hkv, separate):
    n = 900
    cache = _small_cache(2, n, hkv=hkv, batch=2)
    q = W.make_queries(2, n_q_heads=hq, batch=2)
    with G.Index(cache.K, cache.V, "bf16", hq, flags=separate) as ix:
        tau = G.oracle_taus(oracle, ix, q, frac=0.05)
        idx, cnt, out = ix.query(q, tau, fused=True)
        G.check_step(oracle, ix, q, tau, idx, cnt, out, tag=f"hq={hq} hkv={hkv}")
        ref = oracle.dense_attention(ix.K, ix.V, q, ix.sigma, hq)
        assert (np.abs(ix.dense(q) - ref).max(axis=-1) / np.abs(ref).max(axis=-1)).max() <= G.ATTN_TOL


@pytest.mark.parametrize("splits", [-1, 0, 7])
def test_non_default_scale_and_general_fp32_query(G, oracle, splits):
    n = 1200
    cache = _small_cache(2, n)
    q = W.make_queries(2, n_q_heads=8, exact_bf16=False)      # full fp32 query values
    with G.Index(cache.K, cache.V, "bf16", 8, scale=0.031, attn_splits=splits) as ix:
        tau = G.oracle_taus(oracle, ix, q, frac=0.04)
        for fused in (False, True):
            idx, cnt, out = ix.query(q, tau, fused=fused)
            G.check_step(oracle, ix, q, tau, idx, cnt, out, tag=f"scale=0.031 splits={splits} step={fused}")
            assert ix.stats()["keys_emitted"] == int(cnt.sum())


def test_overflow_is_reported_not_silent(G, oracle):
    import paper_2605_06763_amd as L
    n = 512
    cache = _small_cache(2, n)
    q = W.make_queries(2, n_q_heads=8)
    with G.Index(cache.K, cache.V, "bf16", 8) as ix:
        tau = G.oracle_taus(oracle, ix, q, k_count=40)
        idx, cnt, out = ix.query(q, tau, cap=16)
        assert (cnt == 40).all()                      # true sizes even though lists are truncated
        with pytest.raises(L.LouverError) as e:
            ix.stats()
        assert e.value.code == L.LVR_E_OVERFLOW
        for h in range(8):                            # what was written is a subset of the true set
            want = set(oracle.range_query(q[0, h], ix.K[0, h // 4], tau[0, h]).tolist())
            assert set(idx[0, h, :16].tolist()) <= want
        idx, cnt, out = ix.query(q, tau, cap=64)      # flag is cleared, a roomy call is clean
        assert ix.stats()["overflow"] == 0


@pytest.mark.parametrize("splits", [-1, 0, 5, 32], ids=["one_launch", "default", "5_splits", "32_splits"])
def test_sparse_attention_on_caller_lists(G, oracle, splits):
    """lvr_sparse_attention on lists the caller made up (unsorted, with out-of-range entries,
    uneven lengths including empty), in the one-launch form and with partials through HBM."""
    import paper_2605_06763_amd as L
    n = 640
    cache = _small_cache(2, n)
    q = W.make_queries(2, n_q_heads=8)
    g = np.random.default_rng(3)
    with G.Index(cache.K, cache.V, "bf16", 8, attn_splits=splits) as ix:
        cap = 300
        idx = np.zeros((1, 8, cap), dtype=np.int32)
        cnt = np.array([[0, 1, 2, 5, 64, 65, 299, 300]], dtype=np.int32)
        lists = []
        for h in range(8):
            l = g.permutation(n)[:cnt[0, h]].astype(np.int32)
            idx[0, h, :cnt[0, h]] = l
            lists.append(l)
        idx[0, 6, 10] = n + 5          # out of range entries are skipped
        idx[0, 6, 11] = -1
        lists[6] = np.delete(lists[6], [10, 11])
        qd = torch.from_numpy(q).cuda()
        out = torch.zeros((1, 8, 128), device="cuda")
        L.lvr_sparse_attention(ix.h, qd, torch.from_numpy(idx).cuda(), torch.from_numpy(cnt).cuda(), out)
        torch.cuda.synchronize()
        out = out.cpu().numpy()
        for h in range(8):
            ref = oracle.attention_on_list(q[0, h], ix.K[0, h // 4], ix.V[0, h // 4], lists[h], ix.sigma)
            if lists[h].size == 0:
                assert (out[0, h] == 0).all()
            else:
                assert np.abs(out[0, h] - ref).max() / np.abs(ref).max() <= G.ATTN_TOL, h


# ------------------------------------------------------------------ the index itself
def test_index_balls_enclose_members(G, oracle):
    """Eq. (1) on the exported index: stored centres are the group means (to storage rounding),
    stored radii enclose every member measured against the centres AS STORED, and are not
    looser than the documented widening."""
    n, r, S = 1024, 4, 4
    cache = _small_cache(2, n)
    for dtype, Kc in (("bf16", cache.K), ("f32", W.make_cache(1, n=n).K)):
        hkv = Kc.shape[1]
        with G.Index(Kc, Kc, dtype, hkv, group_size=r, n_subspaces=S, index_dtype=G.L.LVR_INDEX_SAME) as ix:
            centres, radii, slot_pos, keys = ix.export()
            for h in range(hkv):
                c = W.bf16_bits_to_f32(centres[0, h]).reshape(n // r, 128) if dtype == "bf16" else centres[0, h]
                label = (np.arange(n) // r).astype(np.int32)
                assert np.array_equal(slot_pos[0, h], np.arange(n))
                mean, _ = oracle.ball_index(Kc[0, h], label, n // r, S)
                ulp = 2.0 ** -8 if dtype == "bf16" else 2.0 ** -22
                # storage rounding of the mean, plus the fp32 summation error of r terms
                absmean = np.abs(Kc[0, h]).reshape(n // r, r, 128).mean(axis=1)
                assert np.all(np.abs(c - mean) <= ulp * np.abs(mean) + r * 2.0 ** -24 * absmean + 1e-30)
                need = oracle.ball_radii_for_centres(Kc[0, h], label, c.astype(np.float64), S)
                assert np.all(radii[0, h] >= need), "a member lies outside its ball"
                cn = np.stack([np.linalg.norm(c[:, lo:hi].astype(np.float64), axis=1)
                               for lo, hi in (oracle.subspace_range(128, S, s) for s in range(S))], axis=1)
                assert np.all(radii[0, h] <= need * (1 + 2.0 ** -11) + cn * 2.0 ** -11 + 1e-30)


@pytest.mark.parametrize("S", [1, 4, 16])
def test_surviving_groups_match_oracle_bounds(G, oracle, S):
    """The number of groups the bound test keeps equals the number whose Eq. (2) bound (per block,
    summed), evaluated by the oracle on the exported index, reaches tau for some head of the KV
    group (up to groups whose bound is within rounding of tau).  Keys with positional locality, so
    that a real share of the balls is pruned."""
    n, r = 4096, 4
    cache = W.make_local_cache(2, n=n)
    K, V = cache.K[:, :1], cache.V[:, :1]
    q = W.make_queries(2, n_q_heads=4)
    with G.Index(K, V, "bf16", 4, group_size=r, n_subspaces=S) as ix:
        centres, radii, _, _ = ix.export()
        a = ix.channel_factors()[0, 0]     # the default index may live in a rescaled space
        c = W.bf16_bits_to_f32(centres[0, 0]).reshape(n // r, 128).astype(np.float64) / a
        seen = []
        for frac in (0.001, 0.02, 0.3):
            t = G.oracle_taus(oracle, ix, q, frac=frac)
            ix.query(q, t)
            st = ix.stats()
            ub = np.stack([oracle.ball_bounds(q[0, h] * a, c, radii[0, 0].astype(np.float64)).sum(0) for h in range(4)])
            te = t[0] - 0.5e-4 * np.abs(t[0])
            lo = int(np.any(ub >= te[:, None] * (1 + 1e-5) + 1e-3, axis=0).sum())
            hi = int(np.any(ub >= te[:, None] * (1 - 1e-5) - 1e-3, axis=0).sum())
            assert lo <= st["groups_surviving"] <= hi, (frac, lo, st["groups_surviving"], hi)
            seen.append(st["groups_surviving"] / st["groups_scored"])
            G.say(f"  S={S} frac={frac}: surviving {st['groups_surviving']} of {st['groups_scored']}")
        assert seen[0] < 0.2 and seen[0] < seen[1] < seen[2]     # the test really exercises pruning


def test_key_on_ball_surface_is_never_lost(G, oracle):
    """Adversarial placement: in every group one member sits exactly at centre + rho * q/|q|,
    so its score equals the ball bound; with tau equal to that score the key must come back."""
    g = np.random.default_rng(11)
    n, r = 512, 4
    qdir = np.zeros(128, dtype=np.float32)
    qdir[[3, 40, 77, 120]] = [1.0, -1.0, 1.0, 1.0]          # |q| = 2, exactly representable
    K = np.zeros((1, 1, n, 128), dtype=np.float32)
    for gi in range(n // r):
        centre = W.round_to_bf16(g.integers(-8, 9, size=128).astype(np.float32))
        step = float(g.integers(1, 5)) * 0.5
        K[0, 0, gi * r + 0] = centre + step * qdir
        K[0, 0, gi * r + 1] = centre - step * qdir
        K[0, 0, gi * r + 2] = centre
        K[0, 0, gi * r + 3] = centre
    V = g.standard_normal((1, 1, n, 128)).astype(np.float32)
    q = (qdir * 3.0)[None, None, :]
    for S in (1, 4, 16):
        with G.Index(K, W.round_to_bf16(V), "bf16", 1, n_subspaces=S) as ix:
            s = oracle.scores_f32(q[0, 0], K[0, 0])
            for tau in np.unique(s)[-6:]:
                t = np.full((1, 1), tau, dtype=np.float32)
                idx, cnt, out = ix.query(q, t)
                G.check_step(oracle, ix, q, t, idx, cnt, out, tag=f"surface S={S} tau={tau}")


@pytest.mark.parametrize("separate", [0, 2], ids=["fused", "two_kernels"])
def test_pruning_happens_on_clustered_keys(G, oracle, separate):
    """Keys with positional locality (consecutive tokens share a slowly changing mean): most
    balls are pruned, the result still equals the oracle's."""
    g = np.random.default_rng(21)
    n, hkv, hq = 8192, 2, 8
    base = np.repeat(g.standard_normal((1, hkv, n // 64, 128)).astype(np.float32) * 3.0, 64, axis=2)
    K = W.round_to_bf16(base + 0.05 * g.standard_normal((1, hkv, n, 128)).astype(np.float32))
    V = W.round_to_bf16(g.standard_normal((1, hkv, n, 128)).astype(np.float32))
    q = W.make_queries(2, n_q_heads=hq)
    with G.Index(K, V, "bf16", hq, n_subspaces=4, flags=separate) as ix:
        tau = G.oracle_taus(oracle, ix, q, frac=0.02)
        idx, cnt, out = ix.query(q, tau, fused=True)
        G.check_step(oracle, ix, q, tau, idx, cnt, out, tag="clustered")
        st = ix.stats()
        G.say("clustered keys:", st)
        assert st["groups_surviving"] < 0.25 * st["groups_scored"]
        assert st["keys_scanned"] == st["groups_surviving"] * 4


@pytest.mark.parametrize("n,r,grouping", [(8192, 4, "contiguous"), (2051, 4, "contiguous"), (1000, 1, "contiguous"),
                                          (1500, 8, "tree"), (40, 16, "contiguous")])
def test_bound_test_switched_off(G, oracle, n, r, grouping):
    """lvr_set_bound_test(0): the exact filter alone.  Same sets and attention as with the bound
    test on; no group is scored, every held key gets the exact dot product; switching the test
    back on restores the pruning.  Also across an append that stays in the buffer."""
    import paper_2605_06763_amd as L
    g = np.random.default_rng(5)
    hkv, hq = 2, 8
    base = np.repeat(g.standard_normal((1, hkv, (n + 63) // 64, 128)).astype(np.float32) * 3.0, 64, axis=2)[:, :, :n]
    K = W.round_to_bf16(base + 0.05 * g.standard_normal((1, hkv, n, 128)).astype(np.float32))
    V = W.round_to_bf16(g.standard_normal((1, hkv, n, 128)).astype(np.float32))
    q = W.make_queries(2, n_q_heads=hq)
    with G.Index(K, V, "bf16", hq, group_size=r, capacity=n + 8,
                 grouping=L.LVR_GROUP_TREE if grouping == "tree" else L.LVR_GROUP_CONTIGUOUS) as ix:
        tau = G.oracle_taus(oracle, ix, q, frac=0.02)
        idx, cnt, out = ix.query(q, tau, fused=True)
        G.check_step(oracle, ix, q, tau, idx, cnt, out, tag="bounds on")
        on = ix.stats()
        L.lvr_set_bound_test(ix.h, False)
        for fused in (True, False):
            idx2, cnt2, out2 = ix.query(q, tau, fused=fused)
            G.check_step(oracle, ix, q, tau, idx2, cnt2, out2, tag=f"bounds off fused={fused}")
            off = ix.stats()
            assert off["groups_scored"] == 0 and off["bytes_index"] == 0
            assert off["keys_scanned"] == hkv * n, (off, n)
            assert off["keys_emitted"] == on["keys_emitted"]
            for h in range(hq):
                assert set(idx[0, h, :cnt[0, h]].tolist()) == set(idx2[0, h, :cnt2[0, h]].tolist())
        ix.append(K[:, :, :3].copy(), V[:, :, :3].copy())
        tau = G.oracle_taus(oracle, ix, q, frac=0.02)
        idx3, cnt3, out3 = ix.query(q, tau, fused=True)
        G.check_step(oracle, ix, q, tau, idx3, cnt3, out3, tag="bounds off, after append")
        assert ix.stats()["keys_scanned"] == hkv * (n + 3)
        L.lvr_set_bound_test(ix.h, True)
        idx4, cnt4, out4 = ix.query(q, tau, fused=True)
        G.check_step(oracle, ix, q, tau, idx4, cnt4, out4, tag="bounds on again")
        again = ix.stats()
        assert again["groups_scored"] == on["groups_scored"]
        if n >= 1000 and r > 1:
            assert again["groups_surviving"] < 0.5 * again["groups_scored"]
    # the two-launch form and fp32 caches have no such switch
    with G.Index(K[:, :, :64], V[:, :, :64], "bf16", hq, flags=L.LVR_SEPARATE_KERNELS) as ix:
        with pytest.raises(L.LouverError) as e:
            L.lvr_set_bound_test(ix.h, False)
        assert e.value.code == L.LVR_E_UNSUPPORTED
        L.lvr_set_bound_test(ix.h, True)


# ------------------------------------------------------------------ append
@pytest.mark.parametrize("flags", [0, 1, 2, 3])
def test_append_matches_oracle_on_grown_cache(G, oracle, flags):
    """Prompt of 200 keys, then single-token appends across several buffer flushes (B = 32);
    after every step the query over the grown cache equals the oracle's.  With the
    attend-buffer flag the not-yet-indexed tail is retrieved whatever its score."""
    n0, steps, B = 203, 75, 32
    cache = _small_cache(5, n0)
    k_new, v_new = W.make_append_stream(5, steps, cache)
    qs = W.drift_queries(5, steps, n_q_heads=8)
    with G.Index(cache.K, cache.V, "bf16", 8, capacity=n0 + steps, buffer_size=B, flags=flags) as ix:
        import paper_2605_06763_amd as L
        for t in range(steps):
            ix.append(k_new[t][:, :, None, :], v_new[t][:, :, None, :])
            n, n_indexed = L.lvr_length(ix.h)
            assert n == n0 + t + 1
            assert n_indexed % 4 == 0 and 0 <= n - n_indexed < B + 4
            if t % 7 == 0 or t == steps - 1:
                tau = G.oracle_taus(oracle, ix, qs[t], frac=0.05)
                idx, cnt, out = ix.query(qs[t], tau, fused=(t % 2 == 0))
                G.check_step(oracle, ix, qs[t], tau, idx, cnt, out, tag=f"append t={t}",
                             extra_from=(n_indexed if flags & 1 else -1))
        assert n_indexed >= n0 // 4 * 4 + 2 * B      # at least two flushes happened
        # bulk append of many tokens at once
    with G.Index(cache.K, cache.V, "bf16", 8, capacity=n0 + steps, buffer_size=B) as ix:
        kk = np.ascontiguousarray(k_new.transpose(1, 2, 0, 3))
        vv = np.ascontiguousarray(v_new.transpose(1, 2, 0, 3))
        ix.append(kk, vv)
        tau = G.oracle_taus(oracle, ix, qs[-1], frac=0.05)
        idx, cnt, out = ix.query(qs[-1], tau)
        G.check_step(oracle, ix, qs[-1], tau, idx, cnt, out, tag="bulk append")
        import paper_2605_06763_amd as L
        with pytest.raises(L.LouverError) as e:
            ix.append(kk[:, :, :1], vv[:, :, :1])
        assert e.value.code == L.LVR_E_CAPACITY


def test_strided_build_input(G, oracle):
    """K and V handed over as views with non-trivial strides (a slice of a longer cache)."""
    import paper_2605_06763_amd as L
    n = 300
    cache = _small_cache(2, 400)
    q = W.make_queries(2, n_q_heads=8)
    Kd = G.to_device(cache.K, "bf16")[:, :, 50:50 + n]
    Vd = G.to_device(cache.V, "bf16")[:, :, 50:50 + n]
    with G.Index(cache.K[:, :, 50:50 + n], cache.V[:, :, 50:50 + n], "bf16", 8) as ix:
        L.lvr_build(ix.h, Kd, Vd)          # rebuild from the strided views
        tau = G.oracle_taus(oracle, ix, q, frac=0.05)
        idx, cnt, out = ix.query(q, tau)
        G.check_step(oracle, ix, q, tau, idx, cnt, out, tag="strided")


# ------------------------------------------------------------------ tree grouping (Alg. 2)
@pytest.mark.parametrize("dtype,n,r", [("bf16", 1024, 4), ("f32", 512, 4), ("bf16", 2048, 8), ("bf16", 256, 2)])
def test_tree_grouping_equals_oracle_tree(G, oracle, dtype, n, r):
    """n = r * 2^k: the arena order produced on the GPU is exactly the left-to-right leaf order of
    the oracle's balanced tree (axis of largest variance, median split, ties by position)."""
    import paper_2605_06763_amd as L
    cache = _small_cache(2 if dtype == "bf16" else 1, n, hkv=2 if dtype == "bf16" else 1)
    hkv = cache.K.shape[1]
    with G.Index(cache.K, cache.V, dtype, hkv, group_size=r, grouping=L.LVR_GROUP_TREE) as ix:
        centres, radii, slot_pos, keys = ix.export()
        for h in range(hkv):
            label, order, leaves = oracle.balanced_tree(cache.K[0, h], r)
            assert leaves == n // r
            assert np.array_equal(slot_pos[0, h], order), (h, np.nonzero(slot_pos[0, h] != order)[0][:8])
            stored = W.bf16_bits_to_f32(keys[0, h]).reshape(n, 128) if dtype == "bf16" else keys[0, h]
            assert np.array_equal(stored, cache.K[0, h][order])        # rows really are regrouped


@pytest.mark.parametrize("n,r,S", [(1500, 4, 4), (777, 8, 2), (64, 4, 16), (5, 4, 4)])
def test_tree_grouping_queries(G, oracle, n, r, S):
    """Ragged sizes (padded tree): the grouping is a valid partition, balls enclose their members,
    and query + attention equal the oracle's in original token positions."""
    import paper_2605_06763_amd as L
    cache = _small_cache(2, n)
    q = W.make_queries(2, n_q_heads=8)
    with G.Index(cache.K, cache.V, "bf16", 8, group_size=r, n_subspaces=S, grouping=L.LVR_GROUP_TREE,
                 buffer_size=64) as ix:
        centres, radii, slot_pos, keys = ix.export()
        n_idx = n // r * r
        for h in range(2):
            assert sorted(slot_pos[0, h, :n_idx].tolist()) == list(range(n_idx))
            assert slot_pos[0, h, n_idx:].tolist() == list(range(n_idx, n))
            if n_idx:
                label = np.empty(n_idx, dtype=np.int32)
                label[slot_pos[0, h, :n_idx]] = np.arange(n_idx) // r
                a = ix.channel_factors()[0, h]
                c = W.bf16_bits_to_f32(centres[0, h]).reshape(n_idx // r, 128).astype(np.float64) / a
                need = oracle.ball_radii_for_centres(cache.K[0, h, :n_idx].astype(np.float64) / a, label, c, S)
                assert np.all(radii[0, h] >= need)
        for frac, fused in ((0.02, True), (0.3, False)):
            tau = G.oracle_taus(oracle, ix, q, frac=frac)
            idx, cnt, out = ix.query(q, tau, fused=fused)
            G.check_step(oracle, ix, q, tau, idx, cnt, out, tag=f"tree n={n} r={r} S={S} frac={frac}")
        ref = oracle.dense_attention(ix.K, ix.V, q, ix.sigma, 8)
        assert (np.abs(ix.dense(q) - ref).max(axis=-1) / np.abs(ref).max(axis=-1)).max() <= G.ATTN_TOL


def test_tree_grouping_append(G, oracle):
    """Appends in tree mode: every chunk of B buffered keys is regrouped on its own; positions
    reported by the query stay the original token positions."""
    import paper_2605_06763_amd as L
    n0, steps, B = 131, 70, 32
    cache = _small_cache(5, n0)
    k_new, v_new = W.make_append_stream(5, steps, cache)
    qs = W.drift_queries(5, steps, n_q_heads=8)
    with G.Index(cache.K, cache.V, "bf16", 8, capacity=n0 + steps, buffer_size=B, grouping=L.LVR_GROUP_TREE) as ix:
        for t in range(steps):
            ix.append(k_new[t][:, :, None, :], v_new[t][:, :, None, :])
            if t % 9 == 0 or t == steps - 1:
                tau = G.oracle_taus(oracle, ix, qs[t], frac=0.06)
                idx, cnt, out = ix.query(qs[t], tau, fused=True)
                G.check_step(oracle, ix, qs[t], tau, idx, cnt, out, tag=f"tree append t={t}")
        n, n_indexed = L.lvr_length(ix.h)
        centres, radii, slot_pos, keys = ix.export()
        assert n_indexed == 128 + 2 * B
        for h in range(2):
            assert sorted(slot_pos[0, h, :128].tolist()) == list(range(128))
            for c0 in (128, 128 + B):                      # each chunk is a permutation of its own rows
                assert sorted(slot_pos[0, h, c0:c0 + B].tolist()) == list(range(c0, c0 + B))
            stored = W.bf16_bits_to_f32(keys[0, h]).reshape(n, 128)
            assert np.array_equal(stored, ix.K[0, h][slot_pos[0, h]])


def test_tree_grouping_prunes_where_contiguous_cannot(G, oracle):
    """Keys drawn from 64 tight clusters but stored in random order: consecutive positions are
    unrelated, so contiguous groups are wide and survive; the tree regroups neighbours in key space."""
    import paper_2605_06763_amd as L
    g = np.random.default_rng(31)
    n, hkv, hq = 4096, 2, 8
    cent = g.standard_normal((hkv, 64, 128)).astype(np.float32) * 3.0
    which = g.integers(0, 64, size=(hkv, n))
    K = np.stack([cent[h][which[h]] for h in range(hkv)])[None]
    K = W.round_to_bf16(K + 0.05 * g.standard_normal(K.shape).astype(np.float32))
    V = W.round_to_bf16(g.standard_normal((1, hkv, n, 128)).astype(np.float32))
    q = W.make_queries(2, n_q_heads=hq)
    surv = {}
    for name, grouping in (("contiguous", L.LVR_GROUP_CONTIGUOUS), ("tree", L.LVR_GROUP_TREE)):
        with G.Index(K, V, "bf16", hq, grouping=grouping) as ix:
            tau = G.oracle_taus(oracle, ix, q, frac=0.02)
            idx, cnt, out = ix.query(q, tau, fused=True)
            G.check_step(oracle, ix, q, tau, idx, cnt, out, tag=name)
            st = ix.stats()
            surv[name] = st["groups_surviving"] / st["groups_scored"]
    G.say("surviving fraction:", surv)
    assert surv["tree"] < 0.5 * surv["contiguous"]


def test_everything_qualifies_large(G, oracle):
    """tau = -inf on 20000 keys: every emission queue flushes hundreds of times; every position
    must come back exactly once per head and the attention equals the dense result."""
    n = 20000
    cache = _small_cache(2, n, hkv=1)
    q = W.make_queries(2, n_q_heads=4)
    for flags in (0, 2):
        with G.Index(cache.K, cache.V, "bf16", 4, flags=flags) as ix:
            tau = np.full((1, 4), -np.inf, dtype=np.float32)
            idx, cnt, out = ix.query(q, tau, fused=True)
            assert (cnt == n).all()
            for h in range(4):
                assert np.array_equal(np.sort(idx[0, h]), np.arange(n))
            ref = oracle.dense_attention(ix.K, ix.V, q, ix.sigma, 4)
            assert (np.abs(out - ref).max(axis=-1) / np.abs(ref).max(axis=-1)).max() <= G.ATTN_TOL


# ------------------------------------------------------------------ box enclosure (Def. 1, AABB)
def _e4m3_values():
    """All finite e4m3 values (OCP: bias 7, subnormals below 2^-6, largest 448), ascending."""
    v = []
    for code in range(0x7f):
        ex, m = code >> 3, code & 7
        v.append(m / 8.0 * 2.0 ** -6 if ex == 0 else (1 + m / 8.0) * 2.0 ** (ex - 7))
    v = np.array(v)
    return np.concatenate([-v[:0:-1], v])


@pytest.mark.parametrize("centres", ["same", "fp8"])
@pytest.mark.parametrize("r,hq,hkv", [(4, 8, 2), (2, 4, 1), (16, 16, 2), (1, 2, 2)])
def test_box_enclosure_index_and_queries(G, oracle, r, hq, hkv, centres):
    """Boxes instead of balls: the stored corners are exactly the per-coordinate extremes of each
    group (bf16 corners) or the nearest e4m3 values outside them (8-bit corners), the number of
    surviving groups matches the oracle's box bound on the stored corners, and query + attention
    equal the oracle's."""
    import paper_2605_06763_amd as L
    n = 1100
    cache = _small_cache(2, n, hkv=hkv)
    q = W.make_queries(2, n_q_heads=hq)
    Gq = hq // hkv
    idt = L.LVR_INDEX_FP8 if centres == "fp8" else L.LVR_INDEX_SAME
    with G.Index(cache.K, cache.V, "bf16", hq, group_size=r, enclosing=L.LVR_ENCLOSE_AABB, buffer_size=64,
                 index_dtype=idt) as ix:
        corners, allow, slot_pos, keys = ix.export()
        n_idx = n // r * r
        label = (np.arange(n_idx) // r).astype(np.int32)
        stored = []
        for h in range(hkv):
            lo, hi = oracle.aabb_index(cache.K[0, h, :n_idx], label, n_idx // r)
            got_hi = W.bf16_bits_to_f32(corners[0, h, :, 0]).reshape(-1, 128)
            got_lo = W.bf16_bits_to_f32(corners[0, h, :, 1]).reshape(-1, 128)
            stored.append((got_lo.astype(np.float64), got_hi.astype(np.float64)))
            if centres == "same":
                assert np.array_equal(got_hi, hi.astype(np.float32)) and np.array_equal(got_lo, lo.astype(np.float32))
            else:
                vals = _e4m3_values()
                want_hi = vals[np.minimum(np.searchsorted(vals, hi, side="left"), len(vals) - 1)]     # smallest value >= hi
                want_lo = vals[np.maximum(np.searchsorted(vals, lo, side="right") - 1, 0)]             # largest value <= lo
                assert np.array_equal(got_hi, want_hi.astype(np.float32)) and np.array_equal(got_lo, want_lo.astype(np.float32))
                assert np.all(got_hi >= hi) and np.all(got_lo <= lo)                                   # these keys stay inside +-448
            a = np.maximum(np.abs(got_lo), np.abs(got_hi))
            # the allowance must exceed the fp32 error bound 2^-16 |a| of the 256-term bound (it is twice that)
            assert np.all(allow[0, h, :, 0] >= 2.0 ** -15 * np.linalg.norm(a, axis=1) * (1 - 1e-5))
            assert np.all(allow[0, h, :, 0] <= 2.0 ** -14 * np.linalg.norm(a, axis=1) + 1e-30)
        for frac in (0.02, 0.4):
            tau = G.oracle_taus(oracle, ix, q, frac=frac)
            for boost in (1.0, 2.5):
                t = (tau * boost).astype(np.float32) if frac < 0.1 else tau
                idx, cnt, out = ix.query(q, t, fused=True)
                G.check_step(oracle, ix, q, t, idx, cnt, out, tag=f"box r={r} frac={frac} boost={boost} {centres}")
                st = ix.stats()
                lo_cnt = hi_cnt = 0
                for h in range(hkv):
                    lo, hi = stored[h]
                    # the kernel adds its rounding allowance (stored per group) times |q| to the box bound
                    ub = np.stack([oracle.aabb_bounds(q[0, h * Gq + g], lo, hi)
                                   + allow[0, h, :, 0].astype(np.float64) * np.linalg.norm(q[0, h * Gq + g].astype(np.float64))
                                   for g in range(Gq)])
                    te = t[0, h * Gq:(h + 1) * Gq]
                    te = (te - 0.5e-4 * np.abs(te))[:, None]
                    lo_cnt += int(np.any(ub >= te * (1 + 1e-5) + 1e-3, axis=0).sum())
                    hi_cnt += int(np.any(ub >= te * (1 - 1e-5) - 1e-3, axis=0).sum())
                assert lo_cnt <= st["groups_surviving"] <= hi_cnt, (lo_cnt, st["groups_surviving"], hi_cnt)


def test_box_8bit_corners_beyond_the_code_range(G, oracle):
    """Members beyond +-448 cannot be enclosed by an e4m3 corner: the corner saturates and what sticks
    out goes into the group's allowance, so no qualifying key is lost; tiny and zero coordinates round
    outwards to the smallest codes."""
    import paper_2605_06763_amd as L
    n, r = 512, 4
    cache = _small_cache(2, n, hkv=1)
    K = cache.K.copy()
    g = np.random.default_rng(5)
    K[0, 0, 8:12, 3] = [500.0, 1000.0, -30.0, 2.0]          # upper corner beyond the range
    K[0, 0, 16:20, 7] = [-600.0, -449.0, 5.0, 0.0]          # lower corner beyond the range
    K[0, 0, 24:28, :] = 0.0                                  # a group of zeros
    K[0, 0, 32:36, 5] = [1e-5, -1e-5, 0.0, 2e-6]            # below the smallest code
    K = W.round_to_bf16(K)
    q = W.make_queries(2, n_q_heads=4)
    with G.Index(K, cache.V, "bf16", 4, group_size=r, enclosing=L.LVR_ENCLOSE_AABB, index_dtype=L.LVR_INDEX_FP8) as ix:
        corners, allow, _, _ = ix.export()
        hi = W.bf16_bits_to_f32(corners[0, 0, :, 0]).reshape(-1, 128).astype(np.float64)
        lo = W.bf16_bits_to_f32(corners[0, 0, :, 1]).reshape(-1, 128).astype(np.float64)
        Kg = K[0, 0].reshape(n // r, r, 128).astype(np.float64)
        out_hi = np.maximum(Kg.max(axis=1) - hi, 0)
        out_lo = np.maximum(lo - Kg.min(axis=1), 0)
        sticks = np.linalg.norm(np.maximum(out_hi, out_lo), axis=1)
        assert sticks[2] > 500 and sticks[4] > 150 and np.count_nonzero(sticks) == 2
        assert hi[2, 3] == 448.0 and lo[4, 7] == -448.0
        assert np.all(allow[0, 0, :, 0] >= sticks)
        assert np.all(hi[6] == 0) and np.all(lo[6] == 0)
        assert hi[8, 5] == 2.0 ** -9 and lo[8, 5] == -2.0 ** -9
        # every member's score stays below its group's bound: exact scores against stored corners + allowance
        for h in range(4):
            ub = oracle.aabb_bounds(q[0, h], lo, hi) + allow[0, 0, :, 0].astype(np.float64) * np.linalg.norm(q[0, h].astype(np.float64))
            sc = oracle.scores_f64(q[0, h], K[0, 0]).reshape(n // r, r)
            assert np.all(sc.max(axis=1) <= ub)
        for frac in (0.01, 0.2):
            tau = G.oracle_taus(oracle, ix, q, frac=frac)
            idx, cnt, out = ix.query(q, tau, fused=True)
            G.check_step(oracle, ix, q, tau, idx, cnt, out, tag=f"box fp8 range frac={frac}")


def test_box_enclosure_with_tree_grouping_and_append(G, oracle):
    import paper_2605_06763_amd as L
    n0, steps, B = 200, 40, 32
    cache = _small_cache(5, n0)
    k_new, v_new = W.make_append_stream(5, steps, cache)
    qs = W.drift_queries(5, steps, n_q_heads=8)
    for grouping, idt in ((L.LVR_GROUP_CONTIGUOUS, L.LVR_INDEX_SAME), (L.LVR_GROUP_TREE, L.LVR_INDEX_SAME),
                          (L.LVR_GROUP_CONTIGUOUS, L.LVR_INDEX_FP8), (L.LVR_GROUP_TREE, L.LVR_INDEX_FP8)):
        with G.Index(cache.K, cache.V, "bf16", 8, capacity=n0 + steps, buffer_size=B, grouping=grouping,
                     enclosing=L.LVR_ENCLOSE_AABB, index_dtype=idt) as ix:
            for t in range(steps):
                ix.append(k_new[t][:, :, None, :], v_new[t][:, :, None, :])
                if t % 13 == 0 or t == steps - 1:
                    tau = G.oracle_taus(oracle, ix, qs[t], frac=0.05)
                    idx, cnt, out = ix.query(qs[t], tau, fused=True)
                    G.check_step(oracle, ix, qs[t], tau, idx, cnt, out, tag=f"box grouping={grouping} t={t}")


def test_box_versus_ball_pruning_on_local_keys(G, oracle):
    import paper_2605_06763_amd as L
    cache = W.make_local_cache(2, n=8192)
    K, V = cache.K[:, :2], cache.V[:, :2]
    q = W.make_queries(2, n_q_heads=8)
    surv = {}
    for name, enc, idt in (("ball", L.LVR_ENCLOSE_BALL, L.LVR_INDEX_SAME), ("box", L.LVR_ENCLOSE_AABB, L.LVR_INDEX_SAME),
                           ("ball8", L.LVR_ENCLOSE_BALL, L.LVR_INDEX_FP8), ("box8", L.LVR_ENCLOSE_AABB, L.LVR_INDEX_FP8)):
        with G.Index(K, V, "bf16", 8, enclosing=enc, index_dtype=idt) as ix:
            tau = G.oracle_taus(oracle, ix, q, frac=0.02)
            idx, cnt, out = ix.query(q, tau, fused=True)
            G.check_step(oracle, ix, q, tau, idx, cnt, out, tag=name)
            st = ix.stats()
            surv[name] = st["groups_surviving"] / st["groups_scored"]
    G.say("surviving fraction on keys with positional locality:", surv)
    assert surv["ball"] < 0.25 and surv["box"] < 0.25 and surv["box8"] < 0.3 and surv["box"] <= surv["box8"]


def test_box_enclosure_unsupported_combinations():
    import ctypes as C
    import paper_2605_06763_amd as L
    for kw in (dict(kv_dtype=L.LVR_F32), dict(flags=L.LVR_SEPARATE_KERNELS)):
        cfg = L.make_config(batch=1, n_q_heads=4, n_kv_heads=1, capacity=64, enclosing=L.LVR_ENCLOSE_AABB, **kw)
        h = C.c_void_p()
        assert L.lib().lvr_create(C.byref(cfg), C.byref(h)) == L.LVR_E_UNSUPPORTED


# ---------------------------------------------------------------------------------------------
# Built-in threshold selection over a reservoir of past keys (appendix "Threshold Oracle Comparison")
# ---------------------------------------------------------------------------------------------
def _check_reservoir(oracle, ix, seed, R):
    res = ix.reservoir()
    m = min(ix.n, R)
    for b in range(ix.batch):
        for g in range(ix.hkv):
            want = oracle.reservoir(seed, b * ix.hkv + g, ix.n, R)
            assert np.array_equal(res[b, g, :m], want), f"reservoir b={b} g={g} n={ix.n}"
            assert (res[b, g, m:] == -1).all()
    return res


@pytest.mark.parametrize("n,R", [(100, 256), (256, 256), (5000, 256), (5000, 64), (40000, 256)])
def test_reservoir_equals_sequential_algorithm_r(G, oracle, n, R):
    """The parallel update (largest position wins a slot) holds exactly what the sequential
    sampler holds, after a build and after chunked and single appends."""
    G.say(f"reservoir n={n} R={R}")
    seed = 0xC0FFEE + n
    c = W.make_cache(2, n=n + 300, n_kv_heads=2, batch=2)
    with G.Index(c.K[:, :, :n], c.V[:, :, :n], "bf16", 8, capacity=n + 300, reservoir_size=R, seed=seed) as ix:
        _check_reservoir(oracle, ix, seed, R)
        ix.append(c.K[:, :, n:n + 257], c.V[:, :, n:n + 257])
        _check_reservoir(oracle, ix, seed, R)
        for i in range(n + 257, n + 300):
            ix.append(c.K[:, :, i:i + 1], c.V[:, :, i:i + 1])
        assert ix.n == n + 300
        _check_reservoir(oracle, ix, seed, R)


@pytest.mark.parametrize("dtype,grouping", [("bf16", "contiguous"), ("bf16", "tree"), ("f32", "contiguous")])
@pytest.mark.parametrize("n", [37, 9000])
def test_threshold_rules_equal_the_oracle(G, oracle, dtype, grouping, n):
    """tau of every rule equals the oracle's rule applied to the oracle's fp32 scores of the
    reservoir keys; a decode step with that tau then meets the parity rule."""
    G.say(f"threshold rules dtype={dtype} grouping={grouping} n={n}")
    seed, R = 77, 256
    cid = 2 if dtype == "bf16" else 1
    c = W.make_cache(cid, n=n, n_kv_heads=2, batch=2)
    q = W.make_queries(cid, n_q_heads=8, batch=2)
    gr = G.L.LVR_GROUP_TREE if grouping == "tree" else G.L.LVR_GROUP_CONTIGUOUS
    with G.Index(c.K, c.V, dtype, 8, grouping=gr, reservoir_size=R, seed=seed) as ix:
        res = _check_reservoir(oracle, ix, seed, R)
        m = min(n, R)
        for mode, param in (("sample-max", 0), ("sample-mean-max", 0), ("sample-gap", 0), ("sample-topk", 1),
                            ("sample-topk", 8), ("sample-topk", 1000), ("budget", 0.02), ("budget", 0.3),
                            ("budget", 1.0)):
            tau = ix.threshold(q, mode, param)
            for b in range(ix.batch):
                for h in range(ix.hq):
                    g = h // ix.G
                    s = oracle.scores_f32(q[b, h], ix.K[b, g][res[b, g, :m]])
                    want = oracle.threshold(s, mode, param)
                    if mode == "sample-gap":
                        # equal largest gaps (to rounding) may cut at either: accept any cut whose
                        # gap is within rounding of the largest
                        sd = np.sort(s.astype(np.float64))[::-1]
                        gaps = sd[:-1] - sd[1:]
                        ok = sd[:-1][gaps >= gaps.max() - 4e-6 * np.abs(sd).max()] if m > 1 else sd[:1]
                        assert np.min(np.abs(ok - tau[b, h])) <= 2e-6 * max(1.0, np.abs(sd).max()), (mode, b, h)
                    else:
                        assert abs(tau[b, h] - want) <= 2e-6 * max(1.0, float(np.abs(s).max())), \
                            (mode, param, b, h, tau[b, h], want)
            if mode in ("sample-topk", "budget", "sample-mean-max"):
                idx, cnt, out = ix.query(q, tau, fused=True)
                G.check_step(oracle, ix, q, tau, idx, cnt, out, tag=f"{mode}/{param}")


def test_threshold_needs_a_reservoir(G):
    c = W.make_cache(2, n=512, n_kv_heads=2)
    q = W.make_queries(2, n_q_heads=8)
    with G.Index(c.K, c.V, "bf16", 8) as ix:
        with pytest.raises(G.L.LouverError):
            ix.threshold(q, "sample-max")
    with G.Index(c.K, c.V, "bf16", 8, reservoir_size=16, seed=1) as ix:
        with pytest.raises(G.L.LouverError):
            ix.threshold(q, "budget", 0.0)
        with pytest.raises(G.L.LouverError):
            ix.threshold(q, "sample-topk", 0.0)


# ---------------------------------------------------------------------------------------------
# Two-stream update (App. "GPU Update"): groups prepared on a side stream, published later
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("grouping", ["contiguous", "tree"])
def test_concurrent_update_half_published_state(G, oracle, grouping):
    """Between the append that fills the buffer and the publish, queries still see the old group
    count and scan the full buffer exactly, so their result is the oracle's; after the publish
    the index equals, bit for bit, the one a single-stream index builds from the same stream."""
    L = G.L
    n0, steps, B = 203, 150, 32
    gr = L.LVR_GROUP_TREE if grouping == "tree" else L.LVR_GROUP_CONTIGUOUS
    cache = _small_cache(5, n0)
    k_new, v_new = W.make_append_stream(5, steps, cache)
    qs = W.drift_queries(5, steps, n_q_heads=8)
    G.say(f"concurrent update grouping={grouping}")
    with G.Index(cache.K, cache.V, "bf16", 8, capacity=n0 + steps, buffer_size=B, grouping=gr,
                 flags=L.LVR_CONCURRENT_UPDATE) as ix, \
         G.Index(cache.K, cache.V, "bf16", 8, capacity=n0 + steps, buffer_size=B, grouping=gr) as ref:
        windows = 0
        for t in range(steps):
            ix.append(k_new[t][:, :, None, :], v_new[t][:, :, None, :])
            ref.append(k_new[t][:, :, None, :], v_new[t][:, :, None, :])
            n, n_indexed = L.lvr_length(ix.h)
            n_ref, n_indexed_ref = L.lvr_length(ref.h)
            assert n == n_ref == n0 + t + 1
            pending = n_indexed != n_indexed_ref
            if pending:
                # the window: the chunk's groups exist (or are being formed) but are not visible
                windows += 1
                assert n_indexed_ref - n_indexed == B and n - n_indexed >= B
                tau = G.oracle_taus(oracle, ix, qs[t], frac=0.05)
                for fused in (True, False):
                    idx, cnt, out = ix.query(qs[t], tau, fused=fused)
                    G.check_step(oracle, ix, qs[t], tau, idx, cnt, out, tag=f"window t={t}")
                st = ix.stats()
                assert st["update_pending"] == 1 and st["n_indexed"] == n_indexed
                assert st["keys_scanned"] >= (n - n_indexed) * ix.batch * ix.hkv
                if windows % 2 == 0:
                    L.lvr_publish(ix.h)                  # explicit phase 2; otherwise the next append does it
                    assert L.lvr_length(ix.h)[1] == n_indexed_ref
                    idx, cnt, out = ix.query(qs[t], tau)
                    G.check_step(oracle, ix, qs[t], tau, idx, cnt, out, tag=f"published t={t}")
                    assert ix.stats()["update_pending"] == 0
            elif t % 11 == 0:
                tau = G.oracle_taus(oracle, ix, qs[t], frac=0.05)
                idx, cnt, out = ix.query(qs[t], tau)
                G.check_step(oracle, ix, qs[t], tau, idx, cnt, out, tag=f"t={t}")
        assert windows >= 4
        L.lvr_publish(ix.h)
        a, b = ix.export(), ref.export()
        for name, x, y in zip(("centres", "radii", "slot_pos", "keys"), a, b):
            assert np.array_equal(np.asarray(x), np.asarray(y)), name
        # a publish with nothing pending, and on an index without the flag, is a no-op
        L.lvr_publish(ix.h)
        L.lvr_publish(ref.h)


def test_concurrent_update_bulk_append_and_rebuild(G, oracle):
    """Several chunks in one append take the single-stream path; a rebuild discards a pending update."""
    L = G.L
    n0, B = 100, 32
    cache = _small_cache(5, n0 + 200)
    q = W.make_queries(5, n_q_heads=8)
    K0, V0 = cache.K[:, :, :n0], cache.V[:, :, :n0]
    with G.Index(K0, V0, "bf16", 8, capacity=n0 + 200, buffer_size=B, flags=L.LVR_CONCURRENT_UPDATE) as ix:
        ix.append(cache.K[:, :, n0:n0 + 40], cache.V[:, :, n0:n0 + 40])          # fills one chunk: pending
        assert ix.stats()["update_pending"] == 1
        ix.append(cache.K[:, :, n0 + 40:n0 + 170], cache.V[:, :, n0 + 40:n0 + 170])   # publishes, then 4 chunks at once
        n, n_indexed = L.lvr_length(ix.h)
        assert n == n0 + 170 and n - n_indexed < B + 4
        tau = G.oracle_taus(oracle, ix, q, frac=0.05)
        idx, cnt, out = ix.query(q, tau)
        G.check_step(oracle, ix, q, tau, idx, cnt, out, tag="bulk")
        ix.append(cache.K[:, :, n0 + 170:n0 + 200], cache.V[:, :, n0 + 170:n0 + 200])
        # rebuild from the prompt alone while an update may be pending
        L.lvr_build(ix.h, ix.Kd, ix.Vd)
        ix.K, ix.V = K0.copy(), V0.copy()
        assert L.lvr_length(ix.h) == (n0, n0 // 4 * 4)
        tau = G.oracle_taus(oracle, ix, q, frac=0.05)
        idx, cnt, out = ix.query(q, tau)
        G.check_step(oracle, ix, q, tau, idx, cnt, out, tag="rebuilt")


# ---------------------------------------------------------------------------------------------
# Query 1 (Sec. 4.2, Alg. 3): per-subspace thresholds
# ---------------------------------------------------------------------------------------------
def _exported_bounds(G, oracle, ix, q, r):
    """Eq. (2) per block, evaluated by the oracle (fp64) on the index as the library stores it:
    f [hq][S][groups] for sequence 0 (one KV head per G query heads)."""
    centres, radii, _, _ = ix.export()
    a = ix.channel_factors()
    out = []
    for h in range(ix.hq):
        g = h // ix.G
        c = W.bf16_bits_to_f32(centres[0, g]).reshape(-1, 128).astype(np.float64) / a[0, g]
        out.append(oracle.ball_bounds(q[0, h] * a[0, g], c, radii[0, g].astype(np.float64)))
    return np.stack(out)


_Q1_CASES = [(1, "local", 4), (2, "local", 4), (4, "local", 4), (1, "workload", 4), (2, "workload", 4), (4, "workload", 4),
             (2, "local", 8), (4, "local", 2), (4, "workload", 1), (8, "local", 4), (16, "local", 4), (8, "workload", 8),
             (16, "workload", 8), (16, "local", 1), (8, "workload", 2)]


# 8-bit centres are built for at most four coordinate blocks
@pytest.mark.parametrize("S,keys,hq,centres", [c + (f,) for c in _Q1_CASES for f in ("fp8", "fp6", "same") if f == "same" or c[0] <= 4])
def test_query1_per_subspace_thresholds(G, oracle, S, keys, hq, centres):
    """Safe thresholds (tau_s = tau minus the largest bounds of the other blocks) must give
    Problem 1's set; arbitrary thresholds must give a set between Alg. 3's candidates (oracle's
    Query 1 on the exported index, thresholds nudged by rounding) filtered at tau, and every key
    the promise covers (all block products reach their thresholds) must be present."""
    n, r = 4096 + 37, 4
    cache = W.make_local_cache(2, n=n) if keys == "local" else W.make_cache(2, n=n)
    K, V = cache.K[:, :1], cache.V[:, :1]
    q = W.make_queries(2, n_q_heads=hq)
    G.say(f"query1 S={S} keys={keys} heads={hq} centres={centres}")
    idt = {"fp8": G.L.LVR_INDEX_FP8, "fp6": G.L.LVR_INDEX_FP6, "same": G.L.LVR_INDEX_SAME}[centres]
    with G.Index(K, V, "bf16", hq, group_size=r, n_subspaces=S, index_dtype=idt) as ix:
        n_groups = n // r
        f = _exported_bounds(G, oracle, ix, q, r)                      # [hq][S][groups]
        label = np.tile(np.arange(n_groups * r, dtype=np.int32) // r, (S, 1))
        ds = S and 128 // S
        Kd = K[0, 0].astype(np.float64)
        tau = G.oracle_taus(oracle, ix, q, frac=0.02)
        # (1) provably safe thresholds
        tau_s = np.empty((1, hq, S), dtype=np.float32)
        for h in range(hq):
            top = f[h].max(axis=1)
            for s in range(S):
                tau_s[0, h, s] = np.float32(tau[0, h] - (top.sum() - top[s]) - 1e-3)
        idx, cnt, out = G.query1(ix, q, tau_s, tau)
        G.check_step(oracle, ix, q, tau, idx, cnt, out, tag=f"query1 safe S={S}")
        st_safe = ix.stats()
        # (1b) the library derives the same thresholds from tau alone: equal to the oracle's on the
        # exported index up to fp32 rounding of the bounds, never above them by more than that, and
        # Query 1 with them returns Problem 1's set
        lib_tau_s = G.subspace_thresholds(ix, q, tau)
        for h in range(hq):
            want = oracle.safe_subspace_thresholds(f[h], float(tau[0, h]))
            scale = abs(float(tau[0, h])) + np.abs(f[h]).max(axis=1).sum()
            assert np.all(np.abs(lib_tau_s[0, h] - want) <= 2e-5 * scale), (h, lib_tau_s[0, h], want)
        idx, cnt, out = G.query1(ix, q, lib_tau_s, tau)
        G.check_step(oracle, ix, q, tau, idx, cnt, out, tag=f"query1 library thresholds S={S}")
        assert ix.stats()["groups_surviving"] <= st_safe["groups_surviving"] * 1.05 + 8
        # (2) thresholds that cut: per block the median of that block's bounds
        for quant in (0.5, 0.9):
            for h in range(hq):
                tau_s[0, h] = np.quantile(f[h], quant, axis=1).astype(np.float32)
            idx, cnt, out = G.query1(ix, q, tau_s, tau)
            st = ix.stats()
            alive_any_lo = np.zeros(n_groups, dtype=bool)
            alive_any_hi = np.zeros(n_groups, dtype=bool)
            for h in range(hq):
                s_f32 = oracle.scores_f32(q[0, h], K[0, 0])
                te = tau_s[0, h].astype(np.float64)
                te = te - 0.5e-4 * np.abs(te)
                slack = 1e-5 * np.abs(te) + 1e-3
                strict = oracle.query1_filter(f[h], label, te + slack)          # certainly candidates
                loose = oracle.query1_filter(f[h], label, te - slack)           # possibly candidates
                alive_any_lo |= strict.reshape(n_groups, r)[:, 0]
                alive_any_hi |= loose.reshape(n_groups, r)[:, 0]
                got = np.zeros(n, dtype=bool)
                got[idx[0, h, :cnt[0, h]]] = True
                assert cnt[0, h] == got.sum()
                band = 1e-4 * abs(float(tau[0, h]))
                tail = np.arange(n) >= n_groups * r                            # buffer keys: tau only
                # zero false negatives inside Alg. 3's candidate set
                must = (s_f32 >= tau[0, h]) & (np.concatenate([strict, np.ones(n - n_groups * r, bool)]) | tail)
                assert not (must & ~got).any(), (S, quant, h)
                # nothing below the threshold band
                assert not (got & (s_f32 < tau[0, h] - band)).any()
                # the promise of Query 1: relevant keys whose block products all reach tau_s
                blocks = (Kd * q[0, h].astype(np.float64)).reshape(n, S, ds).sum(-1)   # [n][S]
                relevant = (s_f32 >= tau[0, h]) & (blocks >= tau_s[0, h][None, :] + 1e-3).all(1)
                assert not (relevant & ~got).any()
            assert alive_any_lo.sum() <= st["groups_surviving"] <= alive_any_hi.sum(), \
                (S, quant, alive_any_lo.sum(), st["groups_surviving"], alive_any_hi.sum())
            G.say(f"  quantile {quant}: {st['groups_surviving']} of {st['groups_scored']} groups are candidates "
                  f"(safe thresholds: {st_safe['groups_surviving']})")
            assert st["groups_surviving"] < st["groups_scored"]


def test_query1_unsupported_configurations(G):
    L = G.L
    cache = _small_cache(2, 512)
    q = torch.zeros((1, 8, 128), device="cuda")
    tau = torch.zeros((1, 8), device="cuda")
    idx = torch.zeros((1, 8, 16), dtype=torch.int32, device="cuda")
    cnt = torch.zeros((1, 8), dtype=torch.int32, device="cuda")
    for kw in (dict(enclosing=L.LVR_ENCLOSE_AABB, n_subspaces=8), dict(flags=L.LVR_SEPARATE_KERNELS)):
        with G.Index(cache.K, cache.V, "bf16", 8, **kw) as ix:
            S = kw.get("n_subspaces", 4)
            with pytest.raises(L.LouverError) as e:
                L.lvr_query1(ix.h, q, torch.zeros((1, 8, S), device="cuda"), tau, idx, cnt)
            assert e.value.code == L.LVR_E_UNSUPPORTED


# ---------------------------------------------------------------------------------------------
# Offloaded mode (Sec. 5 "KV Cache Offloading"): K and V in pinned host memory, index on the GPU
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("grouping,flags", [("contiguous", 0), ("contiguous", 2), ("tree", 0), ("contiguous", 4)])
def test_offloaded_kv_same_results(G, oracle, grouping, flags):
    """With the K/V arena in host memory every entry point gives the results of the resident
    arena: sets and attention against the oracle, exported index bit-equal, appends included;
    device memory then holds the index and work space only."""
    L = G.L
    n0, extra, B = 3000 + 3, 150, 64
    gr = L.LVR_GROUP_TREE if grouping == "tree" else L.LVR_GROUP_CONTIGUOUS
    cache = W.make_local_cache(2, n=n0 + extra)
    K, V = cache.K[:, :2], cache.V[:, :2]
    q = W.make_queries(2, n_q_heads=8)
    G.say(f"offloaded grouping={grouping} flags={flags}")
    kw = dict(capacity=n0 + extra, buffer_size=B, grouping=gr, index_dtype=L.LVR_INDEX_SAME)
    with G.Index(K[:, :, :n0], V[:, :, :n0], "bf16", 8, flags=flags | L.LVR_KV_IN_HOST_MEMORY, **kw) as ix, \
         G.Index(K[:, :, :n0], V[:, :, :n0], "bf16", 8, flags=flags, **kw) as ref:
        kv_bytes = 2 * 2 * ((n0 + extra + 63) // 64 * 64) * 128 * 2
        assert L.lvr_host_bytes(ix.cfg) == kv_bytes and L.lvr_host_bytes(ref.cfg) == 0
        assert L.lvr_arena_bytes(ref.cfg) - L.lvr_arena_bytes(ix.cfg) == kv_bytes
        for step in range(3):
            for frac in (0.01, 0.2):
                tau = G.oracle_taus(oracle, ix, q, frac=frac)
                for fused in (True, False):
                    idx, cnt, out = ix.query(q, tau, fused=fused)
                    G.check_step(oracle, ix, q, tau, idx, cnt, out, tag=f"offloaded step={step} frac={frac}")
                st, st_ref = ix.stats(), None
                ref.query(q, tau)
                st_ref = ref.stats()
                assert st["groups_surviving"] == st_ref["groups_surviving"]
            got = ix.dense(q)
            want = oracle.dense_attention(ix.K, ix.V, q, ix.sigma, 8)
            assert (np.abs(got - want).max(axis=-1) / np.abs(want).max(axis=-1)).max() <= G.ATTN_TOL
            lo, hi = n0 + step * 50, n0 + (step + 1) * 50
            ix.append(K[:, :, lo:hi], V[:, :, lo:hi])
            ref.append(K[:, :, lo:hi], V[:, :, lo:hi])
        L.lvr_publish(ix.h)
        L.lvr_publish(ref.h)
        for name, x, y in zip(("centres", "radii", "slot_pos", "keys"), ix.export(), ref.export()):
            assert np.array_equal(np.asarray(x), np.asarray(y)), name
    # the default centre format: 6-bit in device memory, the cache's own behind the host link
    auto_dev = L.make_config(batch=1, n_q_heads=8, n_kv_heads=2, capacity=1024)
    auto_host = L.make_config(batch=1, n_q_heads=8, n_kv_heads=2, capacity=1024, flags=L.LVR_KV_IN_HOST_MEMORY)
    same_host = L.make_config(batch=1, n_q_heads=8, n_kv_heads=2, capacity=1024, flags=L.LVR_KV_IN_HOST_MEMORY,
                              index_dtype=L.LVR_INDEX_SAME)
    assert L.lvr_arena_bytes(auto_host) == L.lvr_arena_bytes(same_host)
    assert L.lvr_arena_bytes(auto_dev) - 2 * L.lvr_host_bytes(auto_host) // 2 == L.lvr_arena_bytes(auto_host) - 2 * (1024 // 4) * (256 + 16 - 96 - 12)   # 6-bit centres: 96 bytes of codes, 12 of radii (four bf16) and scales, against 256 + four floats


# ---------------------------------------------------------------------------------------------
# Append + decode step in one call (the store of the new rows rides in the query launch)
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("variant", ["plain", "tree", "reservoir", "buffer_dense", "m3"])
def test_append_decode_step_equals_the_two_calls(G, oracle, variant):
    L = G.L
    n0, steps, B = 203, 120, 32
    m = 3 if variant == "m3" else 1
    kw = dict(capacity=n0 + steps * m, buffer_size=B)
    if variant == "tree":
        kw["grouping"] = L.LVR_GROUP_TREE
    if variant == "reservoir":
        kw.update(reservoir_size=64, seed=9)
    if variant == "buffer_dense":
        kw["flags"] = L.LVR_ATTEND_BUFFER_DENSE
    cache = _small_cache(5, n0)
    k_new, v_new = W.make_append_stream(5, steps * m, cache)          # [T][batch][hkv][d]
    qs = W.drift_queries(5, steps, n_q_heads=8)
    G.say(f"append+decode variant={variant}")
    with G.Index(cache.K, cache.V, "bf16", 8, **kw) as ix, G.Index(cache.K, cache.V, "bf16", 8, **kw) as ref:
        cap = n0 + steps * m
        out = torch.zeros((1, 8, 128), device="cuda")
        idx = torch.zeros((1, 8, cap), dtype=torch.int32, device="cuda")
        cnt = torch.zeros((1, 8), dtype=torch.int32, device="cuda")
        for t in range(steps):
            kk = np.ascontiguousarray(k_new[t * m:(t + 1) * m].transpose(1, 2, 0, 3))
            vv = np.ascontiguousarray(v_new[t * m:(t + 1) * m].transpose(1, 2, 0, 3))
            ref.append(kk, vv)
            ix.K, ix.V = ref.K, ref.V                                   # host copies for the oracle
            tau = G.oracle_taus(oracle, ref, qs[t], frac=0.05)
            qd = torch.from_numpy(qs[t]).cuda()
            td = torch.from_numpy(tau).cuda()
            L.lvr_append_decode_step(ix.h, G.to_device(kk, "bf16"), G.to_device(vv, "bf16"), qd, td, out, idx, cnt)
            torch.cuda.synchronize()
            assert L.lvr_length(ix.h) == L.lvr_length(ref.h)
            gi, gc, go = idx.cpu().numpy(), cnt.cpu().numpy(), out.cpu().numpy()
            ri, rc, ro = ref.query(qs[t], tau, cap=cap, fused=True)
            assert np.array_equal(gc, rc)
            for h in range(8):
                assert set(gi[0, h, :gc[0, h]].tolist()) == set(ri[0, h, :rc[0, h]].tolist()), (t, h)
            assert np.abs(go - ro).max() <= 1e-5 * max(1.0, np.abs(ro).max())
            if t % 13 == 0 or t == steps - 1:
                n_indexed = L.lvr_length(ix.h)[1]
                G.check_step(oracle, ix, qs[t], tau, gi, gc, go, tag=f"append+decode {variant} t={t}",
                             extra_from=(n_indexed if variant == "buffer_dense" else -1))
        for name, x, y in zip(("centres", "radii", "slot_pos", "keys"), ix.export(), ref.export()):
            assert np.array_equal(np.asarray(x), np.asarray(y)), name
        if variant == "reservoir":
            assert np.array_equal(ix.reservoir(), ref.reservoir())


# ---------------------------------------------------------------------------------------------
# Centres stored as 8-bit e4m3 codes (LVR_INDEX_FP8)
# ---------------------------------------------------------------------------------------------
def _e4m3_values():
    v = []
    for code in range(127):                      # 0x7f is the NaN code
        e, m = code >> 3, code & 7
        v.append((m / 8.0) * 2.0 ** -6 if e == 0 else (1 + m / 8.0) * 2.0 ** (e - 7))
    return np.array(sorted(set(v + [-x for x in v])))


@pytest.mark.parametrize("S", [1, 2, 4])
def test_fp8_centres_enclose_members(G, oracle, S):
    """Exported 8-bit index: every stored centre coordinate is an e4m3 value and the nearest one
    to the group mean (ties aside), the balls enclose their members measured against the centres
    AS STORED, and are not looser than the documented widening."""
    n, r = 2048, 4
    cache = _small_cache(2, n)
    Kc = cache.K
    with G.Index(Kc, Kc, "bf16", 2, group_size=r, n_subspaces=S, index_dtype=G.L.LVR_INDEX_FP8) as ix:
        centres, radii, slot_pos, keys = ix.export()
        grid = _e4m3_values()
        for h in range(2):
            c = W.bf16_bits_to_f32(centres[0, h]).reshape(n // r, 128).astype(np.float64)
            assert np.isin(c, grid).all(), "a stored centre coordinate is not an e4m3 value"
            label = (np.arange(n) // r).astype(np.int32)
            mean, _ = oracle.ball_index(Kc[0, h], label, n // r, S)
            mean = np.clip(mean, -448, 448)
            # nearest grid value: no other e4m3 value is closer to the mean (up to the fp32 error of the mean)
            pos = np.searchsorted(grid, mean)
            lo = grid[np.clip(pos - 1, 0, grid.size - 1)]
            hi = grid[np.clip(pos, 0, grid.size - 1)]
            best = np.minimum(np.abs(mean - lo), np.abs(mean - hi))
            absmean = np.abs(Kc[0, h]).reshape(n // r, r, 128).mean(axis=1)     # fp32 summation error of the mean
            assert np.all(np.abs(c - mean) <= best + 2 * r * 2.0 ** -24 * absmean + 1e-12)
            need = oracle.ball_radii_for_centres(Kc[0, h], label, c, S)
            assert np.all(radii[0, h] >= need), "a member lies outside its ball"
            cn = np.stack([np.linalg.norm(c[:, a:b], axis=1)
                           for a, b in (oracle.subspace_range(128, S, s) for s in range(S))], axis=1)
            # not loose: the widening of every radius (2^-12 of radius and centre norm, in fp32), then the round-up
            # to the eight significant bits the 8-bit index stores a radius with (at most one part in 2^7)
            assert np.all(radii[0, h] <= (need * (1 + 2.0 ** -11) + cn * 2.0 ** -11) * (1 + 2.0 ** -7) + 1e-30)
            assert np.array_equal(keys[0, h], W.f32_to_bf16_bits(Kc[0, h]).reshape(n, 128))


@pytest.mark.parametrize("n,r,S,hq,grouping", [(1000, 4, 4, 8, "contiguous"), (2051, 4, 4, 16, "contiguous"),
                                               (777, 8, 2, 4, "tree"), (4096, 2, 1, 8, "contiguous"), (3, 4, 4, 8, "contiguous")])
def test_fp8_centres_queries(G, oracle, n, r, S, hq, grouping):
    L = G.L
    cache = _small_cache(2, n)
    q = W.make_queries(2, n_q_heads=hq)
    gr = L.LVR_GROUP_TREE if grouping == "tree" else L.LVR_GROUP_CONTIGUOUS
    G.say(f"fp8 centres n={n} r={r} S={S} hq={hq} {grouping}")
    with G.Index(cache.K, cache.V, "bf16", hq, group_size=r, n_subspaces=S, grouping=gr,
                 index_dtype=L.LVR_INDEX_FP8) as ix:
        for frac in (0.01, 0.2):
            tau = G.oracle_taus(oracle, ix, q, frac=frac)
            for fused in (True, False):
                idx, cnt, out = ix.query(q, tau, fused=fused)
                G.check_step(oracle, ix, q, tau, idx, cnt, out, tag=f"fp8 n={n} frac={frac}")
        st = ix.stats()
        assert st["bytes_index"] == st["groups_scored"] * (128 + 8)     # codes + 8 bytes of radii (four bf16)


@pytest.mark.parametrize("S", [1, 4])
def test_fp8_centres_surviving_groups_and_pruning(G, oracle, S):
    """On keys with positional locality: the groups kept equal those whose Eq. (2) bound on the
    exported 8-bit index reaches tau; coarser centres keep somewhat more groups than bf16 centres,
    never fewer qualifying keys."""
    n, r = 8192, 4
    cache = W.make_local_cache(2, n=n)
    K, V = cache.K[:, :1], cache.V[:, :1]
    q = W.make_queries(2, n_q_heads=4)
    with G.Index(K, V, "bf16", 4, group_size=r, n_subspaces=S, index_dtype=G.L.LVR_INDEX_FP8) as ix, \
         G.Index(K, V, "bf16", 4, group_size=r, n_subspaces=S, index_dtype=G.L.LVR_INDEX_SAME) as ref:
        centres, radii, _, _ = ix.export()
        c = W.bf16_bits_to_f32(centres[0, 0]).reshape(n // r, 128).astype(np.float64)
        for frac in (0.002, 0.02):
            t = G.oracle_taus(oracle, ix, q, frac=frac)
            idx, cnt, out = ix.query(q, t)
            G.check_step(oracle, ix, q, t, idx, cnt, out, tag=f"fp8 local frac={frac}")
            st = ix.stats()
            ref.query(q, t)
            st_ref = ref.stats()
            ub = np.stack([oracle.ball_bounds(q[0, h], c, radii[0, 0].astype(np.float64)).sum(0) for h in range(4)])
            te = t[0] - 0.5e-4 * np.abs(t[0])
            lo = int(np.any(ub >= te[:, None] * (1 + 1e-5) + 1e-3, axis=0).sum())
            hi = int(np.any(ub >= te[:, None] * (1 - 1e-5) - 1e-3, axis=0).sum())
            assert lo <= st["groups_surviving"] <= hi, (frac, lo, st["groups_surviving"], hi)
            G.say(f"  S={S} frac={frac}: surviving with 8-bit centres {st['groups_surviving']}, with bf16 centres "
                  f"{st_ref['groups_surviving']} of {st['groups_scored']}")
            assert st["groups_surviving"] < 0.5 * st["groups_scored"]
            assert st["bytes_index"] < 0.6 * st_ref["bytes_index"]


def test_fp8_centres_surface_keys_saturation_and_append(G, oracle):
    """Keys exactly on ball surfaces, coordinates beyond the e4m3 range (the centre saturates, the
    radius takes up the difference), appends across flushes: nothing is ever lost."""
    L = G.L
    g = np.random.default_rng(12)
    n, r = 512, 4
    qdir = np.zeros(128, dtype=np.float32)
    qdir[[3, 40, 77, 120]] = [1.0, -1.0, 1.0, 1.0]
    K = np.zeros((1, 1, n, 128), dtype=np.float32)
    for gi in range(n // r):
        centre = W.round_to_bf16(g.integers(-8, 9, size=128).astype(np.float32))
        if gi % 7 == 0:
            centre[5] = 1000.0          # beyond 448
            centre[99] = -3000.0
        step = float(g.integers(1, 5)) * 0.5
        K[0, 0, gi * r + 0] = centre + step * qdir
        K[0, 0, gi * r + 1] = centre - step * qdir
        K[0, 0, gi * r + 2] = centre
        K[0, 0, gi * r + 3] = centre
    K = W.round_to_bf16(K)
    V = W.round_to_bf16(g.standard_normal((1, 1, n, 128)).astype(np.float32))
    q = (qdir * 3.0)[None, None, :]
    for S in (1, 4):
        with G.Index(K[:, :, :300], V[:, :, :300], "bf16", 1, n_subspaces=S, capacity=n, buffer_size=32,
                     index_dtype=L.LVR_INDEX_FP8) as ix:
            ix.append(K[:, :, 300:], V[:, :, 300:])
            s = oracle.scores_f32(q[0, 0], K[0, 0])
            for tau in np.unique(s)[-6:]:
                t = np.full((1, 1), tau, dtype=np.float32)
                idx, cnt, out = ix.query(q, t)
                G.check_step(oracle, ix, q, t, idx, cnt, out, tag=f"fp8 surface S={S} tau={tau}")


def test_fp8_centres_unsupported_configurations(G):
    L = G.L
    ok = dict(batch=1, n_q_heads=8, n_kv_heads=2, capacity=1024, index_dtype=L.LVR_INDEX_FP8)
    assert L.lvr_arena_bytes(L.make_config(**ok)) > 0
    assert L.lvr_arena_bytes(L.make_config(**dict(ok, enclosing=L.LVR_ENCLOSE_AABB, n_subspaces=16))) > 0
    for bad in (dict(ok, kv_dtype=L.LVR_F32), dict(ok, n_subspaces=8),
                dict(ok, flags=L.LVR_SEPARATE_KERNELS), dict(ok, index_dtype=4)):
        assert L.lvr_arena_bytes(L.make_config(**bad)) == 0
    # AUTO falls back to the cache's own format where 8-bit centres are not supported
    for kw in (dict(n_subspaces=8), dict(flags=L.LVR_SEPARATE_KERNELS), dict(enclosing=L.LVR_ENCLOSE_AABB)):
        cfg_auto = L.make_config(batch=1, n_q_heads=8, n_kv_heads=2, capacity=1024, **kw)
        cfg_same = L.make_config(batch=1, n_q_heads=8, n_kv_heads=2, capacity=1024, index_dtype=L.LVR_INDEX_SAME, **kw)
        assert L.lvr_arena_bytes(cfg_auto) == L.lvr_arena_bytes(cfg_same) > 0
    cfg_auto = L.make_config(batch=1, n_q_heads=8, n_kv_heads=2, capacity=1024)
    cfg_same = L.make_config(batch=1, n_q_heads=8, n_kv_heads=2, capacity=1024, index_dtype=L.LVR_INDEX_SAME)
    assert L.lvr_arena_bytes(cfg_same) - L.lvr_arena_bytes(cfg_auto) == 2 * (1024 // 4) * (256 + 16 - 96 - 12)   # AUTO: 6-bit centres
    cfg_fp8 = L.make_config(**ok)
    assert L.lvr_arena_bytes(cfg_same) - L.lvr_arena_bytes(cfg_fp8) == 2 * (1024 // 4) * (128 + 8)


# ---------------------------------------------------------------------------------------------
# One-launch attention over lists that carry their scores: set sizes around its batch and round boundaries
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("hkv,gq,n", [(2, 4, 6000), (1, 1, 6000), (3, 2, 6000), (2, 4, 66000), (1, 2, 70001), (1, 2, 140001), (1, 2, 270001)])
def test_decode_step_set_sizes_around_batch_and_round_boundaries(G, oracle, hkv, gq, n):
    """The decode step's attention takes entries in batches of 16 dealt to 16 waves and in rounds of 1024; every
    head of one step gets a different set size around those boundaries (0, 1, 15, 16, 17, 255, 256, 257, 1023, 1024,
    1025, 2047, 2049, 3000), with the list capacity at the context and just above the largest set.  Beyond 65536
    keys of context two workgroups share a head (one per half of the channels); beyond 262144 the attention is two
    launches (partial sums over slices of the list, then a merge), still fed with the carried scores."""
    hq = hkv * gq
    cache = _small_cache(2, n, hkv=hkv)
    g = np.random.default_rng(31 + hq)
    sizes = [0, 1, 15, 16, 17, 255, 256, 257, 1023, 1024, 1025, 2047, 2049, 3000]
    for rep in range(2):
        q = W.make_queries(2, n_q_heads=hq, step=rep)
        with G.Index(cache.K, cache.V, "bf16", hq, group_size=1, buffer_size=64, capacity=n) as ix:
            ks = [sizes[(h * 5 + rep * 3 + int(g.integers(0, 2))) % len(sizes)] for h in range(hq)]
            tau = np.zeros((1, hq), dtype=np.float32)
            for h in range(hq):
                s = oracle.scores_f32(q[0, h], ix.K[0, h // ix.G])
                tau[0, h] = W.tau_for_count(s, ks[h]) if ks[h] > 0 else np.float32(s.max() + 1.0)
            for cap in (n, 3008):
                G.say(f"set sizes {ks} cap {cap}")
                idx, cnt, out = ix.query(q, tau, cap=cap, fused=True)
                # the sizes asked for, plus at most the few keys inside the tolerance band just below a threshold
                assert all(k <= int(c) <= k + 4 for k, c in zip(ks, cnt[0])), (ks, cnt[0].tolist())
                G.check_step(oracle, ix, q, tau, idx, cnt, out, tag=f"sizes hkv={hkv} gq={gq} cap={cap}")


# ---------------------------------------------------------------------------------------------
# Centres stored as 6-bit e2m3 codes with a power-of-two scale per 32 coordinates (LVR_INDEX_FP6)
# ---------------------------------------------------------------------------------------------
_E2M3 = np.array(sorted({s * v for s in (-1.0, 1.0)
                         for v in [m / 8.0 for m in range(8)] + [(1 + m / 8.0) * 2.0 ** (e - 1) for e in (1, 2, 3) for m in range(8)]}))


def _scale_blocks(x):
    """[..., 128] -> [..., 4, 32]: block b holds coordinates 32 kk + 8 b + e (kk = 0..3, e = 0..7)."""
    return np.moveaxis(x.reshape(x.shape[:-1] + (4, 4, 8)), -2, -3).reshape(x.shape[:-1] + (4, 32))


@pytest.mark.parametrize("S", [1, 2, 4])
@pytest.mark.parametrize("r", [1, 4])
def test_fp6_centres_enclose_members(G, oracle, S, r):
    """Exported 6-bit index: within every block of 32 coordinates that share a scale the stored centre is an
    e2m3 value times the smallest power of two that covers the block's largest mean, and the nearest such value;
    the balls enclose their members measured against the centres AS STORED and are not looser than the documented
    widening."""
    n = 2048
    cache = _small_cache(2, n)
    Kc = cache.K
    with G.Index(Kc, Kc, "bf16", 2, group_size=r, n_subspaces=S, index_dtype=G.L.LVR_INDEX_FP6) as ix:
        centres, radii, slot_pos, keys = ix.export()
        st_bytes = G.L.lvr_arena_bytes(G.L.make_config(batch=1, n_q_heads=2, n_kv_heads=2, capacity=n, group_size=r,
                                                       n_subspaces=S, index_dtype=G.L.LVR_INDEX_FP6))
        assert st_bytes > 0
        chan = ix.channel_factors()
        for h in range(2):
            # the index is stored in the space k_c / 2^e_c: the exported centres come back in the keys' own space, the
            # radii, the grid and the scale blocks belong to the stored one
            a = chan[0, h]
            assert np.all(np.log2(a) == np.rint(np.log2(a))) and np.all(np.abs(np.log2(a)) <= 8)
            c = W.bf16_bits_to_f32(centres[0, h]).reshape(n // r, 128).astype(np.float64) / a
            label = (np.arange(n) // r).astype(np.int32)
            Ks = Kc[0, h].astype(np.float64) / a
            mean, _ = oracle.ball_index(Ks, label, n // r, S)
            mb, cb = _scale_blocks(mean), _scale_blocks(c)
            amax = np.abs(mb).max(axis=-1)
            E = np.ceil(np.log2(np.maximum(amax, 1e-300) / 7.5))
            # a block whose largest mean sits within rounding of 7.5 * 2^E may have gone either way: leave it out
            frac = amax / (7.5 * 2.0 ** E)
            sure = (frac < 1 - 1e-5) & (frac > 0.5 + 1e-5)
            assert sure.mean() > 0.99
            scaled = cb / 2.0 ** E[..., None]
            assert np.isin(scaled[sure], _E2M3).all(), "a stored centre coordinate is not an e2m3 value times its block's scale"
            # nearest: no other value of the block's grid is closer to the mean (up to the fp32 error of the mean)
            target = mb / 2.0 ** E[..., None]
            pos = np.searchsorted(_E2M3, target)
            lo = _E2M3[np.clip(pos - 1, 0, _E2M3.size - 1)]
            hi = _E2M3[np.clip(pos, 0, _E2M3.size - 1)]
            best = np.minimum(np.abs(target - lo), np.abs(target - hi))
            assert np.all((np.abs(scaled - target) <= best + 1e-5)[sure])
            need = oracle.ball_radii_for_centres(Ks, label, c, S)
            assert np.all(radii[0, h] >= need), "a member lies outside its ball"
            cn = np.stack([np.linalg.norm(c[:, a:b], axis=1)
                           for a, b in (oracle.subspace_range(128, S, s) for s in range(S))], axis=1)
            assert np.all(radii[0, h] <= (need * (1 + 2.0 ** -11) + cn * 2.0 ** -11) * (1 + 2.0 ** -7) + 1e-30)
            assert np.array_equal(keys[0, h], W.f32_to_bf16_bits(Kc[0, h]).reshape(n, 128))


@pytest.mark.parametrize("n,r,S,hq,grouping", [(1000, 4, 4, 8, "contiguous"), (2051, 1, 4, 16, "contiguous"), (5000, 1, 4, 8, "contiguous"),
                                               (777, 8, 2, 4, "tree"), (4096, 2, 1, 8, "contiguous"), (3, 4, 4, 8, "contiguous"),
                                               (3001, 1, 2, 2, "tree"), (70000, 1, 4, 4, "contiguous")])
def test_fp6_centres_queries(G, oracle, n, r, S, hq, grouping):
    L = G.L
    cache = _small_cache(2, n)
    q = W.make_queries(2, n_q_heads=hq)
    gr = L.LVR_GROUP_TREE if grouping == "tree" else L.LVR_GROUP_CONTIGUOUS
    G.say(f"fp6 centres n={n} r={r} S={S} hq={hq} {grouping}")
    with G.Index(cache.K, cache.V, "bf16", hq, group_size=r, n_subspaces=S, grouping=gr,
                 index_dtype=L.LVR_INDEX_FP6) as ix:
        for frac in (0.01, 0.2):
            tau = G.oracle_taus(oracle, ix, q, frac=frac)
            for fused in (True, False):
                idx, cnt, out = ix.query(q, tau, fused=fused)
                G.check_step(oracle, ix, q, tau, idx, cnt, out, tag=f"fp6 n={n} frac={frac}")
        st = ix.stats()
        assert st["bytes_index"] == st["groups_scored"] * (96 + 12)     # codes + four bf16 radii + four scale bytes


@pytest.mark.parametrize("S", [1, 4])
def test_fp6_centres_surviving_groups_and_pruning(G, oracle, S):
    """On keys with positional locality: the groups kept equal those whose Eq. (2) bound on the exported 6-bit
    index reaches tau; the index is under half the bytes of bf16 centres and still prunes."""
    n, r = 8192, 4
    cache = W.make_local_cache(2, n=n)
    K, V = cache.K[:, :1], cache.V[:, :1]
    q = W.make_queries(2, n_q_heads=4)
    with G.Index(K, V, "bf16", 4, group_size=r, n_subspaces=S, index_dtype=G.L.LVR_INDEX_FP6) as ix, \
         G.Index(K, V, "bf16", 4, group_size=r, n_subspaces=S, index_dtype=G.L.LVR_INDEX_SAME) as ref:
        centres, radii, _, _ = ix.export()
        a = ix.channel_factors()[0, 0]
        c = W.bf16_bits_to_f32(centres[0, 0]).reshape(n // r, 128).astype(np.float64) / a
        for frac in (0.002, 0.02):
            t = G.oracle_taus(oracle, ix, q, frac=frac)
            idx, cnt, out = ix.query(q, t)
            G.check_step(oracle, ix, q, t, idx, cnt, out, tag=f"fp6 local frac={frac}")
            st = ix.stats()
            ref.query(q, t)
            st_ref = ref.stats()
            ub = np.stack([oracle.ball_bounds(q[0, h] * a, c, radii[0, 0].astype(np.float64)).sum(0) for h in range(4)])
            te = t[0] - 0.5e-4 * np.abs(t[0])
            lo = int(np.any(ub >= te[:, None] * (1 + 1e-5) + 1e-3, axis=0).sum())
            hi = int(np.any(ub >= te[:, None] * (1 - 1e-5) - 1e-3, axis=0).sum())
            assert lo <= st["groups_surviving"] <= hi, (frac, lo, st["groups_surviving"], hi)
            G.say(f"  S={S} frac={frac}: surviving with 6-bit centres {st['groups_surviving']}, with bf16 centres "
                  f"{st_ref['groups_surviving']} of {st['groups_scored']}")
            assert st["groups_surviving"] < 0.6 * st["groups_scored"]
            assert st["bytes_index"] < 0.45 * st_ref["bytes_index"]


def test_fp6_centres_surface_keys_wide_range_and_append(G, oracle):
    """Keys exactly on ball surfaces, blocks whose largest coordinate dwarfs the others (they round to zero under
    the shared scale; the radius takes up the difference), all-zero groups, appends across flushes: nothing is
    ever lost."""
    L = G.L
    g = np.random.default_rng(13)
    n, r = 512, 4
    qdir = np.zeros(128, dtype=np.float32)
    qdir[[3, 40, 77, 120]] = [1.0, -1.0, 1.0, 1.0]
    K = np.zeros((1, 1, n, 128), dtype=np.float32)
    for gi in range(n // r):
        centre = W.round_to_bf16(g.integers(-8, 9, size=128).astype(np.float32))
        if gi % 7 == 0:
            centre[5] = 1000.0
            centre[99] = -3.0e6
        if gi % 11 == 0:
            centre[:] = 0.0
        if gi % 13 == 0:
            centre *= 2.0 ** -30
        step = float(g.integers(1, 5)) * 0.5 * (2.0 ** -30 if gi % 13 == 0 else 1.0)
        K[0, 0, gi * r + 0] = centre + step * qdir
        K[0, 0, gi * r + 1] = centre - step * qdir
        K[0, 0, gi * r + 2] = centre
        K[0, 0, gi * r + 3] = centre
    K = W.round_to_bf16(K)
    V = W.round_to_bf16(g.standard_normal((1, 1, n, 128)).astype(np.float32))
    q = (qdir * 3.0)[None, None, :]
    for S, rr in ((1, 4), (4, 4), (4, 1)):
        with G.Index(K[:, :, :300], V[:, :, :300], "bf16", 1, group_size=rr, n_subspaces=S, capacity=n, buffer_size=32,
                     index_dtype=L.LVR_INDEX_FP6) as ix:
            ix.append(K[:, :, 300:], V[:, :, 300:])
            s = oracle.scores_f32(q[0, 0], K[0, 0])
            for tau in np.unique(s)[-6:]:
                t = np.full((1, 1), tau, dtype=np.float32)
                idx, cnt, out = ix.query(q, t)
                G.check_step(oracle, ix, q, t, idx, cnt, out, tag=f"fp6 surface S={S} r={rr} tau={tau}")


def test_fp6_index_follows_channels_of_very_different_size(G, oracle):
    """Keys whose channels span three decades (and queries that weigh the small channels up, so that every channel
    matters to a score): a 6-bit code with one scale per 32 coordinates would round the small channels to zero and
    keep nearly every ball; the index is therefore built on keys divided by a power of two per channel.  The exponents
    follow the channels' sizes, the results are the oracle's, and most balls are pruned, with four heads per KV head and
    with eight (another kernel)."""
    L = G.L
    g = np.random.default_rng(77)
    n, hkv = 4096, 2
    mag = 2.0 ** g.uniform(-5.0, 5.0, size=(hkv, 128))
    K = W.round_to_bf16((g.standard_normal((1, hkv, n, 128)) * mag[None, :, None, :]).astype(np.float32))
    V = W.round_to_bf16(g.standard_normal((1, hkv, n, 128)).astype(np.float32))
    for hq in (8, 16):
        Gq = hq // hkv
        q = (g.standard_normal((1, hq, 128)) / np.repeat(mag, Gq, axis=0)[None]).astype(np.float32)
        with G.Index(K, V, "bf16", hq, group_size=1, index_dtype=L.LVR_INDEX_FP6, capacity=n + 512) as ix:
            e = L.lvr_export_channel_scales(ix.h, ix.cfg).astype(np.float64)
            assert e.shape == (1, hkv, 128)
            rms = np.sqrt((K.astype(np.float64) ** 2).mean(axis=2))     # [1][hkv][128]
            d = e - np.log2(rms)
            # one offset per (sequence, KV head), then rounding to the nearest integer; the library estimates the
            # rms from every row here (4096 is its sample size), in fp32
            from oracle import pruning_power as pp
            for h in range(hkv):
                assert d[0, h].max() - d[0, h].min() <= 1.0 + 1e-3, (h, d[0, h].min(), d[0, h].max())
                # the oracle's rule in fp64: the same exponents up to a common shift (the offset is only defined up to
                # whole numbers), but for a channel that sits on a rounding boundary
                want = np.log2(pp.channel_factors(K[0, h]))
                diff = e[0, h] - want
                shift = np.rint(np.median(diff))
                assert np.all(np.abs(diff - shift) <= 1) and (diff == shift).mean() >= 0.97, (h, diff)
            for frac in (0.003, 0.03):
                tau = G.oracle_taus(oracle, ix, q, frac=frac)
                idx, cnt, out = ix.query(q, tau)
                G.check_step(oracle, ix, q, tau, idx, cnt, out, tag=f"channels hq={hq} frac={frac}")
                st = ix.stats()
                share = st["groups_surviving"] / st["groups_scored"]
                G.say(f"  channels over three decades, {Gq} heads per KV head, frac={frac}: {share:.3f} of the balls survive")
                if frac < 0.01:
                    # what the same code WITHOUT the rescaling keeps (on the CPU: every key rounded to e2m3 with one
                    # scale per 32 coordinates, exact radii, the sum rule over four blocks)
                    kept = 0
                    for kv in range(hkv):
                        Kd = K[0, kv].astype(np.float64)
                        C = pp.code_keys(Kd, "e2m3")
                        rad = np.stack([np.sqrt(((Kd - C)[:, 32 * s:32 * s + 32] ** 2).sum(1)) for s in range(4)])
                        keep = np.zeros(n, dtype=bool)
                        for h in range(kv * Gq, (kv + 1) * Gq):
                            qd = q[0, h].astype(np.float64)
                            ub = C @ qd + sum(rad[s] * np.linalg.norm(qd[32 * s:32 * s + 32]) for s in range(4))
                            keep |= ub >= tau[0, h]
                        kept += int(keep.sum())
                    plain = kept / (hkv * n)
                    G.say(f"    without the rescaling: {plain:.3f}")
                    assert share < 0.2 and share < 0.5 * plain
            # keys appended later are indexed in the same space
            extra = W.round_to_bf16((g.standard_normal((1, hkv, 300, 128)) * mag[None, :, None, :]).astype(np.float32))
            ix.append(extra, W.round_to_bf16(g.standard_normal((1, hkv, 300, 128)).astype(np.float32)))
            tau = G.oracle_taus(oracle, ix, q, frac=0.01)
            idx, cnt, out = ix.query(q, tau)
            G.check_step(oracle, ix, q, tau, idx, cnt, out, tag=f"channels hq={hq} after append")


def test_channel_scales_follow_the_build_and_only_a_6_bit_index_has_them(G, oracle):
    """The exponents belong to the keys of the last lvr_build: a rebuild on keys with other channel sizes replaces them
    (and the queries stay the oracle's); an index in another centre format reports zeros; before any build the call is
    refused."""
    L = G.L
    g = np.random.default_rng(91)
    n, hkv, hq = 2048, 1, 4
    V = W.round_to_bf16(g.standard_normal((1, hkv, n, 128)).astype(np.float32))
    mag1 = 2.0 ** g.integers(-4, 5, size=128).astype(np.float64)
    mag2 = mag1[::-1].copy()
    K1 = W.round_to_bf16((g.standard_normal((1, hkv, n, 128)) * mag1).astype(np.float32))
    K2 = W.round_to_bf16((g.standard_normal((1, hkv, n, 128)) * mag2).astype(np.float32))
    q = g.standard_normal((1, hq, 128)).astype(np.float32)
    with G.Index(K1, V, "bf16", hq, group_size=1) as ix:       # the default format for balls: 6-bit
        e1 = L.lvr_export_channel_scales(ix.h, ix.cfg)[0, 0].astype(np.int64)
        assert np.array_equal(e1 - e1[0], (np.log2(mag1) - np.log2(mag1[0])).astype(np.int64))   # sizes are exact powers of two apart
        tau = G.oracle_taus(oracle, ix, q, frac=0.01)
        idx, cnt, out = ix.query(q, tau)
        G.check_step(oracle, ix, q, tau, idx, cnt, out, tag="scales, first build")
        L.lvr_build(ix.h, G.to_device(K2, "bf16"), G.to_device(V, "bf16"))
        ix.K, ix.V = K2.copy(), V.copy()
        e2 = L.lvr_export_channel_scales(ix.h, ix.cfg)[0, 0].astype(np.int64)
        assert np.array_equal(e2 - e2[0], (np.log2(mag2) - np.log2(mag2[0])).astype(np.int64))
        tau = G.oracle_taus(oracle, ix, q, frac=0.01)
        idx, cnt, out = ix.query(q, tau)
        G.check_step(oracle, ix, q, tau, idx, cnt, out, tag="scales, rebuilt")
    for dt in (L.LVR_INDEX_SAME, L.LVR_INDEX_FP8):
        with G.Index(K1, V, "bf16", hq, group_size=1, index_dtype=dt) as ix:
            assert not L.lvr_export_channel_scales(ix.h, ix.cfg).any()
    cfg = L.make_config(batch=1, n_q_heads=hq, n_kv_heads=hkv, capacity=256)
    h = L.lvr_create(cfg)
    try:
        with pytest.raises(L.LouverError):
            L.lvr_export_channel_scales(h, cfg)
    finally:
        L.lvr_destroy(h)


@pytest.mark.parametrize("index_dtype", ["auto", "same", "fp8"])
@pytest.mark.parametrize("r,hkv,gq", [(1, 2, 4), (4, 1, 8), (2, 1, 2)])
def test_every_segment_size_of_the_query_launch(G, oracle, index_dtype, r, hkv, gq):
    """A query launch cuts the groups of a (sequence, KV head) into segments of 64 * 2^k groups, one workgroup each
    (k = 0..6: 1 to 64 tiles of 16 groups per wave), sized after the number of workgroups it aims at.  Here that
    target is set from 1 (the largest segments, 4096 groups) to far more than there are tiles (the smallest), on a
    cache whose last segment is ragged and which has a buffer; every size must give the oracle's sets."""
    L = G.L
    n = 70001 if r != 2 else 35001
    cache = _small_cache(3, n, hkv=hkv)
    hq = hkv * gq
    q = W.make_queries(2, n_q_heads=hq, step=1)
    dt = {"auto": L.LVR_INDEX_AUTO, "same": L.LVR_INDEX_SAME, "fp8": L.LVR_INDEX_FP8}[index_dtype]
    # with 2 x 70001 groups: 64, 64, 32, 16, 8, 4, 2, 1 tiles per wave
    for wgs in (1, 40, 100, 150, 300, 600, 1200, 100000):
        with G.Index(cache.K, cache.V, "bf16", hq, group_size=r, buffer_size=64, index_dtype=dt, query_workgroups=wgs) as ix:
            tau = G.oracle_taus(oracle, ix, q, frac=0.004)
            idx, cnt, out = ix.query(q, tau, fused=True)
            G.check_step(oracle, ix, q, tau, idx, cnt, out, tag=f"segments r={r} {index_dtype} target {wgs}")


def test_fp6_centres_unsupported_configurations(G):
    L = G.L
    ok = dict(batch=1, n_q_heads=8, n_kv_heads=2, capacity=1024, index_dtype=L.LVR_INDEX_FP6)
    assert L.lvr_arena_bytes(L.make_config(**ok)) > 0
    for bad in (dict(ok, kv_dtype=L.LVR_F32), dict(ok, n_subspaces=8), dict(ok, flags=L.LVR_SEPARATE_KERNELS),
                dict(ok, enclosing=L.LVR_ENCLOSE_AABB), dict(ok, grouping=L.LVR_GROUP_SUBSPACE_TREE, n_q_heads=2, n_kv_heads=2)):
        assert L.lvr_arena_bytes(L.make_config(**bad)) == 0
    cfg_same = L.make_config(batch=1, n_q_heads=8, n_kv_heads=2, capacity=1024, index_dtype=L.LVR_INDEX_SAME)
    # bf16 centres: 256 + 16 bytes per group of four keys; 6-bit: 96 + 12
    assert L.lvr_arena_bytes(cfg_same) - L.lvr_arena_bytes(L.make_config(**ok)) == 2 * (1024 // 4) * (256 + 16 - 96 - 12)


# ---------------------------------------------------------------------------------------------
# Seeded sweep over combinations of the options
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("case", range(160))
def test_option_combinations(G, oracle, case):
    """Group size, subspaces, heads per KV head, grouping, enclosure, centre format, launch form, buffer
    size and cache size drawn from a seeded generator; every combination the library accepts must give
    the oracle's sets and attention, before and after appends."""
    L = G.L
    g = np.random.default_rng(1000 + case)
    r = int(g.choice([1, 2, 4, 8, 16]))
    S = int(g.choice([1, 2, 4, 8, 16]))
    hkv = int(g.choice([1, 2, 3]))
    Gq = int(g.choice([1, 2, 4, 8]))
    hq = hkv * Gq
    batch = int(g.choice([1, 2]))
    grouping = int(g.choice([L.LVR_GROUP_CONTIGUOUS, L.LVR_GROUP_TREE]))
    enclosing = int(g.choice([L.LVR_ENCLOSE_BALL, L.LVR_ENCLOSE_BALL, L.LVR_ENCLOSE_AABB]))
    index_dtype = int(g.choice([L.LVR_INDEX_AUTO, L.LVR_INDEX_SAME, L.LVR_INDEX_FP8]))
    flags = int(g.choice([0, 0, L.LVR_SEPARATE_KERNELS, L.LVR_ATTEND_BUFFER_DENSE, L.LVR_CONCURRENT_UPDATE]))
    attn = int(g.choice([0, -1, 3, 64]))
    B = 16 * int(g.choice([1, 2, 4])) * (r if r > 1 else 1)
    n0 = int(g.integers(0, 3000))
    extra = int(g.integers(0, 3 * B))
    if index_dtype == L.LVR_INDEX_FP8 and case % 2 == 0:
        index_dtype = L.LVR_INDEX_FP6       # every other explicit 8-bit case asks for 6-bit centres instead
    wl = 1 if case % 5 == 4 else 2          # workload 1 is fp32 with iid keys, workload 2 bf16 with channel scales
    dtype = W.CONFIGS[wl]["dtype"]
    cfg = L.make_config(batch=batch, n_q_heads=hq, n_kv_heads=hkv, group_size=r, n_subspaces=S, buffer_size=B,
                        kv_dtype=(L.LVR_F32 if dtype == "f32" else L.LVR_BF16),
                        grouping=grouping, enclosing=enclosing, flags=flags, capacity=max(n0 + extra, 1),
                        attn_splits=attn, index_dtype=index_dtype)
    desc = f"case {case}: {dtype} r={r} S={S} hq={hq} hkv={hkv} batch={batch} grouping={grouping} enclosing={enclosing} " \
           f"centres={index_dtype} flags={flags} attn={attn} B={B} n0={n0} extra={extra}"
    G.say(desc)
    if L.lvr_arena_bytes(cfg) == 0:
        # a combination this build has no kernel for (boxes or 8-bit centres outside the fused bf16
        # path): creation must say so rather than fall back to something else
        h = C.c_void_p()
        assert L.lib().lvr_create(C.byref(cfg), C.byref(h)) == L.LVR_E_UNSUPPORTED and not h.value, desc
        return
    cache = W.make_local_cache(wl, n=n0 + extra, n_kv_heads=hkv, batch=batch) if case % 2 else \
        W.make_cache(wl, n=n0 + extra, n_kv_heads=hkv, batch=batch)
    q = W.make_queries(wl, n_q_heads=hq, batch=batch, step=case)
    with G.Index(cache.K[:, :, :n0], cache.V[:, :, :n0], dtype, hq, capacity=max(n0 + extra, 1), group_size=r,
                 n_subspaces=S, buffer_size=B, flags=flags, grouping=grouping, enclosing=enclosing, attn_splits=attn,
                 index_dtype=index_dtype) as ix:
        steps = [n0] + ([n0 + extra // 2, n0 + extra] if extra else [])
        have = n0
        for upto in steps:
            if upto > have:
                ix.append(cache.K[:, :, have:upto], cache.V[:, :, have:upto])
                have = upto
            if have == 0:
                continue
            n_indexed = L.lvr_length(ix.h)[1]
            for frac in (0.02, 0.3):
                tau = G.oracle_taus(oracle, ix, q, frac=frac)
                idx, cnt, out = ix.query(q, tau, fused=bool(case & 4))
                G.check_step(oracle, ix, q, tau, idx, cnt, out, tag=desc,
                             extra_from=(n_indexed if flags & L.LVR_ATTEND_BUFFER_DENSE else -1))


def test_misaligned_pointers_are_refused_on_the_host(G):
    """A pointer that the kernels could not read with their load widths comes back as LVR_E_INVALID
    from the host-side check; nothing is launched and the index stays usable."""
    L = G.L
    cache = W.make_cache(2, n=512, n_kv_heads=2)
    q = W.make_queries(2, n_q_heads=8)
    with G.Index(cache.K, cache.V, "bf16", 8, capacity=600) as ix:
        raw = torch.zeros(8 * 128 * 4 + 16, dtype=torch.uint8, device="cuda")
        base = raw.data_ptr()
        assert base % 16 == 0
        good = torch.from_numpy(q.astype(np.float32)).cuda()
        tau = torch.zeros((1, 8), dtype=torch.float32, device="cuda")
        out = torch.zeros((1, 8, 128), dtype=torch.float32, device="cuda")
        idx = torch.zeros((1, 8, 512), dtype=torch.int32, device="cuda")
        cnt = torch.zeros((1, 8), dtype=torch.int32, device="cuda")
        lib = L.lib()
        P = C.c_void_p
        bad_q = P(base + 2)
        assert lib.lvr_decode_step(ix.h, bad_q, P(tau.data_ptr()), P(out.data_ptr()), P(idx.data_ptr()),
                                   P(cnt.data_ptr()), 512, None) == L.LVR_E_INVALID
        assert lib.lvr_query(ix.h, P(good.data_ptr()), P(tau.data_ptr() + 1), P(idx.data_ptr()), P(cnt.data_ptr()), 512,
                             None) == L.LVR_E_INVALID
        assert lib.lvr_dense_attention(ix.h, P(good.data_ptr()), P(out.data_ptr() + 3), None) == L.LVR_E_INVALID
        # one appended row whose address is a multiple of 2 but not of 16
        assert lib.lvr_append(ix.h, P(base + 2), P(base), 1, None) == L.LVR_E_INVALID
        assert L.lvr_length(ix.h)[0] == 512
        tau_np = np.full((1, 8), -np.inf, dtype=np.float32)
        idx2, cnt2, _ = ix.query(q, tau_np)
        assert (cnt2 == 512).all()


def test_subspace_thresholds_edge_cases(G, oracle):
    """No indexed group: every threshold is -inf (nothing can be pruned) and Query 1 still returns
    the buffer's qualifying keys; tau = -inf stays -inf; appended groups are taken into account;
    boxes with more than four blocks and the two-launch form have no such entry point."""
    L = G.L
    cache = W.make_cache(2, n=300, n_kv_heads=2)
    q = W.make_queries(2, n_q_heads=8)
    with G.Index(cache.K[:, :, :3], cache.V[:, :, :3], "bf16", 8, capacity=300, buffer_size=32) as ix:
        tau = np.zeros((1, 8), dtype=np.float32)
        ts = G.subspace_thresholds(ix, q, tau)
        assert np.all(np.isneginf(ts))
        idx, cnt, out = G.query1(ix, q, ts, tau)
        G.check_step(oracle, ix, q, tau, idx, cnt, out, tag="query1 without groups")
        ix.append(cache.K[:, :, 3:], cache.V[:, :, 3:])
        tau = G.oracle_taus(oracle, ix, q, frac=0.05)
        tau[0, 3] = -np.inf
        ts = G.subspace_thresholds(ix, q, tau)
        assert np.all(np.isneginf(ts[0, 3])) and np.all(np.isfinite(np.delete(ts[0], 3, axis=0)))
        idx, cnt, out = G.query1(ix, q, ts, tau)
        G.check_step(oracle, ix, q, tau, idx, cnt, out, tag="query1 after append")
        assert cnt[0, 3] == 300
    for kw in (dict(flags=L.LVR_SEPARATE_KERNELS), dict(enclosing=L.LVR_ENCLOSE_AABB, n_subspaces=16)):
        with G.Index(cache.K, cache.V, "bf16", 8, **kw) as ix:
            with pytest.raises(L.LouverError) as e:
                G.subspace_thresholds(ix, q, np.zeros((1, 8), dtype=np.float32))
            assert e.value.code == L.LVR_E_UNSUPPORTED


def test_decode_step_under_graph_capture(G, oracle):
    """lvr_decode_step allocates nothing and never synchronises, so a caller can capture it in a HIP
    graph: every replay (with eager calls and synchronisations in between, fresh q and tau written
    into the captured buffers) must equal the eager call on the same inputs, and the oracle."""
    L = G.L
    cache = W.make_cache(2, n=8192 + 77, n_kv_heads=2)
    steps = 6
    qs = W.drift_queries(3, steps, n_q_heads=8)
    with G.Index(cache.K, cache.V, "bf16", 8) as ix:
        taus = [G.oracle_taus(oracle, ix, qs[t], frac=0.01) for t in range(steps)]
        q_in = torch.zeros((1, 8, 128), dtype=torch.float32, device="cuda")
        tau_in = torch.zeros((1, 8), dtype=torch.float32, device="cuda")
        out = torch.zeros((1, 8, 128), dtype=torch.float32, device="cuda")
        idx = torch.zeros((1, 8, 1024), dtype=torch.int32, device="cuda")
        cnt = torch.zeros((1, 8), dtype=torch.int32, device="cuda")
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):                      # one eager call on the capture stream first
            L.lvr_decode_step(ix.h, q_in, tau_in, out, idx, cnt, stream=side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            L.lvr_decode_step(ix.h, q_in, tau_in, out, idx, cnt, stream=torch.cuda.current_stream())
        for t in range(steps):
            # eager result on the same inputs
            i_e, c_e, o_e = ix.query(qs[t], taus[t], cap=1024, fused=True)
            q_in.copy_(torch.from_numpy(qs[t]))
            tau_in.copy_(torch.from_numpy(taus[t]))
            graph.replay()
            torch.cuda.synchronize()
            c_g, o_g, i_g = cnt.cpu().numpy(), out.cpu().numpy(), idx.cpu().numpy()
            assert np.array_equal(c_g, c_e), t
            for h in range(8):
                assert set(i_g[0, h, :c_g[0, h]].tolist()) == set(i_e[0, h, :c_e[0, h]].tolist()), (t, h)
            np.testing.assert_allclose(o_g, o_e, rtol=1e-5, atol=1e-6)
            G.check_step(oracle, ix, qs[t], taus[t], i_g, c_g, o_g, tag=f"graph replay {t}")
        del graph


# ---------------------------------------------------------------------------------------------
# Seeded random sequences of calls on one index
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("case", range(24))
def test_random_call_sequences(G, oracle, case):
    """A seeded random walk through the entry points on one index (appends of random length, the
    one-call append + step, explicit publishes, rebuilds, queries in both launch forms, Query 1 with the
    library's thresholds, dense attention, the reservoir): after every step the state and every result
    equal the oracle's on the keys held so far."""
    L = G.L
    g = np.random.default_rng(7000 + case)
    hkv, Gq = int(g.choice([1, 2])), int(g.choice([1, 4, 8]))
    hq = hkv * Gq
    r = int(g.choice([1, 4, 8]))
    S = int(g.choice([1, 4]))
    B = int(g.choice([16, 32, 64])) * (r if r > 4 else 1)
    grouping = int(g.choice([L.LVR_GROUP_CONTIGUOUS, L.LVR_GROUP_CONTIGUOUS, L.LVR_GROUP_TREE]))
    flags = int(g.choice([0, 0, L.LVR_CONCURRENT_UPDATE, L.LVR_SEPARATE_KERNELS]))
    idt = int(g.choice([L.LVR_INDEX_AUTO, L.LVR_INDEX_SAME]))
    R = int(g.choice([0, 64]))
    cap = 1500
    pool = W.make_local_cache(2, n=cap, n_kv_heads=hkv) if case % 2 else W.make_cache(2, n=cap, n_kv_heads=hkv)
    n0 = int(g.integers(0, 400))
    desc = f"sequence {case}: hq={hq} hkv={hkv} r={r} S={S} B={B} grouping={grouping} flags={flags} centres={idt} R={R} n0={n0}"
    G.say(desc)
    with G.Index(pool.K[:, :, :n0], pool.V[:, :, :n0], "bf16", hq, capacity=cap, group_size=r, n_subspaces=S,
                 buffer_size=B, grouping=grouping, flags=flags, index_dtype=idt, reservoir_size=R, seed=case) as ix:
        have = n0
        fused_ok = not (flags & L.LVR_SEPARATE_KERNELS)
        for step in range(14):
            op = g.choice(["append", "append", "append_step", "query", "query", "query1", "dense", "publish", "rebuild"])
            q = W.make_queries(2, n_q_heads=hq, step=100 * case + step)
            tag = f"{desc} step {step} {op} n={have}"
            if op == "append" and have < cap:
                m = int(min(g.choice([1, 1, 3, B - 1, B, 2 * B + 5]), cap - have))
                ix.append(pool.K[:, :, have:have + m], pool.V[:, :, have:have + m])
                have += m
            elif op == "append_step" and have < cap:
                m = int(min(g.choice([1, 1, 2, 70]), cap - have))
                kk, vv = pool.K[:, :, have:have + m], pool.V[:, :, have:have + m]
                ix.K = np.concatenate([ix.K, kk], axis=2)
                ix.V = np.concatenate([ix.V, vv], axis=2)
                have += m
                tau = G.oracle_taus(oracle, ix, q, frac=0.05)
                qd, td = torch.from_numpy(q).cuda(), torch.from_numpy(tau).cuda()
                out = torch.full((1, hq, 128), float("nan"), device="cuda")
                idx = torch.full((1, hq, cap), -7, dtype=torch.int32, device="cuda")
                cnt = torch.full((1, hq), -7, dtype=torch.int32, device="cuda")
                L.lvr_append_decode_step(ix.h, G.to_device(kk, "bf16"), G.to_device(vv, "bf16"), qd, td, out, idx, cnt)
                torch.cuda.synchronize()
                G.check_step(oracle, ix, q, tau, idx.cpu().numpy(), cnt.cpu().numpy(), out.cpu().numpy(), tag=tag)
            elif op == "query" and have > 0:
                tau = G.oracle_taus(oracle, ix, q, frac=float(g.choice([0.01, 0.2, 1.0])))
                idx, cnt, out = ix.query(q, tau, fused=bool(g.integers(0, 2)))
                G.check_step(oracle, ix, q, tau, idx, cnt, out, tag=tag)
            elif op == "query1" and have > 0 and fused_ok:
                tau = G.oracle_taus(oracle, ix, q, frac=0.03)
                idx, cnt, out = G.query1(ix, q, G.subspace_thresholds(ix, q, tau), tau)
                G.check_step(oracle, ix, q, tau, idx, cnt, out, tag=tag)
            elif op == "dense" and have > 0:
                ref = oracle.dense_attention(ix.K, ix.V, q, ix.sigma, hq)
                got = ix.dense(q)
                assert (np.abs(got - ref).max(axis=-1) / np.abs(ref).max(axis=-1)).max() <= G.ATTN_TOL, tag
            elif op == "publish":
                L.lvr_publish(ix.h)
                assert ix.stats(raise_on_overflow=False)["update_pending"] == 0, tag
            elif op == "rebuild":
                have = int(g.integers(0, 300))
                ix.K, ix.V = pool.K[:, :, :have].copy(), pool.V[:, :, :have].copy()
                L.lvr_build(ix.h, G.to_device(ix.K, "bf16"), G.to_device(ix.V, "bf16"))
            n, n_indexed = L.lvr_length(ix.h)
            assert n == have == ix.K.shape[2], tag
            assert n_indexed % r == 0 and 0 <= n - n_indexed < 2 * B + r, (tag, n, n_indexed)
            if R:
                _check_reservoir(oracle, ix, case, R)


@pytest.mark.parametrize("hq,hkv", [(8, 1), (16, 2), (4, 1), (4, 2), (1, 1)])
@pytest.mark.parametrize("kind", ["full", "mixed", "sixteen_bits"])
def test_queries_with_full_fp32_precision(G, oracle, hq, hkv, kind):
    """The scoring operand carries an fp32 query exactly (three bf16 terms; with more than four heads per
    KV head the third term travels in an operand of its own that is skipped when every term is zero).
    Queries with 24 significant bits, with 16, and a mix of exact-bf16 and full-precision heads must all
    give the oracle's sets and attention, in both enclosure formats."""
    L = G.L
    n = 3000 + 5
    cache = W.make_cache(2, n=n, n_kv_heads=hkv)
    g = np.random.default_rng(99 + hq)
    q = g.standard_normal((1, hq, 128)).astype(np.float32)                 # 24 significant bits
    if kind == "sixteen_bits":
        q = (q.view(np.uint32) & np.uint32(0xffffff00)).view(np.float32)   # hi + mid terms only
    elif kind == "mixed":
        q[:, ::2] = W.round_to_bf16(q[:, ::2])                             # every other head is bf16-exact
    for idt in (L.LVR_INDEX_AUTO, L.LVR_INDEX_SAME):
        for S in (4, 16):
            with G.Index(cache.K, cache.V, "bf16", hq, n_subspaces=S, index_dtype=idt, buffer_size=64) as ix:
                for frac in (0.01, 0.3):
                    tau = G.oracle_taus(oracle, ix, q, frac=frac)
                    idx, cnt, out = ix.query(q, tau, fused=True)
                    G.check_step(oracle, ix, q, tau, idx, cnt, out, tag=f"fp32 q {kind} hq={hq} S={S} centres={idt} frac={frac}")


@pytest.mark.parametrize("centres", ["same", "fp8"])
@pytest.mark.parametrize("S,keys,hq", [(1, "local", 4), (2, "local", 4), (4, "local", 4), (4, "workload", 4), (2, "workload", 8),
                                       (4, "local", 8), (4, "workload", 1)])
def test_query1_on_boxes(G, oracle, S, keys, hq, centres):
    """Query 1 with box enclosures: a group is a candidate for a head iff in every coordinate block the box
    bound of that block (upper corner against q+, lower corner against q-, plus the group's allowance times
    |q|) reaches the block's threshold.  The library's thresholds equal the oracle's on the exported boxes
    and give Problem 1's set; cutting thresholds keep every key the promise covers, and the number of
    candidate groups matches the oracle's Alg. 3 on the same bounds."""
    L = G.L
    n, r = 4096 + 37, 4
    cache = W.make_local_cache(2, n=n) if keys == "local" else W.make_cache(2, n=n)
    K, V = cache.K[:, :1], cache.V[:, :1]
    q = W.make_queries(2, n_q_heads=hq)
    G.say(f"query1 on boxes S={S} keys={keys} heads={hq} corners={centres}")
    idt = L.LVR_INDEX_FP8 if centres == "fp8" else L.LVR_INDEX_SAME
    with G.Index(K, V, "bf16", hq, group_size=r, n_subspaces=S, enclosing=L.LVR_ENCLOSE_AABB, index_dtype=idt) as ix:
        n_groups = n // r
        corners, allow, _, _ = ix.export()
        hi = W.bf16_bits_to_f32(corners[0, 0, :, 0]).reshape(-1, 128).astype(np.float64)
        lo = W.bf16_bits_to_f32(corners[0, 0, :, 1]).reshape(-1, 128).astype(np.float64)
        ds = 128 // S
        f = np.empty((hq, S, n_groups))
        for h in range(hq):
            qn = np.linalg.norm(q[0, h].astype(np.float64))
            for s_ in range(S):
                qm = np.zeros(128, dtype=np.float32)
                qm[s_ * ds:(s_ + 1) * ds] = q[0, h, s_ * ds:(s_ + 1) * ds]
                f[h, s_] = oracle.aabb_bounds(qm, lo, hi) + allow[0, 0, :, 0].astype(np.float64) * qn
        label = np.tile(np.arange(n_groups * r, dtype=np.int32) // r, (S, 1))
        Kd = K[0, 0].astype(np.float64)
        tau = G.oracle_taus(oracle, ix, q, frac=0.02)
        lib_tau_s = G.subspace_thresholds(ix, q, tau)
        for h in range(hq):
            want = oracle.safe_subspace_thresholds(f[h], float(tau[0, h]))
            scale = abs(float(tau[0, h])) + np.abs(f[h]).max(axis=1).sum()
            assert np.all(np.abs(lib_tau_s[0, h] - want) <= 2e-5 * scale), (h, lib_tau_s[0, h], want)
        idx, cnt, out = G.query1(ix, q, lib_tau_s, tau)
        G.check_step(oracle, ix, q, tau, idx, cnt, out, tag=f"query1 boxes, library thresholds S={S}")
        tau_s = np.empty((1, hq, S), dtype=np.float32)
        for quant in (0.5, 0.9):
            for h in range(hq):
                tau_s[0, h] = np.quantile(f[h], quant, axis=1).astype(np.float32)
            idx, cnt, out = G.query1(ix, q, tau_s, tau)
            st = ix.stats()
            alive_lo = np.zeros(n_groups, dtype=bool)
            alive_hi = np.zeros(n_groups, dtype=bool)
            for h in range(hq):
                s_f32 = oracle.scores_f32(q[0, h], K[0, 0])
                te = tau_s[0, h].astype(np.float64)
                te = te - 0.5e-4 * np.abs(te)
                slack = 1e-5 * np.abs(te) + 1e-5 * np.abs(f[h]).max(axis=1) + 2e-3
                strict = oracle.query1_filter(f[h], label, te + slack)
                loose = oracle.query1_filter(f[h], label, te - slack)
                alive_lo |= strict.reshape(n_groups, r)[:, 0]
                alive_hi |= loose.reshape(n_groups, r)[:, 0]
                got = np.zeros(n, dtype=bool)
                got[idx[0, h, :cnt[0, h]]] = True
                assert cnt[0, h] == got.sum()
                band = 1e-4 * abs(float(tau[0, h]))
                tail = np.arange(n) >= n_groups * r
                must = (s_f32 >= tau[0, h]) & (np.concatenate([strict, np.ones(n - n_groups * r, bool)]) | tail)
                assert not (must & ~got).any(), (S, quant, h)
                assert not (got & (s_f32 < tau[0, h] - band)).any()
                blocks = (Kd * q[0, h].astype(np.float64)).reshape(n, S, ds).sum(-1)
                relevant = (s_f32 >= tau[0, h]) & (blocks >= tau_s[0, h][None, :] + 1e-3).all(1)
                assert not (relevant & ~got).any()
            assert alive_lo.sum() <= st["groups_surviving"] <= alive_hi.sum(), (S, quant, alive_lo.sum(), st["groups_surviving"], alive_hi.sum())
            assert st["groups_surviving"] < st["groups_scored"]


def test_create_destroy_returns_all_memory(G):
    """Device memory in use goes back to where it was after indices of every flavour have been created,
    used and destroyed (arena, index, work space, position maps, reservoir, side stream and events,
    profiling events)."""
    L = G.L
    cache = W.make_cache(2, n=2048, n_kv_heads=2)
    q = W.make_queries(2, n_q_heads=8)
    tau = np.zeros((1, 8), dtype=np.float32)
    flavours = [dict(), dict(grouping=L.LVR_GROUP_TREE), dict(enclosing=L.LVR_ENCLOSE_AABB), dict(reservoir_size=256),
                dict(flags=L.LVR_CONCURRENT_UPDATE, buffer_size=32), dict(flags=L.LVR_SEPARATE_KERNELS),
                dict(flags=L.LVR_KV_IN_HOST_MEMORY), dict(index_dtype=L.LVR_INDEX_SAME, n_subspaces=16)]

    def cycle():
        for kw in flavours:
            with G.Index(cache.K[:, :, :2000], cache.V[:, :, :2000], "bf16", 8, capacity=2048, **kw) as ix:
                L.lvr_profile_enable(ix.h, 16)
                ix.append(cache.K[:, :, 2000:2040], cache.V[:, :, 2000:2040])
                ix.query(q, tau, fused=True)
                L.lvr_profile_read(ix.h)
    cycle()                                   # first use: the runtime's own pools reach their size
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    free0, _ = torch.cuda.mem_get_info()
    for _ in range(5):
        cycle()
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    free1, _ = torch.cuda.mem_get_info()
    assert free0 - free1 < 8 << 20, (free0, free1)


def test_create_beyond_device_memory_fails_cleanly(G):
    """An arena that cannot fit (about a terabyte here) comes back as LVR_E_NOMEM with nothing
    left allocated, and the library keeps working."""
    L = G.L
    torch.cuda.synchronize()
    free0, total = torch.cuda.mem_get_info()
    cfg = L.make_config(batch=8, n_q_heads=32, n_kv_heads=8, capacity=1 << 26)     # 2 * 64 * 2^26 * 256 B = 2 TiB
    assert L.lvr_arena_bytes(cfg) > total
    h = C.c_void_p()
    rc = L.lib().lvr_create(C.byref(cfg), C.byref(h))
    assert rc == L.LVR_E_NOMEM and not h.value, rc
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert free0 - free1 < 8 << 20
    cache = W.make_cache(2, n=256, n_kv_heads=2)
    with G.Index(cache.K, cache.V, "bf16", 8) as ix:
        idx, cnt, _ = ix.query(W.make_queries(2, n_q_heads=8), np.full((1, 8), -np.inf, dtype=np.float32))
        assert (cnt == 256).all()


# ------------------------------------------------------------------ one grouping per subspace (Alg. 1 as printed)
def _subspace_index_from_export(G, ix, S):
    """Exported index of a LVR_GROUP_SUBSPACE_TREE index -> (labels [b][h][S][ni], centres fp32, radii)."""
    import paper_2605_06763_amd as L
    labels = L.lvr_export_labels(ix.h, ix.cfg)
    centres, radii, slot_pos, keys = ix.export()
    return labels, W.bf16_bits_to_f32(centres).reshape(centres.shape), radii


@pytest.mark.parametrize("n,r,S", [(1024, 4, 4), (2048, 4, 16), (512, 2, 8), (256, 8, 1), (1024, 1, 2)])
def test_subspace_tree_index_equals_oracle(G, oracle, n, r, S):
    """n = r * 2^k: in every subspace the labels are the oracle's Alg. 2 leaves on that subspace's
    coordinates; the stored centre is the members' mean rounded to bf16; the stored radius encloses
    the members (measured against the centre as stored) and is not loose."""
    import paper_2605_06763_amd as L
    cache = _small_cache(2, n)
    ds = 128 // S
    with G.Index(cache.K, cache.V, "bf16", 8, group_size=r, n_subspaces=S, grouping=L.LVR_GROUP_SUBSPACE_TREE) as ix:
        labels, centres, radii = _subspace_index_from_export(G, ix, S)
        ng = n // r
        assert labels.shape == (1, 2, S, n)
        for h in range(2):
            K = cache.K[0, h]
            for s in range(S):
                lab, order, leaves = oracle.balanced_tree(K, r, s * ds, (s + 1) * ds)
                assert leaves == ng
                assert np.array_equal(labels[0, h, s], lab), (h, s, np.nonzero(labels[0, h, s] != lab)[0][:8])
                c64, r64 = oracle.ball_index(K, lab, ng, S)
                want_c = W.round_to_bf16(c64[:, s * ds:(s + 1) * ds].astype(np.float32))
                got_c = centres[0, h, :, s * ds:(s + 1) * ds]
                # the mean is summed in fp32 on the GPU: at most one bf16 step from the rounded fp64 mean
                assert np.all(np.abs(got_c - want_c) <= np.abs(want_c) * 2.0 ** -7 + 1e-30), (h, s)
                full = np.zeros((ng, 128))
                full[:, s * ds:(s + 1) * ds] = got_c
                need = oracle.ball_radii_for_centres(K, lab, full, S)[:, s]
                got_r = radii[0, h, :, s].astype(np.float64)
                assert np.all(got_r >= need), (h, s, float((need - got_r).max()))
                cn = np.linalg.norm(got_c.astype(np.float64), axis=1)
                assert np.all(got_r <= need * (1 + 2.0 ** -11) + cn * 2.0 ** -11 + 1e-30), (h, s)


@pytest.mark.parametrize("n,r,S,hq", [(1024, 4, 4, 8), (2048, 4, 16, 8), (1500, 4, 8, 4), (777, 8, 2, 2), (64, 4, 16, 8),
                                      (5, 4, 4, 8), (3, 4, 4, 8), (4096, 2, 16, 8), (1000, 1, 4, 8)])
def test_subspace_tree_queries(G, oracle, n, r, S, hq):
    """Sets and attention equal the oracle's for ragged and tiny sizes; the candidates are what the
    summed bounds of the exported index allow (within rounding), they contain Problem 1's set and
    lie inside the live set of the oracle's depth scan (Alg. 4) on the same index."""
    import paper_2605_06763_amd as L
    cache = _small_cache(2, n)
    q = W.make_queries(2, n_q_heads=hq)
    ds = 128 // S
    Gh = hq // 2
    with G.Index(cache.K, cache.V, "bf16", hq, group_size=r, n_subspaces=S, grouping=L.LVR_GROUP_SUBSPACE_TREE) as ix:
        ni = L.lvr_length(ix.h)[1]
        assert ni == n // r * r
        labels, centres, radii = (None, None, None) if ni == 0 else _subspace_index_from_export(G, ix, S)
        for frac in (0.01, 0.3):
            tau = G.oracle_taus(oracle, ix, q, frac=frac)
            for fused in (False, True):
                idx, cnt, out = ix.query(q, tau, fused=fused)
                G.check_step(oracle, ix, q, tau, idx, cnt, out, tag=f"subspace n={n} r={r} S={S} frac={frac}")
            st = ix.stats()
            assert st["n_indexed"] == ni and st["groups_scored"] == 2 * (ni // r)
            if ni == 0:
                continue
            lo = hi = 0
            for h in range(2):
                K = cache.K[0, h][:ni]
                alive_lo = np.zeros(ni, dtype=bool)
                alive_hi = np.zeros(ni, dtype=bool)
                for hh in range(Gh):
                    qh, t = q[0, h * Gh + hh], float(tau[0, h * Gh + hh])
                    f = oracle.ball_bounds(qh, centres[0, h].astype(np.float64), radii[0, h].astype(np.float64))
                    ub = sum(f[s][labels[0, h, s]] for s in range(S))
                    sc = oracle.scores_f64(qh, K)
                    assert np.all(ub >= sc), "a summed bound below a member's score"
                    te = t - 0.5e-4 * abs(t)
                    alive_lo |= ub >= te * (1 + 1e-5) + 1e-3
                    alive_hi |= ub >= te * (1 - 1e-5) - 1e-3
                    ta_alive, depth = oracle.ta_filter(f, labels[0, h], te * (1 - 1e-5) - 1e-3)
                    assert not np.any((ub >= te * (1 - 1e-5) - 1e-3) & ~ta_alive), "sum rule outside the depth scan's live set"
                lo += int(alive_lo.sum())
                hi += int(alive_hi.sum())
            assert lo <= st["groups_surviving"] <= hi, (frac, lo, st["groups_surviving"], hi)
            assert st["keys_scanned"] == st["groups_surviving"] + 2 * (n - ni)
            G.say(f"  subspace layout n={n} r={r} S={S} frac={frac}: {st['groups_surviving']} of {2 * ni} keys are candidates")


def test_subspace_tree_prunes_where_one_shared_grouping_cannot(G, oracle):
    """Independent structure per coordinate block: block s of key j is u_{s,j} * a_s, a point on a line
    of the block, with the positions u on the 16 lines independent of each other.  One grouping shared by
    all blocks can sort by a few of the lines at best, so its balls stay wide in most blocks; a grouping
    per block sorts every line and gets tight balls everywhere."""
    import paper_2605_06763_amd as L
    g = np.random.default_rng(33)
    n, S, r, hq = 8192, 16, 4, 8
    ds = 128 // S
    K = np.zeros((1, 2, n, 128), dtype=np.float32)
    for h in range(2):
        for s in range(S):
            a = g.standard_normal(ds).astype(np.float32)
            u = g.uniform(-3.0, 3.0, size=n).astype(np.float32)
            K[0, h, :, s * ds:(s + 1) * ds] = u[:, None] * a[None, :]
    K = W.round_to_bf16(K)
    V = W.round_to_bf16(g.standard_normal((1, 2, n, 128)).astype(np.float32))
    q = W.make_queries(2, n_q_heads=hq)
    frac = {}
    for name, grouping in (("per-subspace", L.LVR_GROUP_SUBSPACE_TREE), ("shared tree", L.LVR_GROUP_TREE)):
        with G.Index(K, V, "bf16", hq, group_size=r, n_subspaces=S, grouping=grouping,
                     index_dtype=L.LVR_INDEX_SAME) as ix:
            tau = G.oracle_taus(oracle, ix, q, frac=0.01)
            idx, cnt, out = ix.query(q, tau, fused=True)
            G.check_step(oracle, ix, q, tau, idx, cnt, out, tag=name)
            st = ix.stats()
            frac[name] = st["keys_scanned"] / (2 * n)
            G.say(f"  {name}: {st['keys_scanned']} of {2 * n} keys scanned")
    assert frac["per-subspace"] < 0.2 and frac["shared tree"] > 0.9, frac


@pytest.mark.parametrize("flags", [0, 1])
def test_subspace_tree_append(G, oracle, flags):
    """Appends across several buffer flushes (B = 32): every chunk is grouped block by block; results
    equal the oracle's after every step, through both the two-call and the one-call append."""
    import paper_2605_06763_amd as L
    n0, steps, B = 203, 75, 32
    cache = _small_cache(5, n0)
    k_new, v_new = W.make_append_stream(5, steps, cache)
    qs = W.drift_queries(5, steps, n_q_heads=8)
    with G.Index(cache.K, cache.V, "bf16", 8, capacity=n0 + steps, buffer_size=B, flags=flags, n_subspaces=8,
                 grouping=L.LVR_GROUP_SUBSPACE_TREE) as ix:
        for t in range(steps):
            if t % 3 == 2:      # append + query + attention in one call
                kd, vd = G.to_device(k_new[t][:, :, None, :], "bf16"), G.to_device(v_new[t][:, :, None, :], "bf16")
                ix.K = np.concatenate([ix.K, k_new[t][:, :, None, :]], axis=2)
                ix.V = np.concatenate([ix.V, v_new[t][:, :, None, :]], axis=2)
                n_indexed_before = L.lvr_length(ix.h)[1]
                tau = G.oracle_taus(oracle, ix, qs[t], frac=0.05)
                qd, td = torch.from_numpy(qs[t]).cuda(), torch.from_numpy(tau).cuda()
                idx = torch.full((1, 8, ix.n), -7, dtype=torch.int32, device="cuda")
                cnt = torch.full((1, 8), -7, dtype=torch.int32, device="cuda")
                out = torch.full((1, 8, 128), float("nan"), dtype=torch.float32, device="cuda")
                L.lvr_append_decode_step(ix.h, kd, vd, qd, td, out, idx, cnt)
                torch.cuda.synchronize()
                n, n_indexed = L.lvr_length(ix.h)
                G.check_step(oracle, ix, qs[t], tau, idx.cpu().numpy(), cnt.cpu().numpy(), out.cpu().numpy(),
                             tag=f"subspace append (one call) t={t}", extra_from=(n_indexed if flags & 1 else -1))
                continue
            ix.append(k_new[t][:, :, None, :], v_new[t][:, :, None, :])
            n, n_indexed = L.lvr_length(ix.h)
            assert n == n0 + t + 1 and n_indexed % 4 == 0 and 0 <= n - n_indexed < B + 4
            if t % 7 == 0 or t == steps - 1:
                tau = G.oracle_taus(oracle, ix, qs[t], frac=0.05)
                idx, cnt, out = ix.query(qs[t], tau, fused=(t % 2 == 0))
                G.check_step(oracle, ix, qs[t], tau, idx, cnt, out, tag=f"subspace append t={t}",
                             extra_from=(n_indexed if flags & 1 else -1))
        # the labels of appended chunks name groups of their own chunk
        labels = L.lvr_export_labels(ix.h, ix.cfg)
        n, n_indexed = L.lvr_length(ix.h)
        first = n0 // 4 * 4
        for c0 in range(first, n_indexed, B):
            lab = labels[0, :, :, c0:c0 + B]
            assert lab.min() == c0 // 4 and lab.max() == (c0 + B) // 4 - 1
            for h in range(2):
                for s in range(8):
                    assert np.all(np.bincount(lab[h, s] - c0 // 4, minlength=B // 4) == 4)


def test_subspace_tree_unsupported_combinations(G):
    import paper_2605_06763_amd as L
    base = dict(batch=1, n_q_heads=8, n_kv_heads=2, capacity=1024, grouping=L.LVR_GROUP_SUBSPACE_TREE)
    for bad in (dict(kv_dtype=L.LVR_F32), dict(enclosing=L.LVR_ENCLOSE_AABB), dict(n_q_heads=16),
                dict(flags=L.LVR_SEPARATE_KERNELS), dict(flags=L.LVR_CONCURRENT_UPDATE), dict(flags=L.LVR_KV_IN_HOST_MEMORY),
                dict(index_dtype=L.LVR_INDEX_FP8), dict(capacity=1 << 20, group_size=4)):
        with pytest.raises(L.LouverError) as e:
            L.lvr_create(L.make_config(**{**base, **bad}))
        assert e.value.code == L.LVR_E_UNSUPPORTED, bad
    h = L.lvr_create(L.make_config(**base))
    try:
        K = torch.zeros((1, 2, 64, 128), dtype=torch.bfloat16, device="cuda")
        L.lvr_build(h, K, K)
        with pytest.raises(L.LouverError) as e:
            L.lvr_set_bound_test(h, False)
        assert e.value.code == L.LVR_E_UNSUPPORTED
        q = torch.zeros((1, 8, 128), device="cuda")
        tau = torch.zeros((1, 8), device="cuda")
        ts = torch.zeros((1, 8, 4), device="cuda")
        idx = torch.zeros((1, 8, 64), dtype=torch.int32, device="cuda")
        cnt = torch.zeros((1, 8), dtype=torch.int32, device="cuda")
        with pytest.raises(L.LouverError) as e:
            L.lvr_query1(h, q, ts, tau, idx, cnt)
        assert e.value.code == L.LVR_E_UNSUPPORTED
        with pytest.raises(L.LouverError) as e:
            L.lvr_subspace_thresholds(h, q, tau, ts)
        assert e.value.code == L.LVR_E_UNSUPPORTED
    finally:
        L.lvr_destroy(h)
