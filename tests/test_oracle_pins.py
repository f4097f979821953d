"""Pins for the CPU oracle: every function is checked against something other than itself —
closed forms, exact integer brute force, library routines, printed table values, invariants.
Each pin names the mistake it would catch.  CPU only."""
import itertools
import math
import os

import numpy as np
import pytest
import torch

import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _int_case(seed, n, d, lo=-3, hi=4):
    g = np.random.default_rng(seed)
    K = g.integers(lo, hi, size=(n, d)).astype(np.float32)
    q = g.integers(lo, hi, size=d).astype(np.float32)
    return q, K


# ------------------------------------------------------------------ scores and the range set
def test_scores_exact_integer_bruteforce(oracle):
    """Small integer vectors: Python integer arithmetic gives the exact dot product, both
    score routines must reproduce it exactly (catches wrong index, transposed K, dropped term)."""
    for seed in range(20):
        q, K = _int_case(seed, n=13, d=5)
        exact = [sum(int(q[c]) * int(K[j, c]) for c in range(5)) for j in range(13)]
        assert oracle.scores_f64(q, K).tolist() == exact
        assert oracle.scores_f32(q, K).tolist() == exact


def test_scores_unit_vectors(oracle):
    """Keys that are scaled basis vectors: the score is a single product q_c * a."""
    d = 7
    q = np.arange(1, d + 1, dtype=np.float32) * 0.5
    K = np.zeros((d, d), dtype=np.float32)
    for c in range(d):
        K[c, c] = c - 3.0
    assert np.array_equal(oracle.scores_f32(q, K), q * (np.arange(d) - 3.0))


def test_scores_match_library_matmul(oracle):
    g = np.random.default_rng(1)
    K = g.standard_normal((300, 128)).astype(np.float32)
    q = g.standard_normal(128).astype(np.float32)
    lib = K.astype(np.float64) @ q.astype(np.float64)
    assert np.allclose(oracle.scores_f64(q, K), lib, rtol=0, atol=1e-12 * np.abs(lib).max() + 1e-12)
    # fp32 sequential sum stays within the classical bound d * eps * sum |terms|
    terms = np.abs(K.astype(np.float64) * q.astype(np.float64)).sum(axis=1)
    assert np.all(np.abs(oracle.scores_f32(q, K) - lib) <= 128 * 2.0 ** -24 * terms)


def test_scores_f32_is_sequential_unfused(oracle):
    """(1 + 2^-24) + (-1): a fused or reordered sum gives a different answer from one fp32
    accumulator taken left to right (catches -ffast-math style reassociation and FMA)."""
    q = np.array([1.0, 1.0, 1.0], dtype=np.float32)
    K = np.array([[1.0, 2.0 ** -24, -1.0]], dtype=np.float32)
    assert oracle.scores_f32(q, K)[0] == 0.0          # 1 + 2^-24 rounds to 1 (ties to even)
    assert oracle.scores_f64(q, K)[0] == 2.0 ** -24
    # product rounding: (1+2^-12)^2 = 1 + 2^-11 + 2^-24 rounds to 1 + 2^-11 before the add
    # and -1 + that product: rounding the product first loses the 2^-24 a fused multiply-add
    # (or a wider product) would keep
    a = np.float32(1.0 + 2.0 ** -12)
    q = np.array([1.0, a], dtype=np.float32)
    K = np.array([[-1.0, a]], dtype=np.float32)
    assert oracle.scores_f32(q, K)[0] == 2.0 ** -11
    assert oracle.scores_f64(q, K)[0] == 2.0 ** -11 + 2.0 ** -24


def test_bf16_storage_is_widened_exactly(oracle):
    g = np.random.default_rng(2)
    K = W.round_to_bf16(g.standard_normal((50, 16)).astype(np.float32))
    q = g.standard_normal(16).astype(np.float32)
    bits = W.f32_to_bf16_bits(K).reshape(K.shape)
    assert np.array_equal(oracle.scores_f32(q, bits), oracle.scores_f32(q, K))
    assert np.array_equal(oracle.scores_f64(q, bits), oracle.scores_f64(q, K))


def test_range_set_exhaustive_tiny(oracle):
    """All thresholds between and at the score values of tiny integer cases: the set is
    exactly the positions whose exact integer score is >= tau; a tie at tau is included
    (catches > instead of >=, wrong sign, off-by-one in the compaction)."""
    for seed in range(10):
        q, K = _int_case(100 + seed, n=9, d=3)
        exact = [sum(int(q[c]) * int(K[j, c]) for c in range(3)) for j in range(9)]
        for tau in sorted(set(exact)) + [min(exact) - 1, max(exact) + 1] + [e + 0.5 for e in exact]:
            want = [j for j in range(9) if exact[j] >= tau]
            assert oracle.range_query(q, K, tau).tolist() == want


def test_range_set_count_identity_and_monotone(oracle):
    g = np.random.default_rng(3)
    K = g.standard_normal((2000, 128)).astype(np.float32)
    q = g.standard_normal(128).astype(np.float32)
    s = oracle.scores_f32(q, K)
    prev = None
    for k in (0, 1, 7, 40, 500, 2000):
        tau = W.tau_for_count(s, k)
        got = oracle.range_query(q, K, tau)
        assert got.size == k                      # midpoint threshold -> exactly k keys
        assert np.all(np.diff(got) > 0)           # ascending positions
        if prev is not None:
            assert set(prev.tolist()) <= set(got.tolist())   # lowering tau only adds keys
        prev = got
    assert oracle.range_query(q, K, -np.inf).size == 2000
    assert oracle.range_query(q, K, np.inf).size == 0


def test_planted_keys_are_retrieved(oracle):
    """Config-1 recipe: keys rescaled to score tau + delta are in the set by construction."""
    cache = W.make_cache(1)
    K = cache.K[0, 0]
    q = W.make_queries(1)[0, 0]
    s = oracle.scores_f32(q, K)
    tau = float(W.tau_for_fraction(s, 0.02))
    rows = W.planted_positions(1, K.shape[0], 8)
    W.plant_rows(K, rows, (tau + 0.5) / s[rows], "f32")
    got = set(oracle.range_query(q, K, tau).tolist())
    assert set(rows.tolist()) <= got


# ------------------------------------------------------------------ attention on a set
def _sdpa(q, K, V, sigma):
    qt = torch.tensor(q, dtype=torch.float64)[None, None, None, :]
    Kt = torch.tensor(K, dtype=torch.float64)[None, None]
    Vt = torch.tensor(V, dtype=torch.float64)[None, None]
    return torch.nn.functional.scaled_dot_product_attention(qt, Kt, Vt, scale=sigma)[0, 0, 0].numpy()


def test_attention_full_set_equals_library_sdpa(oracle):
    """tau = -inf retrieves everything, and attention on everything is textbook attention:
    compare with torch's scaled_dot_product_attention in fp64, at the default and at a
    non-default scale (catches K/V swapped, missing scale, wrong normaliser)."""
    g = np.random.default_rng(4)
    K = g.standard_normal((257, 128)).astype(np.float32)
    V = g.standard_normal((257, 128)).astype(np.float32)
    q = g.standard_normal(128).astype(np.float32)
    idx = oracle.range_query(q, K, -np.inf)
    assert idx.tolist() == list(range(257))
    for sigma in (1.0 / math.sqrt(128), 0.37):
        got = oracle.attention_on_list(q, K, V, idx, sigma)
        assert np.allclose(got, _sdpa(q, K, V, sigma), rtol=2e-6, atol=1e-7)


def test_attention_subset_equals_sdpa_on_subset(oracle):
    g = np.random.default_rng(5)
    K = g.standard_normal((100, 32)).astype(np.float32)
    V = g.standard_normal((100, 32)).astype(np.float32)
    q = g.standard_normal(32).astype(np.float32)
    idx = np.array([3, 17, 18, 64, 99], dtype=np.int32)
    got = oracle.attention_on_list(q, K, V, idx, 0.2)
    assert np.allclose(got, _sdpa(q, K[idx], V[idx], 0.2), rtol=2e-6, atol=1e-7)
    # order of the list is irrelevant
    perm = idx[[4, 0, 3, 1, 2]]
    assert np.allclose(oracle.attention_on_list(q, K, V, perm, 0.2), got, rtol=1e-6, atol=1e-7)


def test_attention_closed_forms(oracle):
    g = np.random.default_rng(6)
    K = g.standard_normal((10, 8)).astype(np.float32)
    V = g.standard_normal((10, 8)).astype(np.float32)
    q = g.standard_normal(8).astype(np.float32)
    # one key: the output is its value row
    assert np.array_equal(oracle.attention_on_list(q, K, V, [4], 0.3), V[4])
    # two keys: logistic mix of the two value rows
    s = K.astype(np.float64) @ q.astype(np.float64)
    w = 1.0 / (1.0 + math.exp(-0.3 * (s[2] - s[7])))
    want = w * V[2].astype(np.float64) + (1 - w) * V[7].astype(np.float64)
    assert np.allclose(oracle.attention_on_list(q, K, V, [2, 7], 0.3), want, rtol=1e-6, atol=1e-7)
    # zero query: uniform weights -> plain mean of the selected value rows
    z = np.zeros(8, dtype=np.float32)
    assert np.allclose(oracle.attention_on_list(z, K, V, [1, 2, 3, 9], 0.3), V[[1, 2, 3, 9]].mean(0),
                       rtol=1e-6, atol=1e-7)
    # empty set: zeros
    assert np.array_equal(oracle.attention_on_list(q, K, V, [], 0.3), np.zeros(8, np.float32))
    # huge logits do not overflow (max subtraction)
    big = (K * 1000).astype(np.float32)
    out = oracle.attention_on_list(q * 10, big, V, list(range(10)), 1.0)
    assert np.all(np.isfinite(out))
    assert np.allclose(out, V[int(np.argmax(big.astype(np.float64) @ (q * 10).astype(np.float64)))], atol=1e-6)


def test_decode_step_layout_and_gqa_mapping(oracle):
    """Batched entry point against per-head calls, and the head map h_kv = h_q // G pinned by
    value rows that name their own KV head."""
    g = np.random.default_rng(7)
    batch, hq, hkv, n, d = 2, 6, 3, 40, 16
    K = g.standard_normal((batch, hkv, n, d)).astype(np.float32)
    V = np.zeros((batch, hkv, n, d), dtype=np.float32)
    for b in range(batch):
        for h in range(hkv):
            V[b, h] = 10 * b + h          # every value row of KV head (b,h) is the constant 10b+h
    q = g.standard_normal((batch, hq, d)).astype(np.float32)
    tau = np.full((batch, hq), -np.inf, dtype=np.float32)
    sets, count, out = oracle.decode_step(K, V, q, tau, 0.25, hq)
    for b in range(batch):
        for h in range(hq):
            assert np.allclose(out[b, h], 10 * b + h // 2)
            assert count[b, h] == n
    V = g.standard_normal((batch, hkv, n, d)).astype(np.float32)
    s_all = np.einsum("bhnd,bhgd->bhgn", K.astype(np.float64), q.reshape(batch, hkv, 2, d).astype(np.float64))
    tau = W.tau_for_count(s_all.reshape(batch, hq, n), 5)
    sets, count, out = oracle.decode_step(K, V, q, tau, 0.25, hq)
    for b in range(batch):
        for h in range(hq):
            want = oracle.range_query(q[b, h], K[b, h // 2], tau[b, h])
            assert sets[b][h].tolist() == want.tolist() and count[b, h] == 5
            assert np.array_equal(out[b, h], oracle.attention_on_list(q[b, h], K[b, h // 2], V[b, h // 2], want, 0.25))
    # recent-keys-always-attended variant: positions >= extra_from join the set
    sets2, count2, _ = oracle.decode_step(K, V, q, tau, 0.25, hq, extra_from=n - 3)
    for b in range(batch):
        for h in range(hq):
            assert set(sets2[b][h].tolist()) == set(sets[b][h].tolist()) | {n - 3, n - 2, n - 1}
    # dense entry point = everything retrieved
    dense = oracle.dense_attention(K, V, q, 0.25, hq)
    for b in range(batch):
        for h in range(hq):
            assert np.allclose(dense[b, h], _sdpa(q[b, h], K[b, h // 2], V[b, h // 2], 0.25), rtol=2e-6, atol=1e-7)


# ------------------------------------------------------------------ ball index and bound
def test_subspace_blocks_partition_coordinates(oracle):
    for d, S in [(128, 4), (128, 16), (10, 3), (7, 7), (5, 1)]:
        blocks = [oracle.subspace_range(d, S, s) for s in range(S)]
        assert blocks[0][0] == 0 and blocks[-1][1] == d
        assert all(blocks[i][1] == blocks[i + 1][0] for i in range(S - 1))
        widths = [hi - lo for lo, hi in blocks]
        assert set(widths) <= {d // S, -(-d // S)}


def test_ball_index_closed_forms(oracle):
    """Two-point group: centre = midpoint, radius = half the distance (per subspace).
    One-point group: radius 0.  Catches dividing by r instead of the member count and a
    radius taken over the wrong coordinates."""
    K = np.array([[0, 0, 0, 0], [6, 8, 2, 0], [1, 1, 1, 1]], dtype=np.float32)
    label = np.array([0, 0, 1], dtype=np.int32)
    centre, radius = oracle.ball_index(K, label, 2, S=2)
    assert np.array_equal(centre, [[3, 4, 1, 0], [1, 1, 1, 1]])
    assert np.allclose(radius, [[5.0, 1.0], [0.0, 0.0]])
    centre, radius = oracle.ball_index(K, label, 2, S=1)
    assert np.allclose(radius, [[math.sqrt(26.0)], [0.0]])


def test_ball_enclosure_and_bound_dominate_members(oracle):
    """Eq. (1) enclosure and the upper-bound chain: every member lies in its ball in every
    subspace; each f_{s,a(j)} >= the member's subspace dot product; their sum >= <q,k_j>."""
    g = np.random.default_rng(8)
    n, d, S, r = 96, 16, 4, 4
    K = g.standard_normal((n, d)).astype(np.float32) * g.uniform(0.2, 5, size=d).astype(np.float32)
    label = (g.permutation(n) // r).astype(np.int32)
    centre, radius = oracle.ball_index(K, label, n // r, S)
    for _ in range(5):
        q = g.standard_normal(d).astype(np.float32)
        f = oracle.ball_bounds(q, centre, radius)
        tot = np.zeros(n)
        for s in range(S):
            lo, hi = oracle.subspace_range(d, S, s)
            part = K[:, lo:hi].astype(np.float64) @ q[lo:hi].astype(np.float64)
            dist = np.linalg.norm(K[:, lo:hi] - centre[label, lo:hi], axis=1)
            assert np.all(dist <= radius[label, s] * (1 + 1e-12))
            assert np.all(f[s, label] >= part - 1e-9)
            tot += f[s, label]
        assert np.all(tot >= oracle.scores_f64(q, K) - 1e-9)
    # the radius is attained by some member (it is a max, not a looser bound)
    for s in range(S):
        lo, hi = oracle.subspace_range(d, S, s)
        dist = np.linalg.norm(K[:, lo:hi].astype(np.float64) - centre[label, lo:hi], axis=1)
        for gi in range(n // r):
            assert math.isclose(dist[label == gi].max(), radius[gi, s], rel_tol=1e-12)


def test_ball_bound_is_the_maximum_over_the_ball(oracle):
    """Eq. (2) against brute force: f equals <q, x*> at the maximiser x* = c + rho q/|q| and no
    point sampled on or inside the ball exceeds it (catches minus instead of plus, a missing
    norm, a norm over the full space instead of the subspace)."""
    g = np.random.default_rng(9)
    d = 6
    centre = g.standard_normal((3, d))
    radius = g.uniform(0.1, 2.0, size=(3, 1))
    q = g.standard_normal(d).astype(np.float32)
    f = oracle.ball_bounds(q, centre, radius)[0]
    qd = q.astype(np.float64)
    for i in range(3):
        xstar = centre[i] + radius[i, 0] * qd / np.linalg.norm(qd)
        assert math.isclose(f[i], float(qd @ xstar), rel_tol=1e-12)
        u = g.standard_normal((20000, d))
        u /= np.linalg.norm(u, axis=1, keepdims=True)
        pts = centre[i] + radius[i, 0] * u * g.uniform(0, 1, size=(20000, 1)) ** (1 / d)
        assert np.all(pts @ qd <= f[i] + 1e-12)
        assert (centre[i] + radius[i, 0] * u).dot(qd).max() > f[i] - 0.25 * radius[i, 0] * np.linalg.norm(qd)
    # two subspaces: each bound uses its own coordinate block and its own |pi_s q|
    radius2 = g.uniform(0.1, 2.0, size=(3, 2))
    f2 = oracle.ball_bounds(q, centre, radius2)
    for s, (lo, hi) in enumerate([(0, 3), (3, 6)]):
        want = centre[:, lo:hi] @ qd[lo:hi] + radius2[:, s] * np.linalg.norm(qd[lo:hi])
        assert np.allclose(f2[s], want, rtol=1e-12)


def test_group_of_one_bound_is_exact_score(oracle):
    g = np.random.default_rng(10)
    K = g.standard_normal((30, 12)).astype(np.float32)
    q = g.standard_normal(12).astype(np.float32)
    centre, radius = oracle.ball_index(K, np.arange(30, dtype=np.int32), 30, S=3)
    assert np.all(radius == 0)
    assert np.allclose(oracle.ball_bounds(q, centre, radius).sum(0), oracle.scores_f64(q, K), rtol=1e-12, atol=1e-12)


def test_radii_for_stored_centres(oracle):
    """Moving a centre off the mean must grow the radius by what the enclosure needs."""
    K = np.array([[0.0, 0.0], [2.0, 0.0]], dtype=np.float32)
    label = np.zeros(2, dtype=np.int32)
    assert np.allclose(oracle.ball_radii_for_centres(K, label, np.array([[1.0, 0.0]]), 1), [[1.0]])
    assert np.allclose(oracle.ball_radii_for_centres(K, label, np.array([[1.5, 0.0]]), 1), [[1.5]])


# ------------------------------------------------------------------ TA filter (Alg. 4)
def _ta_bruteforce(f, label, tau):
    """Independent transcription for tiny inputs, written with python lists."""
    S, G = f.shape
    ranked = [sorted(range(G), key=lambda i: (-f[s, i], i)) for s in range(S)]
    seen = [set() for _ in range(S)]
    depth = 0
    while depth < G:
        U = 0.0
        for s in range(S):
            seen[s].add(ranked[s][depth])
            U += f[s, ranked[s][depth]]
        depth += 1
        if U < tau:
            break
    n = label.shape[1]
    return [any(label[s, j] in seen[s] for s in range(S)) for j in range(n)], depth


def test_ta_filter_no_false_negatives_and_sandwich(oracle):
    """K* is inside {j : sum_s f_{s,a(s,j)} >= tau}, which is inside the TA live set; the TA
    live set matches a list-based transcription; the depth grows as tau falls."""
    g = np.random.default_rng(11)
    n, d, S, r = 64, 8, 2, 4
    for trial in range(20):
        K = (g.standard_normal((n, d)) * g.uniform(0.3, 3, size=d)).astype(np.float32)
        q = g.standard_normal(d).astype(np.float32)
        label = np.stack([(g.permutation(n) // r) for _ in range(S)]).astype(np.int32)
        f = np.zeros((S, n // r))
        for s in range(S):
            lo, hi = oracle.subspace_range(d, S, s)
            Ks = np.zeros_like(K)
            Ks[:, lo:hi] = K[:, lo:hi]
            c, rad = oracle.ball_index(Ks, label[s], n // r, S)
            f[s] = oracle.ball_bounds(q, c, rad)[s]
        score = oracle.scores_f64(q, K)
        ub = sum(f[s, label[s]] for s in range(S))
        assert np.all(ub >= score - 1e-9)
        last_depth = 0
        for tau in sorted(np.quantile(score, [0.999, 0.9, 0.5, 0.1]).tolist(), reverse=True):
            alive, depth = oracle.ta_filter(f, label, tau)
            want_alive, want_depth = _ta_bruteforce(f, label, tau)
            assert alive.tolist() == want_alive and depth == want_depth
            assert np.all(alive[score >= tau])                 # zero false negatives
            assert np.all(alive[ub >= tau])                    # per-key sum rule is inside TA's set
            assert depth >= last_depth
            last_depth = depth
        alive, depth = oracle.ta_filter(f, label, -np.inf)
        assert alive.all() and depth == n // r
        alive, depth = oracle.ta_filter(f, label, np.inf)
        assert depth == 1


def test_ta_filter_stops_only_when_strictly_below(oracle):
    """The scan stops at the first depth with U < tau; U == tau must keep scanning, because an
    unseen key may score exactly tau.  Integer bounds make the tie exact."""
    f = np.array([[5.0, 3.0, 1.0]])
    label = np.array([[0, 1, 2]], dtype=np.int32)
    alive, depth = oracle.ta_filter(f, label, 5.0)
    assert depth == 2 and alive.tolist() == [True, True, False]
    alive, depth = oracle.ta_filter(f, label, 5.5)
    assert depth == 1 and alive.tolist() == [True, False, False]
    # two subspaces: U(1) = 4 + 6 = 10 == tau -> continue; U(2) = 2 + 1 = 3 < tau -> stop
    f = np.array([[4.0, 2.0, 0.0], [1.0, 6.0, 0.0]])
    label = np.array([[0, 1, 2], [0, 1, 2]], dtype=np.int32)
    alive, depth = oracle.ta_filter(f, label, 10.0)
    assert depth == 2 and alive.tolist() == [True, True, False]


# ------------------------------------------------------------------ balanced tree (Alg. 2)
def test_tree_on_a_line_is_sorted_chunks(oracle):
    """One informative axis: recursive median splits reduce to cutting the sorted order into
    consecutive runs, so with n = r 2^k every leaf is a run of r consecutive ranks."""
    g = np.random.default_rng(12)
    n, r = 64, 4
    K = np.zeros((n, 3), dtype=np.float32)
    K[:, 1] = g.permutation(n).astype(np.float32)
    label, order, leaves = oracle.balanced_tree(K, r)
    assert leaves == n // r
    assert np.array_equal(K[order, 1], np.arange(n))
    assert np.array_equal(label[order], np.arange(n) // r)


def test_tree_partition_valid_any_n(oracle):
    g = np.random.default_rng(13)
    for n, r in [(1, 4), (3, 4), (24, 4), (37, 4), (100, 8), (31, 2), (16, 1)]:
        K = g.standard_normal((n, 5)).astype(np.float32)
        label, order, leaves = oracle.balanced_tree(K, r)
        sizes = np.bincount(label, minlength=leaves)
        assert sizes.sum() == n and sizes.min() >= 1 and sizes.max() <= r
        assert sorted(order.tolist()) == list(range(n))
        assert np.array_equal(np.unique(label), np.arange(leaves))   # ids are dense, no collisions
        if n % r == 0 and (n // r) & (n // r - 1) == 0:
            assert leaves == n // r and sizes.min() == r


def test_tree_left_subtree_gets_floor_half(oracle):
    """Three points, r = 2: the left child takes floor(3/2) = 1 point (the smallest), the right
    child the other two."""
    K = np.array([[2.0], [0.0], [1.0]], dtype=np.float32)
    label, order, leaves = oracle.balanced_tree(K, r=2)
    assert leaves == 2 and order.tolist() == [1, 2, 0] and label.tolist() == [1, 0, 1]


def test_tree_first_split_uses_max_variance_axis(oracle):
    g = np.random.default_rng(14)
    n = 32
    K = g.standard_normal((n, 4)).astype(np.float32)
    K[:, 2] *= 50                                  # dominant axis
    label, order, leaves = oracle.balanced_tree(K, r=16)
    assert leaves == 2
    med = np.sort(K[:, 2])
    assert np.all(K[label == 0, 2] <= med[15]) and np.all(K[label == 1, 2] >= med[16])
    # restricted to coordinates [0,2) the dominant axis is ignored
    label2, _, _ = oracle.balanced_tree(K, r=16, lo=0, hi=2)
    ax = int(np.argmax(K[:, :2].var(axis=0)))
    med2 = np.sort(K[:, ax])
    assert np.all(K[label2 == 0, ax] <= med2[15]) and np.all(K[label2 == 1, ax] >= med2[16])


# ------------------------------------------------------------------ cost model (printed values)
def test_cost_model_reproduces_printed_table(oracle):
    rows = [l.split() for l in open(os.path.join(GOLDEN, "table7_scan_speedup.txt")) if not l.startswith("#")]
    assert len(rows) == 16
    for _, _, scan, speed in rows:
        # scan is printed to 0.1 %, speed-up to 0.01
        lo = oracle.predicted_speedup(1, 4, (float(scan) + 0.05) / 100)
        hi = oracle.predicted_speedup(1, 4, (float(scan) - 0.05) / 100)
        assert lo - 0.005 <= float(speed) <= hi + 0.005


# ------------------------------------------------------------------ workload generators
def test_generators_are_seeded_and_bf16_exact():
    a = W.make_cache(2, n=64)
    b = W.make_cache(2, n=64)
    assert np.array_equal(a.K, b.K) and np.array_equal(a.V, b.V)
    assert np.array_equal(W.bf16_bits_to_f32(a.K_bits()).reshape(a.K.shape), a.K)
    t = torch.tensor(np.random.default_rng(0).standard_normal(1000).astype(np.float32))
    assert np.array_equal(W.round_to_bf16(t.numpy()), t.to(torch.bfloat16).float().numpy())
    # four dominant channels per head
    sc = a.channel_scale[0, 0]
    assert (sc > 4 * np.median(sc)).sum() >= 3
    q = W.drift_queries(3, 5, n_q_heads=2)
    assert q.shape == (5, 1, 2, 128)
    assert np.array_equal(W.round_to_bf16(q), q)


# ------------------------------------------------------------------ boxes (Def. 1) and Query 1 (Alg. 3)
def test_box_bound_is_the_maximum_over_the_corners(oracle):
    """Brute force over all 2^d corners of tiny boxes: a linear function attains its maximum over
    a box at a corner, so the bound must equal the best corner (catches min instead of max, lo/hi
    swapped, a sign slip for negative q)."""
    g = np.random.default_rng(15)
    d = 6
    K = g.standard_normal((12, d)).astype(np.float32)
    label = np.repeat(np.arange(3), 4).astype(np.int32)
    lo, hi = oracle.aabb_index(K, label, 3)
    for i in range(3):
        assert np.array_equal(lo[i], K[label == i].min(0)) and np.array_equal(hi[i], K[label == i].max(0))
    for _ in range(5):
        q = g.standard_normal(d).astype(np.float32)
        ub = oracle.aabb_bounds(q, lo, hi)
        for i in range(3):
            corners = [sum(float(q[c]) * (hi[i, c] if (mask >> c) & 1 else lo[i, c]) for c in range(d))
                       for mask in range(1 << d)]
            assert math.isclose(ub[i], max(corners), rel_tol=1e-12, abs_tol=1e-12)
            assert np.all(K[label == i].astype(np.float64) @ q.astype(np.float64) <= ub[i] + 1e-12)
    # a one-point group: the box is the point, the bound is its score
    lo1, hi1 = oracle.aabb_index(K, np.arange(12, dtype=np.int32), 12)
    assert np.allclose(oracle.aabb_bounds(q, lo1, hi1), oracle.scores_f64(q, K), rtol=1e-12, atol=1e-12)


def test_box_bound_never_looser_than_needed_and_compares_with_ball(oracle):
    """In one dimension box and ball coincide for a two-point group; in general both dominate
    every member's score."""
    K = np.array([[1.0], [3.0]], dtype=np.float32)
    label = np.zeros(2, dtype=np.int32)
    lo, hi = oracle.aabb_index(K, label, 1)
    c, rad = oracle.ball_index(K, label, 1, 1)
    for qv in (2.0, -0.5):
        q = np.array([qv], dtype=np.float32)
        assert math.isclose(oracle.aabb_bounds(q, lo, hi)[0], oracle.ball_bounds(q, c, rad)[0, 0])
        assert math.isclose(oracle.aabb_bounds(q, lo, hi)[0], max(qv * 1.0, qv * 3.0))


def test_query1_filter_with_valid_thresholds_keeps_every_relevant_key(oracle):
    """Alg. 3: with tau_s = tau - sum over the other subspaces of their largest bound (a valid
    lower bound on a relevant key's subspace term) no relevant key is dropped; with thresholds of
    -inf everything is a candidate; raising one subspace threshold above all bounds drops all."""
    g = np.random.default_rng(16)
    n, d, S, r = 64, 8, 2, 4
    K = (g.standard_normal((n, d)) * g.uniform(0.3, 3, size=d)).astype(np.float32)
    q = g.standard_normal(d).astype(np.float32)
    label = np.stack([(g.permutation(n) // r) for _ in range(S)]).astype(np.int32)
    f = np.zeros((S, n // r))
    for s in range(S):
        lo_, hi_ = oracle.subspace_range(d, S, s)
        Ks = np.zeros_like(K)
        Ks[:, lo_:hi_] = K[:, lo_:hi_]
        c, rad = oracle.ball_index(Ks, label[s], n // r, S)
        f[s] = oracle.ball_bounds(q, c, rad)[s]
    score = oracle.scores_f64(q, K)
    for tau in np.quantile(score, [0.95, 0.5]):
        tau_s = np.array([tau - sum(f[t].max() for t in range(S) if t != s) for s in range(S)])
        alive = oracle.query1_filter(f, label, tau_s)
        assert np.all(alive[score >= tau])
        want = [all(f[s, label[s, j]] >= tau_s[s] for s in range(S)) for j in range(n)]
        assert alive.tolist() == want
    assert oracle.query1_filter(f, label, np.full(S, -np.inf)).all()
    assert not oracle.query1_filter(f, label, np.array([f[0].max() + 1, -np.inf])).any()
    # a ball that exactly touches the threshold is kept (a cluster is pruned only when f < tau_s)
    f1 = np.array([[5.0, 3.0]])
    lab1 = np.array([[0, 1, 1]], dtype=np.int32)
    assert oracle.query1_filter(f1, lab1, np.array([5.0])).tolist() == [True, False, False]
    assert oracle.query1_filter(f1, lab1, np.array([3.0])).tolist() == [True, True, True]


def test_safe_subspace_thresholds(oracle):
    """tau_s = tau - (largest bounds of the OTHER subspaces): hand-computed table; one subspace
    gives tau itself; on random keys with one grouping per subspace the thresholds lose no key
    with <q,k> >= tau, and they are the largest with that guarantee: when one key attains the
    largest bound in every other subspace exactly, its own subspace term equals tau_s."""
    f = np.array([[5.0, 3.0], [2.0, 7.0], [1.0, 1.0]])
    assert oracle.safe_subspace_thresholds(f, 10.0).tolist() == [2.0, 4.0, -2.0]
    assert oracle.safe_subspace_thresholds(np.array([[4.0, 9.0, -1.0]]), 6.5).tolist() == [6.5]
    assert np.all(np.isneginf(oracle.safe_subspace_thresholds(np.zeros((3, 0)), 1.0)))
    # negative bounds subtract as they are (no clamping at zero)
    assert oracle.safe_subspace_thresholds(np.array([[-2.0, -3.0], [1.0, 0.5]]), 0.0).tolist() == [-1.0, 2.0]
    g = np.random.default_rng(23)
    n, d, S, r = 96, 12, 3, 4
    for trial in range(4):
        K = (g.standard_normal((n, d)) * g.uniform(0.3, 3, size=d)).astype(np.float32)
        q = g.standard_normal(d).astype(np.float32)
        label = np.stack([(g.permutation(n) // r) for _ in range(S)]).astype(np.int32)
        f = np.zeros((S, n // r))
        for s in range(S):
            lo_, hi_ = oracle.subspace_range(d, S, s)
            Ks = np.zeros_like(K)
            Ks[:, lo_:hi_] = K[:, lo_:hi_]
            c, rad = oracle.ball_index(Ks, label[s], n // r, S)
            f[s] = oracle.ball_bounds(q, c, rad)[s]
        score = oracle.scores_f64(q, K)
        for tau in np.quantile(score, [0.99, 0.9, 0.3]):
            tau_s = oracle.safe_subspace_thresholds(f, tau)
            assert np.all(oracle.query1_filter(f, label, tau_s)[score >= tau])
    # tightness: groups of one key (bound = the key's own term), a key that is the maximiser of
    # subspaces 1 and 2 and sits exactly at tau has term_0 == tau_0
    terms = np.array([[1.0, 4.0, 2.0], [6.0, 0.0, 1.0], [3.0, 1.0, 0.0]])   # [S][keys]
    tau = terms[:, 0].sum()                                                   # key 0: 1 + 6 + 3
    assert oracle.safe_subspace_thresholds(terms, tau)[0] == terms[0, 0]


# ------------------------------------------------------------------ threshold oracles and reservoir
def test_hash_reference_values(oracle):
    """splitmix64 finaliser: the published generator seeded with 0 produces 0xE220A8397B1DCDAF
    first; our hash32(seed, stream, counter) is that finaliser applied to
    seed + stream*C1 + counter*C2, top 32 bits, so hash32(0, 0, 0) is the top half of that word."""
    assert oracle.hash32(0, 0, 0) == 0xE220A839
    # second output of the published sequence from seed 0 is 0x6E789E6AA1B965F4: counter advances by the same constant
    assert oracle.hash32(0, 0, 1) == 0x6E789E6A


def test_reservoir_is_algorithm_r_and_uniform(oracle):
    R = 16
    assert oracle.reservoir(7, 0, 10, R).tolist() == list(range(10))          # not yet full: arrival order
    assert oracle.reservoir(7, 0, R, R).tolist() == list(range(R))
    # transcription with python integers
    for n in (17, 100, 1000):
        res = list(range(R))
        for i in range(R, n):
            j = (oracle.hash32(7, 3, i) * (i + 1)) >> 32
            if j < R:
                res[j] = i
        assert oracle.reservoir(7, 3, n, R).tolist() == res
    # every position is kept with probability R/n: frequencies over many streams
    n, trials = 200, 4000
    hits = np.zeros(n)
    for t in range(trials):
        hits[oracle.reservoir(123, t, n, R)] += 1
    p = R / n
    sd = math.sqrt(trials * p * (1 - p))
    assert np.all(np.abs(hits - trials * p) < 5 * sd)
    assert len(set(oracle.reservoir(123, 0, n, R).tolist())) == R               # no duplicates


def test_threshold_rules_closed_forms(oracle):
    s = np.array([3.0, 10.0, 9.5, 1.0, 2.0, 9.0, 0.5, 2.5], dtype=np.float32)
    assert oracle.threshold(s, "sample-max") == 10.0
    assert math.isclose(oracle.threshold(s, "sample-mean-max"), 0.5 * (10.0 + s.mean()), rel_tol=1e-6)
    # sorted: 10 9.5 9 | 3 2.5 2 1 0.5  -> largest gap between 9 and 3: tau = 9, three keys qualify
    assert oracle.threshold(s, "sample-gap") == 9.0
    assert (s >= oracle.threshold(s, "sample-gap")).sum() == 3
    # equal largest gaps: the first one from the top is the cut (sorted 10 | 7 | 4 3: gaps 3, 3, 1)
    assert oracle.threshold(np.array([4.0, 10.0, 3.0, 7.0], dtype=np.float32), "sample-gap") == 10.0
    assert oracle.threshold(np.array([5.0], dtype=np.float32), "sample-gap") == 5.0
    for k in (1, 2, 5, 8):
        assert oracle.threshold(s, "sample-topk", k) == np.sort(s)[::-1][k - 1]
    assert oracle.threshold(s, "sample-topk", 100) == 0.5
    # budget(alpha): ceil(alpha m)-th largest, i.e. about a share alpha of the sample qualifies
    assert oracle.threshold(s, "budget", 0.25) == 9.5
    assert oracle.threshold(s, "budget", 0.5) == 3.0
    assert oracle.threshold(s, "budget", 1.0) == 0.5
    g = np.random.default_rng(17)
    x = g.standard_normal(256).astype(np.float32)
    for a in (0.05, 0.10, 0.15):
        t = oracle.threshold(x, "budget", a)
        assert (x >= t).sum() == math.ceil(a * 256)
    assert oracle.threshold(np.zeros(0, np.float32), "sample-max") == -np.inf


def test_threshold_rules_against_the_papers_table(oracle):
    """The appendix table of mean thresholds (tests/golden/threshold_oracle_table.txt) fixes how the
    rank-based rules relate: with a reservoir of 256, budget(alpha) read as the ceil(alpha*256)-th
    largest score puts budget(5 %) = 13th largest below topk(10) and above budget(10 %) = 26th, which
    is the order of the printed means; and sample-mean-max read as (max + mean)/2 is half the
    sample-max when the mean score is near zero (31.3 against 62.0 / 2)."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "threshold_oracle_table.txt")) if l.strip() and l[0] != "#"]
    table = {(r[0], float(r[1])): float(r[2]) for r in rows}
    rank_of = {("sample-max", 0.0): 1, ("sample-topk", 2.0): 2, ("sample-topk", 5.0): 5, ("sample-topk", 10.0): 10,
               ("budget", 0.05): math.ceil(0.05 * 256), ("budget", 0.10): math.ceil(0.10 * 256),
               ("budget", 0.15): math.ceil(0.15 * 256)}
    by_rank = sorted(rank_of, key=lambda k: rank_of[k])
    means = [table[k] for k in by_rank]
    assert means == sorted(means, reverse=True), "printed means must fall as the rank the rule reads grows"
    # the oracle's rules read exactly those ranks of a sample, whatever the sample
    g = np.random.default_rng(5)
    for _ in range(20):
        s = (g.standard_normal(256) * g.uniform(1, 20) + g.uniform(-5, 5)).astype(np.float32)
        srt = np.sort(s)[::-1]
        for (mode, param), rank in rank_of.items():
            assert oracle.threshold(s, mode, param) == srt[rank - 1], (mode, param)
        gap = oracle.threshold(s, "sample-gap")
        assert srt[-1] < gap <= srt[0]
    # (max + mean) / 2: the table's mean-max is half its sample-max up to the (small) mean score
    implied_mean = 2 * table[("sample-mean-max", 0.0)] - table[("sample-max", 0.0)]
    assert abs(implied_mean) < 0.25 * table[("budget", 0.15)]
    # sample-gap's printed mean lies between topk(2) and topk(5): the largest gap sits in the top few
    assert table[("sample-topk", 5.0)] < table[("sample-gap", 0.0)] < table[("sample-topk", 2.0)]


def test_pruning_power_report_runs_on_the_oracle_alone(oracle, capsys):
    """oracle/pruning_power.py (the source of the design notes' pruning table) on a small cache: its
    own check (no summed bound below a key's score) holds, the depth scan's live set contains the
    summed-bound set, and a grouping per subspace with small subspaces keeps fewer keys than one
    shared grouping, which keeps (nearly) all of these keys."""
    from oracle import pruning_power as pp
    pp.run(2, 2048, [4], [4, 16], n_queries=2)
    lines = [l for l in capsys.readouterr().out.splitlines() if l.startswith("config 2")]
    assert len(lines) == 6
    got = {}
    for l in lines:
        name = "per" if "per subspace" in l else ("shared" if "shared tree" in l else "contiguous")
        S = int(l.split("S=")[1].split()[0])
        keep_sum = float(l.split("summed bounds keep")[1].split()[0])
        keep_ta = float(l.split("depth scan keeps")[1].split()[0])
        assert keep_sum <= keep_ta + 1e-12
        got[(name, S)] = keep_sum
    assert got[("contiguous", 4)] > 0.99 and got[("shared", 16)] > 0.99
    assert got[("per", 16)] < got[("per", 4)] <= 1.0 and got[("per", 16)] < 0.9


def test_coded_single_key_balls_on_the_cpu():
    """Groups of one key with coded centres (oracle/pruning_power.py, `codings`): the code grids are the formats'
    (e4m3: 127 magnitudes up to 448 with eight steps per binade; e2m3: 32 magnitudes up to 7.5), every bound lies
    above its key's score (asserted inside), the exact centre keeps exactly the qualifying share per head, and a
    coarser code keeps more keys: bf16 < e4m3 < e2m3 with a scale per 32 coordinates, at radii of a few percent
    of the key's norm; dividing every coordinate by a power of two of its own first ('/chan') brings e2m3 back down."""
    from oracle import pruning_power as pp
    assert pp.E4M3.size == 127 and pp.E4M3[-1] == 448.0 and pp.E4M3[1] == 2.0 ** -9
    assert np.array_equal(pp.E4M3[(pp.E4M3 >= 1) & (pp.E4M3 < 2)], 1 + np.arange(8) / 8)
    assert pp.E2M3.size == 32 and pp.E2M3[-1] == 7.5
    assert np.array_equal(pp.E2M3[:17], np.arange(17) / 8) and np.array_equal(pp.E2M3[16:25], 2 + np.arange(9) / 4)
    # a key that is exactly representable is its own centre: radius 0 in that block
    k = np.zeros((1, 128))
    k[0, :8] = [0.125, -1.5, 3.75, 7.5, 0, 2.25, -6.5, 0.5]
    assert np.array_equal(pp.code_keys(k, "e2m3"), k)
    assert np.array_equal(pp.code_keys(k * 2.0 ** -20, "e2m3"), k * 2.0 ** -20)     # the scale follows the block
    k2 = k.copy()
    k2[0, 8] = 100.0                      # coordinate 8 is in another scale block (block 1): block 0 is untouched
    c2 = pp.code_keys(k2, "e2m3")
    assert np.array_equal(c2[0, :8], k[0, :8]) and c2[0, 8] == 96.0    # 100 / 16 = 6.25 -> 6.0 (ties to even code) * 16
    k3 = k.copy()
    k3[0, 32] = 100.0                     # coordinate 32 shares block 0's scale (16): 0.125 is lost, 7.5 becomes 8
    c3 = pp.code_keys(k3, "e2m3")
    assert c3[0, 0] == 0.0 and c3[0, 3] == 8.0 and c3[0, 32] == 96.0
    r = {c: pp.coded_keep(2, 4096, c, n_queries=2) for c in ("bf16", "e4m3", "e2m3")}
    assert r["bf16"]["relative_radius"] == 0.0 and abs(r["bf16"]["per_head"] - 0.01) < 1e-3
    assert r["bf16"]["per_kv_head"] < r["e4m3"]["per_kv_head"] < r["e2m3"]["per_kv_head"] < 0.3
    assert 0.015 < r["e4m3"]["relative_radius"] < r["e2m3"]["relative_radius"] < 0.06
    # channel factors: powers of two that follow each coordinate's size; coordinates of about the same size get the
    # same factor wherever their common size lies relative to a power of two, a coordinate that is zero keeps 1
    g = np.random.default_rng(3)
    base = g.standard_normal((2000, 128))
    for size in (1.0, 1.4, 0.71, 3.0):          # 1.4 and 0.71 sit next to the rounding boundary of a plain round(log2)
        a = pp.channel_factors(base * size)
        assert np.all(a == a[0]) and np.log2(a[0]) == np.rint(np.log2(a[0]))
    shift = g.integers(-6, 7, size=128)
    a = pp.channel_factors(base * 2.0 ** shift)
    assert np.array_equal(np.log2(a) - np.log2(a[0]), (shift - shift[0]).astype(np.float64))
    z = base.copy()
    z[:, 5] = 0.0
    assert pp.channel_factors(z)[5] == 1.0
    assert np.all(np.abs(np.log2(pp.channel_factors(base * 2.0 ** (3.0 * shift)))) <= 8)
    # the rescaled code keeps fewer keys where the channels differ in size (config 3's keys), and its bounds hold
    # (asserted inside coded_keep)
    plain, chan = (pp.coded_keep(3, 4096, c, n_queries=2) for c in ("e2m3", "e2m3/chan"))
    assert chan["per_kv_head"] < 0.8 * plain["per_kv_head"]
    assert abs(pp.coded_keep(3, 4096, "bf16/chan", n_queries=1)["per_head"] - pp.coded_keep(3, 4096, "bf16", n_queries=1)["per_head"]) < 1e-12
