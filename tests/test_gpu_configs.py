"""The five workloads at their full sizes, checked against the CPU oracle: every head of every
sampled step by the band rule for the retrieved sets and against the oracle's attention on the
same lists.  Five index settings each: the launch configuration bench.py times by default (r = 1:
every key its own group, 6-bit centres, contiguous, fused query kernel, default attention form), the
paper's printed r = 4 / S = 4 with one shared grouping, the paper's own layout (one tree
grouping per subspace, r = 4, S = 16, labels per key), and r = 1 and r = 4 with 8-bit centres."""
import math

import numpy as np
import pytest
import torch

import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import gpu_util
    assert torch.cuda.is_available()
    return gpu_util


def _settings():
    import paper_2605_06763_amd as L
    return {"r1": dict(group_size=1), "r4": dict(group_size=4), "r1_fp8": dict(group_size=1, index_dtype=L.LVR_INDEX_FP8), "r4_fp8": dict(group_size=4, index_dtype=L.LVR_INDEX_FP8),
            "per_subspace_r4_S16": dict(group_size=4, n_subspaces=16, grouping=L.LVR_GROUP_SUBSPACE_TREE)}


SETTINGS = ["r1", "r4", "per_subspace_r4_S16", "r1_fp8", "r4_fp8"]


@pytest.mark.parametrize("setting", SETTINGS)
def test_config2_llama_layer_32k(G, oracle, setting):
    """32 query / 8 KV heads, d=128, 32768 keys, bf16, channel-scaled keys, tau at the 99th percentile."""
    cache = W.make_cache(2)
    q = W.make_queries(2)
    with G.Index(cache.K, cache.V, "bf16", 32, **_settings()[setting]) as ix:
        tau = G.oracle_taus(oracle, ix, q, frac=0.01)
        idx, cnt, out = ix.query(q, tau, cap=2048, fused=True)
        r = G.check_step(oracle, ix, q, tau, idx, cnt, out, tag="config2")
        st = ix.stats()
        assert st["keys_emitted"] == int(cnt.sum()) and 328 * 32 <= st["keys_emitted"] <= 330 * 32 + 64
        G.say("config2", setting, r, st)
        ref = oracle.dense_attention(ix.K, ix.V, q, ix.sigma, 32)
        assert (np.abs(ix.dense(q) - ref).max(axis=-1) / np.abs(ref).max(axis=-1)).max() <= G.ATTN_TOL


@pytest.mark.parametrize("setting", SETTINGS)
def test_config3_128k_drifting_query(G, oracle, setting):
    """131072 keys, 0.5 % qualify, query drifting over 256 steps; three of the steps are checked
    in full, and the retrieved sets must change from step to step."""
    cache = W.make_cache(3)
    qs = W.drift_queries(3, 256)
    with G.Index(cache.K, cache.V, "bf16", 32, **_settings()[setting]) as ix:
        prev = None
        for t in (0, 1, 255):
            tau = G.oracle_taus(oracle, ix, qs[t], k_count=656)
            idx, cnt, out = ix.query(qs[t], tau, cap=4096, fused=True)
            r = G.check_step(oracle, ix, qs[t], tau, idx, cnt, out, tag=f"config3 t={t}")
            assert (cnt >= 656).all() and (cnt <= 656 + 8).all()
            sets = [set(idx[0, h, :cnt[0, h]].tolist()) for h in range(32)]
            if prev is not None:
                turnover = np.mean([len(a ^ b) / (len(a) + len(b)) for a, b in zip(prev, sets)])
                G.say(f"config3 t={t}: set turnover vs previous checked step {turnover:.2f}")
                assert turnover > 0.05
            prev = sets
            G.say(f"config3 t={t}", r)
        G.say("config3", setting, ix.stats())


@pytest.mark.parametrize("setting", SETTINGS)
def test_config4_batch16(G, oracle, setting):
    """16 independent 32k caches, one batched step, tau at the 98th percentile per (sequence, head)."""
    cache = W.make_cache(4)
    q = W.make_queries(4)
    with G.Index(cache.K, cache.V, "bf16", 32, **_settings()[setting]) as ix:
        tau = G.oracle_taus(oracle, ix, q, frac=0.02)
        idx, cnt, out = ix.query(q, tau, cap=2048, fused=True)
        r = G.check_step(oracle, ix, q, tau, idx, cnt, out, tag="config4")
        st = ix.stats()
        assert st["keys_emitted"] == int(cnt.sum())
        G.say("config4", setting, r, st)
        # sequences are independent: swapping the queries of two sequences changes their results
        assert not np.array_equal(idx[0, 0, :16], idx[1, 0, :16])


@pytest.mark.parametrize("setting", SETTINGS)
def test_config5_long_output_decode(G, oracle, setting):
    """Prompt of 16384 keys, then 4096 decode steps, each appending one key/value per KV head and
    issuing query + attention with tau = (max score so far) - 8 per head.  Every step runs on the
    GPU; the oracle checks a sample of steps in full, including the ones around buffer flushes."""
    import paper_2605_06763_amd as L
    steps, n0, hq, hkv, d, B = 4096, 16384, 32, 8, 128, 256
    cache = W.make_cache(5)
    k_new, v_new = W.make_append_stream(5, steps, cache)               # [steps][1][hkv][d]
    qs = W.drift_queries(5, steps)                                     # [steps][1][hq][d]
    K_all = np.concatenate([cache.K, k_new.transpose(1, 2, 0, 3)], axis=2)   # [1][hkv][n0+steps][d]
    V_all = np.concatenate([cache.V, v_new.transpose(1, 2, 0, 3)], axis=2)
    Kd_all, Vd_all = G.to_device(K_all, "bf16"), G.to_device(V_all, "bf16")
    q_dev = torch.from_numpy(qs).cuda()
    cfg = L.make_config(batch=1, n_q_heads=hq, n_kv_heads=hkv, capacity=n0 + steps, buffer_size=B, **_settings()[setting])
    r_grp = cfg.group_size
    h = L.lvr_create(cfg)
    sigma = 1.0 / math.sqrt(d)
    cap = 8192
    out = torch.zeros((1, hq, d), device="cuda")
    idx = torch.zeros((1, hq, cap), dtype=torch.int32, device="cuda")
    cnt = torch.zeros((1, hq), dtype=torch.int32, device="cuda")
    check_at = {0, 1, 254, 255, 256, 257, 511, 512, 1000, 2047, 2048, 3333, 4094, 4095}
    try:
        L.lvr_build(h, Kd_all[:, :, :n0], Vd_all[:, :, :n0])
        total_retrieved, worst = 0, 0.0
        for t in range(steps):
            n_t = n0 + t + 1
            L.lvr_append(h, Kd_all[:, :, n_t - 1:n_t].contiguous(), Vd_all[:, :, n_t - 1:n_t].contiguous())
            # threshold (an input of the method): running max of the raw scores minus 8
            s = torch.einsum("hgd,hnd->hgn", q_dev[t, 0].view(hkv, 4, d), Kd_all[0, :, :n_t].float())
            tau = (s.amax(-1) - 8.0).reshape(1, hq).contiguous()
            L.lvr_decode_step(h, q_dev[t], tau, out, idx, cnt)
            if t in check_at:
                torch.cuda.synchronize()
                n, n_indexed = L.lvr_length(h)
                assert n == n_t and n_indexed % r_grp == 0 and 0 <= n - n_indexed < B
                assert n_indexed == n0 + ((t + 1) // B) * B
                i_np, c_np, o_np, tau_np = idx.cpu().numpy(), cnt.cpu().numpy(), out.cpu().numpy(), tau.cpu().numpy()
                for hh in range(hq):
                    r = G.check_head(oracle, qs[t, 0, hh], K_all[0, hh // 4, :n_t], V_all[0, hh // 4, :n_t],
                                     tau_np[0, hh], i_np[0, hh], int(c_np[0, hh]), o_np[0, hh], sigma,
                                     where=f"config5 t={t} h={hh}")
                    total_retrieved += r["size"]
                    worst = max(worst, r["attn_err"])
                    assert r["size"] >= 1          # the maximum itself always qualifies
                G.say(f"config5 t={t}: n={n_t} indexed={n_indexed} mean set size {c_np.mean():.1f}")
        st = L.lvr_get_stats(h)
        G.say("config5", setting, dict(checked_steps=len(check_at), retrieved=total_retrieved, attn_err=worst), st)
    finally:
        L.lvr_destroy(h)


def test_config2_library_thresholds_query1_and_offload(G, oracle):
    """Full-size config 2 through the rows beyond the core path: tau chosen by the library's
    budget rule over its reservoir (equal to the oracle's rule on the oracle's sample) and used
    for a decode step; Query 1 with safe per-subspace thresholds; the same step with the K/V
    arena in host memory."""
    L = G.L
    seed, R = 20260506, 256
    cache = W.make_cache(2)
    q = W.make_queries(2)
    with G.Index(cache.K, cache.V, "bf16", 32, reservoir_size=R, seed=seed) as ix:
        res = ix.reservoir()
        for g in range(8):
            assert np.array_equal(res[0, g], oracle.reservoir(seed, g, ix.n, R))
        for mode, param in (("budget", 0.02), ("sample-topk", 3), ("sample-max", 0)):
            tau = ix.threshold(q, mode, param)
            for h in range(32):
                s = oracle.scores_f32(q[0, h], ix.K[0, h // 4][res[0, h // 4]])
                assert abs(tau[0, h] - oracle.threshold(s, mode, param)) <= 2e-6 * max(1.0, float(np.abs(s).max()))
            idx, cnt, out = ix.query(q, tau, cap=8192, fused=True)
            r = G.check_step(oracle, ix, q, tau, idx, cnt, out, tag=f"config2 {mode}")
            G.say(f"config2 tau by {mode}({param}): retrieved per head {cnt.mean():.1f}", r)
        # Query 1 with thresholds that cannot lose a qualifying key
        centres, radii, _, _ = ix.export()
        tau = G.oracle_taus(oracle, ix, q, frac=0.01)
        tau_s = np.empty((1, 32, 4), dtype=np.float32)
        chan = ix.channel_factors()   # the default index is stored in a per-channel rescaled space
        for h in range(32):
            c = W.bf16_bits_to_f32(centres[0, h // 4]).reshape(-1, 128).astype(np.float64) / chan[0, h // 4]
            top = oracle.ball_bounds(q[0, h] * chan[0, h // 4], c, radii[0, h // 4].astype(np.float64)).max(axis=1)
            tau_s[0, h] = (tau[0, h] - (top.sum() - top) - 1e-3).astype(np.float32)
        idx, cnt, out = G.query1(ix, q, tau_s, tau, cap=2048)
        G.check_step(oracle, ix, q, tau, idx, cnt, out, tag="config2 query1")
        # the same thresholds derived by the library from tau alone
        lib_tau_s = G.subspace_thresholds(ix, q, tau)
        assert np.all(np.abs(lib_tau_s - (tau_s + 1e-3)) <= 2e-5 * (np.abs(tau)[..., None] + np.abs(tau_s - tau[..., None]) + 1))
        idx, cnt, out = G.query1(ix, q, lib_tau_s, tau, cap=2048)
        G.check_step(oracle, ix, q, tau, idx, cnt, out, tag="config2 query1, library thresholds")
    with G.Index(cache.K, cache.V, "bf16", 32, flags=L.LVR_KV_IN_HOST_MEMORY) as ix:
        assert L.lvr_host_bytes(ix.cfg) == 2 * 8 * 32768 * 128 * 2
        tau = G.oracle_taus(oracle, ix, q, frac=0.01)
        idx, cnt, out = ix.query(q, tau, cap=2048, fused=True)
        G.check_step(oracle, ix, q, tau, idx, cnt, out, tag="config2 offloaded")


def test_config3_threshold_rules_are_stable_over_the_drifting_query(G, oracle):
    """The nine threshold rules of the appendix over the 256 drifting queries of config 3: means
    ordered as the paper's table orders them (rank rules by rank), every rule's threshold moving
    with the query without jumping (the paper reports a coefficient of variation of 8-25 % on model
    traces; these synthetic queries are printed for comparison, not held to that figure), and the
    budget rule's retrieval share close to its target."""
    cache = W.make_cache(3)
    qs = W.drift_queries(3, 256)
    rules = [("sample-max", 0), ("sample-topk", 2), ("sample-gap", 0), ("sample-topk", 5), ("sample-topk", 10),
             ("sample-mean-max", 0), ("budget", 0.05), ("budget", 0.10), ("budget", 0.15)]
    with G.Index(cache.K, cache.V, "bf16", 32, reservoir_size=256, seed=3) as ix:
        taus = {r: np.stack([ix.threshold(qs[t], *r) for t in range(0, 256, 4)]) for r in rules}    # [64][1][32]
        mean = {r: float(v.mean()) for r, v in taus.items()}
        cov = {r: float((v.std(axis=0) / np.abs(v.mean(axis=0))).mean()) for r, v in taus.items()}
        for r in rules:
            G.say(f"  {r[0]}({r[1]}): mean tau {mean[r]:.1f}, CoV over steps {100 * cov[r]:.1f} %")
            # sample-gap cuts at the largest gap wherever it lies; on these symmetric synthetic scores that is
            # as often in the lower tail as in the upper one, so its threshold jumps (the paper's traces are right-skewed)
            assert np.isfinite(mean[r]) and (r[0] == "sample-gap" or cov[r] < 0.6)
        order = [("sample-max", 0), ("sample-topk", 2), ("sample-topk", 5), ("sample-topk", 10), ("budget", 0.05),
                 ("budget", 0.10), ("budget", 0.15)]
        assert [mean[r] for r in order] == sorted((mean[r] for r in order), reverse=True)
        assert mean[("sample-gap", 0)] <= mean[("sample-max", 0)]
        # budget(alpha) aims at a retrieval share of alpha: measured on one step, within sampling error of a 256-key sample
        tau = ix.threshold(qs[0], "budget", 0.05)
        idx, cnt, out = ix.query(qs[0], tau, cap=32768, fused=True)
        share = cnt.mean() / ix.n
        G.say(f"  budget(5 %): retrieved share {100 * share:.2f} %")
        assert 0.02 < share < 0.10
        G.check_step(oracle, ix, qs[0], tau, idx, cnt, out, heads=[0, 13, 31], tag="config3 budget(5%)")


def test_four_million_keys_per_head(G, oracle):
    """Largest size exercised: 4 194 304 keys on each of 8 KV heads (a 16 GiB K/V arena, byte offsets
    far beyond 2^32).  Data is made on the device from a seeded torch generator; the heads of the
    LAST KV head (the largest offsets) are checked against the oracle on the host copy of its keys."""
    L = G.L
    n, hkv, hq, d = 1 << 22, 8, 32, 128
    gen = torch.Generator(device="cuda")
    gen.manual_seed(20260506)
    Kd = torch.randn((1, hkv, n, d), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    Vd = torch.randn((1, hkv, n, d), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    q = W.make_queries(3)                                     # [1][32][128], bf16-representable
    cfg = L.make_config(batch=1, n_q_heads=hq, n_kv_heads=hkv, capacity=n)
    h = L.lvr_create(cfg)
    try:
        L.lvr_build(h, Kd, Vd)
        g = hkv - 1
        K_last = Kd[0, g].float().cpu().numpy()
        V_last = Vd[0, g].float().cpu().numpy()
        heads = list(range(4 * g, 4 * g + 4))
        tau = np.full((1, hq), np.inf, dtype=np.float32)      # other heads: nothing qualifies
        for hh in heads:
            tau[0, hh] = W.tau_for_count(oracle.scores_f32(q[0, hh], K_last), 500)
        qd, td = torch.from_numpy(q).cuda(), torch.from_numpy(tau).cuda()
        out = torch.zeros((1, hq, d), device="cuda")
        idx = torch.zeros((1, hq, 1024), dtype=torch.int32, device="cuda")
        cnt = torch.zeros((1, hq), dtype=torch.int32, device="cuda")
        L.lvr_decode_step(h, qd, td, out, idx, cnt)
        torch.cuda.synchronize()
        gi, gc, go = idx.cpu().numpy(), cnt.cpu().numpy(), out.cpu().numpy()
        assert (gc[0, :4 * g] == 0).all() and np.abs(go[0, :4 * g]).max() == 0.0
        for hh in heads:
            r = G.check_head(oracle, q[0, hh], K_last, V_last, tau[0, hh], gi[0, hh], int(gc[0, hh]), go[0, hh],
                             1.0 / math.sqrt(d), where=f"4M keys head {hh}")
            assert 500 <= r["size"] <= 510
            G.say(f"4M keys, head {hh}:", r)
        st = L.lvr_get_stats(h)
        assert st["n_keys"] == n and st["n_indexed"] == n and st["groups_scored"] == hkv * n // 4
    finally:
        L.lvr_destroy(h)
