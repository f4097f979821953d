#!/usr/bin/env python3
"""Decode-step benchmark of the Louver hot path on one MI355X.

One step = one pass of the per-step hot path over one batch of synthetic input: range query
(bound pruning + exact filter) followed by sparse attention over the retrieved keys, through
the C ABI (lvr_decode_step).  For the append workload (config 5) a step first appends the
step's new key/value (lvr_append_decode_step: both in one call).  Inputs (K, V, all queries,
all thresholds) are resident in HBM before the timed region starts.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config {2,3,4,5}]

Headline workload: config 3 (GQA 32/8 heads, d=128, 131072 keys, batch 1, bf16, 0.5 % of the
keys qualify per head, query drifting over 256 consecutive decode steps) — the 128k-context case
the target is stated on.  The same line also carries, for that workload, the exact filter alone
(no index), the dense baseline, the paper's printed index setting (r = 4) and the CPU oracle,
and a compact block for each of the other workloads (configs 2, 4, 5) measured in the same run.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth
DEFAULT_GROUP_SIZE = 1  # chosen on measured step time over the five workloads


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def kth_midpoint_tau(scores, k):
    """tau midway between the k-th and (k+1)-th largest score along the last axis (torch)."""
    import torch
    top = torch.topk(scores, k + 1, dim=-1).values
    return 0.5 * (top[..., k - 1] + top[..., k])


def scores_on_gpu(Kd, q, G):
    """Raw <q,k> for threshold placement only (the thresholds are inputs of the method):
    Kd [B][Hkv][n][d] bf16, q [B][Hq][d] fp32 -> [B][Hq][n] fp32."""
    import torch
    B, Hkv, n, d = Kd.shape
    out = torch.empty((B, Hkv * G, n), dtype=torch.float32, device=Kd.device)
    for b in range(B):
        for h in range(Hkv):
            out[b, h * G:(h + 1) * G] = q[b, h * G:(h + 1) * G] @ Kd[b, h].float().T
    return out


def timed(fn, n_steps, first=0):
    """ms for n_steps calls of fn(t), t = first .., between two events on the launch stream."""
    import torch
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    ev0.record()
    for t in range(first, first + n_steps):
        fn(t)
    ev1.record()
    torch.cuda.synchronize()
    return ev0.elapsed_time(ev1)


def stream_read_ceiling(L, dev):
    """GB/s of a kernel that only reads (1 GiB, larger than every cache): the best launch shape of
    a few, best of 3 timings of 4 launches each."""
    import torch
    src = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    src.zero_()
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    best, shape = None, None
    for wgs in (1024, 2048, 4096, 8192, 16384):
        L.lvr_stream_read(src, sink, wgs)
        for _ in range(3):
            ms = timed(lambda t: L.lvr_stream_read(src, sink, wgs), 4) / 4
            if best is None or ms < best:
                best, shape = ms, wgs
    del src
    return (1 << 30) / (best * 1e-3) / 1e9, shape


def measure(cid, args, *, group_size, steps, warmup, full, cpu_seconds, legs=True):
    """All measurements of one workload.  full: the headline's extra passes (per-step distribution,
    cache-cold replicas, the paper's printed setting beside the chosen one)."""
    import numpy as np
    import torch

    import paper_2605_06763_amd as L
    import workloads as W

    dev = torch.device("cuda:0")
    c = W.CONFIGS[cid]
    B, Hq, Hkv, d, n0 = c["batch"], c["n_q_heads"], c["n_kv_heads"], c["head_dim"], c["n"]
    if args.q_heads:
        assert args.q_heads in (8, 16, 32, 64) and cid != 5, "--q-heads: 8, 16, 32 or 64, not with the append workload"
        Hq = args.q_heads
    G = Hq // Hkv
    K_steps, W_steps = steps, warmup
    appending = cid == 5
    n_verify = 6 if (appending and cpu_seconds > 0) else 0   # config 5: steps replayed with a sync for the oracle
    # the append workload consumes one new token per step in every pass: warm-up, timed, profiled,
    # exact filter alone, then the steps the oracle checks
    n_passes = 3 if legs else 2
    T_all = W_steps + n_passes * K_steps + n_verify if appending else 0
    log(f"[bench] config {cid} {c['name']}: generating inputs")
    t0 = time.time()
    if args.keys == "local":
        assert not appending, "the supplementary cache has no append stream"
        cache = W.make_local_cache(cid)
    else:
        cache = W.make_cache(cid)
    K_bits, V_bits = cache.K_bits(), cache.V_bits()
    Kd = torch.from_numpy(K_bits.view(np.int16)).view(torch.bfloat16).to(dev)
    Vd = torch.from_numpy(V_bits.view(np.int16)).view(torch.bfloat16).to(dev)

    # distinct queries cycled through the timed steps
    if cid == 3:
        n_distinct = 256
        q_np = W.drift_queries(3, n_distinct, n_q_heads=Hq)        # [T][B][Hq][d]
    elif appending:
        n_distinct = T_all
        q_np = W.drift_queries(5, n_distinct)
    else:
        n_distinct = 16
        q_np = np.stack([W.make_queries(cid, step=t, n_q_heads=Hq) for t in range(n_distinct)])
    q_all = torch.from_numpy(q_np).to(dev)

    capacity = n0 + (T_all + 64 if appending else 0)

    def make_cfg(r, centres=None):
        return L.make_config(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, kv_dtype=L.LVR_BF16,
                             group_size=r, n_subspaces=args.subspaces, buffer_size=256, capacity=capacity,
                             enclosing=L.LVR_ENCLOSE_AABB if args.enclosing == "aabb" else L.LVR_ENCLOSE_BALL,
                             grouping={"contiguous": L.LVR_GROUP_CONTIGUOUS, "tree": L.LVR_GROUP_TREE,
                                       "subspace": L.LVR_GROUP_SUBSPACE_TREE}[args.grouping],
                             attn_splits=args.attn_splits, query_workgroups=args.query_workgroups,
                             index_dtype={"auto": L.LVR_INDEX_AUTO, "bf16": L.LVR_INDEX_SAME, "fp8": L.LVR_INDEX_FP8, "fp6": L.LVR_INDEX_FP6}[centres or args.centres],
                             flags=(L.LVR_CONCURRENT_UPDATE if args.concurrent_update else 0)
                             | (L.LVR_KV_IN_HOST_MEMORY if args.offload else 0)
                             | (L.LVR_SEPARATE_KERNELS if args.separate else 0))
    cfg = make_cfg(group_size)
    h = L.lvr_create(cfg)
    L.lvr_build(h, Kd, Vd)          # first call: the runtime loads the kernels' code
    torch.cuda.synchronize()
    tb = time.time()
    L.lvr_build(h, Kd, Vd)          # a build discards what was there: the same work again, timed
    torch.cuda.synchronize()
    build_ms = (time.time() - tb) * 1e3

    set_turnover = None
    # thresholds (inputs): per step and head, so that the configured share of keys qualifies
    if appending:
        k_new_np, v_new_np = W.make_append_stream(5, T_all, cache)

        def up(x):
            bits = W.f32_to_bf16_bits(x).reshape(x.shape)
            return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(dev)
        k_new = up(k_new_np).unsqueeze(3).contiguous()      # [T][B][Hkv][1][d]
        v_new = up(v_new_np).unsqueeze(3).contiguous()
        # tau_t = (max raw score over the keys present at step t) - 8
        tau_all = torch.empty((T_all, B, Hq), dtype=torch.float32, device=dev)
        Kfull = torch.cat([Kd, k_new[:, :, :, 0].permute(1, 2, 0, 3)], dim=2)     # [B][Hkv][n0+T][d]
        for t in range(T_all):
            s = scores_on_gpu(Kfull[:, :, :n0 + t + 1], q_all[t % n_distinct], G)
            tau_all[t] = s.amax(-1) - c["tau_below_max"]
            if t % 1024 == 1023:
                torch.cuda.synchronize()
                log(f"[bench] thresholds placed for {t + 1} of {T_all} steps")
        del Kfull
    else:
        frac = c["qualify_frac"] if args.qualify_frac is None else args.qualify_frac
        kq = int(math.ceil(frac * n0))
        tau_all = torch.empty((n_distinct, B, Hq), dtype=torch.float32, device=dev)
        prev, turn = None, []
        for t in range(n_distinct):
            sc = scores_on_gpu(Kd, q_all[t], G)
            # --qualify-frac 0: thresholds that no key reaches (the bound phase alone: no survivors, no hits)
            tau_all[t] = kth_midpoint_tau(sc, kq) if kq > 0 else sc.amax(-1) * 1.5 + 1.0
            if cid == 3 and kq > 0:                         # drifting queries: how much of the set is new each step
                cur = sc >= tau_all[t].unsqueeze(-1)
                if prev is not None:
                    turn.append((cur & ~prev).sum(-1).float().div(kq).mean())
                prev = cur
            if t % 64 == 63:
                torch.cuda.synchronize()
                log(f"[bench] thresholds placed for {t + 1} of {n_distinct} queries")
        if turn:
            set_turnover = float(torch.stack(turn).mean())
        del prev
    cap = 4096 if not appending else 8192
    out = torch.zeros((B, Hq, d), dtype=torch.float32, device=dev)
    idx = torch.zeros((B, Hq, cap), dtype=torch.int32, device=dev)
    cnt = torch.zeros((B, Hq), dtype=torch.int32, device=dev)
    torch.cuda.synchronize()
    log(f"[bench] inputs ready in {time.time() - t0:.1f}s; build {build_ms:.2f} ms; arena {L.lvr_arena_bytes(cfg) / 2**20:.0f} MiB")

    # every step's arguments are slices of resident tensors; marshal them once, outside the timed
    # region, so the host loop is the library calls and nothing else
    A = L.tensor_arg
    st_arg = L.stream_arg()
    q_args = [A(q_all[t]) for t in range(n_distinct)]
    tau_args = [A(tau_all[t]) for t in range(tau_all.shape[0])]
    out_a, idx_a, cnt_a = A(out), A(idx), A(cnt)
    if appending:
        k_args = [A(k_new[t]) for t in range(k_new.shape[0])]
        v_args = [A(v_new[t]) for t in range(v_new.shape[0])]

    def step_on(handle):
        def one_step(t):
            if appending:
                # the step's token joins the cache, then the query is answered: one call
                L.lvr_append_decode_step(handle, k_args[t], v_args[t], q_args[t % n_distinct], tau_args[t], out_a, idx_a,
                                         cnt_a, st_arg)
            else:
                L.lvr_decode_step(handle, q_args[t % n_distinct], tau_args[t % n_distinct], out_a, idx_a, cnt_a, st_arg)
        return one_step
    one_step = step_on(h)

    # ---- warm-up, then the timed region: exactly K steps ----
    timed(one_step, W_steps, 0)
    ms_per_step = timed(one_step, K_steps, W_steps) / K_steps
    st = L.lvr_get_stats(h, raise_on_overflow=False)
    if st["overflow"]:
        log("[bench] WARNING: a retrieved set exceeded cap; lists were truncated")
    n_now = st["n_keys"]
    next_t = W_steps + K_steps if appending else W_steps

    # ---- distribution over steps: one event after every step of another pass over the same K steps
    # (each figure includes the event's own cost, about 1 us; the mean above does not) ----
    step_dist = None
    if full and not appending:
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(K_steps + 1)]
        torch.cuda.synchronize()
        evs[0].record()
        for t in range(K_steps):
            one_step(W_steps + t)
            evs[t + 1].record()
        torch.cuda.synchronize()
        per = np.array([evs[t].elapsed_time(evs[t + 1]) * 1e3 for t in range(K_steps)])
        step_dist = {"p10": round(float(np.percentile(per, 10)), 2), "median": round(float(np.median(per)), 2),
                     "p90": round(float(np.percentile(per, 90)), 2), "max": round(float(per.max()), 2)}

    # ---- cache-cold protocol: the same steps over `rotate` replicas of the index in turn, so that a
    # step never finds the previous step's lines of its replica in the 256 MB memory-side cache ----
    cold = None
    if full and not appending and args.rotate > 1:
        reps = [h]
        for _ in range(args.rotate - 1):
            hr = L.lvr_create(cfg)
            L.lvr_build(hr, Kd, Vd)
            reps.append(hr)

        def rot_step(t):
            L.lvr_decode_step(reps[t % len(reps)], q_args[t % n_distinct], tau_args[t % n_distinct], out_a, idx_a,
                              cnt_a, st_arg)
        timed(rot_step, max(W_steps, len(reps)), 0)
        cold_ms = timed(rot_step, K_steps, W_steps) / K_steps
        for hr in reps[1:]:
            L.lvr_destroy(hr)
        cold = {"replicas": len(reps), "us_per_step": round(cold_ms * 1e3, 2)}

    # ---- per-kernel time with HIP events on the launch stream (same K steps again) ----
    L.lvr_profile_enable(h, 8 * K_steps + 64)
    ms_prof_total = timed(one_step, K_steps, next_t)
    prof = L.lvr_profile_read(h)
    L.lvr_profile_enable(h, 0)
    if appending:
        next_t += K_steps
    kern = {k: dict(avg_us=1e3 * ms / max(nl, 1), launches=nl) for k, (ms, nl) in prof.items() if nl}
    st = L.lvr_get_stats(h, raise_on_overflow=False)

    # ---- the exact filter alone on the same arena: no bound test, every held key scored ----
    exact_only = None
    if legs and not args.separate and args.grouping != "subspace":
        L.lvr_set_bound_test(h, False)
        if not appending:
            timed(one_step, max(W_steps // 2, 4), 0)
        ms_x = timed(one_step, K_steps, next_t) / K_steps
        stx = L.lvr_get_stats(h, raise_on_overflow=False)
        L.lvr_set_bound_test(h, True)
        if appending:
            next_t += K_steps
        xb = stx["bytes_keys"] + stx["bytes_attention"]
        exact_only = {"us_per_step": round(ms_x * 1e3, 2), "step_bytes": int(xb),
                      "step_GBs": round(xb / (ms_x * 1e-3) / 1e9, 1),
                      "step_frac_of_peak": round(xb / (ms_x * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                      "index_speedup_over_it": round(ms_x / ms_per_step, 3)}

    # ---- dense full-KV attention on the same arena ----
    def dense_step(t):
        L.lvr_dense_attention(h, q_args[t % n_distinct], out_a, st_arg)
    timed(dense_step, max(W_steps // 2, 4))
    dense_ms = timed(dense_step, K_steps) / K_steps
    n_dense = L.lvr_length(h)[0]
    dense_bytes = B * Hkv * n_dense * 2 * d * 2

    # ---- algorithmic bytes of the dominant kernel ----
    # fused range-query kernel (bound test + exact check): per (sequence, KV head)
    #   groups * (d*c + radii) bytes of centres (c = 1 byte per coordinate as e4m3 codes, 2 as bf16) and radii
    #   +  keys_scanned * d*2 bytes of key rows
    n_bh = B * Hkv
    filt = kern.get("filter", dict(avg_us=float("nan")))
    two_launches = args.separate or args.grouping == "subspace"
    if two_launches and "prune" in kern:
        filt = dict(avg_us=filt["avg_us"] + kern["prune"]["avg_us"])
    query_bytes = st["bytes_index"] + st["bytes_keys"]
    achieved = query_bytes / (filt["avg_us"] * 1e-6) / 1e9
    step_bytes = st["bytes_index"] + st["bytes_keys"] + st["bytes_attention"]
    kernel_name = ("subspace_bounds_kernel+label_filter_kernel" if args.grouping == "subspace"
                   else "prune_mfma_kernel+filter_mfma_kernel" if args.separate else "query_fused_kernel")
    roofline = dict(bound="hbm", kernel=kernel_name, achieved=round(achieved, 1), peak=HBM_PEAK_GBS,
                    unit="GB/s", frac=round(achieved / HBM_PEAK_GBS, 4), traffic=None, traffic_source=None,
                    bytes_per_launch=int(query_bytes), avg_launch_us=round(filt["avg_us"], 2),
                    launch_time_source="a HIP event pair per launch of the kernel, handed to the dispatch itself (hipExtLaunchKernelGGL: "
                                       "the events hold the kernel's own start and end), in a second pass over the timed steps on the "
                                       "library's stream; the events between the kernels keep a step's launches from running back to back, "
                                       "so a launch reads about 1 us more than in a rocprofv3 trace of the same command "
                                       "(profiles/decode_step_config3_kernel_trace.md)")
    # HBM bytes per launch measured OFFLINE with rocprofv3 --pmc on this same command (the counters cannot
    # be read from inside the run); only the default options of a workload have a figure
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    default_opts = (args.subspaces == 4 and args.keys == "workload" and args.query_workgroups == 0 and args.qualify_frac is None
                    and args.enclosing == "ball" and args.centres == "auto" and not args.offload and not args.separate
                    and args.grouping == "contiguous" and not args.q_heads)
    if os.path.exists(tpath) and default_opts:
        for line in open(tpath):
            f = line.split()
            if len(f) == 4 and f[0] == f"config{cid}" and f[1] == f"r{group_size}" and f[2] == "query_fused_kernel":
                roofline["traffic"] = int(f[3])
                roofline["traffic_source"] = ("stored figure, not measured by this run: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE "
                                              "of this command, scaled by a plain copy (profiles/hbm_traffic.txt)")

    res = {
        "cid": cid, "name": c["name"], "B": B, "Hq": Hq, "Hkv": Hkv, "d": d, "n_now": int(n_now),
        "ms_per_step": ms_per_step, "roofline": roofline, "cfg": cfg,
        "step_bytes": {"index": int(st["bytes_index"]), "keys": int(st["bytes_keys"]),
                       "attention": int(st["bytes_attention"]), "total": int(step_bytes),
                       "step_GBs": round(step_bytes / (ms_per_step * 1e-3) / 1e9, 1),
                       "step_frac_of_peak": round(step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
        "set_turnover_per_step": None if set_turnover is None else round(set_turnover, 4),
        "f_scan": round(st["keys_scanned"] / max(n_bh * st["n_keys"], 1), 4),
        "groups_surviving_frac": round(st["groups_surviving"] / max(st["groups_scored"], 1), 4),
        "retrieved_per_head": round(st["keys_emitted"] / (B * Hq), 1),
        "index_bytes_per_key": round(st["bytes_index"] / max(n_bh * st["n_indexed"], 1), 1),
        "kernels_us": {k: round(v["avg_us"], 2) for k, v in kern.items()},
        "profiled_us_per_step": round(ms_prof_total / K_steps * 1e3, 2),
        "exact_filter_only": exact_only,
        "dense_baseline": {"us_per_step": round(dense_ms * 1e3, 2), "bytes": int(dense_bytes),
                           "GBs": round(dense_bytes / (dense_ms * 1e-3) / 1e9, 1),
                           "frac_of_peak": round(dense_bytes / (dense_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                           "speedup_of_sparse_path": round(dense_ms / ms_per_step, 3)},
        "step_us_distribution": step_dist,
        "cache_cold": cold,
        "build_ms": round(build_ms, 3),
        "index_bytes_per_group": st["bytes_index"] // max(st["groups_scored"], 1),
    }

    # ---- the paper's printed setting (r = 4, S = 4) on the same keys, when another one is the default ----
    if full and not appending and group_size != 4 and legs:
        cfg4 = make_cfg(4)
        h4 = L.lvr_create(cfg4)
        L.lvr_build(h4, Kd, Vd)
        step4 = step_on(h4)
        timed(step4, W_steps, 0)
        ms4 = timed(step4, K_steps, W_steps) / K_steps
        st4 = L.lvr_get_stats(h4, raise_on_overflow=False)
        b4 = st4["bytes_index"] + st4["bytes_keys"] + st4["bytes_attention"]
        res["paper_setting_r4"] = {"group_size": 4, "subspaces": args.subspaces, "us_per_step": round(ms4 * 1e3, 2),
                                   "f_scan": round(st4["keys_scanned"] / max(n_bh * st4["n_keys"], 1), 4),
                                   "index_bytes_per_key": round(st4["bytes_index"] / max(n_bh * st4["n_indexed"], 1), 1),
                                   "step_bytes": int(b4),
                                   "step_frac_of_peak": round(b4 / (ms4 * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        L.lvr_destroy(h4)

    # ---- the same keys with 8-bit centres, when the library's choice was 6 bits ----
    if full and not appending and legs and args.centres == "auto" and res["index_bytes_per_group"] == 108:
        h8 = L.lvr_create(make_cfg(group_size, "fp8"))
        L.lvr_build(h8, Kd, Vd)
        step8 = step_on(h8)
        timed(step8, W_steps, 0)
        ms8 = timed(step8, K_steps, W_steps) / K_steps
        st8 = L.lvr_get_stats(h8, raise_on_overflow=False)
        res["centres_fp8"] = {"us_per_step": round(ms8 * 1e3, 2),
                              "f_scan": round(st8["keys_scanned"] / max(n_bh * st8["n_keys"], 1), 4),
                              "index_bytes_per_key": round(st8["bytes_index"] / max(n_bh * st8["n_indexed"], 1), 1)}
        L.lvr_destroy(h8)

    # ---- CPU oracle on a bounded sample of the same workload (also checks recall) ----
    if cpu_seconds > 0:
        import oracle
        threads = oracle.max_threads()
        sigma = 1.0 / math.sqrt(d)
        tau_np = tau_all.cpu().numpy()
        done, cpu_s, recall_num, recall_den, spurious, worst = 0, 0.0, 0, 0, 0, 0.0
        sample_steps = []

        def compare(sets, o_ref, nb):
            nonlocal recall_num, recall_den, spurious, worst
            gi, gc, go = idx.cpu().numpy(), cnt.cpu().numpy(), out.cpu().numpy()
            for b in range(nb):
                for hh in range(Hq):
                    want = set(sets[b][hh].tolist())
                    got = set(gi[b, hh, :gc[b, hh]].tolist())
                    recall_num += len(want & got)
                    recall_den += len(want)
                    spurious += len(got - want)
                    if want == got:
                        e = float(np.abs(go[b, hh] - o_ref[b, hh]).max() / max(np.abs(o_ref[b, hh]).max(), 1e-30))
                        worst = max(worst, e)
        if appending:
            # the steps after the timed passes, one at a time with a synchronisation: the GPU's cache
            # after step t holds the prompt plus t+1 appended tokens, and so does the oracle's copy
            nb = B
            Kh = np.concatenate([K_bits, W.f32_to_bf16_bits(k_new_np).reshape(k_new_np.shape).transpose(1, 2, 0, 3)], axis=2)
            Vh = np.concatenate([V_bits, W.f32_to_bf16_bits(v_new_np).reshape(v_new_np.shape).transpose(1, 2, 0, 3)], axis=2)
            for t in range(next_t, next_t + n_verify):
                one_step(t)
                torch.cuda.synchronize()
                n_t = n0 + t + 1
                assert L.lvr_length(h)[0] == n_t
                tc = time.time()
                sets, counts, o_ref = oracle.decode_step(np.ascontiguousarray(Kh[:, :, :n_t]), np.ascontiguousarray(Vh[:, :, :n_t]),
                                                         q_np[t], tau_np[t], sigma, Hq, cap=cap)
                cpu_s += time.time() - tc
                compare(sets, o_ref, nb)
                sample_steps.append(t)
                done += 1
            what = f"{done} append+decode steps of config {cid} at {n0 + next_t + 1}..{n0 + next_t + n_verify} keys"
        else:
            # one sequence of the batch per sampled step keeps the sample bounded for batch 16
            nb = 1 if B > 1 else B
            while cpu_s < cpu_seconds and done < 8 * n_distinct:   # wraps around the distinct steps if they are few
                t = (done * 37) % n_distinct
                tc = time.time()
                sets, counts, o_ref = oracle.decode_step(K_bits[:nb], V_bits[:nb], q_np[t][:nb], tau_np[t][:nb], sigma, Hq, cap=cap)
                cpu_s += time.time() - tc
                L.lvr_decode_step(h, q_all[t], tau_all[t], out, idx, cnt)   # GPU result for the same step
                torch.cuda.synchronize()
                compare(sets, o_ref, nb)
                sample_steps.append(t)
                done += 1
            what = f"{done} decode steps of config {cid} (steps {sample_steps[:6]}...)"
        frac_of_step = nb / B
        res["cpu_baseline"] = {"value": round(done * frac_of_step / max(cpu_s, 1e-9), 4), "unit": "steps/s", "cores": threads,
                               "kind": "oracle",
                               "sample": f"{what}, {nb} of {B} sequences each, all {Hq} heads, brute force + attention"}
        res["recall"] = round(recall_num / max(recall_den, 1), 6)
        res["borderline_extra_keys"] = spurious
        res["max_attention_rel_err"] = float(f"{worst:.3e}")
    L.lvr_destroy(h)
    del Kd, Vd, q_all, tau_all
    torch.cuda.empty_cache()
    return res


def compact(r):
    """The block of a workload that is not the headline."""
    keep = {"us_per_step": round(r["ms_per_step"] * 1e3, 2), "steps_per_sec": round(1e3 / r["ms_per_step"], 1),
            "context": r["n_now"], "batch": r["B"],
            "kernel_frac_of_peak": r["roofline"]["frac"], "kernel_us": r["roofline"]["avg_launch_us"],
            "step_frac_of_peak": r["step_bytes"]["step_frac_of_peak"], "step_bytes": r["step_bytes"]["total"],
            "f_scan": r["f_scan"], "retrieved_per_head": r["retrieved_per_head"], "kernels_us": r["kernels_us"],
            "exact_filter_only_us": None if not r["exact_filter_only"] else r["exact_filter_only"]["us_per_step"],
            "dense_us": r["dense_baseline"]["us_per_step"],
            "speedup_over_dense": r["dense_baseline"]["speedup_of_sparse_path"]}
    for k in ("recall", "max_attention_rel_err", "cpu_baseline"):
        if k in r:
            keep[k] = r[k]
    return keep


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--config", type=int, default=3, choices=[2, 3, 4, 5])
    ap.add_argument("--group-size", type=int, default=DEFAULT_GROUP_SIZE,
                    help="r; 1 = every key its own group (centre = the key in 8 bits, radius = its rounding error)")
    ap.add_argument("--subspaces", type=int, default=4)
    ap.add_argument("--enclosing", choices=["ball", "aabb"], default="ball")
    ap.add_argument("--grouping", choices=["contiguous", "tree", "subspace"], default="contiguous",
                    help="'subspace': one tree grouping per subspace with per-key labels (the paper's own layout)")
    ap.add_argument("--centres", choices=["auto", "bf16", "fp8", "fp6"], default="auto",
                    help="storage of the centres: the cache's bf16, 8-bit e4m3 codes, or 6-bit e2m3 codes with a scale per 32 "
                         "coordinates; auto = the library's default (6-bit for single-key groups, else 8-bit, where supported)")
    ap.add_argument("--q-heads", type=int, default=0,
                    help="supplementary: query heads per sequence (8, 16, 32 or 64 over the workload's 8 KV heads; "
                         "default: the workload's 32)")
    ap.add_argument("--keys", choices=["workload", "local"], default="workload",
                    help="'local': supplementary cache whose keys have positional locality; not one of the five workloads")
    ap.add_argument("--concurrent-update", action="store_true",
                    help="group full buffers on a side stream (two-stream update); matters for --config 5")
    ap.add_argument("--offload", action="store_true",
                    help="offloaded mode: K and V in pinned host memory, only the index in HBM")
    ap.add_argument("--separate", action="store_true",
                    help="bound test and exact check as two launches (times the index search apart)")
    ap.add_argument("--attn-splits", type=int, default=0,
                    help="lvr_config.attn_splits: 0 = chosen per call, -1 = one workgroup per head, one launch")
    ap.add_argument("--rotate", type=int, default=4,
                    help="replicas of the index cycled through by the cache-cold pass (1 = skip that pass)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="CPU time budget of the oracle sample")
    ap.add_argument("--qualify-frac", type=float, default=None,
                    help="share of the keys that qualifies per head (default: the workload's); 0 = thresholds that nothing "
                         "reaches, which times the bound phase alone; not for the append workload")
    ap.add_argument("--query-workgroups", type=int, default=0,
                    help="lvr_config.query_workgroups: workgroups a range-query launch aims at (0 = the library's default)")
    ap.add_argument("--only", action="store_true", help="measure --config alone (no block for the other workloads)")
    ap.add_argument("--no-legs", action="store_true",
                    help="skip the exact-filter-only pass and the r = 4 pass (they launch the same kernel as the timed steps; "
                         "a profile of the run then shows the timed steps' launches alone)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the hot path is a single-GPU kernel pipeline; "
              "no collective or multi-rank code exists). Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2605_06763_amd as L

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = torch.device("cuda:0")
    cid = args.config
    steps = args.steps
    if cid == 5 and steps == 256 and not any(a.startswith("--steps") for a in sys.argv[1:]):
        steps = 1024                     # the append workload: a longer run, the cache grows as it goes
    cpu_s = 0.0 if args.no_cpu_baseline else args.cpu_seconds
    r = measure(cid, args, group_size=args.group_size, steps=steps, warmup=args.warmup, full=True, cpu_seconds=cpu_s,
                legs=not args.no_legs)
    ms_per_step = r["ms_per_step"]
    B, Hq = r["B"], r["Hq"]
    appending = cid == 5
    fp8 = r["index_bytes_per_group"] < (512 if args.enclosing == "aabb" else 256)
    result = {
        "metric": "decode steps/sec (index query + sparse attention)",
        "value": round(1e3 / ms_per_step, 2),
        "unit": "steps/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "us_per_step": round(ms_per_step * 1e3, 2),
        "queries_per_sec": round(1e3 / ms_per_step * B * Hq, 1),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"config{cid}:{r['name']}" + (" [supplementary: keys with positional locality]" if args.keys == "local" else "") + (f" [supplementary: {Hq} query heads]" if args.q_heads else "")
                               + (f" [supplementary: {args.qualify_frac} of the keys qualify]" if args.qualify_frac is not None else ""), "batch": B, "n_q_heads": Hq, "n_kv_heads": r["Hkv"],
                   "head_dim": r["d"], "context": r["n_now"], "kv_storage": "bf16", "group_size": args.group_size,
                   "subspaces": args.subspaces, "attn_splits": args.attn_splits, "grouping": args.grouping,
                   "centres": "fp6" if r["index_bytes_per_group"] == 108 else ("fp8" if fp8 else "bf16"), "enclosing": args.enclosing,
                   "index_bytes_per_key": r["index_bytes_per_key"],
                   "step": "append+query+attention" if appending else "query+attention",
                   "update": "two-stream" if args.concurrent_update else "single-stream",
                   "kv_memory": "host (pinned, read in place)" if args.offload else "hbm",
                   "device_bytes": int(L.lvr_arena_bytes(r["cfg"])), "host_bytes": int(L.lvr_host_bytes(r["cfg"]))},
    }
    for k in ("roofline", "step_bytes", "set_turnover_per_step", "f_scan", "groups_surviving_frac", "retrieved_per_head",
              "kernels_us", "profiled_us_per_step", "exact_filter_only", "dense_baseline", "paper_setting_r4", "centres_fp8",
              "step_us_distribution", "cache_cold", "build_ms", "cpu_baseline", "recall", "borderline_extra_keys",
              "max_attention_rel_err"):
        if k in r:
            result[k] = r[k]

    # ---- one plain device copy of known size (256 MiB read, 256 MiB written): the dispatch the offline
    # counter runs (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this command) are calibrated against ----
    src = torch.empty(1 << 28, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    dst.copy_(src)
    ms_copy = timed(lambda t: dst.copy_(src), 4) / 4
    result["device_copy_GBs"] = round(2 * src.numel() / (ms_copy * 1e-3) / 1e9, 1)
    del src, dst

    # ---- the read-only streaming rate of this machine: the practical ceiling of the HBM-bound kernels ----
    ceiling, shape = stream_read_ceiling(L, dev)
    result["stream_read_GBs"] = round(ceiling, 1)
    result["stream_read_workgroups"] = shape
    result["roofline"]["frac_of_stream_read"] = round(result["roofline"]["achieved"] / ceiling, 4)

    # ---- the other workloads, compactly, in the same run ----
    if not args.only and args.keys == "workload" and not args.q_heads and not args.offload:
        others = {}
        for oc in (2, 4, 5):
            if oc == cid:
                continue
            o_steps = {2: 256, 4: 64, 5: 1024}[oc]
            ro = measure(oc, args, group_size=args.group_size, steps=o_steps, warmup=args.warmup, full=False,
                         cpu_seconds=0.0 if args.no_cpu_baseline else min(args.cpu_seconds, 5.0))
            others[f"config{oc}"] = compact(ro)
        result["other_configs"] = others
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
