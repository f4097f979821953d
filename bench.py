#!/usr/bin/env python3
"""Decode-step benchmark of the Louver hot path on one MI355X.

One step = one pass of the per-step hot path over one batch of synthetic input: range query
(bound pruning + exact filter) followed by sparse attention over the retrieved keys, through
the C ABI (lvr_decode_step).  For the append workload (config 5) a step first appends the
step's new key/value (lvr_append_decode_step: both in one call).  Inputs (K, V, all queries, all thresholds) are resident in HBM
before the timed region starts.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config {2,3,4,5}]

Default workload: config 3 (GQA 32/8 heads, d=128, 131072 keys, batch 1, bf16, 0.5 % of the
keys qualify per head, query drifting over 256 consecutive steps) — the 128k-context case the
target is stated on.
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--config", type=int, default=3, choices=[2, 3, 4, 5])
    ap.add_argument("--group-size", type=int, default=4)
    ap.add_argument("--subspaces", type=int, default=4)
    ap.add_argument("--enclosing", choices=["ball", "aabb"], default="ball")
    ap.add_argument("--grouping", choices=["contiguous", "tree"], default="contiguous")
    ap.add_argument("--centres", choices=["auto", "bf16", "fp8"], default="auto",
                    help="storage of the centres: the cache's bf16, or 8-bit e4m3 codes (half the index read); "
                         "auto = the library's default (8-bit where supported)")
    ap.add_argument("--q-heads", type=int, default=0,
                    help="supplementary: query heads per sequence (8, 16, 32 or 64 over the workload's 8 KV heads; "
                         "default: the workload's 32)")
    ap.add_argument("--keys", choices=["workload", "local"], default="workload",
                    help="'local': supplementary cache whose keys have positional locality (the pruned regime); "
                         "not one of the five workloads")
    ap.add_argument("--concurrent-update", action="store_true",
                    help="group full buffers on a side stream (two-stream update); matters for --config 5")
    ap.add_argument("--offload", action="store_true",
                    help="offloaded mode: K and V in pinned host memory, only the index in HBM")
    ap.add_argument("--separate", action="store_true",
                    help="bound test and exact check as two launches (times the index search apart)")
    ap.add_argument("--attn-splits", type=int, default=0,
                    help="lvr_config.attn_splits: 0 = default (64 splits + combine launch), -1 = one workgroup per head, one launch")
    ap.add_argument("--rotate", type=int, default=4,
                    help="replicas of the index cycled through by the cache-cold pass (1 = skip that pass)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="CPU time budget of the oracle sample")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the hot path is a single-GPU kernel pipeline; "
              "no collective or multi-rank code exists). Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2605_06763_amd as L
    import workloads as W

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = torch.device("cuda:0")
    cid = args.config
    c = W.CONFIGS[cid]
    B, Hq, Hkv, d, n0 = c["batch"], c["n_q_heads"], c["n_kv_heads"], c["head_dim"], c["n"]
    if args.q_heads:
        assert args.q_heads in (8, 16, 32, 64) and cid != 5, "--q-heads: 8, 16, 32 or 64, not with the append workload"
        Hq = args.q_heads
    G = Hq // Hkv
    K_steps, W_steps = args.steps, args.warmup
    total_steps = K_steps + W_steps
    appending = cid == 5
    log(f"[bench] config {cid} {c['name']}: generating inputs")
    t0 = time.time()
    if args.keys == "local":
        assert not (cid == 5), "the supplementary cache has no append stream"
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
        n_distinct = total_steps
        q_np = W.drift_queries(5, n_distinct)
    else:
        n_distinct = 16
        q_np = np.stack([W.make_queries(cid, step=t, n_q_heads=Hq) for t in range(n_distinct)])
    q_all = torch.from_numpy(q_np).to(dev)

    capacity = n0 + (total_steps + K_steps + 64 if appending else 0)
    cfg = L.make_config(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, kv_dtype=L.LVR_BF16,
                        group_size=args.group_size, n_subspaces=args.subspaces, buffer_size=256, capacity=capacity,
                        enclosing=L.LVR_ENCLOSE_AABB if args.enclosing == "aabb" else L.LVR_ENCLOSE_BALL,
                        grouping=L.LVR_GROUP_TREE if args.grouping == "tree" else L.LVR_GROUP_CONTIGUOUS,
                        attn_splits=args.attn_splits,
                        index_dtype={"auto": L.LVR_INDEX_AUTO, "bf16": L.LVR_INDEX_SAME, "fp8": L.LVR_INDEX_FP8}[args.centres],
                        flags=(L.LVR_CONCURRENT_UPDATE if args.concurrent_update else 0)
                        | (L.LVR_KV_IN_HOST_MEMORY if args.offload else 0)
                        | (L.LVR_SEPARATE_KERNELS if args.separate else 0))
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
        T_all = total_steps + K_steps                       # timed pass, then the profiled pass
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
            if t % 512 == 511:
                torch.cuda.synchronize()
                log(f"[bench] thresholds placed for {t + 1} of {T_all} steps")
        del Kfull
    else:
        kq = int(math.ceil(c["qualify_frac"] * n0))
        tau_all = torch.empty((n_distinct, B, Hq), dtype=torch.float32, device=dev)
        prev, turn = None, []
        for t in range(n_distinct):
            sc = scores_on_gpu(Kd, q_all[t], G)
            tau_all[t] = kth_midpoint_tau(sc, kq)
            if cid == 3:                                    # drifting queries: how much of the set is new each step
                cur = sc >= tau_all[t].unsqueeze(-1)
                if prev is not None:
                    turn.append((cur & ~prev).sum(-1).float().div(kq).mean())
                prev = cur
            if t % 32 == 31:
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

    def one_step(t):
        if appending:
            # the step's token joins the cache, then the query is answered: one call
            L.lvr_append_decode_step(h, k_args[t], v_args[t], q_args[t % n_distinct], tau_args[t], out_a, idx_a, cnt_a,
                                     st_arg)
        else:
            L.lvr_decode_step(h, q_args[t % n_distinct], tau_args[t % n_distinct], out_a, idx_a, cnt_a, st_arg)

    def run(n_steps, first):
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        ev0.record()
        for t in range(first, first + n_steps):
            one_step(t)
        ev1.record()
        torch.cuda.synchronize()
        return ev0.elapsed_time(ev1)

    # ---- warm-up, then the timed region: exactly K steps ----
    run(W_steps, 0)
    ms_total = run(K_steps, W_steps)
    ms_per_step = ms_total / K_steps
    st = L.lvr_get_stats(h, raise_on_overflow=False)
    if st["overflow"]:
        log("[bench] WARNING: a retrieved set exceeded cap; lists were truncated")
    n_now = st["n_keys"]

    # ---- distribution over steps: one event after every step of another pass over the same K steps
    # (each figure includes the event's own cost, about 1 us; the mean above does not) ----
    step_dist = None
    if not appending:
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
    if not appending and args.rotate > 1:
        reps = [h]
        for _ in range(args.rotate - 1):
            hr = L.lvr_create(cfg)
            L.lvr_build(hr, Kd, Vd)
            reps.append(hr)
        def run_rot(n_steps, first):
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            ev0.record()
            for t in range(first, first + n_steps):
                L.lvr_decode_step(reps[t % len(reps)], q_args[t % n_distinct], tau_args[t % n_distinct], out_a, idx_a,
                                  cnt_a, st_arg)
            ev1.record()
            torch.cuda.synchronize()
            return ev0.elapsed_time(ev1)
        run_rot(max(W_steps, len(reps)), 0)
        cold_ms = run_rot(K_steps, W_steps) / K_steps
        for hr in reps[1:]:
            L.lvr_destroy(hr)
        cold = {"replicas": len(reps), "us_per_step": round(cold_ms * 1e3, 2)}

    # ---- per-kernel time with HIP events on the launch stream (same K steps again) ----
    L.lvr_profile_enable(h, 8 * K_steps + 64)
    first = total_steps if appending else W_steps
    ms_prof_total = run(K_steps, first)
    prof = L.lvr_profile_read(h)
    L.lvr_profile_enable(h, 0)
    kern = {k: dict(avg_us=1e3 * ms / max(nl, 1), launches=nl) for k, (ms, nl) in prof.items() if nl}
    st = L.lvr_get_stats(h, raise_on_overflow=False)

    # ---- dense full-KV attention on the same arena ----
    def run_dense(n_steps):
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        ev0.record()
        for t in range(n_steps):
            L.lvr_dense_attention(h, q_args[t % n_distinct], out_a, st_arg)
        ev1.record()
        torch.cuda.synchronize()
        return ev0.elapsed_time(ev1) / n_steps
    run_dense(max(W_steps, 4))
    dense_ms = run_dense(K_steps)
    n_dense = L.lvr_length(h)[0]
    dense_bytes = B * Hkv * n_dense * 2 * d * 2

    # ---- a plain device copy, for the box's achievable streaming rate ----
    src = torch.empty(1 << 28, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    dst.copy_(src)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    ev0.record()
    for _ in range(10):
        dst.copy_(src)
    ev1.record()
    torch.cuda.synchronize()
    copy_gbs = 10 * 2 * src.numel() / (ev0.elapsed_time(ev1) * 1e-3) / 1e9
    del src, dst

    index_bytes_per_group = st["bytes_index"] // max(st["groups_scored"], 1)
    # ---- algorithmic bytes of the dominant kernel ----
    # fused range-query kernel (bound test + exact check): per (sequence, KV head)
    #   groups * (d*c + S*4) bytes of centres (c = 1 byte per coordinate as e4m3 codes, 2 as bf16) and radii
    #   +  keys_scanned * d*2 bytes of key rows
    n_bh = B * Hkv
    filt = kern.get("filter", dict(avg_us=float("nan")))
    if args.separate and "prune" in kern:
        filt = dict(avg_us=filt["avg_us"] + kern["prune"]["avg_us"])
    query_bytes = st["bytes_index"] + st["bytes_keys"]
    achieved = query_bytes / (filt["avg_us"] * 1e-6) / 1e9
    step_bytes = st["bytes_index"] + st["bytes_keys"] + st["bytes_attention"]
    roofline = dict(bound="hbm", kernel="prune_mfma_kernel+filter_mfma_kernel" if args.separate else "query_fused_kernel", achieved=round(achieved, 1), peak=HBM_PEAK_GBS,
                    unit="GB/s", frac=round(achieved / HBM_PEAK_GBS, 4), traffic=None,
                    bytes_per_launch=int(query_bytes), avg_launch_us=round(filt["avg_us"], 2))
    # HBM bytes per launch measured offline with rocprofv3 --pmc (profiles/), when this workload was profiled
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if (os.path.exists(tpath) and args.group_size == 4 and args.subspaces == 4 and args.keys == "workload"
            and args.enclosing == "ball" and args.centres == "auto" and not args.offload and not args.separate and args.grouping == "contiguous"
            and not args.q_heads):
        for line in open(tpath):
            f = line.split()
            if len(f) == 3 and f[0] == f"config{cid}" and f[1] == "query_fused_kernel":
                roofline["traffic"] = int(f[2])

    result = {
        "metric": "decode steps/sec (index query + sparse attention)",
        "value": round(1e3 / ms_per_step, 2),
        "unit": "steps/s",
        "n_gpus": 1,
        "steps": K_steps,
        "warmup": W_steps,
        "ms_per_step": round(ms_per_step, 5),
        "us_per_step": round(ms_per_step * 1e3, 2),
        "queries_per_sec": round(1e3 / ms_per_step * B * Hq, 1),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"config{cid}:{c['name']}" + (" [supplementary: keys with positional locality]" if args.keys == "local" else "") + (f" [supplementary: {Hq} query heads]" if args.q_heads else ""), "batch": B, "n_q_heads": Hq, "n_kv_heads": Hkv,
                   "head_dim": d, "context": int(n_now), "kv_storage": "bf16", "group_size": args.group_size,
                   "subspaces": args.subspaces, "attn_splits": args.attn_splits, "grouping": args.grouping,
                   "centres": ("fp8" if index_bytes_per_group < (512 if args.enclosing == "aabb" else 256) else "bf16"), "enclosing": args.enclosing,
                   "step": "append+query+attention" if appending else "query+attention",
                   "update": "two-stream" if args.concurrent_update else "single-stream",
                   "kv_memory": "host (pinned, read in place)" if args.offload else "hbm",
                   "device_bytes": int(L.lvr_arena_bytes(cfg)), "host_bytes": int(L.lvr_host_bytes(cfg))},
        "roofline": roofline,
        "step_bytes": {"index": int(st["bytes_index"]), "keys": int(st["bytes_keys"]),
                       "attention": int(st["bytes_attention"]), "total": int(step_bytes),
                       "step_GBs": round(step_bytes / (ms_per_step * 1e-3) / 1e9, 1),
                       "step_frac_of_peak": round(step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
        "set_turnover_per_step": None if set_turnover is None else round(set_turnover, 4),
        "f_scan": round(st["keys_scanned"] / max(n_bh * st["n_keys"], 1), 4),
        "groups_surviving_frac": round(st["groups_surviving"] / max(st["groups_scored"], 1), 4),
        "retrieved_per_head": round(st["keys_emitted"] / (B * Hq), 1),
        "kernels_us": {k: round(v["avg_us"], 2) for k, v in kern.items()},
        "profiled_us_per_step": round(ms_prof_total / K_steps * 1e3, 2),
        "dense_baseline": {"us_per_step": round(dense_ms * 1e3, 2), "bytes": int(dense_bytes),
                           "GBs": round(dense_bytes / (dense_ms * 1e-3) / 1e9, 1),
                           "frac_of_peak": round(dense_bytes / (dense_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                           "speedup_of_sparse_path": round(dense_ms / ms_per_step, 3)},
        "step_us_distribution": step_dist,
        "cache_cold": cold,
        "device_copy_GBs": round(copy_gbs, 1),
        "build_ms": round(build_ms, 3),
    }

    # ---- CPU oracle on a bounded sample of the same workload (also checks recall) ----
    if not args.no_cpu_baseline and not appending:
        import oracle
        threads = oracle.max_threads()
        sigma = 1.0 / math.sqrt(d)
        tau_np = tau_all.cpu().numpy()
        # one sequence of the batch per sampled step keeps the sample bounded for batch 16
        nb = 1 if B > 1 else B
        done, cpu_s, recall_num, recall_den, spurious, worst = 0, 0.0, 0, 0, 0, 0.0
        sample_steps = []
        while cpu_s < args.cpu_seconds and done < 8 * n_distinct:   # wraps around the distinct steps if they are few
            t = (done * 37) % n_distinct
            tc = time.time()
            sets, counts, o_ref = oracle.decode_step(K_bits[:nb], V_bits[:nb], q_np[t][:nb], tau_np[t][:nb], sigma, Hq, cap=cap)
            cpu_s += time.time() - tc
            # GPU result for the same step
            L.lvr_decode_step(h, q_all[t], tau_all[t], out, idx, cnt)
            torch.cuda.synchronize()
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
            sample_steps.append(t)
            done += 1
        frac_of_step = nb / B
        result["cpu_baseline"] = {"value": round(done * frac_of_step / cpu_s, 4), "unit": "steps/s", "cores": threads,
                                  "kind": "oracle",
                                  "sample": f"{done} decode steps of config {cid} (steps {sample_steps[:6]}...), "
                                            f"{nb} of {B} sequences each, all {Hq} heads, brute force + attention"}
        result["recall"] = round(recall_num / max(recall_den, 1), 6)
        result["borderline_extra_keys"] = spurious
        result["max_attention_rel_err"] = float(f"{worst:.3e}")
    L.lvr_destroy(h)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
