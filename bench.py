#!/usr/bin/env python3
"""Benchmark of the CSAttention decode step on one MI355X.

A "step" is one pass of the whole hot path through the C-ABI library - the decode step (centroid
scoring, row gather + score accumulation, Top-K, gathered attention) followed by the append of the
next K/V row, as the one call csa_decode_step_append (or, with --two-calls, csa_decode_step then
csa_append_kv) - over one batch of synthetic input that is already resident in HBM.  Every step
uses a fresh query, so the 256 MiB last-level cache cannot replay the previous step.

Prints ONE JSON line.  One GPU only.
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBPS = 8000.0  # MI355X published HBM3E bandwidth


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="cfg4",
                    help="benchmark configuration cfg1..cfg4, or paper_s8 (the paper's default geometry)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--partition-keys", type=int, default=0)
    ap.add_argument("--centroids", default="library", choices=("library", "sample"),
                    help="library: the centroids come from the library's own clustering of the prefill "
                         "queries (csa_prefill; --cluster-iters steps, --cluster-batches classes); sample: "
                         "normalised prefill queries picked at random, then csa_build_tables")
    ap.add_argument("--search-period", type=int, default=1,
                    help="schedule 'keep ratio + search period': search every P-th step, reuse the "
                         "index set in between (csa_decode_step_reuse)")
    ap.add_argument("--keep-ratio", type=float, default=0.0,
                    help="budget k = round(ratio * N_pre) instead of the config's (0 = config)")
    ap.add_argument("--stream-window", type=int, default=0,
                    help="R > 0: streaming updates - csa_append_kv try-inserts every new key into the "
                         "tables and only the last R positions are attended unconditionally")
    ap.add_argument("--cluster", action="store_true",
                    help="measure the offline query clustering (csa_cluster_queries) of ONE sequence of "
                         "the config instead of the decode step: seeding + Lloyd steps, and the "
                         "assignment kernel against the bf16 matrix-core peak")
    ap.add_argument("--cluster-iters", type=int, default=10)
    ap.add_argument("--cluster-batches", type=int, default=8,
                    help="mini-batch clustering: the points are dealt into this many classes, the seeding "
                         "runs over the first and step t over class t %% batches (1 = full batch)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run three plain 1 GiB device-to-device copies before the timed region, "
                         "so that a counter run has a kernel of known HBM traffic to scale by")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--row-gather-floor", action="store_true",
                    help="also time bench_aids/row_gather_probe.hip (bare fetches of K and V rows) over the distinct "
                         "rows the last step's attention had to read, and report it as row_gather_floor")
    ap.add_argument("--graph-iters", type=int, default=8,
                    help="also time the steps as replays of a captured HIP graph of this many iterations "
                         "(csa_decode_step_append_replayable); 0 = off")
    ap.add_argument("--also", default="auto",
                    help="a second workload measured in the same process and reported under 'also' "
                         "(auto = cfg2 when the main workload is cfg4; none = off)")
    ap.add_argument("--two-calls", action="store_true",
                    help="csa_decode_step then csa_append_kv instead of the one-call csa_decode_step_append")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU (no collectives, no sharding); "
            f"--gpus {args.gpus} is not supported. The path shards over (sequence, KV head) "
            "with no exchange between GPUs.")
        sys.exit(2)

    import torch
    from paper_2604_08584_amd import binding
    from paper_2604_08584_amd.workload import CONFIGS
    binding.lib()  # fail loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    if args.cluster:
        return cluster_bench(args, CONFIGS[args.config])
    result = decode_bench(args, args.config, args.steps, args.warmup, not args.no_cpu_baseline)
    # the other headline configuration of the metric (batch 1 at 128K next to batch 8), in the same
    # process, after the first one's buffers are gone; config.workload stays the first one
    also = args.also if args.also != "auto" else ("cfg2" if args.config == "cfg4" else "none")
    plain = (args.search_period == 1 and args.keep_ratio == 0 and args.stream_window == 0)
    if also != "none" and also != args.config and plain:
        import gc
        gc.collect()
        torch.cuda.empty_cache()
        r2 = decode_bench(args, also, min(args.steps, CONFIGS[also].steps), args.warmup, False)
        keep = ("value", "unit", "steps", "warmup", "ms_per_step", "config", "tokens_per_s", "step_algorithmic_bytes",
                "step_hbm_gbps", "step_frac_of_peak", "step_us_percentiles", "host_issue_us_per_step", "graph_replay_us_per_step", "stage_us",
                "search_us", "roofline", "footprint")
        result["also"] = {also: {k_: r2[k_] for k_ in keep if k_ in r2}}
    print(json.dumps(result, ensure_ascii=False), flush=True)


def source_sha():
    """Hash of the kernel sources: a stored counter figure is only quoted for the kernels it was taken on."""
    import hashlib
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2604_08584_amd", "csrc")
    for f in ("attention.hip", "common.h"):
        h.update(open(os.path.join(d, f), "rb").read())
    return h.hexdigest()[:12]


def decode_bench(args, name, K, W, with_cpu):
    """One workload: K timed steps after W warm-up steps; returns the result dictionary."""
    import torch
    from paper_2604_08584_amd import binding
    from paper_2604_08584_amd.workload import (CONFIGS, algorithmic_bytes_per_head, make_inputs,
                                                 paginate)
    dev = "cuda"
    base = CONFIGS[name]
    streaming = args.stream_window > 0
    # with streaming updates the tables keep the appended keys, so the context cannot be rewound
    # after the warm-up: the timed steps simply continue from there
    K_prof = min(K, 16) if streaming else K   # steps of the per-kernel event pass
    w = dataclasses.replace(base, steps=(W + K + K_prof) if streaming else max(K, W, 1))
    if args.keep_ratio > 0:
        w = dataclasses.replace(w, k=int(round(args.keep_ratio * w.n_pre)))
    period = max(1, args.search_period)
    B, Hq, Hkv, G = w.batch, w.n_q_heads, w.n_kv_heads, w.group
    log(f"[bench] workload {w.name}: B={B} Hq={Hq} Hkv={Hkv} N_pre={w.n_pre} C={w.C} L={w.L} "
        f"m={w.m} k={w.k} pre_appended={w.pre_appended} page={w.page_size} steps={K} warmup={W}")

    t0 = time.time()
    library_centroids = args.centroids == "library"
    inp = make_inputs(w, seed=args.seed, device=dev, keep_q_pre=library_centroids)
    torch.cuda.synchronize()
    log(f"[bench] synthetic inputs: {time.time() - t0:.1f} s")
    if w.page_size:
        k_store, bt = paginate(inp["k_cache"], w.page_size, args.seed, w.name)
        v_store, _ = paginate(inp["v_cache"], w.page_size, args.seed, w.name, bt)
    else:
        k_store, v_store, bt = inp["k_cache"], inp["v_cache"], None
    ctx = binding.Context(k_store, v_store, bt, batch=B, n_q_heads=Hq, n_kv_heads=Hkv,
                          n_centroids=w.C, list_len=w.L, n_probe=w.m, budget_k=w.k,
                          max_ctx=w.max_ctx, page_size=w.page_size, score_frac_bits=-1,
                          partition_keys=args.partition_keys, n_subspaces=w.n_sub,
                          stream_window=args.stream_window)
    t0 = time.time()
    if library_centroids:
        # the offline prefill as the library does it (Sec. 3.2): clustering of the prefill queries, then
        # the table build, in one call
        import numpy as np
        S_ = w.n_sub
        cent = torch.empty(B, Hkv, S_, w.C, w.head_dim // S_, dtype=torch.bfloat16, device=dev)
        u_seed = np.random.default_rng(args.seed).uniform(size=(B, Hkv, S_, w.C)).astype(np.float32)
        binding.csa_prefill(ctx.ctx, inp["q_pre"], w.n_pre, args.cluster_iters, max(1, args.cluster_batches), u_seed, cent)
        inp["centroids"] = cent.view(B, Hkv, w.C, w.head_dim) if S_ == 1 else cent
        del inp["q_pre"]
    else:
        ctx.build_tables(inp["centroids"], w.n_pre)
    torch.cuda.synchronize()
    t_build = time.time() - t0
    log(f"[bench] {'csa_prefill (clustering + tables)' if library_centroids else 'csa_build_tables'}: {t_build:.2f} s "
        f"(F = {binding.csa_score_frac_bits(ctx.ctx)})")

    q_steps, k_new, v_new = inp["q_steps"], inp["k_new"], inp["v_new"]

    done = [0]   # decode steps taken since the last rewind

    def reset():
        if streaming:   # never rewinds; only the keys appended before the first step are due once
            if binding.csa_context_len(ctx.ctx)[1] == w.n_pre:
                for t in range(w.pre_appended):
                    ctx.append_kv(k_new[t], v_new[t])
            return
        done[0] = 0
        binding.csa_set_context_len(ctx.ctx, w.n_pre)
        for t in range(w.pre_appended):
            ctx.append_kv(k_new[t], v_new[t])

    def run(n_steps):
        first = done[0]
        done[0] += n_steps
        for s in range(first, first + n_steps):
            t = w.pre_appended + s
            if args.two_calls:
                if s % period == 0:
                    ctx.decode_step(q_steps[t])
                else:
                    ctx.decode_step_reuse(q_steps[t])
                ctx.append_kv(k_new[t], v_new[t])
            elif s % period == 0:
                ctx.decode_step_append(q_steps[t], k_new[t], v_new[t])
            else:
                ctx.decode_step_reuse_append(q_steps[t], k_new[t], v_new[t])

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)          # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    # ---- clocks: the chip has idled through the host-side set-up, and a short warm-up (a few steps are
    # a few milliseconds) leaves it short of its sustained clock; some tens of milliseconds of the same
    # steps first, untimed like the warm-up
    if not streaming:
        n_ramp = min(64, w.steps)
        for _ in range((128 + n_ramp - 1) // n_ramp):
            reset()
            run(n_ramp)
        torch.cuda.synchronize()
    # ---- warm-up, then the timed region (exactly K steps)
    reset()
    run(W)
    reset()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(K)
    issued = time.perf_counter() - t0       # host time to enqueue the K steps (no waiting)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    us_per_step = elapsed / K * 1e6
    sel_mean = float(ctx.sel_count.float().mean().item())
    # a cheap sanity check of the last timed step (parity proper is the tests' job)
    sel_t, cnt_t = ctx.sel, ctx.sel_count
    n_end = binding.csa_context_len(ctx.ctx)[1]
    valid = torch.arange(sel_t.shape[-1], device=dev).view(1, 1, -1) < cnt_t.unsqueeze(-1)
    checks = dict(finite_out=bool(torch.isfinite(ctx.out).all().item()),
                  sel_count_min=int(cnt_t.min().item()), sel_count_max=int(cnt_t.max().item()),
                  sel_ascending=bool((~(valid[..., 1:]) | (sel_t[..., 1:] > sel_t[..., :-1])).all().item()),
                  sel_in_range=bool((~valid | ((sel_t >= 0) & (sel_t < n_end))).all().item()),
                  sel_padded=bool((valid | (sel_t == -1)).all().item()) if w.k else True)
    assert all(v for k_, v in checks.items() if isinstance(v, bool)), f"last step failed its sanity check: {checks}"

    # ---- the same K steps as replays of a captured HIP graph of `graph_iters` iterations
    # (csa_decode_step_append_replayable: the position lives on the device), each iteration of the
    # graph with its own query, so the host issues one launch per graph_iters steps
    graph_us = None
    gi = args.graph_iters
    if gi > 0 and period == 1 and not streaming and not args.two_calls and K >= gi:
        reset()
        run(1)                      # (first-use paths run outside the capture)
        reset()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.graph(g, stream=side):
            for t in range(gi):
                ctx.decode_step_append_replayable(q_steps[w.pre_appended + t], k_new[w.pre_appended + t],
                                                  v_new[w.pre_appended + t])
        reset()                     # (the capture advanced the host-side count only)
        for _ in range(max(1, W // gi)):
            g.replay()
        reset()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(K // gi):
            g.replay()
        torch.cuda.synchronize()
        graph_us = (time.perf_counter() - t0) / (K // gi * gi) * 1e6
        binding.csa_sync_context_len(ctx.ctx)
        del g

    # ---- per-step latency spread: an event pair around every step of one more pass (the library
    # launches on torch's current stream, so torch events bracket its kernels); streaming runs,
    # which cannot replay their steps, skip it
    step_pct = None
    if not streaming:
        reset()
        torch.cuda.synchronize()
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(K + 1)]
        marks[0].record()
        for i in range(K):
            run(1)
            marks[i + 1].record()
        torch.cuda.synchronize()
        per = sorted(marks[i].elapsed_time(marks[i + 1]) * 1e3 for i in range(K))
        step_pct = {f"p{q_}": round(per[min(K - 1, int(q_ / 100.0 * K))], 2) for q_ in (50, 90, 99)}

    # ---- second pass with per-kernel HIP events: over the same K steps, or - with streaming
    # updates, where steps cannot be replayed - over the next K_prof steps
    reset()
    binding.csa_profile_enable(ctx.ctx, True)
    run(K_prof)
    torch.cuda.synchronize()
    prof = binding.csa_profile_read(ctx.ctx)
    binding.csa_profile_enable(ctx.ctx, False)
    # per launch of each kernel (search kernels run on every period-th step only)
    stage_us = {name: (ms / max(n, 1) * 1e3) for name, (ms, n) in prof.items() if n > 0}

    # ---- algorithmic bytes (per step, mean appended count over the timed steps)
    # keys attended unconditionally: all appended ones, or the recent window
    t_mean = float(args.stream_window) if streaming else w.pre_appended + (K - 1) / 2.0
    per_head = algorithmic_bytes_per_head(w, t_mean)
    n_search = (K + period - 1) // period
    step_bytes = B * Hq * ((per_head["centroids"] + per_head["table_rows"]) * n_search / K
                           + per_head["kv_rows"] + per_head["io"])
    step_bytes_are = "per query head (rows shared by the heads of a KV head counted per head)"
    # dominant kernel = the gathered attention.  Its algorithmic bytes per launch: per query head the
    # K and V rows it attends, q and the index list - every head's rows counted separately, as the
    # method's cost model counts them (a row picked by several heads of a KV head counts once per
    # head, although it comes from HBM once and from L2 for the others).  Beside it, measured live:
    # the DISTINCT rows per (sequence, KV head) - the union of the G heads' index sets of the last
    # step - which is what must come from HBM (distinct_*), and the counter traffic of a stored
    # rocprofv3 run when it was taken on these kernel sources (traffic_*).  Schedule runs (larger
    # keep ratios), where the heads overlap so much that the per-head rate exceeds the HBM peak, take
    # the distinct rows for `achieved`.
    att_us = stage_us["attention_split"]
    n_now = binding.csa_context_len(ctx.ctx)[1]
    ws_now = max(0, n_now - args.stream_window) if streaming else w.n_pre
    sel_l = ctx.sel.view(B, Hkv, G * max(w.k, 1)).long()
    need = torch.zeros(B, Hkv, w.max_ctx + 1, dtype=torch.bool, device=dev)
    if w.k:
        need.scatter_(2, torch.where(sel_l >= 0, sel_l, torch.full_like(sel_l, w.max_ctx)), True)
    need[:, :, w.max_ctx] = False
    distinct_sel = int(need.sum().item())
    sum_sel = int(ctx.sel_count.sum().item())
    del need, sel_l
    # (the window of the last step is the largest of the run; scaled to the run's mean window)
    share = distinct_sel / max(sum_sel, 1)               # distinct / per-head selected rows
    rows_per_head = w.k * share + t_mean / G
    att_bytes = B * Hq * (2 * rows_per_head * w.head_dim * 2 + w.head_dim * 2 + w.k * 4)
    per_head_bytes = B * Hq * (per_head["kv_rows"] + w.head_dim * 2 + w.k * 4)
    schedule_run = period > 1 or args.keep_ratio > 0
    if schedule_run:   # (the per-head count would exceed the HBM peak: count the distinct K/V rows)
        step_bytes = B * Hq * ((per_head["centroids"] + per_head["table_rows"]) * n_search / K
                               + 2 * rows_per_head * w.head_dim * 2 + per_head["io"])
        step_bytes_are = "K/V rows as the union of the heads' index sets per KV head; tables, centroids, q, out, sel per head"
    main_bytes = att_bytes if schedule_run else per_head_bytes
    achieved = main_bytes / (att_us * 1e-6) / 1e9
    traffic = traffic_src = None
    tf = os.path.join(ROOT, "profiles", f"attention_split_{w.name}_hbm_traffic.txt")
    if os.path.exists(tf) and not schedule_run and not streaming:
        txt = open(tf).read()
        mt = re.search(r"traffic_bytes_per_launch:\s*([0-9.eE+]+)", txt)
        ms = re.search(r"kernel_source_sha:\s*([0-9a-f]+)", txt)
        if mt and ms and ms.group(1) == source_sha():
            traffic = float(mt.group(1))
            traffic_src = f"profiles/{os.path.basename(tf)} (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE; kernel sources {ms.group(1)})"
        else:
            traffic_src = (f"profiles/{os.path.basename(tf)} was taken on other kernel sources "
                           f"({ms.group(1) if ms else 'unstamped'} != {source_sha()}): not quoted")
    roofline = dict(kernel="k_attention_split", bound="hbm", achieved=round(achieved, 1),
                    peak=PEAK_HBM_GBPS, unit="GB/s", frac=round(achieved / PEAK_HBM_GBPS, 4),
                    traffic=traffic, traffic_source=traffic_src,
                    algorithmic_bytes_per_launch=int(main_bytes),
                    algorithmic_bytes_are=("K/V rows of the union of the G heads' index sets per KV head + window rows + q "
                                           "+ index lists" if schedule_run else
                                           "per query head: 2 (k + t) rows of 256 B + q + index list, times B Hq heads "
                                           "(rows shared by the heads of a KV head counted once per head)"),
                    distinct_bytes_per_launch=int(att_bytes),
                    distinct_gbps=round(att_bytes / (att_us * 1e-6) / 1e9, 1),
                    distinct_frac=round(att_bytes / (att_us * 1e-6) / 1e9 / PEAK_HBM_GBPS, 4),
                    distinct_bytes_are="K/V rows of the union of the G heads' index sets per KV head (counted from "
                                       "the last step's sel) + window rows + q + index lists: what must come from HBM",
                    distinct_over_per_head_rows=round(share, 4),
                    avg_launch_us=round(att_us, 2),
                    measured="HIP events around each launch, second pass over the same steps")
    if traffic:
        roofline["traffic_gbps"] = round(traffic / (att_us * 1e-6) / 1e9, 1)
        roofline["traffic_frac"] = round(traffic / (att_us * 1e-6) / 1e9 / PEAK_HBM_GBPS, 4)
    search = ("score_centroids", "top_centroids", "accumulate", "select_threshold", "select_emit")
    # table footprint against the K/V cache (the paper's memory-footprint appendix: 3 S C alpha / (2 d)
    # with 6-byte entries; the device entry here is 4 bytes, the canonical export 8)
    tb, _ = binding.csa_workspace_bytes(ctx.ctx)
    kv_bytes = 2 * B * Hkv * w.n_pre * w.head_dim * 2
    alpha = w.L / w.n_pre
    footprint = dict(tables_bytes=int(tb), kv_bytes_at_n_pre=int(kv_bytes), tables_over_kv=round(tb / kv_bytes, 4),
                     paper_formula_6B=round(3 * w.n_sub * w.C * alpha / (2 * w.head_dim), 4),
                     same_formula_4B_entries=round(2 * w.n_sub * w.C * alpha / (2 * w.head_dim), 4),
                     note="tables_bytes also holds the centroids and the per-row block offsets")

    result = {
        "metric": "decode-step latency (µs) and achieved HBM GB/s at 128K ctx, 95% sparsity",
        "value": round(us_per_step, 2),
        "unit": "us/step",
        "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(us_per_step / 1e3, 5),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16 K/V/q/centroids, int32 table scores, fp32 accumulate",
        "data": "synthetic",
        "config": {"workload": w.name, "batch": B, "n_q_heads": Hq, "n_kv_heads": Hkv,
                   "head_dim": w.head_dim, "n_pre": w.n_pre, "subspaces": w.n_sub, "C": w.C, "L": w.L, "m": w.m,
                   "k": w.k, "pre_appended": w.pre_appended, "page_size": w.page_size,
                   "sparsity": round(1 - w.k / w.n_pre, 4), "mean_selected": sel_mean,
                   "search_period": period,
                   "calls_per_step": "csa_decode_step + csa_append_kv" if args.two_calls else "csa_decode_step_append"},
        "last_step_checks": checks,
        "tokens_per_s": round(B / (us_per_step * 1e-6), 1),
        "step_algorithmic_bytes": int(step_bytes),
        "step_algorithmic_bytes_are": step_bytes_are,
        "step_hbm_gbps": round(step_bytes / (us_per_step * 1e-6) / 1e9, 1),
        "step_frac_of_peak": round(step_bytes / (us_per_step * 1e-6) / 1e9 / PEAK_HBM_GBPS, 4),
        "step_us_percentiles": step_pct,
        "host_issue_us_per_step": round(issued / K * 1e6, 2),
        "graph_replay_us_per_step": None if graph_us is None else round(graph_us, 2),
        "stage_us": {k_: round(v, 2) for k_, v in stage_us.items()},
        "search_us": round(sum(stage_us.get(k_, 0.0) for k_ in search), 2),
        "footprint": footprint,
        "centroids": ("csa_prefill: k-means++ seeding + %d steps, %d mini-batch classes" % (args.cluster_iters, max(1, args.cluster_batches)))
                     if library_centroids else "random sample of the prefill queries",
        "prefill_s" if library_centroids else "build_tables_s": round(t_build, 2),
        "roofline": roofline,
    }

    if args.row_gather_floor:
        result["row_gather_floor"] = row_gather_floor(ctx, w, k_store, v_store, bt, att_us)
    if streaming:
        result["config"]["stream_window"] = args.stream_window
        binding.csa_streaming_status(ctx.ctx)
    if with_cpu and not streaming:
        result["cpu_baseline"] = cpu_baseline(ctx, w, inp, args.cpu_seconds)
    ctx.close()
    return result


def row_gather_floor(ctx, w, k_store, v_store, bt, att_us, reps=20):
    """Time of fetching, and doing nothing else with, the distinct K and V rows the attention kernel
    of the last step had to read: per (sequence, KV head) the union of its query heads' selected
    keys and the appended keys, in ascending order."""
    import torch
    from bench_aids import probe_row_gather
    from paper_2604_08584_amd import binding
    B, Hkv, G = w.batch, w.n_kv_heads, w.group
    n = binding.csa_context_len(ctx.ctx)[1]
    sel = ctx.sel.view(B, Hkv, G * w.k).long()
    need = torch.zeros(B, Hkv, w.max_ctx + 1, dtype=torch.bool, device=sel.device)
    need.scatter_(2, torch.where(sel >= 0, sel, torch.full_like(sel, w.max_ctx)), True)
    need = need[:, :, :w.max_ctx]
    need[:, :, w.n_pre:n] = True
    idx = need.reshape(-1).nonzero().squeeze(1)                      # row number in [B*Hkv*max_ctx)
    if bt is not None:      # paged pools [n_pages][Hkv][page][128]: the row a (b, g, key) triple lives in
        key, bg = idx % w.max_ctx, idx // w.max_ctx
        page = bt.view(B, -1).long()[bg // Hkv, key // w.page_size]
        idx = (page * Hkv + bg % Hkv) * w.page_size + key % w.page_size
    idx = idx.to(torch.int32)
    check = torch.empty((idx.numel() + 63) // 64, dtype=torch.int32, device=sel.device)
    kc, vc = k_store.view(-1, w.head_dim), v_store.view(-1, w.head_dim)
    for _ in range(3):
        probe_row_gather(kc, vc, idx, check)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        probe_row_gather(kc, vc, idx, check)
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / reps
    nbytes = idx.numel() * 2 * w.head_dim * 2
    return {"distinct_rows": int(idx.numel()), "bytes": int(nbytes), "us": round(us, 2),
            "gbps": round(nbytes / (us * 1e-6) / 1e9, 1), "attention_split_us": round(att_us, 2),
            "floor_over_attention": round(us / att_us, 4),
            "what": "bench_aids.probe_row_gather over the union of the selected and appended rows per KV head "
                    "(last step), K and V, HIP events"}


def cluster_bench(args, w):
    """Offline clustering of one sequence's prefill queries (Sec. 3.2 (1)): k-means++ seeding plus
    `--cluster-iters` Lloyd steps for every KV head and subspace.  Prints one JSON line."""
    import numpy as np
    import torch
    from paper_2604_08584_amd import binding
    from paper_2604_08584_amd.workload import make_inputs
    Hq, Hkv, G, S, C, d = w.n_q_heads, w.n_kv_heads, w.group, w.n_sub, w.C, w.head_dim
    iters = args.cluster_iters
    # the prefill queries of one sequence, by the workload's own recipe
    q = make_inputs(dataclasses.replace(w, batch=1, steps=1, pre_appended=0), seed=args.seed, device="cuda",
                    keep_q_pre=True)["q_pre"]
    ctx = binding.csa_create(batch=1, n_q_heads=Hq, n_kv_heads=Hkv, n_centroids=C, list_len=w.L, n_probe=w.m,
                             budget_k=w.k, max_ctx=w.max_ctx, n_subspaces=S)
    work = torch.empty(binding.csa_cluster_workspace_bytes(ctx, w.n_pre), dtype=torch.uint8, device="cuda")
    cent = torch.empty(1, Hkv, S, C, d // S, dtype=torch.bfloat16, device="cuda")
    mean_cos = torch.zeros(1, Hkv, S, max(iters, 1), device="cuda")
    useed = np.random.default_rng(args.seed).uniform(size=(1, Hkv, S, C)).astype(np.float32)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    nb = max(1, args.cluster_batches)
    binding.csa_cluster_queries(ctx, q, w.n_pre, 0, useed, None, cent, None, None, work, n_batches=nb)   # seeding only
    torch.cuda.synchronize()
    t_seed = time.perf_counter() - t0
    seeds = cent.clone()
    t0 = time.perf_counter()
    binding.csa_cluster_queries(ctx, q, w.n_pre, iters, None, seeds, cent, mean_cos, None, work, n_batches=nb)
    torch.cuda.synchronize()
    t_lloyd = time.perf_counter() - t0
    n_pool = G * w.n_pre
    flops = 2.0 * (n_pool / nb) * C * (d // S) * Hkv * S * iters          # the assignment contraction
    mc = mean_cos.mean(dim=(0, 1, 2)).cpu().numpy()
    binding.csa_destroy(ctx)
    peak = 2500.0
    print(json.dumps({
        "metric": "offline query clustering of one sequence (s): k-means++ seeding + Lloyd steps",
        "value": round(t_seed + t_lloyd, 4), "unit": "s", "n_gpus": 1, "higher_is_better": False,
        "dtype": "bf16 operands, fp32 accumulate", "data": "synthetic",
        "config": {"workload": w.name, "n_q_heads": Hq, "n_kv_heads": Hkv, "n_pre": w.n_pre, "subspaces": S,
                   "C": C, "iters": iters, "points_per_problem": n_pool, "batches": nb,
                   "problems_side_by_side": Hkv * S},
        "seeding_s": round(t_seed, 4), "lloyd_s": round(t_lloyd, 4),
        "mean_cos_first_last": [round(float(mc[0]), 4), round(float(mc[-1]), 4)],
        "roofline": lloyd_roofline(flops, t_lloyd, n_pool / nb, C, d // S, Hkv * S, iters, peak),
    }), flush=True)


def lloyd_roofline(flops, t_lloyd, n_pts, C, db, n_prob, iters, peak):
    """The Lloyd steps against the bound that governs them: the bf16 matrix-core peak when the
    contraction is large against the bytes of the points (long sub-vectors, many centroids), else the
    HBM stream of the points (every step reads each point's sub-vector once for the assignment and
    once for the member sums: 2 * d_b * 2 bytes per point)."""
    point_bytes = 2.0 * n_pts * db * 2 * n_prob * iters
    t_mfma, t_hbm = flops / (peak * 1e12), point_bytes / (PEAK_HBM_GBPS * 1e9)
    if t_mfma >= t_hbm:
        return {"kernel": "k_km_assign (+ member sums, k_km_finish)", "bound": "mfma",
                "achieved": round(flops / t_lloyd / 1e12, 2), "peak": peak, "unit": "TFLOP/s",
                "frac": round(flops / t_lloyd / 1e12 / peak, 4), "traffic": None,
                "measured": "wall clock over all Lloyd steps of all problems, synchronised"}
    return {"kernel": "k_km_assign (+ member sums, k_km_finish)", "bound": "hbm",
            "achieved": round(point_bytes / t_lloyd / 1e9, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
            "frac": round(point_bytes / t_lloyd / 1e9 / PEAK_HBM_GBPS, 4), "traffic": None,
            "note": "the contraction is tiny against the bytes of the points (%.1f flop per byte): the steps "
                    "are bound by the stream of the points and by their launches, not by the matrix cores"
                    % (flops / point_bytes),
            "measured": "wall clock over all Lloyd steps of all problems, synchronised"}


def cpu_baseline(ctx, w, inp, budget_s):
    """The oracle, as it stands, on the host cores: the first decode step of the run (context =
    N_pre + pre_appended) for the query heads of the first KV heads, scaled to the whole batch.
    The oracle reads tables it builds itself (the rows its sampled heads probe, at the grid the
    library reports); building them is set-up and not timed, like the GPU's build."""
    import numpy as np
    from oracle import oracle
    from paper_2604_08584_amd import binding
    n_groups = max(1, min(w.batch * w.n_kv_heads, 16 // w.group))
    t = w.pre_appended
    n = w.n_pre + t
    F = binding.csa_score_frac_bits(ctx.ctx)
    qh = oracle.bf16_bits(inp["q_steps"][t])
    items = []
    for s in range(n_groups):
        b, g = divmod(s, w.n_kv_heads)
        K = oracle.bf16_bits(inp["k_cache"][b, g])
        V = oracle.bf16_bits(inp["v_cache"][b, g])
        # rows [n_pre, n) of the logical cache: the keys appended before the first step
        K[w.n_pre:n] = oracle.bf16_bits(inp["k_new"][:t, b, g])
        V[w.n_pre:n] = oracle.bf16_bits(inp["v_new"][:t, b, g])
        cent = oracle.bf16_bits(inp["centroids"][b, g])
        heads = range(g * w.group, (g + 1) * w.group)
        probed = np.unique(np.concatenate(
            [oracle.top_centroids(np.ascontiguousarray(qh[b, h]), cent, w.m)[0] for h in heads]))
        idx = np.full((w.n_sub * w.C, w.L), -1, np.int32)
        score = np.zeros((w.n_sub * w.C, w.L), np.float32)
        idx[probed], score[probed], _ = oracle.build_rows(np.ascontiguousarray(K[:w.n_pre]), w.n_pre, cent,
                                                          probed, w.L, F)
        for h in heads:
            items.append(dict(q=np.ascontiguousarray(qh[b, h]), cent=cent, tbl_idx=idx,
                              tbl_score=score, K=K, V=V))
    oracle.decode_items(items[:1], w.m, w.k, w.n_pre, n)  # page the library in

    def timed(its, n_threads, budget):
        reps, spent, used = 0, 0.0, 1
        while spent < budget and reps < 100000:
            t0 = time.perf_counter()
            *_, used = oracle.decode_items(its, w.m, w.k, w.n_pre, n, n_threads=n_threads)
            spent += time.perf_counter() - t0
            reps += 1
        return spent / reps / len(its), reps, int(used)

    scale = w.batch * w.n_q_heads
    per_head_s, reps, used = timed(items, 0, 0.6 * budget_s)            # all host threads
    one_head_s, _, _ = timed(items[:2], 1, 0.2 * budget_s)               # one thread
    # dense attention over the whole context (Sec. 3.1, the definition the method approximates) on one
    # thread, for the dense-to-sparse ratio on the same cores
    it = items[0]
    reps_d, spent_d = 0, 0.0
    while spent_d < 0.2 * budget_s and reps_d < 1000:
        t0 = time.perf_counter()
        oracle.dense_attention(it["q"], it["K"], it["V"], n)
        spent_d += time.perf_counter() - t0
        reps_d += 1
    return dict(value=round(per_head_s * scale * 1e6, 1), unit="us/step", cores=used, kind="oracle",
                sample=f"{len(items)} of {scale} (sequence, query head) items of the "
                       f"first step, {reps} repetitions, all {used} host threads, scaled by "
                       f"{scale}/{len(items)}",
                single_thread_us_step=round(one_head_s * scale * 1e6, 1),
                dense_attention_single_thread_us_step=round(spent_d / reps_d * scale * 1e6, 1),
                host_cpus=os.cpu_count())


if __name__ == "__main__":
    main()
