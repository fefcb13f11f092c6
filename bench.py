#!/usr/bin/env python3
"""Benchmark of the verify -> select -> draft hot path on one MI355X.

A "step" is one decoding iteration's attention work for one layer on the 32K-context workload
(batch 1, 32 query / 8 KV heads, head_dim 128, 16-token pages, gamma = 4, KV budget 2048):
one vegas_verify_attention, one vegas_select_blocks and gamma+1 vegas_draft_attention calls,
all through the C ABI on one stream, inputs resident in HBM before the timed region.

Cold-cache protocol: the 128 MiB of K+V of this workload would fit in the last-level cache, which a
serving engine never enjoys (dozens of layers' caches pass between two visits of the same layer),
so consecutive steps rotate over several device copies of the cache (>= 1 GiB in total).

Prints ONE JSON line: whole-path us per iteration (timed region = K iterations, nothing else on the
stream), the roofline of the dominant kernel (the KV-streaming verification kernel: K back-to-back
launches of that kernel alone over the same rotating caches, bracketed by two HIP events on the
launch stream) and the CPU oracle timed on the host cores as a reported baseline.

Beyond the default run:
  --workload NAME      another synthetic workload (ctx4k, ctx128k_drift, ragged16, stack32; extras: hd64_ctx32k, the
                       head-dimension-64 shape at 32K context, and ctx32k_batch4); the
                       CPU baseline and the counter-derived traffic belong to the default workload only
  --extras             adds per-iteration percentiles, the warm-cache figure (one cache copy) and the
                       iteration replayed from captured HIP graphs to the same JSON line
  --live               the drafting phase as it runs live: every draft step first appends the drafted token's K/V rows
                       (vegas_append_kv) and grows the selection by them (vegas_extend_selection)
  --all-layers         a multi-layer workload (stack32) with every layer's cache resident: a step is one pass over all
                       layers
  --timeline           per-wave phase times of the two KV-streaming kernels (profiling build of the library)
  --no-all-workloads   the default run appends one compact record per other workload (`workloads`); this skips them
  --sweep page_size    draft attention latency versus the page size (1..16 tokens) of the selection table in the
                       set-up of App. D / Table 5 (batch 16, 8192 selected tokens per request, random positions)
  --sweep collect      the collection-overhead curve (Sec. 3.3, Fig. 6 analogue): the verification call
                       at G = 2..12 rows for collect_rows = none / all rows (Eq. 2) / first + bonus
                       row (Eq. 3); prints one JSON line holding the table
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
# HBM bytes per launch of the verification streaming kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# runs, each scaled by what the same counter reads for a plain 64 MiB copy (factors 1.9990 and 1.0); the figures are
# the `traffic_bytes_per_launch[...]` lines of the two summaries (tests/test_profiles_match_bench.py compares them).
VERIFY_TRAFFIC_BYTES = {
    "ctx32k": 138574632,       # (131447 KiB fetched + 3880 KiB written), profiles/ctx32k_hbm_traffic_pmc.md
    "ragged16": 2434575050,    # (2312055 KiB fetched + 65460 KiB written), profiles/ragged16_hbm_traffic_pmc.md
}
DEFAULT_WORKLOAD = "ctx32k"
ROTATE_BYTES = 1.2e9           # rotate cache copies up to about this much K+V in total


def all_workloads(synth):
    return {**synth.CONFIGS, **synth.EXTRA_CONFIGS}


def cpu_baseline(L, budget: int, workload: str, target_seconds: float = 12.0):
    """Time the oracle as it stands on the host cores: whole iterations of the same workload."""
    from oracle import vegas_oracle as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([int(p.get("num_threads", 1)) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    max_sel = (budget + 15) // 16 + 2

    def one():
        O.decoding_iteration(L.q_verify, L.q_draft, L.k_cache, L.v_cache, L.block_table, L.seq_lens,
                             L.softmax_scale, budget, max_sel)
    t0 = time.perf_counter()
    one()
    first = time.perf_counter() - t0
    reps = max(1, min(40, int(target_seconds / max(first, 1e-3))))
    t0 = time.perf_counter()
    for _ in range(reps):
        one()
    dt = (time.perf_counter() - t0) / reps
    return {"value": dt * 1e6, "unit": "us", "cores": threads, "kind": "oracle",
            "sample": f"{reps} whole iterations of the {workload} workload (verify + select + "
                      f"{L.spec.num_queries} draft steps), float64 NumPy oracle, mean"}


def oracle_iteration_us(L, budget: int, threads: int = 0) -> dict:
    """One whole iteration of the oracle on the host (as it stands), timed once; threads > 0 limits the BLAS pool."""
    from oracle import vegas_oracle as O
    max_sel = (budget + 15) // 16 + 2

    def one():
        t0 = time.perf_counter()
        O.decoding_iteration(L.q_verify, L.q_draft, L.k_cache, L.v_cache, L.block_table, L.seq_lens,
                             L.softmax_scale, budget, max_sel)
        return (time.perf_counter() - t0) * 1e6
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        if threads > 0:
            with threadpool_limits(limits=threads):
                return {"us": one(), "threads": threads}
        used = max([int(p.get("num_threads", 1)) for p in threadpool_info()] or [1])
        return {"us": one(), "threads": used}
    except ImportError:
        return {"us": one(), "threads": os.cpu_count() or 1}


def compact_workload(name: str, args, torch, vb, harness, synth, with_oracle: bool) -> dict:
    """One workload through the same protocol as the headline one (cold rotating caches, whole iterations, then the
    two KV-streaming kernels alone), as one compact record for the `workloads` array."""
    spec = all_workloads(synth)[name]
    L = synth.make_layer(spec, 0)
    dev = torch.device("cuda:0")
    base = harness.DeviceLayer.upload(L, dev)
    copies = device_copies(harness, base, copies_for(base, args.copies))
    path = harness.VegasPath.for_layer(L)
    G = spec.num_queries
    stream = int(torch.cuda.current_stream(dev).cuda_stream)
    n_tokens = int(L.seq_lens.sum())
    bpt = 2 * spec.num_kv_heads * spec.head_dim * 2
    big = n_tokens * bpt > 1e9
    K, W = (20, 3) if big else (100, 10)

    def timed(fn, reps, warm):
        for i in range(warm):
            fn(i)
        torch.cuda.synchronize()
        e0, e1 = vb.HipEvent(), vb.HipEvent()
        e0.record(stream)
        for i in range(reps):
            fn(i)
        e1.record(stream)
        e1.synchronize()
        return e0.elapsed_ms(e1) / reps * 1e3
    for i in range(W):
        path.iteration(copies[i % len(copies)])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        path.iteration(copies[i % len(copies)])
    torch.cuda.synchronize()
    it_us = (time.perf_counter() - t0) / K * 1e6
    v_us = timed(lambda i: path.verify(copies[i % len(copies)], stages=vb.STAGE_STREAM), K, 3)
    d_us = timed(lambda i: path.draft(copies[i % len(copies)], i % G, stages=vb.STAGE_STREAM), K, 3)
    verify_bytes = n_tokens * bpt
    draft_bytes = int(path.sel_seq_lens.sum().item()) * bpt
    rec = {"workload": name, "batch": spec.batch, "context_tokens_total": n_tokens, "draft_steps": G,
           "kv_budget_tokens": spec.budget_tokens, "steps": K, "us_per_iteration": it_us,
           "iteration_gbps": (verify_bytes + G * draft_bytes) / (it_us * 1e-6) / 1e9,
           "verify_kernel_us": v_us, "verify_frac_of_peak": verify_bytes / (v_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
           "draft_kernel_us": d_us, "draft_frac_of_peak": draft_bytes / (d_us * 1e-6) / 1e9 / HBM_PEAK_GBS}
    if spec.layers > 1:
        rec["note"] = f"one of {spec.layers} independent layers (layer 0); --all-layers times the whole stack"
    del copies, base, path
    torch.cuda.empty_cache()
    if with_oracle:
        o = oracle_iteration_us(L, spec.budget_tokens)
        rec["cpu_oracle_us"], rec["cpu_oracle_threads"] = o["us"], o["threads"]
        if spec.config_id in (1, 2):
            rec["cpu_oracle_us_single_thread"] = oracle_iteration_us(L, spec.budget_tokens, threads=1)["us"]
    return rec


def all_layers(args, torch, vb, harness, synth) -> int:
    """The multi-layer workload as its definition reads: every layer's K/V resident at once (32 x 1.07 GB), one
    iteration = layers x (verify + select + G draft calls), each layer on its own cache.  Prints one JSON line."""
    spec = all_workloads(synth)[args.workload]
    dev = torch.device("cuda:0")
    layers = []
    t0 = time.perf_counter()
    for l in range(spec.layers):
        L = synth.make_layer(spec, l)
        layers.append(harness.DeviceLayer.upload(L, dev))
        if l == 0:
            path = harness.VegasPath.for_layer(L)
            n_tokens = int(L.seq_lens.sum())
        print(f"layer {l} resident ({time.perf_counter() - t0:.0f} s)", file=sys.stderr, flush=True)
        del L
    G = spec.num_queries
    K, W = args.steps, args.warmup

    def iteration():
        for dl in layers:
            path.iteration(dl)
    for _ in range(W):
        iteration()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(K):
        iteration()
    torch.cuda.synchronize()
    us = (time.perf_counter() - t0) / K * 1e6
    bpt = 2 * spec.num_kv_heads * spec.head_dim * 2
    resident = sum(2 * dl.k_cache.numel() * dl.k_cache.element_size() for dl in layers)
    it_bytes = spec.layers * (n_tokens + G * int(path.sel_seq_lens.sum().item())) * bpt
    print(json.dumps({
        "metric": "us_per_verify_select_draft_iteration", "value": us, "unit": "us", "n_gpus": 1, "steps": K,
        "warmup": W, "ms_per_step": us / 1e3, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload, "layers": spec.layers, "all_layers_resident": True, "batch": spec.batch,
                   "context": spec.seq_len, "num_q_heads": spec.num_q_heads, "num_kv_heads": spec.num_kv_heads,
                   "head_dim": spec.head_dim, "page_size": 16, "gamma": spec.gamma,
                   "kv_budget_tokens": spec.budget_tokens, "draft_steps": G,
                   "step": f"{spec.layers} x (verify + select + {G} draft calls), one layer after the other"},
        "kv_bytes_resident": resident, "iteration_kv_bytes": it_bytes,
        "iteration_gbps": it_bytes / (us * 1e-6) / 1e9,
        "iteration_frac_of_hbm_peak": it_bytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS,
        "us_per_layer": us / spec.layers}), flush=True)
    return 0


TIMELINE_EVENTS = ["wave entry", "length known", "first tile's loads issued", "queries in LDS (first barrier passed)",
                   "first tile done", "last tile done", "merge barrier passed", "partial stored (exit)"]


def timeline_table(buf, label: str) -> dict:
    """Per-phase summary of one launch's stamps ([records][8] uint64 at 100 MHz; records never written stay zero):
    event times relative to the first wave's entry, and per-wave phase durations, in microseconds."""
    import numpy as np
    raw = buf.cpu().numpy().view(np.uint64).reshape(-1, 8)
    live = raw[:, 0] > 0
    rec = raw[live].astype(np.float64)
    if rec.shape[0] == 0:
        return {"kernel": label, "waves": 0}
    t0 = rec[:, 0].min()
    rel = (rec - t0) / 100.0
    # Workgroup ids are dealt round-robin to the 8 XCDs (record index = 4 * workgroup id + wave): when each XCD's
    # waves are done streaming, which is what a static partition of the work has to live with.
    xcd = ((np.nonzero(live)[0] // 4) % 8)
    by_xcd = [float(rel[xcd == x, 5].mean()) if np.any(xcd == x) else None for x in range(8)]

    def summary(col):
        c = np.sort(col)
        return {"min": float(c[0]), "p50": float(c[len(c) // 2]), "p90": float(c[int(0.9 * (len(c) - 1))]), "max": float(c[-1])}
    events = {name: summary(rel[:, i]) for i, name in enumerate(TIMELINE_EVENTS)}
    phases = {f"{TIMELINE_EVENTS[i]} -> {TIMELINE_EVENTS[i + 1]}": summary(rel[:, i + 1] - rel[:, i]) for i in range(7)}
    return {"kernel": label, "waves": int(rec.shape[0]), "unit": "us",
            "events_after_first_entry": events, "phase_durations_per_wave": phases,
            "last_tile_done_mean_by_xcd": by_xcd}


def run_timeline(args, torch, vb, harness, synth) -> int:
    """Per-wave phase timeline of the two KV-streaming kernels on the workload (profiling build of the library)."""
    spec = all_workloads(synth)[args.workload]
    L = synth.make_layer(spec, args.layer)
    dev = torch.device("cuda:0")
    base = harness.DeviceLayer.upload(L, dev)
    copies = device_copies(harness, base, copies_for(base, args.copies))
    path = harness.VegasPath.for_layer(L, verify_chunk=args.verify_chunk, draft_chunk=args.draft_chunk)
    G = spec.num_queries
    buf = torch.zeros(4 << 20, dtype=torch.int64, device=dev)              # 32 MiB: 65536 workgroups of 4 waves
    out = {"timeline": True, "workload": args.workload, "clock": "100 MHz wall clock (10 ns steps)", "kernels": []}
    for i in range(6):                                                     # cold caches as in the timed runs
        path.iteration(copies[i % len(copies)])
    torch.cuda.synchronize()
    vb.vegas_debug_set_timeline(buf)
    path.verify(copies[6 % len(copies)], stages=vb.STAGE_STREAM)
    torch.cuda.synchronize()
    vb.vegas_debug_set_timeline(None)
    out["kernels"].append(timeline_table(buf, "KV-streaming kernel of vegas_verify_attention"))
    path.iteration(copies[7 % len(copies)])                                # the selection a draft call walks
    path.draft(copies[7 % len(copies)], 0)
    torch.cuda.synchronize()
    buf.zero_()
    torch.cuda.synchronize()
    vb.vegas_debug_set_timeline(buf)
    path.draft(copies[7 % len(copies)], 1 % G, stages=vb.STAGE_STREAM)     # a second draft step, as in an iteration
    torch.cuda.synchronize()
    vb.vegas_debug_set_timeline(None)
    out["kernels"].append(timeline_table(buf, "KV-streaming kernel of vegas_draft_attention (second draft step)"))
    for k in out["kernels"]:
        print(f"== {k['kernel']}: {k['waves']} waves", file=sys.stderr)
        for name, v in k.get("events_after_first_entry", {}).items():
            print(f"   at   {name:40s} min {v['min']:6.2f}  p50 {v['p50']:6.2f}  p90 {v['p90']:6.2f}  max {v['max']:6.2f}", file=sys.stderr)
        for name, v in k.get("phase_durations_per_wave", {}).items():
            print(f"   took {name:80s} p50 {v['p50']:6.2f}  p90 {v['p90']:6.2f}  max {v['max']:6.2f}", file=sys.stderr)
        if k.get("last_tile_done_mean_by_xcd"):
            print("   last tile done, mean over the waves of XCD 0..7 (workgroup id mod 8): " +
                  "  ".join("   -  " if v is None else f"{v:6.2f}" for v in k["last_tile_done_mean_by_xcd"]), file=sys.stderr)
    print(json.dumps(out), flush=True)
    return 0


def device_copies(harness, base, want: int):
    """`want` device layers that share queries and tables with `base` but own their K/V caches."""
    copies = [base]
    for _ in range(want - 1):
        copies.append(harness.DeviceLayer(q_verify=base.q_verify, q_draft=base.q_draft,
                                          k_cache=base.k_cache.clone(), v_cache=base.v_cache.clone(),
                                          block_table=base.block_table, seq_lens=base.seq_lens,
                                          k_new=base.k_new, v_new=base.v_new, seq_lens_live=base.seq_lens_live))
    return copies


def copies_for(base, asked: int) -> int:
    kv_bytes = 2 * base.k_cache.numel() * base.k_cache.element_size()
    return max(1, min(asked, int(ROTATE_BYTES // kv_bytes) + 1))


def percentile(sorted_vals, q: float) -> float:
    i = min(len(sorted_vals) - 1, max(0, int(round(q * (len(sorted_vals) - 1)))))
    return sorted_vals[i]


def sweep_collect(args, torch, vb, harness, synth) -> int:
    """Collection-overhead curve: time of the verification call versus the number of verification
    rows G and what is collected.  Sec. 3.3 measures that cost for an instrumented dense kernel
    (all rows against two rows); this is the same question asked of the kernel here."""
    dev = torch.device("cuda:0")
    base_spec = all_workloads(synth)[args.workload]
    stream = int(torch.cuda.current_stream(dev).cuda_stream)
    K = args.steps
    rows = []
    modes = ((vb.COLLECT_NONE, "none"), (vb.COLLECT_ALL_ROWS, "all_rows"), (vb.COLLECT_FIRST_LAST, "first_last"))
    for G in range(2, 13):
        spec = synth.scaled(base_spec, gamma=G - 1)
        L = synth.make_layer(spec)
        base = harness.DeviceLayer.upload(L, dev)
        copies = device_copies(harness, base, copies_for(base, args.copies))
        verify_bytes = int(L.seq_lens.sum()) * 2 * spec.num_kv_heads * spec.head_dim * 2
        entry = {"G": G, "rows_per_kv_head": G * spec.num_q_heads // spec.num_kv_heads}
        for mode, name in modes:
            path = harness.VegasPath.for_layer(L, collect_rows=mode, verify_chunk=args.verify_chunk)

            def leg(stages: int) -> float:
                e0, e1 = vb.HipEvent(), vb.HipEvent()
                for i in range(5):
                    path.verify(copies[i % len(copies)], stages=stages)
                torch.cuda.synchronize()
                e0.record(stream)
                for i in range(K):
                    path.verify(copies[i % len(copies)], stages=stages)
                e1.record(stream)
                e1.synchronize()
                return e0.elapsed_ms(e1) / K * 1e3
            call_us, stream_us = leg(0), leg(vb.STAGE_STREAM)
            entry[name] = {"call_us": call_us, "stream_kernel_us": stream_us,
                           "stream_gbps": verify_bytes / (stream_us * 1e-6) / 1e9}
            del path
        for name in ("all_rows", "first_last"):
            entry[name]["overhead_pct_call"] = 100.0 * (entry[name]["call_us"] / entry["none"]["call_us"] - 1.0)
            entry[name]["overhead_pct_stream_kernel"] = 100.0 * (entry[name]["stream_kernel_us"]
                                                                 / entry["none"]["stream_kernel_us"] - 1.0)
        rows.append(entry)
        print(f"G={G:2d} none {entry['none']['call_us']:7.1f} us | all rows {entry['all_rows']['call_us']:7.1f} us "
              f"({entry['all_rows']['overhead_pct_call']:+.1f}%) | first+last {entry['first_last']['call_us']:7.1f} us "
              f"({entry['first_last']['overhead_pct_call']:+.1f}%)", file=sys.stderr, flush=True)
        del copies, base, L
        torch.cuda.empty_cache()
    print(json.dumps({"sweep": "collect", "workload": args.workload, "steps": K, "unit": "us",
                      "what": "vegas_verify_attention per call (streaming kernel + merge/score kernel) and its "
                              "streaming kernel alone, cold caches, versus verification rows G and collect_rows",
                      "rows": rows}), flush=True)
    return 0


PAPER_TABLE5_H100_US = {1: 197.6, 2: 197.6, 4: 197.1, 8: 198.1, 16: 198.3}   # App. D, Table 5, first row (another machine: context)


def sweep_page_size(args, torch, vb) -> int:
    """Sparse (draft) attention latency versus the page size of the selection table, in the set-up of
    App. D / Table 5: batch 16, a K/V pool of 16 x 128K tokens, 8192 selected tokens per request
    (8192 / page_size pages at random positions of the whole pool), 32 query / 8 KV heads, head_dim 128."""
    import numpy as np
    dev = torch.device("cuda:0")
    B, Hq, Hkv, D, sel_tokens = 16, 32, 8, 128, 8192
    pool_tokens = B * 131072
    stream = int(torch.cuda.current_stream(dev).cuda_stream)
    gen = torch.Generator(device=dev)
    gen.manual_seed(7223900)
    k_pool = torch.empty((pool_tokens, Hkv, D), dtype=torch.bfloat16, device=dev)
    v_pool = torch.empty((pool_tokens, Hkv, D), dtype=torch.bfloat16, device=dev)
    step = 1 << 20
    for t0 in range(0, pool_tokens, step):                       # N(0,1)/sqrt(D), drawn on the device piece by piece
        k_pool[t0:t0 + step].normal_(0.0, D ** -0.5, generator=gen)
        v_pool[t0:t0 + step].normal_(0.0, D ** -0.5, generator=gen)
    q = torch.empty((B, Hq, D), dtype=torch.bfloat16, device=dev).normal_(0.0, D ** -0.5, generator=gen)
    out = torch.empty((B, Hq, D), dtype=torch.bfloat16, device=dev)
    rng = np.random.default_rng(7223901)
    K = args.steps
    rows = []
    bytes_per_call = B * sel_tokens * 2 * Hkv * D * 2
    for P in (1, 2, 4, 8, 16):
        n_sel = sel_tokens // P
        pool_pages = pool_tokens // P
        tables = []
        for _ in range(3):                                       # rotate over three selections: nothing stays cached
            ids = rng.choice(pool_pages, size=B * n_sel, replace=False).astype(np.int32).reshape(B, n_sel)
            ids.sort(axis=1)
            tables.append(torch.from_numpy(ids).to(dev))
        ssl = torch.full((B,), sel_tokens, dtype=torch.int32, device=dev)
        desc = vb.make_desc(batch=B, num_q_heads=Hq, num_kv_heads=Hkv, num_queries=1, max_blocks=n_sel,
                            max_sel_blocks=n_sel, max_seq_len=sel_tokens, num_pages=pool_pages,
                            softmax_scale=D ** -0.5, page_size=P, kv_chunk_tokens=args.draft_chunk)
        ws = torch.empty(vb.vegas_workspace_bytes(desc), dtype=torch.uint8, device=dev)
        addr = dict(q=q.data_ptr(), k=k_pool.data_ptr(), v=v_pool.data_ptr(), ssl=ssl.data_ptr(), out=out.data_ptr(),
                    ws=ws.data_ptr(), t=[t.data_ptr() for t in tables])

        def call(i: int, stages: int) -> None:
            vb.vegas_draft_attention(desc, addr["q"], addr["k"], addr["v"], addr["t"][i % 3], addr["ssl"], addr["out"],
                                     addr["ws"], stream=stream, workspace_bytes=ws.numel(), stages=stages)

        def leg(stages: int) -> float:
            e0, e1 = vb.HipEvent(), vb.HipEvent()
            for i in range(5):
                call(i, stages)
            torch.cuda.synchronize()
            e0.record(stream)
            for i in range(K):
                call(i, stages)
            e1.record(stream)
            e1.synchronize()
            return e0.elapsed_ms(e1) / K * 1e3
        call_us, stream_us = leg(0), leg(vb.STAGE_STREAM)
        rows.append({"page_size": P, "call_us": call_us, "stream_kernel_us": stream_us,
                     "call_gbps": bytes_per_call / (call_us * 1e-6) / 1e9,
                     "stream_kernel_gbps": bytes_per_call / (stream_us * 1e-6) / 1e9,
                     "stream_kernel_frac_of_peak": bytes_per_call / (stream_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                     "paper_h100_us": PAPER_TABLE5_H100_US[P]})
        print(f"page_size={P:2d} call {call_us:7.1f} us ({rows[-1]['call_gbps']:.0f} GB/s) | streaming kernel "
              f"{stream_us:7.1f} us ({rows[-1]['stream_kernel_gbps']:.0f} GB/s, "
              f"{100 * rows[-1]['stream_kernel_frac_of_peak']:.1f}% of peak) | paper, H100: {PAPER_TABLE5_H100_US[P]} us",
              file=sys.stderr, flush=True)
    print(json.dumps({"sweep": "page_size", "steps": K, "unit": "us", "kv_bytes_per_call": bytes_per_call,
                      "what": "vegas_draft_attention, batch 16, 8192 selected tokens per request at random pool "
                              "positions, K/V pool of 16 x 128K tokens (App. D, Table 5 set-up)",
                      "rows": rows}), flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD)
    ap.add_argument("--layer", type=int, default=0, help="layer of a multi-layer workload (own seed each)")
    ap.add_argument("--copies", type=int, default=8, help="device copies of the KV cache to rotate over (at most)")
    ap.add_argument("--verify-chunk", type=int, default=0)
    ap.add_argument("--draft-chunk", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-legs", action="store_true",
                    help="skip the legs that time the KV-streaming kernels alone (counter runs want the plain iteration)")
    ap.add_argument("--extras", action="store_true")
    ap.add_argument("--variant", choices=["page", "token"], default="page",
                    help="page: 16-token pages scored by softmax weights (the default path); token: the paper's own "
                         "variant -- averaged logits per token (Eq. 3 rows), top-k over tokens, one-token pages")
    ap.add_argument("--budget", type=int, default=0, help="KV budget in tokens (0: the workload's)")
    ap.add_argument("--live", action="store_true",
                    help="a live drafting phase: before each draft call the drafted token's K/V is appended to the cache "
                         "(vegas_append_kv) and the selection grows by it (vegas_extend_selection); the step then is "
                         "verify + select + G x (append + extend + draft) + one small copy that rewinds the lengths")
    ap.add_argument("--all-layers", action="store_true",
                    help="a multi-layer workload (stack32) as its definition reads: all layers resident, one step = "
                         "layers x (verify + select + G draft calls); takes a few minutes of host time to generate")
    ap.add_argument("--no-all-workloads", action="store_true",
                    help="skip the compact records of the other workloads that the default run appends")
    ap.add_argument("--timeline", action="store_true",
                    help="per-wave phase timeline of the two KV-streaming kernels; needs the profiling build "
                         "(python -m paper_2602_07223_amd.build --timeline), which this option loads")
    ap.add_argument("--sweep", choices=["collect", "page_size"], default=None)
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              "use --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2602_07223_amd import binding as vb
    from paper_2602_07223_amd import harness, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    if args.timeline:
        from paper_2602_07223_amd import build as vbuild
        vb.load_library(vbuild.TIMELINE_LIB_PATH)       # the profiling build; raises if it has not been built
    vb.load_library()                                   # fail loudly if the HIP library is not built
    if args.workload not in all_workloads(synth):
        print(f"bench.py: unknown workload {args.workload!r}; one of {sorted(all_workloads(synth))}", file=sys.stderr)
        return 2
    if args.timeline:
        return run_timeline(args, torch, vb, harness, synth)
    if args.sweep == "collect":
        return sweep_collect(args, torch, vb, harness, synth)
    if args.sweep == "page_size":
        return sweep_page_size(args, torch, vb)

    if args.all_layers:
        if args.steps == 200:
            args.steps, args.warmup = 5, 1
        return all_layers(args, torch, vb, harness, synth)

    workload = args.workload
    spec = all_workloads(synth)[workload]
    L = synth.make_layer(spec, args.layer)
    if args.live:
        L = synth.with_growth(L, spec.num_queries)
    dev = torch.device("cuda:0")
    base = harness.DeviceLayer.upload(L, dev)
    copies = device_copies(harness, base, copies_for(base, args.copies))
    token = args.variant == "token"
    budget = args.budget or spec.budget_tokens
    path = harness.VegasPath.for_layer(L, budget_tokens=budget, verify_chunk=args.verify_chunk,
                                       draft_chunk=args.draft_chunk, token_granular=token,
                                       growth=spec.num_queries if args.live else 0,
                                       collect_rows=vb.COLLECT_FIRST_LAST if token else vb.COLLECT_ALL_ROWS)
    G = spec.num_queries
    stream = int(torch.cuda.current_stream(dev).cuda_stream)

    K, W = args.steps, args.warmup

    def run_one(c) -> None:
        if args.live:
            path.live_iteration(c)
        else:
            path.iteration(c)

    def step(i: int) -> None:
        run_one(copies[i % len(copies)])

    for i in range(W):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        step(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    us_per_step = dt / K * 1e6

    n_tokens = int(L.seq_lens.sum())
    bytes_per_token = 2 * spec.num_kv_heads * spec.head_dim * 2          # K and V, bf16: 4096 B
    verify_bytes = n_tokens * bytes_per_token                            # algorithmic bytes of one launch
    sel_tokens = int(path.sel_seq_lens.sum().item())
    draft_bytes = sel_tokens * bytes_per_token

    def kernel_leg(call, reps: int) -> float:
        """Average duration of one KV-streaming kernel: `reps` back-to-back launches of that kernel
        alone (the debug entry point with stages = STREAM), bracketed by two HIP events on the launch stream."""
        e0, e1 = vb.HipEvent(), vb.HipEvent()
        for i in range(5):
            call(i)
        torch.cuda.synchronize()
        e0.record(stream)
        for i in range(reps):
            call(i)
        e1.record(stream)
        e1.synchronize()
        return e0.elapsed_ms(e1) / reps * 1e3

    traffic = VERIFY_TRAFFIC_BYTES.get(workload) if args.verify_chunk == 0 and not token else None
    rows_per_kv_head = G * (spec.num_q_heads // spec.num_kv_heads)
    vkernel = "attn_pair_kernel<collect>" if 32 < rows_per_kv_head <= 64 else "attn_split_kernel<causal, collect>"
    roofline = {"bound": "hbm", "kernel": vkernel + " (KV-streaming kernel of vegas_verify_attention)",
                "achieved": None, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": None, "traffic": traffic,
                "bytes_per_launch": verify_bytes}
    roofline_draft = None
    if not args.no_kernel_legs:
        v_us = kernel_leg(lambda i: path.verify(copies[i % len(copies)], stages=vb.STAGE_STREAM), K)
        roofline["kernel_us"] = v_us
        roofline["achieved"] = verify_bytes / (v_us * 1e-6) / 1e9
        roofline["frac"] = roofline["achieved"] / HBM_PEAK_GBS
        d_reps = max(K, 100)              # (a 7 us kernel: twenty launches are too few for a stable mean)
        d_us = kernel_leg(lambda i: path.draft(copies[i % len(copies)], i % G, stages=vb.STAGE_STREAM), d_reps)
        dkernel = "attn_draft16_kernel" if spec.num_q_heads // spec.num_kv_heads <= 16 and not token else "attn_split_kernel"
        roofline_draft = {"bound": "hbm", "kernel": dkernel + " (KV-streaming kernel of vegas_draft_attention)",
                          "kernel_us": d_us, "achieved": draft_bytes / (d_us * 1e-6) / 1e9, "peak": HBM_PEAK_GBS,
                          "unit": "GB/s", "frac": draft_bytes / (d_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                          "bytes_per_launch": draft_bytes, "traffic": None, "launches": d_reps}
        roofline["launches"] = K
        # The yardstick: a kernel that only reads the same K and V caches (cold, rotating over the same copies), plain
        # coalesced 16-byte non-temporal loads, best of several grid sizes.  What it reaches is what this memory system
        # gives a launch of this footprint; the verification kernel is held against it beside the published peak.
        cache_bytes = base.k_cache.numel() * base.k_cache.element_size()
        sink = torch.empty(4096 * 256, dtype=torch.int32, device=dev)
        best = None
        for wgs in (256, 512, 1024, 2048, 4096):
            r_us = kernel_leg(lambda i: vb.vegas_debug_stream_read(copies[i % len(copies)].k_cache.data_ptr(),
                                                                    copies[i % len(copies)].v_cache.data_ptr(),
                                                                    cache_bytes, wgs, True, sink.data_ptr(), stream=stream), K)
            if best is None or r_us < best[0]:
                best = (r_us, wgs)
        ceil_gbps = 2 * cache_bytes / (best[0] * 1e-6) / 1e9
        roofline["plain_read"] = {"what": "a kernel that only reads the same K and V caches (non-temporal 16-byte loads), "
                                          "cold, same rotation, best grid", "bytes_per_launch": 2 * cache_bytes,
                                  "kernel_us": best[0], "workgroups": best[1], "achieved": ceil_gbps,
                                  "frac_of_peak": ceil_gbps / HBM_PEAK_GBS,
                                  "verify_kernel_vs_plain_read": (verify_bytes / (v_us * 1e-6) / 1e9) / ceil_gbps}
    iter_bytes = verify_bytes + G * draft_bytes
    out = {
        "metric": "us_per_verify_select_draft_iteration", "value": us_per_step, "unit": "us",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": us_per_step / 1e3,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": workload, "batch": spec.batch, "context": int(L.seq_lens.max()),
                   "context_tokens_total": n_tokens, "layer": args.layer,
                   "num_q_heads": spec.num_q_heads, "num_kv_heads": spec.num_kv_heads,
                   "head_dim": spec.head_dim, "page_size": 16, "gamma": spec.gamma,
                   "kv_budget_tokens": budget, "draft_steps": G, "variant": args.variant,
                   "live_drafting": bool(args.live),
                   "kv_cache_copies_rotated": len(copies)},
        "iteration_kv_bytes": iter_bytes,
        "iteration_gbps": iter_bytes / (us_per_step * 1e-6) / 1e9,
        "roofline": roofline,
    }
    if roofline_draft is not None:
        out["roofline_draft"] = roofline_draft

    if args.extras:
        # (1) per-iteration HIP events: spread of single iterations (the events add a little to each)
        evs = [(vb.HipEvent(), vb.HipEvent()) for _ in range(K)]
        torch.cuda.synchronize()
        for i in range(K):
            evs[i][0].record(stream)
            step(i)
            evs[i][1].record(stream)
        torch.cuda.synchronize()
        per = sorted(a.elapsed_ms(b) * 1e3 for a, b in evs)
        # (2) warm caches: every step reads the same cache copy
        for i in range(W):
            run_one(copies[0])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(K):
            run_one(copies[0])
        torch.cuda.synchronize()
        warm_us = (time.perf_counter() - t0) / K * 1e6
        # (3) the iteration replayed from ONE captured HIP graph that holds an iteration for every cache copy (a serving
        #     engine captures a whole decoding step, hundreds of kernels, not 13: a graph launch has a fixed cost)
        side = torch.cuda.Stream(device=dev)
        side.wait_stream(torch.cuda.current_stream(dev))
        with torch.cuda.stream(side):
            for c in copies:
                run_one(c)                             # settle one-time set-up outside capture
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for c in copies:
                run_one(c)
        torch.cuda.synchronize()
        replays = max(1, K // len(copies))
        for i in range(max(1, W // len(copies))):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(replays):
            graph.replay()
        torch.cuda.synchronize()
        graph_us = (time.perf_counter() - t0) / (replays * len(copies)) * 1e6
        # (4) the launch floor: the library's smallest kernel (selection growth on an empty selection: it reads one
        #     length and returns), 200 dependent launches replayed from a graph, and the same calls issued eagerly
        #     through the binding (which measures the host: the GPU is waiting)
        tiny = vb.make_desc(batch=1, num_q_heads=spec.num_q_heads, num_kv_heads=spec.num_kv_heads, num_queries=1,
                            max_blocks=64, max_sel_blocks=64, max_seq_len=1024, num_pages=64,
                            softmax_scale=1.0, head_dim=spec.head_dim)
        t_table = torch.zeros((1, 64), dtype=torch.int32, device=dev)
        t_lens = torch.full((1,), 100, dtype=torch.int32, device=dev)
        t_sel = torch.full((1, 64), -1, dtype=torch.int32, device=dev)
        t_ssl = torch.zeros((1,), dtype=torch.int32, device=dev)
        tiny_args = (tiny, t_table.data_ptr(), t_lens.data_ptr(), 1, t_sel.data_ptr(), t_ssl.data_ptr())
        with torch.cuda.stream(side):
            vb.vegas_extend_selection(*tiny_args, stream=side.cuda_stream)
        torch.cuda.synchronize()
        floor_graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(floor_graph, stream=side):
            for _ in range(200):
                vb.vegas_extend_selection(*tiny_args, stream=side.cuda_stream)
        torch.cuda.synchronize()
        floor_graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(20):
            floor_graph.replay()
        torch.cuda.synchronize()
        floor_graph_us = (time.perf_counter() - t0) / (20 * 200) * 1e6
        t0 = time.perf_counter()
        for _ in range(2000):
            vb.vegas_extend_selection(*tiny_args, stream=stream)
        torch.cuda.synchronize()
        floor_eager_us = (time.perf_counter() - t0) / 2000 * 1e6
        out["extras"] = {"iteration_us_p10": percentile(per, 0.1), "iteration_us_p50": percentile(per, 0.5),
                         "iteration_us_p90": percentile(per, 0.9), "iteration_us_warm_cache": warm_us,
                         "iteration_us_hip_graph": graph_us,
                         "launch_floor_us_graph_replay": floor_graph_us,
                         "launch_floor_us_eager_through_binding": floor_eager_us}

    default_run = (workload == DEFAULT_WORKLOAD and args.layer == 0 and not token and not args.budget and not args.live
                   and args.verify_chunk == 0 and args.draft_chunk == 0)
    if not args.no_cpu_baseline and default_run:
        out["cpu_baseline"] = cpu_baseline(L, spec.budget_tokens, workload)
        out["cpu_baseline"]["us_single_thread"] = oracle_iteration_us(L, spec.budget_tokens, threads=1)["us"]
    if default_run and not args.no_all_workloads:
        # The other baseline configurations (and the two extra shapes) through the same door, one compact record each;
        # a failure there is reported in its record and never costs the headline line.
        del copies, base, path
        torch.cuda.empty_cache()
        out["workloads"] = []
        for name in all_workloads(synth):
            if name == workload:
                continue
            try:
                out["workloads"].append(compact_workload(name, args, torch, vb, harness, synth,
                                                         with_oracle=not args.no_cpu_baseline and name in synth.CONFIGS))
            except Exception as exc:                     # noqa: BLE001 (reported, not hidden)
                out["workloads"].append({"workload": name, "error": f"{type(exc).__name__}: {exc}"})
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
