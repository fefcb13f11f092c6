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
# runs, each scaled by what the same counter reads for a plain 64 MiB copy (factors 1.9990 and 1.0).
VERIFY_TRAFFIC_BYTES = 138_504_192   # (131378 KiB fetched + 3880 KiB written), profiles/ctx32k_hbm_traffic_pmc.md
WORKLOAD = "ctx32k"


def cpu_baseline(L, budget: int, target_seconds: float = 12.0):
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
            "sample": f"{reps} whole iterations of the {WORKLOAD} workload (verify + select + "
                      f"{L.spec.num_queries} draft steps), float64 NumPy oracle, mean"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--copies", type=int, default=8, help="device copies of the KV cache to rotate over")
    ap.add_argument("--verify-chunk", type=int, default=0)
    ap.add_argument("--draft-chunk", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-events", action="store_true")
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
    vb.load_library()                                   # fail loudly if the HIP library is not built
    spec = synth.CONFIGS[WORKLOAD]
    L = synth.make_layer(spec)
    dev = torch.device("cuda:0")
    base = harness.DeviceLayer.upload(L, dev)
    copies = [base]
    for _ in range(max(1, args.copies) - 1):
        copies.append(harness.DeviceLayer(q_verify=base.q_verify, q_draft=base.q_draft,
                                          k_cache=base.k_cache.clone(), v_cache=base.v_cache.clone(),
                                          block_table=base.block_table, seq_lens=base.seq_lens))
    path = harness.VegasPath.for_layer(L, verify_chunk=args.verify_chunk, draft_chunk=args.draft_chunk)
    G = spec.num_queries
    stream = int(torch.cuda.current_stream(dev).cuda_stream)

    K, W = args.steps, args.warmup

    def step(i: int) -> None:
        path.iteration(copies[i % len(copies)])

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

    def kernel_leg(call, desc, reps: int) -> float:
        """Average duration of one KV-streaming kernel: `reps` back-to-back launches of that kernel
        alone (launch_stages = STREAM), bracketed by two HIP events on the launch stream."""
        desc.launch_stages = vb.STAGE_STREAM
        e0, e1 = vb.HipEvent(), vb.HipEvent()
        for i in range(5):
            call(i)
        torch.cuda.synchronize()
        e0.record(stream)
        for i in range(reps):
            call(i)
        e1.record(stream)
        e1.synchronize()
        desc.launch_stages = 0
        return e0.elapsed_ms(e1) / reps * 1e3

    roofline = {"bound": "hbm", "kernel": "attn_split_kernel<causal, collect> (KV-streaming kernel of vegas_verify_attention)",
                "achieved": None, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": None, "traffic": VERIFY_TRAFFIC_BYTES,
                "bytes_per_launch": verify_bytes}
    roofline_draft = None
    if not args.no_kernel_events:
        v_us = kernel_leg(lambda i: path.verify(copies[i % len(copies)]), path.desc_verify, K)
        roofline["kernel_us"] = v_us
        roofline["achieved"] = verify_bytes / (v_us * 1e-6) / 1e9
        roofline["frac"] = roofline["achieved"] / HBM_PEAK_GBS
        d_us = kernel_leg(lambda i: path.draft(copies[i % len(copies)], i % G), path.desc_draft, K)
        roofline_draft = {"bound": "hbm", "kernel": "attn_split_kernel (KV-streaming kernel of vegas_draft_attention)",
                          "kernel_us": d_us, "achieved": draft_bytes / (d_us * 1e-6) / 1e9, "peak": HBM_PEAK_GBS,
                          "unit": "GB/s", "frac": draft_bytes / (d_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                          "bytes_per_launch": draft_bytes, "traffic": None}
    iter_bytes = verify_bytes + G * draft_bytes
    out = {
        "metric": "us_per_verify_select_draft_iteration", "value": us_per_step, "unit": "us",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": us_per_step / 1e3,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": WORKLOAD, "batch": spec.batch, "context": int(L.seq_lens.max()),
                   "num_q_heads": spec.num_q_heads, "num_kv_heads": spec.num_kv_heads,
                   "head_dim": spec.head_dim, "page_size": 16, "gamma": spec.gamma,
                   "kv_budget_tokens": spec.budget_tokens, "draft_steps": G,
                   "kv_cache_copies_rotated": len(copies)},
        "iteration_kv_bytes": iter_bytes,
        "iteration_gbps": iter_bytes / (us_per_step * 1e-6) / 1e9,
        "roofline": roofline,
    }
    if roofline_draft is not None:
        out["roofline_draft"] = roofline_draft
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(L, spec.budget_tokens)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
