#!/usr/bin/env python3
"""Benchmark of the paged decode attention step on one MI355X.

A step is one pass of the whole hot path -- pa_decode(): partition kernel (block-table walk,
K/V loads, scores, online softmax, PV, partial write) followed by the log-sum-exp merge kernel
-- over one synthetic Llama-3-8B-shaped decode batch (64 sequences, 32 query / 8 KV heads,
head_dim 128, block_size 16, context lengths uniform in [512, 4096], bf16 KV, randomly permuted
physical blocks).  Inputs are resident in HBM before the timed region starts.  Consecutive steps
read different copies of the KV pool so that the 256 MB last-level cache cannot serve them.

Prints ONE JSON line.  `value` is algorithmic KV bytes (valid tokens only) per second over the
whole step; `roofline` prices the partition kernel alone against the 8 TB/s HBM peak;
`cpu_baseline` is the float64 oracle timed on this machine's host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

HBM_PEAK_GBPS = 8000.0
METRIC = "paged decode attention achieved HBM GB/s (% of peak) + decode tokens/s, 1 GPU"


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", type=int, default=2, choices=[1, 2, 3, 4, 5, 6],
                    help="named config (default 2: the Llama-3-8B-shaped batch the metric is quoted on; 6: the "
                         "prompt-caching batch, 20 sequences over one shared 32k-token prefix)")
    ap.add_argument("--no-shared-prefix", action="store_true",
                    help="workload 6: do not tell the library about the shared prefix (every sequence reads it)")
    ap.add_argument("--seed", type=int, default=None)
    ap.add_argument("--pools", type=int, default=0, help="KV pool copies to rotate over (0 = enough for >= 2 GB)")
    ap.add_argument("--partitions", type=int, default=0, help="force the number of partitions (0 = library heuristic)")
    ap.add_argument("--q-len", type=int, default=1,
                    help="query tokens per sequence (default 1: plain decode, the metric's workload; 2..16 times "
                         "the multi-token verification call over the same KV cache instead)")
    ap.add_argument("--window", type=int, default=0, help="sliding window in tokens (default 0: none)")
    ap.add_argument("--num-q-heads", type=int, default=None, help="override the workload's query heads")
    ap.add_argument("--num-kv-heads", type=int, default=None, help="override the workload's KV heads")
    ap.add_argument("--head-dim", type=int, default=None, choices=[64, 128], help="override the workload's head_dim")
    ap.add_argument("--kv-dtype", default=None, choices=["bf16", "fp8"], help="override the workload's KV type")
    ap.add_argument("--length-scale", type=float, default=1.0, help="scale every context length of the workload")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    return ap.parse_args()


def recorded_traffic(workload_name: str):
    """HBM bytes per launch of the partition kernel, from the committed counter summary
    (profiles/partition_<workload>.txt, partition_wide_<workload>.txt or prefix_<workload>.txt, the
    workload named as in this run's config: FETCH_SIZE and WRITE_SIZE, scaled by what the same
    counters read for a copy of known size).  None when there is no summary for this workload or
    the kernel sources changed since the counters were taken."""
    from paper_2605_06068_amd import build as pa_build

    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles")
    path = None
    for prefix in ("partition", "partition_wide", "prefix"):  # one-wave kernel, multi-wave kernel, shared-prefix pass
        cand = os.path.join(here, f"{prefix}_{workload_name}.txt")
        if os.path.exists(cand):
            path = cand
    if path is None:
        return None
    kv = {}
    with open(path) as fh:
        for line in fh:
            if ":" in line and not line.startswith("#"):
                k, v = line.split(":", 1)
                kv[k.strip()] = v.strip()
    if kv.get("kernel_source_sha256") != pa_build.source_digest() or kv.get("workload") != workload_name:
        return None
    try:
        return int(float(kv["traffic_bytes_per_launch"]))
    except (KeyError, ValueError):
        return None


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs on exactly one GPU (no sharding or collectives are part of it); "
              "use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2605_06068_amd import binding as pa
    from paper_2605_06068_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    pa.lib()  # fail loudly if the HIP library is missing
    torch.cuda.set_device(0)

    t0 = time.time()
    kv_override = None if args.kv_dtype is None else (W.KV_BF16 if args.kv_dtype == "bf16" else W.KV_FP8_E4M3)
    batch = W.make_config(args.workload, seed=args.seed, poison=False, q_len=args.q_len, window=args.window,
                          length_scale=args.length_scale, num_q_heads=args.num_q_heads,
                          num_kv_heads=args.num_kv_heads, head_dim=args.head_dim, kv_dtype=kv_override)
    gen_s = time.time() - t0
    shared_blocks = 0 if args.no_shared_prefix else batch.shared_prefix_blocks
    # bytes the step has to read: every valid K/V slot once per sequence that owns it, a declared shared prefix once
    kv_bytes = batch.kv_bytes_unique if shared_blocks > 0 else batch.kv_bytes_visible
    pool_bytes = batch.k_cache.nbytes + batch.v_cache.nbytes
    n_pools = args.pools if args.pools > 0 else max(2, min(8, -(-(2 << 30) // max(pool_bytes, 1))))

    dev = pa.DeviceBatch(batch, num_partitions=args.partitions, shared_prefix_blocks=shared_blocks)
    pools = [(dev.k_cache, dev.v_cache)]
    for _ in range(n_pools - 1):
        pools.append((dev.k_cache.clone(), dev.v_cache.clone()))
    stream = torch.cuda.current_stream()

    def step(i):
        k, v = pools[i % n_pools]
        pa.pa_decode(dev.q, k, v, dev.block_tables, dev.context_lens, dev.scale, dev.kv_dtype, dev.out, dev.k_scale,
                     dev.v_scale, shape=dev.shape, workspace=dev.workspace, stream=stream)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    t_wall = time.perf_counter()
    ev0.record(stream)
    for i in range(args.steps):
        step(i)
    ev1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t_wall) * 1e3
    ms_per_step = ev0.elapsed_time(ev1) / args.steps

    # per-kernel durations: HIP events recorded by the library around each launch, on the same
    # stream, rotating over the same pools
    def profile_round():
        a_sum = b_sum = 0.0
        for i, (k, v) in enumerate(pools):  # one timed launch per pool per round keeps the last-level cache cold
            # an untimed step on the previous pool goes first, so that the timed kernels start on a busy
            # queue as they do in the timed region above (the profile call synchronises afterwards)
            step(i - 1)
            a, b = pa.pa_decode_profile(dev.q, k, v, dev.block_tables, dev.context_lens, dev.scale, dev.kv_dtype,
                                        dev.out, dev.k_scale, dev.v_scale, shape=dev.shape, workspace=dev.workspace,
                                        stream=stream, steps=1)
            a_sum += a
            b_sum += b
        return a_sum, b_sum

    profile_round()
    part_ms = merge_ms = 0.0
    reps = max(1, args.steps // n_pools)
    for _ in range(reps):
        a, b = profile_round()
        part_ms += a
        merge_ms += b
    part_ms /= reps * n_pools
    merge_ms /= reps * n_pools

    gbps = kv_bytes / (ms_per_step * 1e-3) / 1e9
    workload = batch.name + (f"_qlen{args.q_len}" if args.q_len > 1 else "") + (f"_window{args.window}" if args.window > 0 else "")
    n_layers = 80 if batch.num_q_heads >= 64 else 32  # 70B-shaped heads, else 8B-shaped
    tokens_read = kv_bytes / (batch.num_kv_heads * batch.head_dim * 2 * batch.kv_elem_bytes)  # tokens whose K and V the step reads
    part_gbps = kv_bytes / (part_ms * 1e-3) / 1e9
    result = {
        "metric": METRIC,
        "value": round(gbps, 2),
        "unit": "GB/s",
        "pct_of_hbm_peak": round(100.0 * gbps / HBM_PEAK_GBPS, 2),
        "tokens_per_s": round(batch.batch / (ms_per_step * 1e-3), 1),  # attention-layer tokens/s: sequences per step / step time
        # the same divided over the layers of a model of this head shape: an upper bound from attention alone
        "model_equivalent_tokens_per_s": {"n_layers": n_layers, "value": round(batch.batch / (n_layers * ms_per_step * 1e-3), 1),
                                          "note": "attention only, no other layer counted"},
        # 2 flop per multiply-add, q.K and P.V, every query row against every token read: far below any matrix peak
        "attention_tflops": round(4.0 * batch.head_dim * batch.num_q_heads * args.q_len * tokens_read
                                  / (ms_per_step * 1e-3) / 1e12, 2),
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "wall_ms_per_step": round(wall_ms / args.steps, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if batch.kv_dtype == W.KV_BF16 else "fp8_e4m3",
        "data": "synthetic",
        "config": {
            "workload": workload,
            "q_len": args.q_len, "window": args.window,
            "batch": batch.batch, "num_q_heads": batch.num_q_heads,
            "num_kv_heads": batch.num_kv_heads, "head_dim": batch.head_dim, "block_size": batch.block_size,
            "total_context_tokens": batch.total_tokens, "kv_bytes": kv_bytes, "seed": batch.seed,
            "kv_pool_copies": n_pools, "num_partitions": pa.pa_num_partitions(dev.shape, dev.kv_dtype),
            "kernel_variant": pa.pa_kernel_variant(dev.shape, dev.kv_dtype),
            "shared_prefix_blocks": shared_blocks, "kv_bytes_if_nothing_shared": batch.kv_bytes,
        },
        "roofline": {
            "bound": "hbm", "kernel": "partition", "achieved": round(part_gbps, 2), "peak": HBM_PEAK_GBPS,
            "unit": "GB/s", "frac": round(part_gbps / HBM_PEAK_GBPS, 4), "traffic": recorded_traffic(workload),
            "partition_ms": round(part_ms, 5), "merge_ms": round(merge_ms, 5),
        },
    }

    if not args.no_cpu_baseline:
        # CPU-baseline leg: the float64 oracle on the host cores.  Its result also checks that the
        # timed launches produced the right answer (last step's output, every row).
        from oracle import pa_oracle

        pa_oracle.build()
        t = time.perf_counter()
        want = pa_oracle.decode_batch(batch)["out"]
        first = time.perf_counter() - t
        n = int(max(1, min(400, 12.0 / max(first, 1e-3))))  # about 12 s of CPU work
        t = time.perf_counter()
        for _ in range(n):
            pa_oracle.decode_batch(batch)
        per = (time.perf_counter() - t) / n
        err = float(np.max(np.abs(dev.out.cpu().numpy() - want)))
        tol = 1e-2 if batch.kv_dtype == W.KV_BF16 else 5e-2
        result["cpu_baseline"] = {
            "value": round(kv_bytes / per / 1e9, 3), "unit": "GB/s", "cores": pa_oracle.num_threads(),
            "kind": "oracle", "tokens_per_s": round(batch.batch / per, 1), "s_per_step": round(per, 4),
            "sample": f"the full {batch.name} batch (all {batch.batch * args.q_len * batch.num_q_heads} output rows), "
                      f"{n} repetitions, float64, OpenMP over rows",
            "gpu_vs_oracle_max_abs_err": err,
        }
        if not (err <= tol):
            print(f"bench.py: output check failed: max_abs_err {err} > {tol}", file=sys.stderr)
            return 1
    result["setup"] = {"generate_s": round(gen_s, 1), "host_cpus": os.cpu_count()}
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
