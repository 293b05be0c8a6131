#!/usr/bin/env python3
"""Benchmark of the paged decode attention step on one MI355X.

A step is one pass of the whole hot path -- pa_decode(): partition kernel (block-table walk,
K/V loads, scores, online softmax, PV, partial write) followed by the log-sum-exp merge kernel
-- over one synthetic Llama-3-8B-shaped decode batch (64 sequences, 32 query / 8 KV heads,
head_dim 128, block_size 16, context lengths uniform in [512, 4096], bf16 KV, randomly permuted
physical blocks).  Inputs are resident in HBM before the timed region starts.  Consecutive steps
read different copies of the KV pool so that the 256 MB last-level cache cannot serve them.

Prints ONE JSON line.  `value` is algorithmic KV bytes (valid tokens only) per second over the
whole step (K steps between one pair of events); `per_call` times the same calls one by one, each
between its own pair of events, and gives the median beside the mean; `roofline` prices the
partition kernel alone against the 8 TB/s HBM peak; `cpu_baseline` is the float64 oracle timed on
this machine's host cores, with all threads and with one; `others` carries the same measurements
(step time, GB/s, fraction of peak, kernel times, error against the oracle on sampled rows) for
the other workloads: the long-context, ragged and fp8 batches, the prompt-cache batch with its
shared prefix, 16-token verification and a 1024-token sliding window on the 8B-shaped batch.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

HBM_PEAK_GBPS = 8000.0
METRIC = "paged decode attention achieved HBM GB/s (% of peak) + decode tokens/s, 1 GPU"

# (workload, q_len, window): what `others` reports beside the headline
OTHER_WORKLOADS = [(3, 1, 0), (4, 1, 0), (5, 1, 0), (6, 1, 0), (2, 16, 0), (5, 4, 0), (5, 8, 0), (5, 16, 0), (2, 1, 1024)]


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
    ap.add_argument("--no-others", action="store_true", help="time the named workload only")
    return ap.parse_args()


def recorded_traffic(workload_name: str):
    """(HBM bytes per launch of the partition kernel, where that figure is recorded): from the
    committed counter summary (profiles/partition_<workload>.txt, partition_wide_<workload>.txt,
    partition_staged_<workload>.txt or prefix_<workload>.txt, the workload named as in this run's config: FETCH_SIZE and WRITE_SIZE,
    scaled by what the same counters read for a copy of known size).  (None, why) when there is no
    summary for this workload or the kernel sources changed since the counters were taken.  The
    counters are never collected inside a timed run."""
    from paper_2605_06068_amd import build as pa_build

    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles")
    path = None
    # one-wave kernel, multi-wave kernel, stage-split kernel, shared-prefix pass
    for prefix in ("partition", "partition_wide", "partition_staged", "prefix"):
        cand = os.path.join(here, f"{prefix}_{workload_name}.txt")
        if os.path.exists(cand):
            path = cand
    if path is None:
        return None, "no counter summary for this workload under profiles/"
    kv = {}
    with open(path) as fh:
        for line in fh:
            if ":" in line and not line.startswith("#"):
                k, v = line.split(":", 1)
                kv[k.strip()] = v.strip()
    rel = os.path.relpath(path, os.path.dirname(here))
    if kv.get("kernel_source_sha256") != pa_build.source_digest() or kv.get("workload") != workload_name:
        return None, f"{rel} was recorded for other kernel sources"
    try:
        return int(float(kv["traffic_bytes_per_launch"])), f"recorded in {rel} (rocprofv3 --pmc, the same kernel sources)"
    except (KeyError, ValueError):
        return None, f"{rel} holds no traffic figure"


def cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as fh:
            for line in fh:
                if line.lower().startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def workload_name(batch, q_len, window):
    return batch.name + (f"_qlen{q_len}" if q_len > 1 else "") + (f"_window{window}" if window > 0 else "")


def measure(pa, torch, batch, *, steps, warmup, calls, pools=0, partitions=0, shared_blocks=None):
    """Put the batch on the device, rotate over copies of its KV pool, and time pa_decode three ways:
    `steps` calls between one pair of events (after `warmup` untimed ones); `calls` calls each between
    its own pair of events; the partition and merge kernels alone (events recorded by the library
    around each launch).  Returns the figures and the device batch (whose `out` holds the last
    step's result)."""
    shared = batch.shared_prefix_blocks if shared_blocks is None else shared_blocks
    # bytes the step has to read: every valid K/V slot once per sequence that owns it, a declared shared prefix once
    kv_bytes = batch.kv_bytes_unique if shared > 0 else batch.kv_bytes_visible
    pool_bytes = batch.k_cache.nbytes + batch.v_cache.nbytes
    n_pools = pools if pools > 0 else max(2, min(8, -(-(2 << 30) // max(pool_bytes, 1))))
    dev = pa.DeviceBatch(batch, num_partitions=partitions, shared_prefix_blocks=shared)
    kv_pools = [(dev.k_cache, dev.v_cache)]
    for _ in range(n_pools - 1):
        kv_pools.append((dev.k_cache.clone(), dev.v_cache.clone()))
    stream = torch.cuda.current_stream()

    def step(i):
        k, v = kv_pools[i % n_pools]
        pa.pa_decode(dev.q, k, v, dev.block_tables, dev.context_lens, dev.scale, dev.kv_dtype, dev.out, dev.k_scale,
                     dev.v_scale, shape=dev.shape, workspace=dev.workspace, stream=stream)

    # ---- K steps between one pair of events
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    t_wall = time.perf_counter()
    ev0.record(stream)
    for i in range(steps):
        step(i)
    ev1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t_wall) * 1e3
    ms_per_step = ev0.elapsed_time(ev1) / steps

    # ---- every call between its own pair of events (one event between consecutive calls serves both)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(calls + 1)]
    marks[0].record(stream)
    for i in range(calls):
        step(i)
        marks[i + 1].record(stream)
    torch.cuda.synchronize()
    per_call = [marks[i].elapsed_time(marks[i + 1]) for i in range(calls)]

    # ---- per-kernel durations: HIP events recorded by the library around each launch, on the same
    # stream, rotating over the same pools
    def profile_round():
        a_sum = b_sum = 0.0
        for i, (k, v) in enumerate(kv_pools):  # one timed launch per pool per round keeps the last-level cache cold
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
    reps = max(1, min(steps, calls) // n_pools)
    for _ in range(reps):
        a, b = profile_round()
        part_ms += a
        merge_ms += b
    part_ms /= reps * n_pools
    merge_ms /= reps * n_pools
    step(0)  # leave the result of a plain call in dev.out
    torch.cuda.synchronize()
    del kv_pools[1:]
    return {"dev": dev, "kv_bytes": kv_bytes, "n_pools": n_pools, "ms_per_step": ms_per_step, "wall_ms": wall_ms,
            "per_call": per_call, "partition_ms": part_ms, "merge_ms": merge_ms, "shared_blocks": shared}


def per_call_summary(per_call):
    return {"calls": len(per_call), "median_ms": round(statistics.median(per_call), 5),
            "mean_ms": round(statistics.fmean(per_call), 5), "min_ms": round(min(per_call), 5),
            "max_ms": round(max(per_call), 5)}


def sampled_error(np, pa_oracle, batch, got, n_rows, seed):
    """max |GPU - oracle| over a seeded sample of output rows (every sequence at least once)."""
    rng = np.random.default_rng(seed)
    Q, Hq = batch.q_len, batch.num_q_heads
    seqs = list(range(batch.batch)) + [int(x) for x in rng.integers(0, batch.batch, size=max(0, n_rows - batch.batch))]
    seqs = seqs[:max(n_rows, 1)]
    if Q > 1:
        rows = [(s, int(rng.integers(0, Q)), int(rng.integers(0, Hq))) for s in seqs]
        sel = np.stack([got[s, i, h] for s, i, h in rows])
    else:
        rows = [(s, int(rng.integers(0, Hq))) for s in seqs]
        sel = np.stack([got[s, h] for s, h in rows])
    want = pa_oracle.decode_batch(batch, rows=rows)["out"]
    return float(np.max(np.abs(sel.astype(np.float64) - want))), len(rows)


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
    t_start = time.time()

    kv_override = None if args.kv_dtype is None else (W.KV_BF16 if args.kv_dtype == "bf16" else W.KV_FP8_E4M3)
    batch = W.make_config(args.workload, seed=args.seed, poison=False, q_len=args.q_len, window=args.window,
                          length_scale=args.length_scale, num_q_heads=args.num_q_heads,
                          num_kv_heads=args.num_kv_heads, head_dim=args.head_dim, kv_dtype=kv_override)
    gen_s = time.time() - t_start
    calls = max(50, args.steps)  # at least 50 individually timed calls
    m = measure(pa, torch, batch, steps=args.steps, warmup=max(args.warmup, 0), calls=calls, pools=args.pools,
                partitions=args.partitions, shared_blocks=0 if args.no_shared_prefix else None)
    dev, kv_bytes, ms_per_step = m["dev"], m["kv_bytes"], m["ms_per_step"]
    part_ms, merge_ms = m["partition_ms"], m["merge_ms"]

    gbps = kv_bytes / (ms_per_step * 1e-3) / 1e9
    workload = workload_name(batch, args.q_len, args.window)
    n_layers = 80 if batch.num_q_heads >= 64 else 32  # 70B-shaped heads, else 8B-shaped
    tokens_read = kv_bytes / (batch.num_kv_heads * batch.head_dim * 2 * batch.kv_elem_bytes)  # tokens whose K and V the step reads
    part_gbps = kv_bytes / (part_ms * 1e-3) / 1e9
    traffic, traffic_source = recorded_traffic(workload)
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
        "wall_ms_per_step": round(m["wall_ms"] / args.steps, 5),
        "per_call": per_call_summary(m["per_call"]),
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
            "kv_pool_copies": m["n_pools"], "num_partitions": pa.pa_num_partitions(dev.shape, dev.kv_dtype),
            "kernel_variant": pa.pa_kernel_variant(dev.shape, dev.kv_dtype),
            "shared_prefix_blocks": m["shared_blocks"], "kv_bytes_if_nothing_shared": batch.kv_bytes,
        },
        "roofline": {
            "bound": "hbm", "kernel": "partition", "achieved": round(part_gbps, 2), "peak": HBM_PEAK_GBPS,
            "unit": "GB/s", "frac": round(part_gbps / HBM_PEAK_GBPS, 4), "traffic": traffic,
            "traffic_source": traffic_source,
            "partition_ms": round(part_ms, 5), "merge_ms": round(merge_ms, 5),
            "timing": "HIP events recorded by the library around single launches; each pair adds about 3 us to its kernel, so "
                      "partition_ms + merge_ms exceeds ms_per_step; rocprofv3 durations of the same kernels are under profiles/",
        },
    }

    pa_oracle = None
    if not args.no_cpu_baseline or not args.no_others:
        from oracle import pa_oracle

        pa_oracle.build()
    tol = lambda b: 1e-2 if b.kv_dtype == W.KV_BF16 else 5e-2

    if not args.no_cpu_baseline:
        # CPU-baseline leg: the float64 oracle on the host cores, with all threads on the whole batch
        # and with one thread on a sample of its rows.  Its result also checks that the timed
        # launches produced the right answer (last step's output, every row).
        threads_all = pa_oracle.num_threads()
        t = time.perf_counter()
        want = pa_oracle.decode_batch(batch)["out"]
        first = time.perf_counter() - t
        n = int(max(1, min(400, 8.0 / max(first, 1e-3))))  # about 8 s of CPU work
        t = time.perf_counter()
        for _ in range(n):
            pa_oracle.decode_batch(batch)
        per = (time.perf_counter() - t) / n
        # one thread: a strided sample of the output rows sized for about 8 s, scaled to the whole
        # batch by the tokens the rows attend over
        Hq, Q = batch.num_q_heads, batch.q_len
        n_out = batch.batch * Q * Hq
        stride = int(max(1, min(n_out, round(first * threads_all / 8.0))))
        picks = list(range(0, n_out, stride))
        rows = [(r // (Q * Hq), (r // Hq) % Q, r % Hq) for r in picks] if Q > 1 else [(r // Hq, r % Hq) for r in picks]
        lens = batch.context_lens.astype(np.int64)
        frac = float(sum(int(lens[r[0]]) for r in rows)) / max(1.0, float(lens.sum()) * Q * Hq)
        pa_oracle.set_num_threads(1)
        t = time.perf_counter()
        pa_oracle.decode_batch(batch, rows=rows)
        one = (time.perf_counter() - t) / max(frac, 1e-12)
        pa_oracle.set_num_threads(threads_all)
        err = float(np.max(np.abs(dev.out.cpu().numpy() - want)))
        result["cpu_baseline"] = {
            "value": round(kv_bytes / per / 1e9, 3), "unit": "GB/s", "cores": threads_all,
            "kind": "oracle", "tokens_per_s": round(batch.batch / per, 1), "s_per_step": round(per, 4),
            "sample": f"the full {batch.name} batch (all {n_out} output rows), "
                      f"{n} repetitions, float64, OpenMP over rows",
            "cpu_model": cpu_model(), "host_cpus": os.cpu_count(),
            "threads_all": {"threads": threads_all, "value": round(kv_bytes / per / 1e9, 3), "unit": "GB/s",
                            "s_per_step": round(per, 4), "tokens_per_s": round(batch.batch / per, 1)},
            "threads_1": {"threads": 1, "value": round(kv_bytes / one / 1e9, 4), "unit": "GB/s",
                          "s_per_step": round(one, 3), "tokens_per_s": round(batch.batch / one, 2),
                          "sample": f"every {stride}th output row ({len(rows)} rows, {100 * frac:.2f} % of the batch's "
                                    f"row-tokens), one repetition, scaled to the whole batch by row-tokens"},
            "gpu_vs_oracle_max_abs_err": err,
        }
        if not (err <= tol(batch)):
            print(f"bench.py: output check failed: max_abs_err {err} > {tol(batch)}", file=sys.stderr)
            return 1

    if not args.no_others:
        # the other workloads, each measured like the headline (fewer calls) and checked against the
        # oracle on a seeded sample of output rows
        others = []
        del m, dev
        torch.cuda.empty_cache()
        for cfg, q_len, window in OTHER_WORKLOADS:
            if (cfg, q_len, window) == (args.workload, args.q_len, args.window):
                continue
            t0 = time.time()
            b = W.make_config(cfg, poison=False, q_len=q_len, window=window)
            om = measure(pa, torch, b, steps=50, warmup=30, calls=50)
            odev = om["dev"]
            err, n_rows = sampled_error(np, pa_oracle, b, odev.out.cpu().numpy(), 48, 1000 + cfg)
            med = statistics.median(om["per_call"])
            name = workload_name(b, q_len, window)
            tr, tr_src = recorded_traffic(name)
            others.append({
                "workload": name, "dtype": "bf16" if b.kv_dtype == W.KV_BF16 else "fp8_e4m3",
                "batch": b.batch, "num_q_heads": b.num_q_heads, "num_kv_heads": b.num_kv_heads, "head_dim": b.head_dim,
                "q_len": q_len, "window": window, "shared_prefix_blocks": om["shared_blocks"],
                "total_context_tokens": b.total_tokens, "kv_bytes": om["kv_bytes"],
                "num_partitions": pa.pa_num_partitions(odev.shape, odev.kv_dtype),
                "kernel_variant": pa.pa_kernel_variant(odev.shape, odev.kv_dtype),
                "ms_per_step": round(om["ms_per_step"], 5), "per_call": per_call_summary(om["per_call"]),
                "value": round(om["kv_bytes"] / (om["ms_per_step"] * 1e-3) / 1e9, 2), "unit": "GB/s",
                "frac_of_hbm_peak": round(om["kv_bytes"] / (om["ms_per_step"] * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                "frac_of_hbm_peak_median_call": round(om["kv_bytes"] / (med * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                "tokens_per_s": round(b.batch / (om["ms_per_step"] * 1e-3), 1),
                "partition_ms": round(om["partition_ms"], 5), "merge_ms": round(om["merge_ms"], 5),
                "partition_frac_of_hbm_peak": round(om["kv_bytes"] / (om["partition_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                "traffic": tr, "traffic_source": tr_src,
                "max_abs_err": err, "rows_checked": n_rows, "tolerance": tol(b),
                "seconds": round(time.time() - t0, 1),
            })
            if not (err <= tol(b)):
                print(f"bench.py: output check failed on {name}: max_abs_err {err} > {tol(b)}", file=sys.stderr)
                return 1
            del om, odev, b
            torch.cuda.empty_cache()
        result["others"] = others
    result["setup"] = {"generate_s": round(gen_s, 1), "host_cpus": os.cpu_count(), "total_s": round(time.time() - t_start, 1)}
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
