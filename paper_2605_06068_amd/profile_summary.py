"""Writes a rocprofv3 summary of one bench.py workload: kernel durations, HBM traffic and, on
request, the issue / LDS / occupancy / cache counters of its kernels.

    python3 -m paper_2605_06068_amd.profile_summary --out profiles/NAME.txt [--counters] -- <bench.py arguments>

runs, each as a child process of its own (this process never touches the GPU),

    rocprofv3 --kernel-trace --stats ... -- python3 bench.py <arguments> --steps 50 --warmup 10
    rocprofv3 --pmc FETCH_SIZE      ... -- python3 bench.py <arguments> --steps 6 --warmup 2 --pools 2
    rocprofv3 --pmc WRITE_SIZE      ... -- python3 bench.py <arguments> --steps 6 --warmup 2 --pools 2
    (--counters)  one rocprofv3 --pmc run per counter set of COUNTER_SETS, same bench arguments

and reduces their CSV output to a text file of `key: value` lines (bench.py reads
`traffic_bytes_per_launch`, `workload` and `kernel_source_sha256` back from it).  FETCH_SIZE and
WRITE_SIZE (KiB per dispatch) are scaled by what the same counters read, in the same run, for the
largest device-to-device copy of a KV pool, whose size is known.  Raw profiler output goes to a
scratch directory under gpurun_out/ and is deleted afterwards.

Two more modes need no GPU:  --resources OUT.txt  tabulates registers, LDS and scratch of every kernel
from the compiler's remarks;  --index FOLDER  writes FOLDER/INDEX.md from the summaries in it.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os
import shutil
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BENCH_FIXED = ["--no-cpu-baseline", "--no-others"]

# one rocprofv3 --pmc run each (at most 8 SQ counters, or 4 TCC counters, per run)
COUNTER_SETS = [
    ["SQ_LDS_BANK_CONFLICT", "SQ_LDS_IDX_ACTIVE", "SQ_LDS_ADDR_CONFLICT", "SQ_INSTS_LDS", "SQ_INSTS_VALU", "SQ_INSTS_MFMA",
     "SQ_INSTS_SALU", "SQ_INSTS_VMEM"],
    ["SQ_BUSY_CYCLES", "SQ_WAVE_CYCLES", "SQ_ACTIVE_INST_VALU", "SQ_ACTIVE_INST_LDS", "SQ_VALU_MFMA_BUSY_CYCLES",
     "SQ_WAIT_INST_ANY", "SQ_WAIT_INST_LDS", "SQ_ACTIVE_INST_ANY"],
    ["SQ_WAVES", "SQ_BUSY_CU_CYCLES", "SQ_INSTS_SMEM", "SQ_INSTS_VALU_CVT", "SQ_INSTS_VALU_TRANS_F32", "SQ_ACTIVE_INST_SCA",
     "SQ_VALU_MFMA_COEXEC_CYCLES"],
    ["SQC_DCACHE_REQ", "SQC_DCACHE_HITS", "SQC_DCACHE_MISSES", "SQC_TC_DATA_READ_REQ"],
    ["TCC_HIT_sum", "TCC_MISS_sum", "TCC_REQ_sum"],
]


def rocprof(out_dir, tool_args, bench_args, log, limit):
    """One rocprofv3 run of bench.py; returns the JSON line bench.py printed."""
    cmd = ["rocprofv3", *tool_args, "--output-format", "csv", "-d", out_dir, "-o", "run", "--",
           "python3", os.path.join(ROOT, "bench.py"), *bench_args]
    env = dict(os.environ, TMPDIR="/tmp")
    with open(log, "w") as fh:
        rc = subprocess.run(["timeout", "-s", "KILL", str(limit), *cmd], stdout=fh, stderr=subprocess.STDOUT, cwd=ROOT,
                            env=env).returncode
    if rc != 0:
        raise RuntimeError(f"rocprofv3 run failed (exit {rc}); see {log}: {' '.join(cmd)}")
    line = None
    with open(log) as fh:
        for text in fh:
            if text.startswith("{"):
                line = json.loads(text)
    return line


def find_csv(out_dir, suffix):
    hits = glob.glob(os.path.join(out_dir, "**", f"*{suffix}"), recursive=True)
    if not hits:
        raise RuntimeError(f"no *{suffix} under {out_dir}")
    return hits[0]


def counter_means(out_dir):
    """{kernel name: {counter: (dispatches, mean, max)}} from a --pmc run."""
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    with open(find_csv(out_dir, "counter_collection.csv")) as fh:
        for r in csv.DictReader(fh):
            agg[r["Kernel_Name"]][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return {k: {c: (len(v), sum(v) / len(v), max(v)) for c, v in d.items()} for k, d in agg.items()}


def short(name):
    return name.replace("void ", "").replace("(pa::Params)", "").replace("(pa::CheckParams)", "")


def write_resources(out_path):
    """Registers, LDS and scratch of every kernel as the compiler reports them (no GPU needed)."""
    import re

    sys.path.insert(0, ROOT)
    from paper_2605_06068_amd import build as pa_build

    cmd = [pa_build.hipcc(), pa_build.ARCH, *pa_build.COMMON_FLAGS, *pa_build.DEVICE_ONLY_FLAGS, "--cuda-device-only",
           "-Rpass-analysis=kernel-resource-usage", f"-I{pa_build.INCLUDE}", f"-I{pa_build.CSRC}", "-S", "-o", os.devnull,
           *pa_build.sources()]
    text = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, check=True).stdout.decode()
    rows, cur = [], None
    for line in text.splitlines():
        m = re.search(r"remark:\s+(.*?): (.*?) \[-Rpass", line)
        if not m:
            continue
        k, v = m.group(1).strip(), m.group(2).strip()
        if k == "Function Name":
            cur = {"name": v}
            rows.append(cur)
        elif cur is not None:
            cur[k] = v
    names = subprocess.run(["c++filt"] + [r["name"] for r in rows], stdout=subprocess.PIPE, check=True).stdout.decode().splitlines()
    table = []
    for r, n in zip(rows, names):
        n = re.sub(r"\(.*\)$", "", n.replace("void pa::", "")).strip()
        table.append((n, r["TotalSGPRs"], r["VGPRs"], r["AGPRs"], r["ScratchSize [bytes/lane]"],
                      r["SGPRs Spill"] + "/" + r["VGPRs Spill"], r["LDS Size [bytes/block]"], r["Occupancy [waves/SIMD]"]))
    scratch_free = all(t[4] == "0" and t[5].endswith("/0") for t in table)
    w = max(len(t[0]) for t in table)
    fmt = "%-*s %5s %5s %5s %7s %7s %7s %4s\n"
    with open(out_path, "w") as fh:
        fh.write("# Register, LDS and scratch use of every kernel of the library, as the compiler reports it (gfx950).\n"
                 "# Command (from the repository root; no GPU needed):\n"
                 f"#   python3 -m paper_2605_06068_amd.profile_summary --resources {os.path.relpath(out_path, ROOT)}\n"
                 "# which compiles the device code with -Rpass-analysis=kernel-resource-usage and tabulates the remarks: TotalSGPRs, VGPRs,\n"
                 "# AGPRs, ScratchSize [bytes/lane], spills (SGPR/VGPR), LDS Size [bytes/block], and the occupancy the compiler derives\n"
                 "# from registers and LDS (waves/SIMD).\n"
                 "# Template arguments: partition_mfma_kernel<D, NSTAGE, CPAD, KV(0 bf16, 1 fp8), TRACE, PRECISE>;\n"
                 "#                     partition_mfma_wide_kernel<D, NW, NCT, NSTAGE, KV, TRACE, PREFIX, PRECISE>;\n"
                 "#                     partition_mfma_staged_kernel<D, NS, NCT, KV, TRACE>.\n"
                 + ("# No kernel uses scratch memory or spills a vector register.  The scalar registers counted under spills live in\n"
                    "# lanes of a vector register (v_writelane / v_readlane), not in memory.\n" if scratch_free else
                    "# SOME KERNELS USE SCRATCH MEMORY OR SPILL VECTOR REGISTERS: see the scratch and spills columns.\n"))
        fh.write(f"kernel_source_sha256: {pa_build.source_digest()}\n")
        fh.write(fmt % (w, "kernel", "sgpr", "vgpr", "agpr", "scratch", "spills", "lds", "occ"))
        for t in sorted(table):
            fh.write(fmt % ((w,) + t))
    print(f"{out_path}: {len(table)} kernels, scratch-free: {scratch_free}")


def write_index(folder):
    """INDEX.md: one line per summary in `folder`."""
    rows = []
    for f in sorted(os.listdir(folder)):
        if not f.endswith(".txt") or f.startswith("kernel_resources"):
            continue
        kv = {}
        with open(os.path.join(folder, f)) as fh:
            for line in fh:
                if ":" in line and not line.startswith("#"):
                    k, v = line.split(":", 1)
                    kv[k.strip()] = v.strip()
        if "partition_avg_ns" not in kv:
            continue
        counters = "yes" if any(k.startswith("partition_SQ_") for k in kv) else ""
        rows.append(f"| `{f}` | `{kv.get('partition_kernel', '?')}` | {float(kv['partition_avg_ns']) / 1e3:.1f} µs | "
                    f"{100 * float(kv['partition_frac_of_8000_GBps']):.1f} % | {float(kv['all_kernels_avg_ns_per_step']) / 1e3:.1f} µs | "
                    f"{kv.get('traffic_over_algorithmic', '-')} | {counters} |")
    with open(os.path.join(folder, "INDEX.md"), "w") as fh:
        fh.write("# rocprofv3 summaries in this folder\n\n"
                 "One file per kernel and workload, written by `python3 -m paper_2605_06068_amd.profile_summary` (each file names its\n"
                 "full command, which runs `bench.py` of this repository under rocprofv3, and the hash of the kernel sources the figures\n"
                 "belong to). Durations are rocprofv3 averages per launch; the fraction is algorithmic KV bytes / duration / 8000 GB/s;\n"
                 "traffic is measured HBM bytes (FETCH_SIZE + WRITE_SIZE, calibrated on a copy of known size) over algorithmic KV bytes;\n"
                 "files marked under *counters* also hold the issue / LDS / occupancy / cache counters of their kernels.\n"
                 "`kernel_resources_gfx950.txt` lists registers, LDS and scratch of every kernel as the compiler reports them.\n"
                 "This index: `python3 -m paper_2605_06068_amd.profile_summary --index profiles`.\n\n"
                 "| file | dominant kernel | its time | of HBM peak | all kernels of a step | traffic / algorithmic | counters |\n"
                 "|---|---|---|---|---|---|---|\n" + "\n".join(rows) + "\n")
    print(f"{folder}/INDEX.md: {len(rows)} summaries")


def main():
    argv = sys.argv[1:]
    if len(argv) == 2 and argv[0] == "--resources":
        return write_resources(os.path.abspath(argv[1]))
    if len(argv) == 2 and argv[0] == "--index":
        return write_index(os.path.abspath(argv[1]))
    bench_args = []
    if "--" in argv:
        i = argv.index("--")
        argv, bench_args = argv[:i], argv[i + 1:]
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", required=True, help="summary file to write (profiles/NAME.txt)")
    ap.add_argument("--title", default=None)
    ap.add_argument("--counters", action="store_true", help="also collect the counter sets of COUNTER_SETS")
    ap.add_argument("--scratch", default=os.path.join(ROOT, "gpurun_out", "profile_scratch"))
    args = ap.parse_args(argv)
    sys.path.insert(0, ROOT)
    from paper_2605_06068_amd import build as pa_build

    scratch = args.scratch
    shutil.rmtree(scratch, ignore_errors=True)
    os.makedirs(scratch)
    bench = BENCH_FIXED + bench_args
    line = rocprof(os.path.join(scratch, "stats"), ["--kernel-trace", "--stats"], bench + ["--steps", "50", "--warmup", "10"],
                   os.path.join(scratch, "stats.log"), 400)
    with open(find_csv(os.path.join(scratch, "stats"), "kernel_stats.csv")) as fh:
        stats = [r for r in csv.DictReader(fh) if r["Name"].startswith("void pa::")]
    stats.sort(key=lambda r: -float(r["TotalDurationNs"]))
    short_run = bench + ["--steps", "6", "--warmup", "2", "--pools", "2"]
    pmc = {}
    for c in ("FETCH_SIZE", "WRITE_SIZE"):
        rocprof(os.path.join(scratch, c), ["--pmc", c], short_run, os.path.join(scratch, c + ".log"), 300)
        pmc[c] = counter_means(os.path.join(scratch, c))
    copy = next(k for k in pmc["WRITE_SIZE"] if "copyBuffer" in k)
    copy_w, copy_f = pmc["WRITE_SIZE"][copy]["WRITE_SIZE"][2], pmc["FETCH_SIZE"][copy]["FETCH_SIZE"][2]
    fscale = copy_w / copy_f

    cfg = line["config"]
    kv_bytes = cfg["kv_bytes"]
    self_cmd = "python3 -m paper_2605_06068_amd.profile_summary --out " + os.path.relpath(args.out, ROOT) + \
               (" --counters" if args.counters else "") + " -- " + " ".join(bench_args)
    out = [f"# rocprofv3 summary: {args.title or cfg['workload']} (MI355X, one GPU)",
           '# Command (from the repository root, after `python -c "import __graft_entry__ as g; g.build()"`):',
           f"#   {self_cmd}",
           "# which runs rocprofv3 --kernel-trace --stats (50 steps after 10), --pmc FETCH_SIZE and --pmc WRITE_SIZE (6 steps,",
           "# two pool copies)" + (" and one --pmc run per counter set below" if args.counters else "") +
           f" on: python3 bench.py {' '.join(bench)}",
           "# Counter values are means over the dispatches of a run (KiB per dispatch for FETCH_SIZE / WRITE_SIZE);",
           "# durations from the kernel-trace run's kernel_stats.csv.",
           f"workload: {cfg['workload']}",
           f"kernel_source_sha256: {pa_build.source_digest()}",
           f"algorithmic_kv_bytes_per_launch: {kv_bytes}",
           f"total_context_tokens: {cfg['total_context_tokens']}",
           f"num_partitions: {cfg['num_partitions']}"]
    total_ns = 0.0
    traffic = None
    names = []
    for i, r in enumerate(stats):
        pre = "partition" if i == 0 else f"kernel{i + 1}"
        avg = float(r["AverageNs"])
        total_ns += avg
        names.append((pre, r["Name"]))
        out += [f"{pre}_kernel: {short(r['Name'])}", f"{pre}_calls: {r['Calls']}", f"{pre}_avg_ns: {avg:.1f}",
                f"{pre}_min_ns: {r['MinNs']}", f"{pre}_max_ns: {r['MaxNs']}"]
        f = pmc["FETCH_SIZE"].get(r["Name"], {}).get("FETCH_SIZE")
        w = pmc["WRITE_SIZE"].get(r["Name"], {}).get("WRITE_SIZE")
        if f:
            out.append(f"{pre}_FETCH_SIZE_KiB: {f[1]:.1f}")
        if w:
            out.append(f"{pre}_WRITE_SIZE_KiB: {w[1]:.1f}")
        if i == 0:
            out += [f"partition_achieved_GBps: {kv_bytes / avg:.1f}", f"partition_frac_of_8000_GBps: {kv_bytes / avg / 8000:.4f}"]
            if f and w:
                traffic = (f[1] * fscale + w[1]) * 1024
    out += [f"all_kernels_avg_ns_per_step: {total_ns:.1f}", f"all_kernels_achieved_GBps: {kv_bytes / total_ns:.1f}",
            f"# calibration: the largest device-to-device copy of a KV pool in the same runs ({copy_w:.0f} KiB known size)",
            f"FETCH_SIZE_copy_KiB: {copy_f:.1f}", f"WRITE_SIZE_copy_KiB: {copy_w:.1f}", f"fetch_scale: {fscale:.5f}",
            "write_scale: 1.00000"]
    if traffic is not None:
        out += [f"traffic_bytes_per_launch: {traffic:.0f}", f"traffic_over_algorithmic: {traffic / kv_bytes:.4f}"]
    out += ["# bench.py line of the kernel-trace run (event timings are inflated under the profiler):",
            f"bench_ms_per_step_under_profiler: {line['ms_per_step']}"]

    if args.counters:
        got = collections.defaultdict(dict)  # kernel -> counter -> mean per dispatch
        for n, cset in enumerate(COUNTER_SETS):
            d = os.path.join(scratch, f"set{n}")
            try:
                rocprof(d, ["--pmc", *cset], short_run, os.path.join(scratch, f"set{n}.log"), 120)
            except RuntimeError as e:
                out.append(f"# counter set {' '.join(cset)}: not collected ({str(e).split(';')[0]})")
                continue
            for k, cs in counter_means(d).items():
                for c, v in cs.items():
                    got[k][c] = v[1]
        out.append("# counters: whole-GPU totals per dispatch (means over the dispatches of a 6-step run), one --pmc run per set:")
        for cset in COUNTER_SETS:
            out.append("#   " + " ".join(cset))
        for pre, name in names:
            c = got.get(name, {})
            if not c:
                continue
            for k in sorted(c):
                out.append(f"{pre}_{k}: {c[k]:.1f}")

            def ratio(a, b, fmt="{:.4f}", times=1.0):
                return fmt.format(times * c[a] / c[b]) if a in c and b in c and c[b] else None

            derived = [
                ("lds_bank_conflict_cycles_per_lds_active_cycle", ratio("SQ_LDS_BANK_CONFLICT", "SQ_LDS_IDX_ACTIVE")),
                ("lds_active_cycles_per_lds_instruction", ratio("SQ_LDS_IDX_ACTIVE", "SQ_INSTS_LDS", "{:.2f}")),
                # SQ_BUSY_CYCLES counts per shader engine (32 of them), SQ_ACTIVE_INST_VALU in units of four
                # cycles and SQ_VALU_MFMA_BUSY_CYCLES in cycles, both summed over the 1024 SIMDs
                ("valu_pipe_issuing_share_of_kernel_time_per_simd", ratio("SQ_ACTIVE_INST_VALU", "SQ_BUSY_CYCLES", "{:.4f}", 4.0 * 32 / 1024)),
                ("matrix_pipe_busy_share_of_kernel_time_per_simd", ratio("SQ_VALU_MFMA_BUSY_CYCLES", "SQ_BUSY_CYCLES", "{:.4f}", 32.0 / 1024)),
                ("matrix_pipe_busy_cycles_with_a_vector_instruction_issuing_share", ratio("SQ_VALU_MFMA_COEXEC_CYCLES", "SQ_VALU_MFMA_BUSY_CYCLES")),
                ("resident_waves_per_simd_while_busy", ratio("SQ_WAVE_CYCLES", "SQ_BUSY_CYCLES", "{:.2f}", 4.0 * 32 / 1024)),
                ("wave_cycles_waiting_on_any_instruction_share", ratio("SQ_WAIT_INST_ANY", "SQ_WAVE_CYCLES")),
                ("wave_cycles_waiting_on_lds_share", ratio("SQ_WAIT_INST_LDS", "SQ_WAVE_CYCLES")),
                ("scalar_cache_hit_rate", ratio("SQC_DCACHE_HITS", "SQC_DCACHE_REQ")),
                ("scalar_cache_reads_sent_to_l2_per_request", ratio("SQC_TC_DATA_READ_REQ", "SQC_DCACHE_REQ")),
                ("l2_hit_rate_all_requests", ratio("TCC_HIT_sum", "TCC_REQ_sum")),
                ("valu_instructions_per_wave", ratio("SQ_INSTS_VALU", "SQ_WAVES", "{:.1f}")),
                ("salu_instructions_per_wave", ratio("SQ_INSTS_SALU", "SQ_WAVES", "{:.1f}")),
                ("mfma_instructions_per_wave", ratio("SQ_INSTS_MFMA", "SQ_WAVES", "{:.1f}")),
                ("lds_instructions_per_wave", ratio("SQ_INSTS_LDS", "SQ_WAVES", "{:.1f}")),
            ]
            for k, v in derived:
                if v is not None:
                    out.append(f"{pre}_{k}: {v}")
    os.makedirs(os.path.dirname(os.path.abspath(args.out)), exist_ok=True)
    with open(args.out, "w") as fh:
        fh.write("\n".join(out) + "\n")
    shutil.rmtree(scratch, ignore_errors=True)
    avg0 = float(stats[0]["AverageNs"])
    print(f"{os.path.basename(args.out)}: {short(stats[0]['Name'])} {avg0 / 1000:.1f} us = {kv_bytes / avg0 / 8000:.3f} of peak; "
          f"step {total_ns / 1000:.1f} us" + (f"; traffic/algorithmic {traffic / kv_bytes:.4f}" if traffic else ""), flush=True)


if __name__ == "__main__":
    main()
