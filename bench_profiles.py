#!/usr/bin/env python3
"""Turns rocprofv3 output of a bench.py run into the short text summaries kept under profiles/ (measurement side,
beside bench.py; no part of the library).

  python bench_profiles.py trace <results.db> [--top N] --bench-args '<bench.py arguments of the profiled run>'
      per-kernel totals of a `rocprofv3 --kernel-trace --stats` run (the rocpd database it writes)
  python bench_profiles.py hbm --fetch F.csv --write W.csv --copy-gib G --workload NAME --steps N [--json OUT.json]
      HBM bytes per launch and kernel family from a `--pmc FETCH_SIZE` run and a `--pmc WRITE_SIZE` run of
      `bench.py --ceilings` (both counters are KiB per dispatch; the stream_copy_kernel dispatches of gm_ceilings, which
      read and write G GiB each -- "copy_buffer_bytes" of the bench line -- are the transfers of known size that scale them)
  python bench_profiles.py mfma --csv C.csv --workload NAME
      matrix-core busy share per kernel from a `--pmc SQ_VALU_MFMA_BUSY_CYCLES GRBM_GUI_ACTIVE
      SQ_INSTS_VALU_MFMA_MOPS_BF16 SQ_INSTS_VALU_MFMA_MOPS_I8` run
"""
from __future__ import annotations

import argparse
import collections
import csv
import json
import re
import sqlite3

# regular expressions over kernel names for each kernel family that bench.py reports (launches of one family are averaged)
FAMILIES = {
    "pair_hop": r"pair_hop_kernel",
    "pair_count": r"pair_count_kernel",
    "two_hop": r"two_hop_kernel",
    "seg_reduce": r"seg_reduce_(chunks|join)_kernel",
    "gather_pool": r"gather_pool(_xcd)?_kernel|dense_tail_kernel",
    # radix_*_kernel<BITS, BYTASK>: the pass by task belongs to the per-(task, field) dictionaries (with the join that reads
    # them off the ordered list), the passes by row key to the ordering of the lookups by row
    "tf_sort": r"tf_sort_kernel|tf_join_kernel|radix_(hist|scatter)_kernel<\d+, true>",
    "tf_count": r"tf_count_kernel",
    "global_sort": r"build_keys_kernel|build_keys_fm_kernel|field_(offsets|table)_kernel|radix_(hist|scatter)_kernel<\d+, false>|seg_flags_kernel|seg_emit_kernel",
    "task_colsum": r"task_colsum_kernel",
    "reduce_tasks": r"reduce_tasks_kernel",
    "axpy_gx": r"axpy_kernel",
    "last_layer": r"last_fwd_kernel|last_bwd",
    # gemm_bf16_kernel<BM, BN, DB, KA, KB, EP>: which operand is read contraction-slowest tells the product's kind;
    # gemm_bf16_pipe_kernel<KA, KB, EP, ..>: the pipelined 256 x 256 kernel, the same two flags
    "gemm_wgrad": r"gemm_bf16_kernel<\d+, \d+, false, true, true|gemm_bf16_pipe_kernel<true, true",
    "gemm_fwd": r"gemm_bf16_kernel<\d+, \d+, false, false, true|gemm_bf16_pipe_kernel<false, true",
    "gemm_bwd": r"gemm_bf16_kernel<\d+, \d+, false, false, false|gemm_bf16_pipe_kernel<false, false",
    "gemm_f32 (all launches)": r"gemm_f32_kernel",
}


def _is_framework(name: str) -> bool:
    return name.startswith("void at::") or "at::native" in name or "rocprim" in name or "hipcub" in name


def trace(a):
    con = sqlite3.connect(a.db)
    rows = list(con.execute("select name, total_calls, total_duration, average, percentage from top_kernels"))
    ours, other_ns, other_calls, probe_ns, probe_calls = [], 0.0, 0, 0.0, 0
    for name, calls, total, avg, _pct in rows:
        if _is_framework(name):
            other_ns += total
            other_calls += calls
        elif re.search(r"mfma_loop(_random)?_kernel|stream_copy_kernel|stream_read_kernel", name):
            probe_ns += total      # bench.py --ceilings: the on-box ceiling probes, not part of the step
            probe_calls += calls
        else:
            ours.append((name.split("(")[0].replace("void ", ""), calls, total, avg))
    tot = sum(r[2] for r in ours)
    ba = a.bench_args or "<bench arguments>"
    print("# rocprofv3 kernel trace of gm_meta_step (per-kernel totals over the whole run: warm-up, timed and event-timed steps)")
    print(f"# command (from /tmp, TMPDIR=/tmp): rocprofv3 --kernel-trace --stats -d <out> -o <name> -- python3 /root/repo/bench.py {ba}")
    print(f"# summary made with: python bench_profiles.py trace <out>/<name>_results.db --top {a.top} --bench-args '{ba}'")
    print(f"{'kernel':56s} {'calls':>6s} {'total_us':>10s} {'avg_us':>10s}   share_of_library_time")
    for name, calls, total, avg in ours[:a.top]:
        print(f"{name[:56]:56s} {calls:6d} {total:10.1f} {avg:10.2f} {100.0 * total / tot:8.2f}%")
    print(f"(ceiling probes of bench.py --ceilings: {probe_calls} calls, {probe_ns:.1f} us)")
    print(f"(input generation and other framework kernels: {other_calls} calls, {other_ns:.1f} us)")


def _read_counter(path, counter):
    per_kernel = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] == counter:
            per_kernel[r["Kernel_Name"]].append(float(r["Counter_Value"]))
    return per_kernel


def hbm(a):
    fetch = {k: [x * 1024.0 for x in v] for k, v in _read_counter(a.fetch, "FETCH_SIZE").items()}
    write = {k: [x * 1024.0 for x in v] for k, v in _read_counter(a.write, "WRITE_SIZE").items()}
    known = a.copy_gib * 2 ** 30

    def copy_reading(tab):
        # the library's own copy kernel (bench.py --ceilings) when the run has it, else the largest copy-like dispatch
        for k, v in tab.items():
            if "stream_copy_kernel" in k:
                return sum(v) / len(v)
        best = 0.0
        for k, v in tab.items():
            if "copy" in k.lower() or "elementwise" in k.lower():
                best = max(best, max(v))
        return best

    cf, cw = copy_reading(fetch), copy_reading(write)
    sf, sw = (known / cf if cf > 0 else 1.0), (known / cw if cw > 0 else 1.0)
    ba = a.bench_args or "<bench arguments>"
    print(f"# HBM traffic per kernel family, workload {a.workload}")
    print("# commands (from /tmp, TMPDIR=/tmp), one counter per run:")
    print(f"#   rocprofv3 --pmc FETCH_SIZE --output-format csv -d <f> -o p -- python3 /root/repo/bench.py {ba}")
    print(f"#   rocprofv3 --pmc WRITE_SIZE --output-format csv -d <w> -o p -- python3 /root/repo/bench.py {ba}")
    print(f"#   python bench_profiles.py hbm --fetch <f>/.../p_counter_collection.csv --write <w>/.../p_counter_collection.csv "
          f"--copy-gib {a.copy_gib:g} --workload {a.workload} --steps {a.steps} --bench-args '{ba}' --json <json>")
    print(f"# {a.steps} meta steps per run (timed + warm-up + event-timed).  FETCH_SIZE / WRITE_SIZE are KiB per dispatch; the run's "
          f"{a.copy_gib:g} GiB device copies (a kernel that reads and")
    print("# writes that much) are the transfers of known size that scale them.  \"bytes/launch\" is per kernel dispatch of the family.")
    print(f"# copy probe of {known:.0f} B read as FETCH_SIZE {cf:.0f} B, WRITE_SIZE {cw:.0f} B -> scale factors {sf:.3f}, {sw:.3f}")
    print(f"# {'family':24s} {'dispatches/step':>16s} {'fetch GB/step':>14s} {'write GB/step':>14s} {'bytes/launch':>14s}")
    out, per_step = {}, {}
    for fam, pattern in FAMILIES.items():
        fb = wb = 0.0
        n = 0
        rx = re.compile(pattern)
        for k, v in fetch.items():
            if rx.search(k):
                fb += sum(v) * sf
                n += len(v)
        for k, v in write.items():
            if rx.search(k):
                wb += sum(v) * sw
        if n == 0:
            continue
        out[fam] = (fb + wb) / n
        per_step[fam] = (fb + wb) / a.steps
        print(f"  {fam:24s} {n / a.steps:16.1f} {fb / a.steps / 1e9:14.3f} {wb / a.steps / 1e9:14.3f} {out[fam]:14.4g}")
    if a.json:
        with open(a.json, "w") as fh:
            json.dump({"workload": a.workload, "unit": "bytes", "scale_fetch": sf, "scale_write": sw,
                       "bytes_per_launch": out, "bytes_per_step": per_step, "steps": a.steps,
                       "tasks_in_the_profiled_run": a.tasks}, fh, indent=1)


def mfma(a):
    names = ["SQ_VALU_MFMA_BUSY_CYCLES", "GRBM_GUI_ACTIVE", "SQ_INSTS_VALU_MFMA_MOPS_BF16", "SQ_INSTS_VALU_MFMA_MOPS_I8"]
    tabs = {n: _read_counter(a.csv, n) for n in names}
    ba = a.bench_args or "<bench arguments>"
    print(f"# Matrix-core utilisation per kernel, workload {a.workload}")
    print("# command (from /tmp, TMPDIR=/tmp):")
    print(f"#   rocprofv3 --pmc {' '.join(names)} --output-format csv -d <dir> -o p -- python3 /root/repo/bench.py {ba}")
    print(f"#   python bench_profiles.py mfma --csv <dir>/.../p_counter_collection.csv --workload {a.workload} --bench-args '{ba}'")
    print("# values are averages per dispatch.  GRBM_GUI_ACTIVE is summed over the 8 XCDs (divided by 8 below),")
    print("# SQ_VALU_MFMA_BUSY_CYCLES over the 1024 SIMDs:")
    print("#   MFMA busy % = SQ_VALU_MFMA_BUSY_CYCLES / (GRBM_GUI_ACTIVE / 8 * 1024) * 100   (rocprofv3's own MfmaUtil expression)")
    print("#   matrix-core ops = (SQ_INSTS_VALU_MFMA_MOPS_BF16 + SQ_INSTS_VALU_MFMA_MOPS_I8) * 512")
    print(f"# {'kernel':60s} {'dispatches':>10s} {'active cycles':>14s} {'MFMA busy cycles':>16s} {'MFMA busy %':>11s} {'ops/dispatch':>14s}")
    rows = []
    for k, busy in tabs[names[0]].items():
        if _is_framework(k) or sum(busy) == 0:
            continue
        act = tabs[names[1]].get(k, [])
        n = len(busy)
        mb, ma = sum(busy) / n, (sum(act) / max(len(act), 1))
        ops = (sum(tabs[names[2]].get(k, [0])) + sum(tabs[names[3]].get(k, [0]))) / n * 512
        rows.append((sum(act), k.split("(")[0].replace("void ", ""), n, ma, mb, 100.0 * mb / (ma / 8 * 1024) if ma > 0 else 0.0, ops))
    for _, k, n, ma, mb, pct, ops in sorted(rows, reverse=True):
        print(f"  {k[:60]:60s} {n:10d} {ma:14.4g} {mb:16.4g} {pct:11.1f} {ops:14.4g}")
    print("# gemm_bf16_kernel<BM,BN,false,KA,KB,EP>: KA,KB = false,true forward products; false,false backward (dA) products;")
    print("# true,true weight gradients.  gemm_bf16_pipe_kernel<KA,KB,EP,..>: the pipelined 256 x 256 kernel, the same two flags.")
    print("# EP encodes the fused epilogue of the launch.")


def main():
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="cmd", required=True)
    t = sub.add_parser("trace")
    t.add_argument("db")
    t.add_argument("--top", type=int, default=40)
    t.add_argument("--bench-args", default="")
    h = sub.add_parser("hbm")
    h.add_argument("--fetch", required=True)
    h.add_argument("--write", required=True)
    h.add_argument("--copy-gib", type=float, required=True)
    h.add_argument("--workload", required=True)
    h.add_argument("--steps", type=int, default=1, help="meta steps the profiled run made (timed + warm-up + event-timed)")
    h.add_argument("--json", default=None)
    h.add_argument("--tasks", type=int, default=None, help="tasks of the profiled run (when it was a share of the workload)")
    h.add_argument("--bench-args", default="")
    m = sub.add_parser("mfma")
    m.add_argument("--csv", required=True)
    m.add_argument("--workload", required=True)
    m.add_argument("--bench-args", default="")
    a = ap.parse_args()
    {"trace": trace, "hbm": hbm, "mfma": mfma}[a.cmd](a)


if __name__ == "__main__":
    main()
