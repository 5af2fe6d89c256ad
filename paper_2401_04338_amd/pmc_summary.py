"""Summarises rocprofv3 counter runs of bench.py into HBM bytes per launch and kernel family.

Input: the counter_collection CSV of a `rocprofv3 --pmc FETCH_SIZE` run and of a `--pmc WRITE_SIZE` run of
`bench.py --copy-probe-gib G` (both counters are in KiB per dispatch).  The device copy of G GiB that the
bench performs is a transfer of known size: its reading gives the factor that scales the other kernels'.

    python -m paper_2401_04338_amd.pmc_summary --fetch F.csv --write W.csv --copy-gib 1 --workload c3_medium \
        --json profiles/hbm_traffic_c3_medium.json > profiles/hbm_traffic_c3_medium.txt
"""
from __future__ import annotations

import argparse
import collections
import csv
import json

# kernel-name fragments of each kernel family that bench.py reports (launches of one family are averaged)
FAMILIES = {
    "pair_hop": ["pair_hop_kernel"],
    "pair_count": ["pair_count_kernel"],
    "two_hop": ["two_hop_kernel"],
    "seg_reduce": ["seg_reduce_chunks_kernel", "seg_reduce_join_kernel"],
    "gather_pool": ["gather_pool_kernel", "dense_tail_kernel"],
    "tf_sort": ["tf_sort_kernel"],
    "tf_count": ["tf_count_kernel"],
    "global_sort": ["build_keys_kernel", "radix_hist_kernel", "radix_scatter_kernel", "seg_flags_kernel", "seg_emit_kernel"],
    "transpose_act": ["transpose_bf16_kernel"],
    "task_colsum": ["task_colsum_kernel"],
    "reduce_tasks": ["reduce_tasks_kernel"],
    "axpy_gx": ["axpy_kernel"],
    # template flags of gemm_bf16_kernel<BM, BN, DB, KA, KB>: which operand is read contraction-slowest
    "gemm_wgrad": ["false, true, true>"],
    "gemm_fwd": ["false, false, true>"],
    "gemm_bwd": ["false, false, false>"],
    "gemm_f32 (all launches)": ["gemm_f32_kernel"],
}


def read(path, counter):
    per_kernel = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] != counter:
            continue
        per_kernel[r["Kernel_Name"]].append(float(r["Counter_Value"]) * 1024.0)
    return per_kernel


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--fetch", required=True)
    ap.add_argument("--write", required=True)
    ap.add_argument("--copy-gib", type=float, required=True)
    ap.add_argument("--workload", required=True)
    ap.add_argument("--steps", type=int, default=1, help="meta steps the profiled run made (timed + warm-up + 2 profiling)")
    ap.add_argument("--json", default=None)
    ap.add_argument("--bench-args", default="", help="bench.py arguments of the two profiled runs (for the header)")
    a = ap.parse_args()
    fetch, write = read(a.fetch, "FETCH_SIZE"), read(a.write, "WRITE_SIZE")
    known = a.copy_gib * 2 ** 30

    def copy_reading(tab):
        # the probe is the largest single copy-like dispatch of the run
        best = 0.0
        for k, v in tab.items():
            if "copy" in k.lower() or "elementwise" in k.lower():
                best = max(best, max(v))
        return best

    cf, cw = copy_reading(fetch), copy_reading(write)
    sf, sw = (known / cf if cf > 0 else 1.0), (known / cw if cw > 0 else 1.0)
    print(f"# HBM traffic per kernel family, workload {a.workload}")
    ba = a.bench_args or "<bench arguments>"
    print("# commands (from /tmp, TMPDIR=/tmp), one counter per run:")
    print(f"#   rocprofv3 --pmc FETCH_SIZE --output-format csv -d <f> -o p -- python3 /root/repo/bench.py {ba}")
    print(f"#   rocprofv3 --pmc WRITE_SIZE --output-format csv -d <w> -o p -- python3 /root/repo/bench.py {ba}")
    print(f"#   python -m paper_2401_04338_amd.pmc_summary --fetch <f>/.../p_counter_collection.csv --write <w>/.../p_counter_collection.csv "
          f"--copy-gib {a.copy_gib:g} --workload {a.workload} --steps {a.steps} --bench-args '{ba}' --json <json>")
    print(f"# {a.steps} meta steps per run (timed + warm-up + 2 event-timed).  FETCH_SIZE / WRITE_SIZE are KiB per dispatch; the run's "
          f"{a.copy_gib:g} GiB device copy (--copy-probe-gib) is the")
    print("# transfer of known size that scales them.  \"bytes/launch\" is per kernel dispatch of the family.")
    print(f"# copy probe of {known:.0f} B read as FETCH_SIZE {cf:.0f} B, WRITE_SIZE {cw:.0f} B -> scale factors {sf:.3f}, {sw:.3f}")
    print(f"# {'family':24s} {'dispatches/step':>16s} {'fetch GB/step':>14s} {'write GB/step':>14s} {'bytes/launch':>14s}")
    out = {}
    for fam, frags in FAMILIES.items():
        fb = wb = 0.0
        n = 0
        for k, v in fetch.items():
            if any(x in k for x in frags):
                fb += sum(v) * sf
                n += len(v)
        for k, v in write.items():
            if any(x in k for x in frags):
                wb += sum(v) * sw
        if n == 0:
            continue
        per_launch = (fb + wb) / n
        out[fam] = per_launch
        print(f"  {fam:24s} {n / a.steps:16.1f} {fb / a.steps / 1e9:14.3f} {wb / a.steps / 1e9:14.3f} {per_launch:14.4g}")
    if a.json:
        with open(a.json, "w") as fh:
            json.dump({"workload": a.workload, "unit": "bytes", "scale_fetch": sf, "scale_write": sw,
                       "bytes_per_launch": out}, fh, indent=1)


if __name__ == "__main__":
    main()
