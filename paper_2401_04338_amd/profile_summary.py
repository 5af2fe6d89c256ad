"""Turns the rocpd database that `rocprofv3 --kernel-trace --stats` writes into a short text summary.

Usage: python -m paper_2401_04338_amd.profile_summary <results.db> [top_n] [bench arguments of the profiled run]
Only this package's kernels are listed by name; everything else (PyTorch's generator kernels that
build the synthetic inputs) is summed into one line.  The header states the command that made the trace.
"""
import sqlite3
import sys


def summarize(db_path: str, top_n: int = 40) -> str:
    con = sqlite3.connect(db_path)
    rows = list(con.execute("select name, total_calls, total_duration, average, percentage from top_kernels"))
    ours, other_ns, other_calls = [], 0.0, 0
    for name, calls, total, avg, pct in rows:
        if name.startswith("void at::") or "at::native" in name or "rocprim" in name or "hipcub" in name:
            other_ns += total
            other_calls += calls
        else:
            ours.append((name.split("(")[0].replace("void ", ""), calls, total, avg))
    tot = sum(r[2] for r in ours)
    lines = [f"{'kernel':56s} {'calls':>6s} {'total_us':>10s} {'avg_us':>10s}   share_of_library_time"]
    for name, calls, total, avg in ours[:top_n]:
        lines.append(f"{name[:56]:56s} {calls:6d} {total:10.1f} {avg:10.2f} {100.0 * total / tot:8.2f}%")
    lines.append(f"(input generation and other framework kernels: {other_calls} calls, {other_ns:.1f} us)")
    return "\n".join(lines)


if __name__ == "__main__":
    top = int(sys.argv[2]) if len(sys.argv) > 2 else 40
    bench_args = " ".join(sys.argv[3:]) or "<bench arguments>"
    print("# rocprofv3 kernel trace of gm_meta_step (per-kernel totals over the whole run: warm-up, timed and event-timed steps)")
    print(f"# command (from /tmp, TMPDIR=/tmp): rocprofv3 --kernel-trace --stats -d <out> -o <name> -- python3 /root/repo/bench.py {bench_args}")
    print(f"# summary made with: python -m paper_2401_04338_amd.profile_summary <out>/<name>_results.db {top} {bench_args}")
    print(summarize(sys.argv[1], top))
