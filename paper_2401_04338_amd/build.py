"""Builds libgmeta.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

Every source is compiled to an object of its own (in parallel) and the objects are linked into the shared library.
`python -m paper_2401_04338_amd.build --incremental` recompiles only sources newer than their objects (for work on
one kernel file); build() itself, which the driver calls, compiles everything every time.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libgmeta.so")
SOURCES = ["gmeta.hip", "index_kernels.hip", "embed_kernels.hip", "mlp_kernels.hip", "gemm_bf16.hip", "twohop_kernels.hip",
           "pairhop_kernels.hip", "ceiling_kernels.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-result", "-Wno-unused-value", "-Wno-unknown-warning-option"]


def _newer(a: str, b: str) -> bool:
    return not os.path.exists(b) or os.path.getmtime(a) > os.path.getmtime(b)


def build(verbose: bool = True, incremental: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    headers = [os.path.join(CSRC, "gm_internal.h"), os.path.join(HERE, "..", "include", "gmeta.h")]
    jobs = []
    for s in SOURCES:
        src, obj = os.path.join(CSRC, s), os.path.join(OBJ, s.replace(".hip", ".o"))
        if incremental and not _newer(src, obj) and not any(_newer(h, obj) for h in headers):
            continue
        jobs.append([hipcc] + FLAGS + ["-c", src, "-o", obj])

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        # (hipcc's host pass warns that it does not know the packed-fp32 feature: harmless, filtered from the output)
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
        if out.strip():
            print(out, flush=True)
        if r.returncode:
            raise subprocess.CalledProcessError(r.returncode, cmd)

    with ThreadPoolExecutor(max_workers=min(8, max(1, len(jobs)))) as ex:
        list(ex.map(run, jobs))
    run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] +
        [os.path.join(OBJ, s.replace(".hip", ".o")) for s in SOURCES] + ["-o", LIB])
    return LIB


if __name__ == "__main__":
    build(incremental="--incremental" in sys.argv[1:])
    print("built", LIB)
