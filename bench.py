#!/usr/bin/env python3
"""Benchmark of gm_meta_step on one MI355X: meta-train samples/sec (support + query).

A step is one whole pass of the hot path (index preparation, prefetch + pooling, inner loop, overlap update, outer
forward, meta-gradient with the second-order chain, cross-task reduction, coalesced sparse gradient) over one
synthetic batch that is already resident in HBM.  The default workload is the largest configuration (c5_large, whole:
8,192 tasks x (512 + 512) samples, 64 fields x 4 Mi rows x 64, second order, sparse gradient added into a table-shaped
accumulator); the other configurations are reachable with --config.

Prints ONE JSON line: metric/value/unit, ms_per_step, config.workload, plus
  "roofline":      the kernel family with the most time in the step against the roofline that binds it (durations
                   measured live with HIP events on the library's stream; `traffic` from the committed counter summary),
  "roofline_gemm": all grouped-GEMM launches together against the matrix-core peak of their operand type,
  "kernels":       every family: algorithmic bytes or flops per launch / average launch duration / published peak,
  "ceilings":      (--ceilings) what a streaming copy / read and a register-resident MFMA loop of the library reach here,
  "cpu_baseline":  the CPU oracle timed on a bounded task subset of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK = {"hbm": (8000.0, "GB/s"), "mfma_bf16": (2500.0, "TFLOP/s"), "fp32": (157.3, "TFLOP/s")}
GEMM_FAMILIES = {"gemm_fwd", "gemm_bwd", "gemm_wgrad"}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="c5_large", help="c1_tiny | c2_small | c3_medium | c4_coldstart | c5_large")
    ap.add_argument("--order", type=int, default=None)
    ap.add_argument("--tasks", type=int, default=None,
                    help="run only the first N tasks of the config (same per-task data: a share of the workload)")
    ap.add_argument("--workspace-gib", type=float, default=None)
    ap.add_argument("--sparse-out", choices=("list", "table"), default=None,
                    help="list: coalesced (rows, gradient) lists; table: added into a table-shaped accumulator wave by wave "
                         "(default: list while the call has fewer than 2^31 lookups per set)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-outer-update", action="store_true", help="skip the separate timing of gm_scatter_add")
    ap.add_argument("--group-batch", action="store_true",
                    help="also time gm_group_batch (the record-grouping step before the hot path) on this workload's records")
    ap.add_argument("--train", type=float, default=None, metavar="OUTER_LR",
                    help="time whole training iterations (the step and the outer update with this step size, parameters "
                         "updated in place) instead of the step alone")
    ap.add_argument("--cpu-seconds", type=float, default=20.0)
    ap.add_argument("--batches", type=int, default=None,
                    help="distinct pre-generated batches cycled through (default: 2, or 1 when two do not fit beside the tables)")
    ap.add_argument("--configure", action="append", default=[], metavar="KEY=VALUE",
                    help="gm_configure setting for the run (e.g. row_path=1, gemm_tile_n=256); may be repeated")
    ap.add_argument("--vendor-gemm", action="store_true",
                    help="also time the vendor library (torch.bmm, bf16) on the first layer's forward product of this workload")
    ap.add_argument("--ceilings", action="store_true",
                    help="also measure this GPU's streaming copy / read rate and its register-resident bf16 MFMA rate with "
                         "the library's own kernels (gm_ceilings): the on-box denominators beside the published peaks")
    ap.add_argument("--copy-probe-gib", type=float, default=0.0,
                    help="also run one device copy of this size (a known transfer that calibrates rocprofv3 byte counters)")
    ap.add_argument("--save-inputs", default=None, metavar="DIR", help="write the generated batches to DIR and exit")
    ap.add_argument("--load-inputs", default=None, metavar="DIR",
                    help="read the batches from DIR instead of generating them, and fill the tables with one library call "
                         "(values differ from the seeded ones; for profiler runs, which must not see the generator's "
                         "tens of thousands of small dispatches)")
    return ap.parse_args()


def save_batches(batches, path):
    import numpy as np
    import torch
    os.makedirs(path, exist_ok=True)
    for i, (s, q) in enumerate(batches):
        for name, sd in (("sup", s), ("qry", q)):
            np.save(os.path.join(path, f"b{i}_{name}_task_offsets.npy"), np.asarray(sd.task_offsets))
            torch.save({"bag_offsets": sd.bag_offsets.cpu(), "indices": sd.indices.cpu(), "dense": sd.dense.cpu(),
                        "labels": sd.labels.cpu()}, os.path.join(path, f"b{i}_{name}.pt"))


def load_batches(path, n, dev):
    import numpy as np
    import torch
    from synth import SetData
    out = []
    for i in range(n):
        pair = []
        for name in ("sup", "qry"):
            toff = np.load(os.path.join(path, f"b{i}_{name}_task_offsets.npy"))
            d = torch.load(os.path.join(path, f"b{i}_{name}.pt"), weights_only=True)
            pair.append(SetData(toff, d["bag_offsets"].to(dev), d["indices"].to(dev), d["dense"].to(dev), d["labels"].to(dev)))
        out.append(tuple(pair))
    return out


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures ONE GPU: this build has no multi-GPU path (every box has one GPU); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from synth import CONFIGS, make_batch, make_params
    from paper_2401_04338_amd import GMeta

    cfg = cfg_gen = CONFIGS[args.config]
    task_ids = None
    if args.tasks is not None and args.tasks < cfg.n_tasks:
        # inputs are generated from the full config's streams, so the share holds exactly the full batch's values
        task_ids = list(range(args.tasks))
        cfg = cfg.with_(n_tasks=args.tasks, name=f"{cfg.name}[first {args.tasks} of {cfg.n_tasks} tasks]")
    order = cfg.order if args.order is None else args.order
    K = cfg.inner_steps
    dev = torch.device("cuda", 0)
    torch.cuda.set_device(dev)

    # how many distinct batches fit beside the tables (and the table-shaped accumulator, when that output is used)
    lookups_est = cfg.n_tasks * (cfg.n_support + cfg.n_query) * cfg.n_fields * (cfg.bag_max + 1) / 2
    batch_bytes_est = lookups_est * 4 + cfg.n_tasks * (cfg.n_support + cfg.n_query) * (cfg.n_fields * 8 + cfg.n_dense * 4 + 4)
    table_bytes = cfg.total_rows * cfg.emb_dim * 4
    table_out_est = (args.sparse_out == "table") or (args.sparse_out is None and lookups_est / 2 >= 2 ** 31 * 0.98)
    n_batches = args.batches
    if n_batches is None:
        total_b = torch.cuda.get_device_properties(dev).total_memory
        left = total_b - table_bytes * (2 if table_out_est else 1) - 2 * batch_bytes_est
        n_batches = 2 if (left > 0.2 * total_b or left > 64e9) else 1
    n_batches = max(1, n_batches)

    t0 = time.time()
    if args.load_inputs:
        from synth import Params
        batches = load_batches(args.load_inputs, n_batches, dev)
        small = make_params(cfg.with_(rows_per_field=1), dev)                    # seeded dense parameters
        emb = torch.empty(cfg.total_rows, cfg.emb_dim, dtype=torch.float32, device=dev).normal_(0.0, 0.05)
        params = Params(emb=emb, W=small.W, b=small.b)
    else:
        params = make_params(cfg, dev, chunk=1 << 27)
        batches = [make_batch(cfg_gen, it, dev, task_ids) for it in range(n_batches)]
    torch.cuda.synchronize()
    gen_s = time.time() - t0
    if args.save_inputs:
        save_batches(batches, args.save_inputs)
        print(json.dumps({"saved": args.save_inputs, "batches": len(batches), "input_generation_s": gen_s}))
        return
    sup0, qry0 = batches[0]
    S = sup0.n_samples + qry0.n_samples
    nnz = sup0.nnz + qry0.nnz

    probe = GMeta.from_config(cfg, workspace_bytes=1 << 20)
    need = max(probe.workspace_bytes(cfg.n_tasks, s.n_samples, q.n_samples, s.nnz, q.nnz, K, order) for s, q in batches)
    probe.close()
    sparse_out = args.sparse_out or ("table" if max(sup0.nnz, qry0.nnz) >= 2 ** 31 else "list")
    table = torch.zeros_like(params.emb) if sparse_out == "table" else None
    free_b, _total = torch.cuda.mem_get_info()
    cap_rows = 0 if table is not None else min(nnz, cfg.total_rows)
    out_bytes = cap_rows * (cfg.emb_dim * 4 + 8)
    ws = int(need * 1.02)
    if args.train is not None and table is None:   # the meta-gradient lists and a second set of index structures then live in the workspace
        ws += 2 * out_bytes + int(need * 0.35) + (64 << 20)
        cap_rows, out_bytes = 0, 0
    if args.workspace_gib is not None:
        ws = int(args.workspace_gib * 2 ** 30)
    ws = min(ws, int(free_b - out_bytes - (4 << 30)))
    ctx = GMeta.from_config(cfg, workspace_bytes=ws)
    if cfg.name == "c5_large" and not any(kv.startswith("max_wave_tasks=") for kv in args.configure):
        # waves of 256 tasks: the share of the workload that the committed counter profiles were taken on, so that their
        # bytes per launch apply to this run's launches
        args.configure.append("max_wave_tasks=256")
    for kv in args.configure:
        key, _, val = kv.partition("=")
        ctx.configure(key, int(val))
    out = ctx.alloc_outputs(cfg.n_tasks, cap_rows)

    def step(i):
        s, q = batches[i % len(batches)]
        if args.train is not None and table is not None:   # (the table-shaped accumulator is cleared by the update)
            ctx.meta_train_step_table(s, q, params, cfg.inner_lr, K, order, args.train, table, loss=out["loss"])
            return out
        if args.train is not None:
            ctx.meta_train_step(s, q, params, cfg.inner_lr, K, order, args.train, loss=out["loss"])
            return out
        return ctx.meta_step(s, q, params, cfg.inner_lr, K, order, out=out, emb_grad_table=table)

    def train_loop(n):   # n iterations of Alg. 1 in one call (gm_meta_train), cycling through the batches
        if table is not None:   # batches beyond the row-list form: one call per iteration
            for i in range(n):
                step(i)
            return
        losses = ctx.meta_train([batches[i % len(batches)] for i in range(n)], params, cfg.inner_lr, K, order, args.train)
        out["loss"][:1] = losses[-1:]

    if args.train is not None:
        train_loop(max(args.warmup, 1))
    else:
        for i in range(args.warmup):
            step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    if args.train is not None:
        train_loop(args.steps)
    else:
        for i in range(args.steps):
            step(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    value = S * args.steps / dt
    loss = float(out["loss"].item())

    # kernel families, timed live with HIP events on the library's stream (separate, untimed pass)
    ctx.profile(True)
    n_prof = 2 if ms_per_step < 500 else 1
    for i in range(n_prof):
        step(i)
    ctx.profile(False)
    rep = ctx.profile_report()
    ceilings = ctx.ceilings() if args.ceilings else None

    gather_launches = rep.get("gather_pool", {}).get("launches", 0) // n_prof
    tasks_per_wave = cfg.n_tasks if gather_launches <= 0 else -(-cfg.n_tasks // max(gather_launches, 1))
    workload = cfg_gen.name
    ridge = PEAK["mfma_bf16"][0] * 1e12 / (PEAK["hbm"][0] * 1e9) if cfg.mlp_dtype else PEAK["fp32"][0] * 1e12 / (PEAK["hbm"][0] * 1e9)
    fams = []
    for name, r in rep.items():
        sec = r["ms"] * 1e-3
        launches = max(r["launches"], 1)
        ach_b = r["bytes"] / sec / 1e9 if sec > 0 else 0.0
        f = dict(kernel=name, launches=r["launches"] // n_prof, ms_per_step=r["ms"] / n_prof, avg_launch_ms=r["ms"] / launches,
                 algorithmic_bytes_per_launch=r["bytes"] / launches, flops_per_launch=r["flops"] / launches)
        traffic = measured_traffic(workload, name, r["launches"] / n_prof, cfg.n_tasks, tasks_per_wave)
        if name in GEMM_FAMILIES:
            # A grouped GEMM is held against the roofline that its arithmetic intensity puts it under: products whose
            # flops per algorithmic byte reach the ridge (peak flops / peak bytes) are matrix-core bound, the others
            # (per-task weight gradients: a contraction over one task's rows, then theta' written) are HBM bound.
            pk_f, un_f = PEAK["mfma_bf16"] if cfg.mlp_dtype else PEAK["fp32"]
            ach_f = r["flops"] / sec / 1e12 if sec > 0 else 0.0
            intensity = r["flops"] / r["bytes"] if r["bytes"] > 0 else 0.0
            f.update(intensity_flop_per_byte=intensity, ridge_flop_per_byte=ridge,
                     frac_of_matrix_peak=ach_f / pk_f, frac_of_hbm_peak=ach_b / PEAK["hbm"][0])
            if intensity >= ridge:
                f.update(bound="mfma" if cfg.mlp_dtype else "alu", achieved=ach_f, peak=pk_f, unit=un_f, frac=ach_f / pk_f)
            else:
                f.update(bound="hbm", achieved=ach_b, peak=PEAK["hbm"][0], unit="GB/s", frac=ach_b / PEAK["hbm"][0])
        else:
            f.update(bound="hbm", achieved=ach_b, peak=PEAK["hbm"][0], unit="GB/s",
                     frac=ach_b / PEAK["hbm"][0] if r["bytes"] > 0 else None)
        f["traffic"] = traffic
        if traffic is not None and f["avg_launch_ms"] > 0:
            f["frac_by_counters"] = traffic / (f["avg_launch_ms"] * 1e-3) / 1e9 / PEAK["hbm"][0]
        fams.append(f)
    fams.sort(key=lambda f: -f["ms_per_step"])

    vendor = None
    if args.vendor_gemm and cfg.mlp_dtype:
        vendor = vendor_gemm(cfg, dev)
    ctx_ws = ws
    ctx.close()
    torch.cuda.empty_cache()

    # The prefetch reads hot rows from the caches: its logical bytes (4 D per lookup) can exceed what HBM delivers.  Its
    # fraction of the roofline is therefore taken on the COMPULSORY bytes of a launch: every distinct row once, the
    # indices, the offsets and the pooled outputs (counted here for the first wave of tasks of each set).
    for f in fams:
        if f["kernel"] != "gather_pool" or cfg.n_fields == 0:
            continue
        comp = compulsory_gather_bytes(cfg, sup0, qry0, min(tasks_per_wave, cfg.n_tasks))
        f["frac_of_logical_bytes"] = f["frac"]
        f["logical_bytes_per_launch"] = f["algorithmic_bytes_per_launch"]
        f["algorithmic_bytes_per_launch"] = comp
        f["achieved"] = comp / (f["avg_launch_ms"] * 1e-3) / 1e9
        f["frac"] = f["achieved"] / PEAK["hbm"][0]
        f["note"] = ("frac: compulsory bytes (distinct rows of a launch once + indices + offsets + pooled outputs); "
                     "frac_of_logical_bytes counts 4 D bytes per lookup, which caches serve for hot rows; "
                     "frac_by_counters: HBM bytes read by rocprofv3 counters")

    gemm = [f for f in fams if f["kernel"] in GEMM_FAMILIES]
    gemm_ms = sum(f["ms_per_step"] for f in gemm)
    gemm_flops = sum(rep[f["kernel"]]["flops"] for f in gemm) / n_prof
    gemm_launches = sum(f["launches"] for f in gemm)
    peak_m, unit_m = PEAK["mfma_bf16"] if cfg.mlp_dtype else PEAK["fp32"]
    gemm_ach = gemm_flops / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 else 0.0
    roof_gemm = dict(kernel="gemm_bf16_kernel (all launches)" if cfg.mlp_dtype else "gemm_f32_kernel (all launches)",
                     bound="mfma" if cfg.mlp_dtype else "alu", achieved=gemm_ach, peak=peak_m, unit=unit_m,
                     frac=gemm_ach / peak_m, traffic=None, ms_per_step=gemm_ms, avg_launch_ms=gemm_ms / max(gemm_launches, 1),
                     compute_bound_launches={f["kernel"]: f["frac_of_matrix_peak"] for f in gemm if f["bound"] != "hbm"})
    top = next((f for f in fams if f["frac"] is not None), None)
    roof = roof_gemm if top is None else {k: top.get(k) for k in ("kernel", "bound", "achieved", "peak", "unit", "frac", "traffic",
                                                                 "ms_per_step", "avg_launch_ms", "algorithmic_bytes_per_launch",
                                                                 "flops_per_launch", "launches")}
    top_hbm = next((f for f in fams if f["bound"] == "hbm" and f["frac"] is not None), None)

    outer = grouping = None
    if table is None and cfg.n_fields > 0 and not args.no_outer_update and args.train is None:
        outer = outer_update_timing(cfg, params, out, ctx_ws)
    if args.group_batch:
        grouping = group_batch_timing(cfg, sup0, qry0, ctx_ws)

    if args.copy_probe_gib > 0:
        n = int(args.copy_probe_gib * 2 ** 30)
        src = torch.ones(n, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(cfg, cfg_gen, K, order, args.cpu_seconds, params, adapt_rows="adapt_rows=0" not in args.configure)

    line = {
        "metric": "meta-train samples/sec (support+query) on 1 GPU", "value": value, "unit": "samples/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.mlp_dtype else "f32", "data": "synthetic",
        "config": {"workload": cfg.name, "n_tasks": cfg.n_tasks, "samples_per_step": S, "lookups_per_step": nnz,
                   "n_fields": cfg.n_fields, "rows_per_field": cfg.rows_per_field, "emb_dim": cfg.emb_dim,
                   "mlp": list(cfg.layer_dims), "inner_steps": K, "order": order, "inner_lr": cfg.inner_lr,
                   "outer_update": None if args.train is None else {"fused": True, "outer_lr": args.train,
                                                                     "loop": "gm_meta_train: one call per timed region" if table is None
                                                                     else "gm_meta_train_step_table: one call per iteration"},
                   "sparse_out": sparse_out, "configure": args.configure, "workspace_gib": ctx_ws / 2 ** 30,
                   "tasks_per_wave": tasks_per_wave, "batches_cycled": len(batches), "loss": loss,
                   "input_generation_s": gen_s, "inputs": "loaded" if args.load_inputs else "generated"},
        "roofline": roof,
        "roofline_gemm": roof_gemm,
        "roofline_hbm": top_hbm,
        "kernels": fams,
        "ceilings": ceilings,
        "outer_update_sparse": outer,
        "group_batch": grouping,
        "vendor_gemm": vendor,
        "cpu_baseline": cpu,
    }
    print(json.dumps(line))


def measured_traffic(workload, family, launches_per_step, n_tasks, tasks_per_wave):
    """HBM bytes per timed launch of a kernel family from the committed rocprofv3 counter summary (FETCH_SIZE and
    WRITE_SIZE runs, scaled by a copy of known size), or None when no such summary is committed for this workload.
    The summary holds a family's bytes per meta step of the profiled run; a timed launch here is one bracket of HIP
    events (which may hold several dispatches of the family).  A summary taken on a share of the workload's tasks
    applies when this run processes that many tasks per wave (then the launches have the same shape)."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.json")
    try:
        with open(path) as fh:
            d = json.load(fh)
    except (OSError, ValueError):
        return None
    per_step = d.get("bytes_per_step", {}).get(family)
    if per_step is None or launches_per_step <= 0:
        return None
    share = d.get("tasks_in_the_profiled_run")
    if share in (None, n_tasks):
        return per_step / launches_per_step
    if share == tasks_per_wave:   # the profiled run was one wave of this run
        return per_step / max(1.0, launches_per_step / (-(-n_tasks // tasks_per_wave)))
    return None


def compulsory_gather_bytes(cfg, sup, qry, n_tasks):
    """Bytes one prefetch launch cannot avoid moving, averaged over the two launches (support, query) of the first
    n_tasks tasks: distinct table rows * 4 D + 4 per lookup + 8 per bag + the pooled rows written (fp32, and the bf16
    operand copy when the MLP runs on bf16 operands)."""
    import torch
    F, R, D = cfg.n_fields, cfg.rows_per_field, cfg.emb_dim
    ld0 = -(-cfg.layer_dims[0] // 32) * 32
    total = 0.0
    for sd in (sup, qry):
        s1 = int(sd.task_offsets[n_tasks])
        lo, hi = int(sd.bag_offsets[0].item()), int(sd.bag_offsets[s1 * F].item())
        mark = torch.zeros(cfg.total_rows, dtype=torch.bool, device=sd.indices.device)
        step_bags = max(1, (1 << 24) // max(cfg.bag_max, 1))
        for b0 in range(0, s1 * F, step_bags):      # in pieces: the per-lookup field ids are 8 bytes each
            b1 = min(s1 * F, b0 + step_bags)
            offs = sd.bag_offsets[b0: b1 + 1]
            lens = offs[1:] - offs[:-1]
            field = (torch.arange(b0, b1, device=lens.device) % F).repeat_interleave(lens)
            mark[sd.indices[int(offs[0].item()): int(offs[-1].item())].long() + field * R] = True
        distinct = int(mark.sum().item())
        del mark
        total += distinct * 4.0 * D + (hi - lo) * 4.0 + s1 * F * 8.0 + s1 * ld0 * (4.0 + (2.0 if cfg.mlp_dtype else 0.0))
    return total / 2.0


def outer_update_timing(cfg, params, out, ws):
    """The outer update's sparse half (Alg. 1, global back-propagation on xi with the coalesced gradient): outside the
    step, timed on its own with HIP events around the call, on a copy of the tables."""
    import torch
    from paper_2401_04338_amd import GMeta
    free_now, _ = torch.cuda.mem_get_info()
    if free_now <= params.emb.numel() * 4 + (2 << 30):
        return None
    ctx = GMeta.from_config(cfg, workspace_bytes=1 << 20)
    n_rows = int(out["n_emb_rows"].item())
    tbl = params.emb.clone()
    rows_v, grad_v = out["emb_rows"][:n_rows], out["emb_grad"][:n_rows]
    ctx.scatter_add(tbl, rows_v, grad_v, -1e-3)   # warm-up
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 5
    torch.cuda.synchronize()
    ev0.record()
    for _ in range(reps):
        ctx.scatter_add(tbl, rows_v, grad_v, -1e-3)
    ev1.record()
    torch.cuda.synchronize()
    ctx.close()
    ms = ev0.elapsed_time(ev1) / reps
    by = n_rows * (3 * cfg.emb_dim * 4 + 8)   # row read + gradient read + row written + row id
    pk, un = PEAK["hbm"]
    return dict(kernel="scatter_add_kernel (gm_scatter_add, outside the step)", bound="hbm", rows=n_rows, ms=ms,
                achieved=by / (ms * 1e-3) / 1e9, peak=pk, unit=un, frac=by / (ms * 1e-3) / 1e9 / pk,
                algorithmic_bytes_per_launch=by)


def group_batch_timing(cfg, sup0, qry0, ws):
    """The step before the hot path: the batch's records as one flat stream (support records, then query records, each
    with its task id), regrouped into one-task batches and split again; wall time of the call (host ordering + device
    copies), outside the step."""
    import numpy as np
    import torch
    from paper_2401_04338_amd import GMeta
    ctx = GMeta.from_config(cfg, workspace_bytes=min(ws, 8 << 30))
    sizes_s, sizes_q = np.diff(sup0.task_offsets), np.diff(qry0.task_offsets)
    task_of = np.concatenate([np.repeat(np.arange(cfg.n_tasks), sizes_s), np.repeat(np.arange(cfg.n_tasks), sizes_q)])
    bo = torch.cat([sup0.bag_offsets, qry0.bag_offsets[1:] + sup0.bag_offsets[-1]])
    idx = torch.cat([sup0.indices, qry0.indices])
    dn, lb = torch.cat([sup0.dense, qry0.dense]), torch.cat([sup0.labels, qry0.labels])
    num, den = int(sizes_s.sum()), int(sizes_s.sum() + sizes_q.sum())
    ctx.group_batch(task_of, np.zeros_like(task_of), bo, idx, dn, lb, num, den)   # warm-up
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    reps = 3
    for _ in range(reps):
        gs, gq = ctx.group_batch(task_of, np.zeros_like(task_of), bo, idx, dn, lb, num, den)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / reps * 1e3
    same = bool(torch.equal(gs.indices, sup0.indices) and torch.equal(gq.bag_offsets, qry0.bag_offsets)) \
        if np.all(sizes_s * den == (sizes_s + sizes_q) * num) else None
    ctx.close()
    return dict(op="gm_group_batch (outside the step; includes the binding's output allocation)", records=int(task_of.size),
                lookups=int(idx.numel()), ms=ms, records_per_s=task_of.size / (ms * 1e-3), reproduces_the_batch=same)


def vendor_gemm(cfg, dev):
    """Context for roofline_gemm, not part of the path: the vendor library's batched bf16 GEMM on the first layer's
    forward product (per-task weights [d0, d1], one set's rows per task, random values)."""
    import torch
    Tg = min(cfg.n_tasks, 256)
    rows, d0, d1 = int(cfg.n_support), -(-int(cfg.layer_dims[0]) // 32) * 32, int(cfg.layer_dims[1])
    xa = torch.randn(Tg, rows, d0, device=dev, dtype=torch.bfloat16)
    wb = torch.randn(Tg, d0, d1, device=dev, dtype=torch.bfloat16)
    best = None
    for _ in range(5):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        torch.bmm(xa, wb)
        e1.record()
        torch.cuda.synchronize()
        best = e0.elapsed_time(e1) if best is None else min(best, e0.elapsed_time(e1))
    fl = 2.0 * Tg * rows * d0 * d1
    return dict(op="torch.bmm bf16 (vendor library), first layer forward", tasks=Tg, m=rows, k=d0, n=d1, ms=best,
                achieved=fl / (best * 1e-3) / 1e12, unit="TFLOP/s", frac_of_mfma_peak=fl / (best * 1e-3) / 2.5e15)


def cpu_baseline(cfg, cfg_gen, K, order, budget_s, params, adapt_rows=True):
    """The CPU oracle, as it stands, on a task subset of the same workload (about budget_s of CPU work).  The oracle
    sees the table rows the subset looks up (re-indexed: the full tables of the larger workloads do not fit a host
    copy, and the result depends on no other row)."""
    from oracle import maml_dlrm as O
    from synth import compact_tasks, make_batch
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    W = [w.cpu().numpy() for w in params.W]
    b = [x.cpu().numpy() for x in params.b]
    operand = "bf16" if cfg.mlp_dtype else "fp64"
    done, spent, samples, n = 0, 0.0, 0, 1
    while done < cfg.n_tasks and spent < budget_s:
        tasks = list(range(done, min(cfg.n_tasks, done + n)))
        sup, qry = make_batch(cfg_gen, 0, "cpu", tasks)
        counts, emb, sd, qd, _rows = compact_tasks(cfg_gen, sup, qry, params.emb)
        model = O.Model(rows_per_field=counts, emb_dim=cfg.emb_dim, n_dense=cfg.n_dense, layer_dims=list(cfg.layer_dims))
        t0 = time.perf_counter()
        O.meta_step(model, dict(emb=emb, W=W, b=b), sd, qd, cfg.inner_lr, K, order, operand=operand, adapt_rows=adapt_rows)
        dt = time.perf_counter() - t0
        spent += dt
        samples += sup.n_samples + qry.n_samples
        done += len(tasks)
        per_task = spent / done
        n = max(1, min(cfg.n_tasks - done, int((budget_s - spent) / max(per_task, 1e-6) / 2)))
    return {"value": samples / spent, "unit": "samples/s", "cores": cores, "kind": "oracle",
            "sample": f"tasks 0..{done - 1} of {cfg.n_tasks} ({samples} samples, {spent:.1f} s of oracle time, "
                      f"float64 numpy, operand rounding {operand})"}


if __name__ == "__main__":
    main()
