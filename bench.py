#!/usr/bin/env python3
"""Benchmark of gm_meta_step on one MI355X: meta-train samples/sec (support + query).

A step is one whole pass of the hot path (index preparation, prefetch + pooling, inner loop,
overlap update, outer forward, meta-gradient with the second-order chain, cross-task reduction,
coalesced sparse gradient) over one synthetic batch that is already resident in HBM.

Prints ONE JSON line: metric/value/unit, ms_per_step, config.workload, plus
  "roofline":     the dominant kernel family of the step against the chip's published peak
                  (durations measured live with HIP events on the library's stream),
  "cpu_baseline": the CPU oracle timed on a bounded task subset of the same workload.
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
HBM_FAMILIES = {"gather_pool", "pool_slots", "slot_segsum", "seg_reduce", "global_sort", "tf_sort", "tf_count",
                "transpose_act", "transpose_w", "reduce_tasks", "axpy_gx"}
GEMM_FAMILIES = {"gemm_fwd", "gemm_bwd", "gemm_wgrad"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default="c3_medium", help="c1_tiny | c2_small | c3_medium | c4_coldstart | c5_large (with --tasks)")
    ap.add_argument("--order", type=int, default=None)
    ap.add_argument("--tasks", type=int, default=None,
                    help="run only the first N tasks of the config (same per-task data; a share of a config too large for one call)")
    ap.add_argument("--workspace-gib", type=float, default=None)
    ap.add_argument("--sparse-out", choices=("list", "table"), default=None,
                    help="list: coalesced (rows, gradient) lists; table: added into a table-shaped accumulator wave by wave "
                         "(default: list while the call has fewer than 2^31 lookups per set)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-outer-update", action="store_true", help="skip the separate timing of gm_scatter_add")
    ap.add_argument("--group-batch", action="store_true",
                    help="also time gm_group_batch (the record-grouping step before the hot path) on this workload's records")
    ap.add_argument("--train", type=float, default=None, metavar="OUTER_LR",
                    help="time whole training iterations (gm_meta_train_step: the step and the outer update with this step "
                         "size, parameters updated in place) instead of the step alone")
    ap.add_argument("--cpu-seconds", type=float, default=20.0)
    ap.add_argument("--batches", type=int, default=2, help="distinct pre-generated batches cycled through")
    ap.add_argument("--configure", action="append", default=[], metavar="KEY=VALUE",
                    help="gm_configure setting for the run (e.g. row_path=1, gemm_tile_n=256); may be repeated")
    ap.add_argument("--vendor-gemm", action="store_true",
                    help="also time the vendor library (torch.bmm, bf16) on the first layer's forward product of this workload: "
                         "what a grouped GEMM with per-task weights reaches on this GPU with the same shapes and random values")
    ap.add_argument("--copy-probe-gib", type=float, default=0.0,
                    help="also run one device copy of this size (a known transfer that calibrates rocprofv3 byte counters)")
    args = ap.parse_args()
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

    t0 = time.time()
    params = make_params(cfg, dev)
    batches = [make_batch(cfg_gen, it, dev, task_ids) for it in range(max(1, args.batches))]
    torch.cuda.synchronize()
    gen_s = time.time() - t0
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
    if args.train is not None:   # the meta-gradient lists then live in the workspace, not in caller buffers
        ws += out_bytes + (1 << 20)
        if table is not None:
            print("--train uses the row-list output (fewer than 2^31 lookups per set)", file=sys.stderr)
            sys.exit(2)
        cap_rows, out_bytes = 0, 0
    if args.workspace_gib is not None:
        ws = int(args.workspace_gib * 2 ** 30)
    ws = min(ws, int(free_b - out_bytes - (4 << 30)))
    ctx = GMeta.from_config(cfg, workspace_bytes=ws)
    for kv in args.configure:
        key, _, val = kv.partition("=")
        ctx.configure(key, int(val))
    out = ctx.alloc_outputs(cfg.n_tasks, cap_rows)

    def step(i):
        s, q = batches[i % len(batches)]
        if args.train is not None:
            ctx.meta_train_step(s, q, params, cfg.inner_lr, K, order, args.train, loss=out["loss"])
            return out
        return ctx.meta_step(s, q, params, cfg.inner_lr, K, order, out=out, emb_grad_table=table)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    value = S * args.steps / dt
    loss = float(out["loss"].item())

    # kernel families, timed live with HIP events on the library's stream (separate, untimed pass)
    ctx.profile(True)
    n_prof = 2
    for i in range(n_prof):
        step(i)
    ctx.profile(False)
    rep = ctx.profile_report()
    fams = []
    for name, r in rep.items():
        if name in GEMM_FAMILIES:
            # a grouped GEMM with short contractions (per-task weight gradients) is bound by its outputs, not by
            # the matrix cores: report against whichever roofline it sits closer to
            pk_f, un_f = PEAK["mfma_bf16"] if cfg.mlp_dtype else PEAK["fp32"]
            pk_b, un_b = PEAK["hbm"]
            ach_f = r["flops"] / (r["ms"] * 1e-3) / 1e12 if r["ms"] > 0 else 0.0
            ach_b = r["bytes"] / (r["ms"] * 1e-3) / 1e9 if r["ms"] > 0 else 0.0
            if ach_b / pk_b > ach_f / pk_f:
                bound, work, peak, unit, ach = "hbm", r["bytes"], pk_b, un_b, ach_b
            else:
                bound, work, peak, unit, ach = ("mfma" if cfg.mlp_dtype else "alu"), r["flops"], pk_f, un_f, ach_f
        else:
            bound, work = "hbm", r["bytes"]
            peak, unit = PEAK["hbm"]
            ach = work / (r["ms"] * 1e-3) / 1e9 if r["ms"] > 0 else 0.0
        fams.append(dict(kernel=name, bound=bound, launches=r["launches"] // n_prof, ms_per_step=r["ms"] / n_prof,
                         avg_launch_ms=r["ms"] / max(r["launches"], 1), achieved=ach, peak=peak, unit=unit,
                         frac=ach / peak if work > 0 else None,
                         algorithmic_bytes_per_launch=r["bytes"] / max(r["launches"], 1),
                         flops_per_launch=r["flops"] / max(r["launches"], 1)))
    fams.sort(key=lambda f: -f["ms_per_step"])
    # dominant family: all GEMM launches are one kernel (same code, three operand set-ups)
    gemm_ms = sum(f["ms_per_step"] for f in fams if f["kernel"] in GEMM_FAMILIES)
    gemm_flops = sum(rep[n]["flops"] for n in GEMM_FAMILIES if n in rep)
    gemm_launches = sum(rep[n]["launches"] for n in GEMM_FAMILIES if n in rep)
    top_hbm = next((f for f in fams if f["bound"] == "hbm" and f["frac"] is not None), None)
    peak_m, unit_m = PEAK["mfma_bf16"] if cfg.mlp_dtype else PEAK["fp32"]
    gemm_ach = gemm_flops / n_prof / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 else 0.0
    roof_gemm = dict(kernel="gemm_bf16_kernel" if cfg.mlp_dtype else "gemm_f32_kernel",
                     bound="mfma" if cfg.mlp_dtype else "alu", achieved=gemm_ach, peak=peak_m, unit=unit_m,
                     frac=gemm_ach / peak_m, traffic=None, ms_per_step=gemm_ms,
                     avg_launch_ms=gemm_ms * n_prof / max(gemm_launches, 1))
    # the dominant kernel family of the step, against the roofline that binds it
    top = fams[0] if fams else None
    roof = roof_gemm
    if top is not None and top["frac"] is not None:
        roof = dict(kernel=top["kernel"], bound=top["bound"], achieved=top["achieved"], peak=top["peak"], unit=top["unit"],
                    frac=top["frac"], traffic=measured_traffic(cfg.name, top["kernel"]), ms_per_step=top["ms_per_step"],
                    avg_launch_ms=top["avg_launch_ms"])

    # The outer update's sparse half (Alg. 1, global back-propagation on xi with the coalesced gradient): outside the
    # step, timed on its own with HIP events around the call, on a copy of the tables
    outer = None
    if table is None and cfg.n_fields > 0 and not args.no_outer_update and args.train is None:
        free_now, _ = torch.cuda.mem_get_info()
        if free_now > params.emb.numel() * 4 + (2 << 30):
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
            ms = ev0.elapsed_time(ev1) / reps
            by = n_rows * (3 * cfg.emb_dim * 4 + 8)   # row read + gradient read + row written + row id
            pk, un = PEAK["hbm"]
            outer = dict(kernel="scatter_add_kernel (gm_scatter_add, outside the step)", bound="hbm", rows=n_rows, ms=ms,
                         achieved=by / (ms * 1e-3) / 1e9, peak=pk, unit=un, frac=by / (ms * 1e-3) / 1e9 / pk,
                         algorithmic_bytes_per_launch=by)
            del tbl

    # The step before the hot path: the batch's records as one flat stream (support records, then query records, each
    # with its task id), regrouped into one-task batches and split again; wall time of the call (host ordering +
    # device copies), outside the step
    grouping = None
    if args.group_batch:
        F = cfg.n_fields
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
        grouping = dict(op="gm_group_batch (outside the step; includes the binding's output allocation)", records=int(task_of.size),
                        lookups=int(idx.numel()), ms=ms, records_per_s=task_of.size / (ms * 1e-3),
                        reproduces_the_batch=same)
        del bo, idx, dn, lb, gs, gq

    if args.copy_probe_gib > 0:
        n = int(args.copy_probe_gib * 2 ** 30)
        src = torch.ones(n, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    vendor = None
    if args.vendor_gemm and cfg.mlp_dtype:
        # context for roofline_gemm, not part of the path: per-task weights [d0, d1], one set's rows per task
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
        vendor = dict(op="torch.bmm bf16 (vendor library), first layer forward", tasks=Tg, m=rows, k=d0, n=d1, ms=best,
                      achieved=fl / (best * 1e-3) / 1e12, unit="TFLOP/s", frac_of_mfma_peak=fl / (best * 1e-3) / 2.5e15)
        del xa, wb

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(cfg, cfg_gen, K, order, args.cpu_seconds, params.numpy(),
                           adapt_rows="adapt_rows=0" not in args.configure)

    line = {
        "metric": "meta-train samples/sec (support+query) on 1 GPU", "value": value, "unit": "samples/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.mlp_dtype else "f32", "data": "synthetic",
        "config": {"workload": cfg.name, "n_tasks": cfg.n_tasks, "samples_per_step": S, "lookups_per_step": nnz,
                   "n_fields": cfg.n_fields, "rows_per_field": cfg.rows_per_field, "emb_dim": cfg.emb_dim,
                   "mlp": list(cfg.layer_dims), "inner_steps": K, "order": order, "inner_lr": cfg.inner_lr,
                   "outer_update": None if args.train is None else {"fused": True, "outer_lr": args.train},
                   "sparse_out": sparse_out, "configure": args.configure, "workspace_gib": ws / 2 ** 30, "batches_cycled": len(batches), "loss": loss,
                   "input_generation_s": gen_s},
        "roofline": roof,
        "roofline_gemm": roof_gemm,
        "roofline_hbm": top_hbm,
        "kernels": fams,
        "outer_update_sparse": outer,
        "group_batch": grouping,
        "vendor_gemm": vendor,
        "cpu_baseline": cpu,
    }
    print(json.dumps(line))


def measured_traffic(workload, family):
    """HBM bytes per launch of a kernel family from the committed rocprofv3 counter summary (FETCH_SIZE and WRITE_SIZE
    runs, scaled by a copy of known size), or None when no such summary is committed for this workload."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", f"hbm_traffic_{workload}.json")
    try:
        with open(path) as fh:
            return json.load(fh).get("bytes_per_launch", {}).get(family)
    except (OSError, ValueError):
        return None


def cpu_baseline(cfg, cfg_gen, K, order, budget_s, params, adapt_rows=True):
    """The CPU oracle, as it stands, on a task subset of the same workload (about budget_s of CPU work)."""
    import numpy as np
    from oracle import maml_dlrm as O
    from synth import make_batch
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    model = O.Model(rows_per_field=[cfg.rows_per_field] * cfg.n_fields, emb_dim=cfg.emb_dim, n_dense=cfg.n_dense,
                    layer_dims=list(cfg.layer_dims))
    operand = "bf16" if cfg.mlp_dtype else "fp64"
    done, spent, samples, n = 0, 0.0, 0, 1
    t_all = time.perf_counter()
    while done < cfg.n_tasks and spent < budget_s:
        tasks = list(range(done, min(cfg.n_tasks, done + n)))
        sup, qry = make_batch(cfg_gen, 0, "cpu", tasks)
        t0 = time.perf_counter()
        O.meta_step(model, params, sup.numpy(), qry.numpy(), cfg.inner_lr, K, order, operand=operand, adapt_rows=adapt_rows)
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
