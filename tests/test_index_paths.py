"""The two ways the HIP path builds the per-(task, field) row dictionaries, lookup lists and the overlap join of
Sec. 2.1.2: every (task, field) sorted by itself (gm_configure("index_path", 1)), or read off the row order of the wave's
lookups plus one stable pass by task ("index_path", 2; that row order from one sort on (field, row) or, "sort_fields",
from the fields' ranges sorted by row alone).  All must give the oracle's integer structures bit for bit,
and a meta step must come out identical whichever built them.
"""
import numpy as np
import pytest
import torch

from oracle import maml_dlrm as O
from synth import SMALL, TINY
from tests.helpers import oracle_model, small_cfg
from tests.test_gpu_parity import TOL_FP32, _compare_step, _inputs, _params_dev, _to_dev, gm  # noqa: F401

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("path,by_field", [(1, 1), (2, 0), (2, 1)], ids=["per_task_field", "row_order", "row_order_by_field"])
@pytest.mark.parametrize("cfg", [small_cfg(n_tasks=5, rows_per_field=12, bag_max=5), TINY, SMALL.with_(n_tasks=6),
                                 small_cfg(n_tasks=1, n_fields=1, rows_per_field=3, bag_max=1, n_support=9, n_query=4),
                                 small_cfg(n_tasks=700, n_fields=2, rows_per_field=9, bag_max=3, n_support=3, n_query=2)],
                         ids=["mini", "tiny", "small6", "one_field_one_lookup", "700_tasks"])
def test_index_prep_bit_exact_on_both_paths(gm, cfg, path, by_field):
    """Slots, row lists, the slot of every lookup and the batch-wide segments against the oracle.  "700_tasks" needs two
    passes to order the lookups by task (more than 512 tasks); "one_field_one_lookup" has no field or position bits.
    The row order itself is made either by one sort on (field, row) or ("sort_fields", the default) field by field."""
    print("index_prep", cfg.name, "index_path", path, "sort_fields", by_field, flush=True)
    sup, qry, _ = _inputs(cfg)
    ctx = gm.from_config(cfg, workspace_bytes=1 << 30)
    ctx.configure("index_path", path)
    ctx.configure("sort_fields", by_field)
    got = ctx.index_prep(_to_dev(sup, ctx.device), _to_dev(qry, ctx.device))
    ref = O.index_prep(oracle_model(cfg), sup.numpy(), qry.numpy())
    for k in ("slot_counts", "slot_rows", "sup_slot", "qry_slot", "emb_rows", "seg_counts"):
        assert np.array_equal(got[k].cpu().numpy(), ref[k]), k
    ctx.close()


def _same_bits(a, b, n_layers, table_a=None, table_b=None):
    assert torch.equal(a["loss"], b["loss"])
    assert torch.equal(a["task_loss"], b["task_loss"])
    for l in range(n_layers):
        assert torch.equal(a["dW"][l], b["dW"][l]) and torch.equal(a["db"][l], b["db"][l]), l
    if table_a is not None:
        assert torch.equal(table_a, table_b)
        return
    n = int(a["n_emb_rows"].item())
    assert n == int(b["n_emb_rows"].item())
    assert torch.equal(a["emb_rows"][:n], b["emb_rows"][:n]) and torch.equal(a["emb_grad"][:n], b["emb_grad"][:n])


CASES = {
    # configs[1]'s shape, pair-count row path, row-list output
    "small8": (SMALL.with_(n_tasks=8), 2, 2, 2 << 30, False),
    # the same with the table-shaped output in several waves of tasks (every wave orders its own lookups)
    "small8_table_waves": (SMALL.with_(n_tasks=8), 2, 2, None, True),
    # more than 512 tasks (two passes by task), ragged tiny tasks, bf16 operands
    "many_tiny_tasks": (SMALL.with_(n_tasks=530, n_support=5, n_query=3, n_fields=3, emb_dim=32, rows_per_field=50, bag_max=4,
                                    layer_dims=(3 * 32 + 13, 32, 16, 1), mlp_dtype=1, inner_lr=0.05), 1, 2, 1 << 30, False),
    # counts above a byte: found by the counting kernel, the sparse row kernel then needs the slot of every lookup
    "pair_overflow": (SMALL.with_(n_tasks=3, n_support=40, n_query=30, n_fields=4, emb_dim=32, rows_per_field=1, bag_max=24,
                                  layer_dims=(4 * 32 + 13, 32, 16, 1), inner_lr=0.01), 2, 2, 1 << 30, False),
    # tasks above 512 samples per set: the sparse row kernel, which reads the slot of every lookup
    "sparse_row_path": (SMALL.with_(n_tasks=3, n_support=530, n_query=70, n_fields=3, emb_dim=64, rows_per_field=900,
                                    layer_dims=(3 * 64 + 13, 32, 16, 1), inner_lr=0.05), 1, 2, 2 << 30, False),
}


@pytest.mark.parametrize("case", list(CASES))
def test_step_is_identical_on_both_index_paths(gm, case):
    cfg, K, order, ws, table = CASES[case]
    print("index paths", case, flush=True)
    sup, qry, params = _inputs(cfg)
    if ws is None:   # a third of what one wave of all tasks needs: several waves
        probe = gm.from_config(cfg, workspace_bytes=2 << 30)
        ws = int(probe.workspace_bytes(cfg.n_tasks, sup.n_samples, qry.n_samples, sup.nnz, qry.nnz, K, order) * 0.3)
        probe.close()
    ctx = gm.from_config(cfg, workspace_bytes=ws)
    dev = ctx.device
    ds, dq, dp = _to_dev(sup, dev), _to_dev(qry, dev), _params_dev(params, dev)
    res, tables = [], []
    for path, by_field in ((1, 1), (2, 1), (2, 0), (0, 1)):
        ctx.configure("index_path", path)
        ctx.configure("sort_fields", by_field)
        t = torch.zeros_like(dp.emb) if table else None
        out = ctx.meta_step(ds, dq, dp, cfg.inner_lr, K, order, emb_grad_table=t)
        res.append({k: (v.clone() if torch.is_tensor(v) else [x.clone() for x in v] if isinstance(v, (list, tuple)) else v)
                    for k, v in out.items()})
        tables.append(t)
    nl = len(cfg.layer_dims) - 1
    for i in (1, 2, 3):
        _same_bits(res[0], res[i], nl, tables[0], tables[i])
    if not table and cfg.mlp_dtype == 0:
        ctx.configure("index_path", 2)
        _compare_step(cfg, ctx, sup, qry, params, K, order, TOL_FP32, f"{case} index_path=2")
    ctx.close()


def test_row_order_path_refuses_a_row_list_over_several_waves(gm):
    """The row-list output orders the lookups of the whole batch, which is not the order of any one wave of tasks: the
    forced path refuses, the default takes the per-(task, field) sort."""
    from paper_2401_04338_amd.binding import GMetaError
    cfg = SMALL.with_(n_tasks=8)
    sup, qry, params = _inputs(cfg)
    probe = gm.from_config(cfg, workspace_bytes=2 << 30)
    need = probe.workspace_bytes(8, sup.n_samples, qry.n_samples, sup.nnz, qry.nnz, 1, 2)
    probe.close()
    ctx = gm.from_config(cfg, workspace_bytes=int(need * 0.6))
    dev = ctx.device
    ctx.configure("index_path", 2)
    with pytest.raises(GMetaError):
        ctx.meta_step(_to_dev(sup, dev), _to_dev(qry, dev), _params_dev(params, dev), cfg.inner_lr, 1, 2)
    ctx.configure("index_path", 0)
    _compare_step(cfg, ctx, sup, qry, params, 1, 2, TOL_FP32, "row list over several waves, default path")
    ctx.close()
