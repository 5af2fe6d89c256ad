"""Test-only helpers: small hand-made batches, oracle model construction, error norms."""
from __future__ import annotations

import numpy as np

from oracle.maml_dlrm import Model
from synth import Config, make_batch, make_params


def oracle_model(cfg: Config) -> Model:
    return Model(rows_per_field=[cfg.rows_per_field] * cfg.n_fields, emb_dim=cfg.emb_dim,
                 n_dense=cfg.n_dense, layer_dims=list(cfg.layer_dims))


def small_cfg(**kw) -> Config:
    """A multi-hot, Zipf-skewed miniature with overlapping support/query rows."""
    base = dict(name="mini", n_tasks=3, n_fields=3, rows_per_field=40, emb_dim=4,
                layer_dims=(3 * 4 + 5, 8, 6, 1), bag_max=4, zipf_s=1.05, n_support=7, n_query=5,
                inner_steps=2, order=2, n_dense=5, inner_lr=0.1, seed=3)
    base.update(kw)
    if "layer_dims" not in kw:
        d0 = base["n_fields"] * base["emb_dim"] + base["n_dense"]
        base["layer_dims"] = (d0, 8, 6, 1)
    return Config(**base)


def oracle_inputs(cfg: Config, iteration: int = 0, tasks=None, emb_std: float = 0.05):
    sup, qry = make_batch(cfg, iteration, "cpu", tasks)
    params = make_params(cfg, "cpu", emb_std=emb_std)
    return oracle_model(cfg), params.numpy(), sup.numpy(), qry.numpy()


def rel_err(a, b):
    """(relative L2 error, max-abs error relative to max-abs of the reference b)."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    nb = np.linalg.norm(b)
    mb = np.max(np.abs(b)) if b.size else 0.0
    if b.size == 0:
        return 0.0, 0.0
    l2 = np.linalg.norm(a - b) / nb if nb > 0 else np.linalg.norm(a - b)
    mx = np.max(np.abs(a - b)) / mb if mb > 0 else np.max(np.abs(a - b))
    return float(l2), float(mx)


def compact_task(cfg: Config, sup_t, qry_t, emb_dev, W, b):
    """Oracle inputs of a task subset over only the table rows it looks up (synth.compact_tasks does the re-indexing):
    returns (Model with per-field row counts, params dict, sup dict, qry dict, global_rows) where global_rows[i] is the
    full-size table row behind compact row i.  Lets the oracle check tasks of a configuration whose tables do not fit
    host-side copies."""
    from synth import compact_tasks
    counts, emb, sd, qd, global_rows = compact_tasks(cfg, sup_t, qry_t, emb_dev)
    model = Model(rows_per_field=counts, emb_dim=cfg.emb_dim, n_dense=cfg.n_dense, layer_dims=list(cfg.layer_dims))
    params = dict(emb=emb, W=[w.cpu().numpy() for w in W], b=[x.cpu().numpy() for x in b])
    return model, params, sd, qd, global_rows
