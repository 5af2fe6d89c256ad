"""Re-indexing of a task subset onto the table rows it looks up (pure index bookkeeping, none of the method's arithmetic).

The step's result for a set of tasks depends on no table row that those tasks do not look up.  A checker that cannot
hold a configuration's full tables on the host (40 fields x 4 M rows, 64 x 4 M rows) can therefore run on a compacted
copy: per field, the distinct rows the subset looks up, renumbered 0..n_f-1 in ascending order.
"""
from __future__ import annotations

import numpy as np
import torch

from .configs import Config


def compact_tasks(cfg: Config, sup, qry, emb_dev: torch.Tensor):
    """sup, qry: SetData of the task subset (as make_batch(cfg, it, "cpu", tasks) returns them); emb_dev: the full
    tables [F*R, D] on any device.

    Returns (rows_per_field [F] (each >= 1), emb [sum rows_per_field, D] float32 numpy, sup dict, qry dict,
    global_rows) where the dicts are the sets with indices renumbered and global_rows[i] is the full-size global row
    (field * R + index) behind compact global row i."""
    F, R = cfg.n_fields, cfg.rows_per_field
    sd, qd = sup.numpy(), qry.numpy()

    def fields_of(d):
        lens = d["bag_offsets"][1:] - d["bag_offsets"][:-1]
        return np.repeat(np.arange(lens.size, dtype=np.int64) % F, lens)

    fs, fq = fields_of(sd), fields_of(qd)
    counts, rows_all = [], []
    new_s, new_q = np.empty_like(sd["indices"]), np.empty_like(qd["indices"])
    for f in range(F):
        ms, mq = fs == f, fq == f
        u = np.unique(np.concatenate([sd["indices"][ms], qd["indices"][mq]]).astype(np.int64))
        if u.size == 0:
            u = np.zeros(1, dtype=np.int64)
        new_s[ms] = np.searchsorted(u, sd["indices"][ms]).astype(new_s.dtype)
        new_q[mq] = np.searchsorted(u, qd["indices"][mq]).astype(new_q.dtype)
        counts.append(int(u.size))
        rows_all.append(u + f * R)
    global_rows = np.concatenate(rows_all)
    emb = emb_dev[torch.from_numpy(global_rows).to(emb_dev.device)].cpu().numpy()
    sd["indices"], qd["indices"] = new_s, new_q
    return counts, emb, sd, qd, global_rows
