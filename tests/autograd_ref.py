"""Test-only third opinion: the MAML step reduced to a library autograd (float64, CPU).

Only the forward model is written here, with library routines for the loss
(binary_cross_entropy_with_logits) and for every derivative (autograd with
create_graph for the second-order term).  It differentiates with respect to the
WHOLE embedding table, so it also checks the oracle's row-dictionary logic.
Used to cross-check the oracle, never as the oracle.
"""
from __future__ import annotations

import numpy as np
import torch
import torch.nn.functional as Fn


def _set_tensors(model, s, lo, hi):
    F = model.n_fields
    off = s["bag_offsets"]
    p0, p1 = int(off[lo * F]), int(off[hi * F])
    lens = torch.from_numpy(np.diff(off[lo * F: hi * F + 1]))
    bag = torch.repeat_interleave(torch.arange((hi - lo) * F), lens)
    base = torch.from_numpy(np.asarray(model.field_base[:-1], dtype=np.int64))
    rows = base[bag % F] + torch.from_numpy(s["indices"][p0:p1].astype(np.int64))
    dense = torch.from_numpy(s["dense"][lo:hi].astype(np.float64))
    y = torch.from_numpy(s["labels"][lo:hi].astype(np.float64))
    return rows, bag, dense, y


def _loss(model, emb, W, b, rows, bag, dense, y):
    n = dense.shape[0]
    pooled = torch.zeros(n * model.n_fields, model.emb_dim, dtype=torch.float64)
    pooled = pooled.index_add(0, bag, emb[rows])
    a = torch.cat([pooled.reshape(n, -1), dense], dim=1)
    L = len(W)
    for l in range(L):
        a = a @ W[l] + b[l]
        if l < L - 1:
            a = torch.relu(a)
    return Fn.binary_cross_entropy_with_logits(a[:, 0], y, reduction="mean")


def meta_step_autograd(model, params, sup, qry, alpha, K, order, adapt_emb=True):
    emb0 = torch.tensor(params["emb"], dtype=torch.float64, requires_grad=True)
    W0 = [torch.tensor(w, dtype=torch.float64, requires_grad=True) for w in params["W"]]
    b0 = [torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in params["b"]]
    L = len(W0)
    T = len(sup["task_offsets"]) - 1
    total = 0.0
    task_loss = []
    for t in range(T):
        rs, bs, ds, ys = _set_tensors(model, sup, int(sup["task_offsets"][t]), int(sup["task_offsets"][t + 1]))
        rq, bq, dq, yq = _set_tensors(model, qry, int(qry["task_offsets"][t]), int(qry["task_offsets"][t + 1]))
        emb, W, b = emb0, list(W0), list(b0)
        for _ in range(K):
            ls = _loss(model, emb, W, b, rs, bs, ds, ys)
            gs = torch.autograd.grad(ls, [emb] + W + b, create_graph=(order == 2))
            if order == 1:
                gs = [g.detach() for g in gs]
            if adapt_emb:
                emb = emb - alpha * gs[0]
            W = [w - alpha * g for w, g in zip(W, gs[1:1 + L])]
            b = [x - alpha * g for x, g in zip(b, gs[1 + L:])]
        lq = _loss(model, emb, W, b, rq, bq, dq, yq)
        task_loss.append(float(lq.detach()))
        total = total + lq
    total.backward()
    return dict(loss=float(total.detach()), task_loss=np.array(task_loss),
                dW=[w.grad.numpy() for w in W0], db=[x.grad.numpy() for x in b0],
                emb_grad_full=emb0.grad.numpy())
