"""CPU oracle of the per-task MAML step over a DLRM-style model (float64, numpy).

TEST INFRASTRUCTURE ONLY.  This file defines what the HIP path must compute; it
is imported by tests/, by __graft_entry__.smoke() and by bench.py's
cpu_baseline leg, never by the product package, and it shares no code with it.

What it follows (G-Meta, Algorithm 1, worker i == task t; MAML after Finn et
al. as the paper adopts it in Section 2):
  * prefetch of the support and query embedding rows        (Alg. 1, prefetch step)
  * inner forward L^Sup, local back-propagation on the looked-up rows xi^Sup and
    on theta with step size alpha                            (Alg. 1, inner steps)
  * overlap update: query rows that also occur in the support set take the
    adapted value, all others keep the prefetched one        (Section 2.1.2)
  * outer forward L^Query with (xi'^Query, theta')           (Alg. 1, outer forward)
  * gradients of L^Query w.r.t. the META parameters, summed over tasks
    (Alg. 1, the two global back-propagation steps; Section 2.1.3: the sum of
    per-task gradients equals the gradient of the sum).
The beta update itself is not part of the step: the step returns the summed
gradients.

Model f (the paper says only "embedding layer + dense layers", Section 2.1):
  x_s = concat_f( sum_{r in bag(s,f)} xi_f[r] ) || dense_s
  MLP with ReLU on hidden layers, one logit, L = mean over the set's samples of
  the binary cross-entropy with logits.

Readings where the paper is silent: loss is the MEAN over a set's samples; tasks
are SUMMED; `inner_steps` repeats the inner update on the whole support set;
order=1 drops the Hessian term; ReLU'(0) = 0; duplicate indices count with
multiplicity; an empty bag pools to zero; the sparse output lists every row
looked up by any support or query sample, ascending by global row id
(field_base[f] + index).

Operand precision.  By default everything is float64.  With operand="bf16" the
operands of the hidden-layer matrix products -- the model input x, the weights
W_l (l < L), the activations a_l, the deltas delta_l (l < L), and their tangent
counterparts -- are rounded to bfloat16 (round to nearest even) at the points
where a mixed-precision kernel would store them; sums, biases, the last layer,
the loss, the SGD updates and the embedding-row arithmetic stay float64.  This
exists because a ReLU mask is a yes/no decision taken on a floating-point
value: a path that stores bf16 activations decides it on the rounded operands,
and a float64 oracle compared with it would differ by whole gradient terms
wherever a pre-activation sits within rounding distance of zero.  Both sides
must take that decision in the same precision; the rounding below is the only
place where the oracle departs from float64, and q = identity recovers it.

ReLU decisions given from outside (relu_masks).  The mode above rounds operands
throughout, so a comparison against it cannot tell whether the rounding points
themselves are right.  relu_masks="bf16" therefore separates the two things:
the task is first run once in the bf16-operand mode only to record the ReLU
gates of every forward pass (each inner step's support pass, the query pass);
then ALL arithmetic runs in float64, with no rounding anywhere, using those
gates as given 0/1 factors (a_l = z_l * m_l; the backward and tangent passes
gate with the same m_l).  This is the reference a reduced-precision path is
held against at the bf16 tolerance: the yes/no decisions are taken where such a
path takes them, and every rounding it makes has to fit inside the tolerance by
itself.  relu_masks may also be an explicit list of masks per forward pass
(tests freeze the gates that way and take central differences of the
frozen-gate objective).

Pins (tests/test_oracle_*.py): central finite differences of the loss and of
the meta-objective, K=0 and alpha=0 identities, the K=1 relation
order2 = (I - alpha*H) order1 with H pinned by differences of the gradient,
closed-form logistic regression, full-table brute force for the overlap update,
task additivity, multiplicity, gradient-mass conservation, pure-Python loops on
a tiny case and a library autograd (double backward) cross-check.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence

import numpy as np


# --------------------------------------------------------------------------
# model description and small helpers
# --------------------------------------------------------------------------
@dataclass
class Model:
    rows_per_field: Sequence[int]
    emb_dim: int
    n_dense: int
    layer_dims: Sequence[int]          # d_0 .. d_L, d_0 = F*D + n_dense, d_L = 1

    @property
    def n_fields(self) -> int:
        return len(self.rows_per_field)

    @property
    def field_base(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(np.asarray(self.rows_per_field, dtype=np.int64))])

    @property
    def n_layers(self) -> int:
        return len(self.layer_dims) - 1


def round_bf16(x):
    """Round float values to the nearest bfloat16 (ties to even), returned as float64."""
    a = np.ascontiguousarray(np.asarray(x, dtype=np.float64).astype(np.float32))
    u = a.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(np.float64).reshape(np.shape(x))


def _identity(x):
    return x


def quantizer(operand: str):
    if operand == "fp64":
        return _identity
    if operand == "bf16":
        return round_bf16
    raise ValueError("operand must be 'fp64' or 'bf16'")


def sigmoid(z):
    return 0.5 * (1.0 + np.tanh(0.5 * z))


def bce_with_logits(z, y):
    """Per-sample binary cross-entropy on a logit, numerically stable form."""
    return np.maximum(z, 0.0) - y * z + np.log1p(np.exp(-np.abs(z)))


def lookup_rows(model: Model, s: Dict[str, np.ndarray], lo: int, hi: int):
    """Global row id and bag id (relative to sample `lo`) of every lookup of samples [lo, hi)."""
    F = model.n_fields
    off = s["bag_offsets"]
    p0, p1 = int(off[lo * F]), int(off[hi * F])
    lens = np.diff(off[lo * F: hi * F + 1])
    bag = np.repeat(np.arange((hi - lo) * F, dtype=np.int64), lens)
    field = bag % F
    rows = model.field_base[field] + s["indices"][p0:p1].astype(np.int64)
    return rows, bag


# --------------------------------------------------------------------------
# the DLRM on one set of samples, with the embedding rows given as a dictionary
# --------------------------------------------------------------------------
def pool(model: Model, E: np.ndarray, loc: np.ndarray, bag: np.ndarray, n: int) -> np.ndarray:
    """e[s,f] = sum over the bag's lookups of E[loc] (multiplicity counted); -> [n, F*D]."""
    out = np.zeros((n * model.n_fields, model.emb_dim))
    np.add.at(out, bag, E[loc])
    return out.reshape(n, model.n_fields * model.emb_dim)


def _w(W, l, q):
    """Weights of layer l as the matrix product reads them: rounded for hidden layers, exact for the last."""
    return q(W[l]) if l < len(W) - 1 else W[l]


def forward(x: np.ndarray, W: List[np.ndarray], b: List[np.ndarray], q=_identity, masks=None, pre_out=None):
    """a_0 = x; z_l = a_{l-1} W_l + b_l; a_l = z_l * m_l for l < L, with m_l = [z_l > 0] (ReLU) unless the
    gates are given (masks[l-1] for hidden layer l).  Returns ([a_0..a_{L-1}], z_L, [m_1..m_{L-1}]).
    pre_out, if a list, receives the hidden layers' pre-activations [z_1..z_{L-1}] (what the gates were decided
    on: a test can tell from them which gates sit within rounding distance of zero)."""
    acts = [q(x)]
    used = []
    L = len(W)
    for l in range(L):
        z = acts[-1] @ _w(W, l, q) + b[l]
        if l < L - 1:
            m = (z > 0.0) if masks is None else np.asarray(masks[l], dtype=bool)
            used.append(m)
            if pre_out is not None:
                pre_out.append(z.copy())
            acts.append(q(np.where(m, z, 0.0)))
    return acts, z[:, 0], used


def set_loss(z: np.ndarray, y: np.ndarray) -> float:
    return float(np.mean(bce_with_logits(z, y))) if len(y) else 0.0


def backward(acts, z, y, W, masks, q=_identity):
    """Gradient of the mean BCE w.r.t. W_l, b_l and the input x (masks: the gates of the forward pass).
    Also returns the deltas."""
    n = len(y)
    L = len(W)
    delta = ((sigmoid(z) - y) / max(n, 1))[:, None]
    dW, db, deltas = [None] * L, [None] * L, [None] * L
    for l in range(L - 1, -1, -1):
        deltas[l] = delta
        dW[l] = acts[l].T @ delta
        db[l] = delta.sum(axis=0)
        da = delta @ _w(W, l, q).T
        if l > 0:
            delta = q(da * masks[l - 1])
    return dW, db, da, deltas


def hvp(acts, z, y, W, deltas, masks, vW, vb, vx, q=_identity):
    """Hessian of the mean BCE (w.r.t. W, b and the input x) times (vW, vb, vx).

    Tangent (forward) pass through the forward AND the backward pass of the
    network; ReLU has no second-derivative term.  Returns (hW, hb, hx).
    """
    n = len(y)
    L = len(W)
    sg = sigmoid(z)
    # tangent of the forward pass
    ta = [q(vx)]
    for l in range(L):
        tz = ta[-1] @ _w(W, l, q) + acts[l] @ _w(vW, l, q) + vb[l]
        if l < L - 1:
            ta.append(q(tz * masks[l]))
    tdelta = (sg * (1.0 - sg) * tz[:, 0] / max(n, 1))[:, None]
    hW, hb = [None] * L, [None] * L
    for l in range(L - 1, -1, -1):
        hW[l] = ta[l].T @ deltas[l] + acts[l].T @ tdelta
        hb[l] = tdelta.sum(axis=0)
        tda = tdelta @ _w(W, l, q).T + deltas[l] @ _w(vW, l, q).T
        if l > 0:
            tdelta = q(tda * masks[l - 1])
    return hW, hb, tda


# --------------------------------------------------------------------------
# one task
# --------------------------------------------------------------------------
def task_meta_grad(model: Model, params, sup, qry, t: int, alpha: float, K: int, order: int,
                   full_table: bool = False, operand: str = "fp64", adapt_rows: bool = True,
                   relu_masks=None, masks_out: Optional[list] = None, pre_out: Optional[list] = None):
    """MAML for task t.  Returns (L^Query, gW, gb, rows, gxi[rows]) w.r.t. the META parameters.

    adapt_rows=False is the variant that adapts the dense parameters only (the way the paper's framework
    also hosts MeLU, Sec. 3.1: embeddings are meta-parameters that the inner loop reads but does not update):
    phi_k = (theta_k, xi), theta_{k+1} = theta_k - alpha grad_theta L^Sup(theta_k, xi).  The meta-gradient
    w.r.t. xi is then the query loss's own plus, for order 2, the path through every theta_k:
    -alpha * d/dxi <grad_theta L^Sup(theta_k, xi), v_theta,k+1>.

    full_table=True copies the whole table into the task (brute force: phi_0 is
    all of xi); the default keeps only the rows the task looks up.  Both must agree.

    relu_masks: None -- every forward pass decides its own ReLU gates (z > 0); "bf16" -- the gates are those of a
    run of the task with operand="bf16", recorded first, while the arithmetic itself follows `operand`; a list of
    K + 1 entries (the K support passes, then the query pass), each the list of hidden
    layers' boolean masks -- gates given from outside.  masks_out, if a list, receives the gates used, in that form;
    pre_out, if a list, the pre-activations those gates belong to (same form).
    """
    F, D = model.n_fields, model.emb_dim
    FD = F * D
    q = quantizer(operand)
    if isinstance(relu_masks, str):
        if relu_masks != "bf16":
            raise ValueError("relu_masks must be None, 'bf16' or a list of masks")
        recorded: list = []
        task_meta_grad(model, params, sup, qry, t, alpha, K, 1, full_table, "bf16", adapt_rows, None, recorded)
        relu_masks = recorded
    s_lo, s_hi = int(sup["task_offsets"][t]), int(sup["task_offsets"][t + 1])
    q_lo, q_hi = int(qry["task_offsets"][t]), int(qry["task_offsets"][t + 1])
    ns, nq = s_hi - s_lo, q_hi - q_lo
    rows_s, bag_s = lookup_rows(model, sup, s_lo, s_hi)
    rows_q, bag_q = lookup_rows(model, qry, q_lo, q_hi)
    if full_table:
        rows = np.arange(model.field_base[-1], dtype=np.int64)
    else:
        rows = np.unique(np.concatenate([rows_s, rows_q]))
    loc_s = np.searchsorted(rows, rows_s)
    loc_q = np.searchsorted(rows, rows_q)
    ys = sup["labels"][s_lo:s_hi].astype(np.float64)
    yq = qry["labels"][q_lo:q_hi].astype(np.float64)
    dense_s = sup["dense"][s_lo:s_hi].astype(np.float64)
    dense_q = qry["dense"][q_lo:q_hi].astype(np.float64)

    # phi_0 = the meta parameters (task-local copies; the meta table is never written)
    E = params["emb"][rows].astype(np.float64)
    W = [w.astype(np.float64) for w in params["W"]]
    b = [x.astype(np.float64) for x in params["b"]]

    def rows_grad(dx, loc, bag):
        g = np.zeros_like(E)
        np.add.at(g, loc, dx[:, :FD].reshape(-1, D)[bag])
        return g

    def gated_forward(x, W, b, i):
        """Forward pass number i of the task (support passes 0..K-1, query pass K) with its gates."""
        pre = [] if pre_out is not None else None
        acts, z, used = forward(x, W, b, q, None if relu_masks is None else relu_masks[i], pre)
        if masks_out is not None:
            masks_out.append(used)
        if pre_out is not None:
            pre_out.append(pre)
        return acts, z, used

    # inner loop on the support set
    tape = []
    for k in range(K):
        x = np.concatenate([pool(model, E, loc_s, bag_s, ns), dense_s], axis=1)
        acts, z, masks = gated_forward(x, W, b, k)
        dW, db, dx, deltas = backward(acts, z, ys, W, masks, q)
        tape.append((acts, z, W, deltas, masks))
        if adapt_rows:
            E = E - alpha * rows_grad(dx, loc_s, bag_s)
        W = [w - alpha * g for w, g in zip(W, dW)]
        b = [v - alpha * g for v, g in zip(b, db)]

    # outer forward/backward on the query set with the adapted parameters
    xq = np.concatenate([pool(model, E, loc_q, bag_q, nq), dense_q], axis=1)
    acts, z, masks = gated_forward(xq, W, b, K)
    loss_q = set_loss(z, yq)
    vW, vb, dx, _ = backward(acts, z, yq, W, masks, q)
    vE = rows_grad(dx, loc_q, bag_q)

    # chain back through the inner steps: v_k = v_{k+1} - alpha * H_k v_{k+1}
    if order == 2:
        for acts_k, z_k, W_k, deltas_k, masks_k in reversed(tape):
            if adapt_rows:
                vx = np.concatenate([pool(model, vE, loc_s, bag_s, ns), np.zeros_like(dense_s)], axis=1)
            else:   # xi is not a state of the inner loop: no direction on the inputs
                vx = np.zeros((ns, FD + dense_s.shape[1]))
            hW, hb, hx = hvp(acts_k, z_k, ys, W_k, deltas_k, masks_k, vW, vb, vx, q)
            hE = rows_grad(hx, loc_s, bag_s)
            vW = [v - alpha * h for v, h in zip(vW, hW)]
            vb = [v - alpha * h for v, h in zip(vb, hb)]
            vE = vE - alpha * hE
    elif order != 1:
        raise ValueError("order must be 1 or 2")
    if full_table:
        touched = np.unique(np.concatenate([rows_s, rows_q]))
        return loss_q, vW, vb, touched, vE[touched]
    return loss_q, vW, vb, rows, vE


# --------------------------------------------------------------------------
# the whole step
# --------------------------------------------------------------------------
def meta_step(model: Model, params, sup, qry, alpha: float, K: int, order: int,
              tasks: Optional[Sequence[int]] = None, full_table: bool = False, operand: str = "fp64",
              adapt_rows: bool = True, relu_masks=None, masks_out: Optional[dict] = None,
              pre_out: Optional[dict] = None):
    """Sum of the per-task meta-gradients (Alg. 1, global back-propagation steps).

    relu_masks: None, "bf16", or {task: list of masks per forward pass} (see task_meta_grad); masks_out, if a
    dict, receives {task: gates used}; pre_out, if a dict, {task: the pre-activations they were decided on}.

    Returns dict(loss, task_loss[T], dW[l], db[l], emb_rows (ascending unique
    global rows looked up by any sample), emb_grad[len(emb_rows), D]).
    """
    T = len(sup["task_offsets"]) - 1
    tasks = list(range(T)) if tasks is None else list(tasks)
    L = model.n_layers
    gW = [np.zeros((model.layer_dims[l], model.layer_dims[l + 1])) for l in range(L)]
    gb = [np.zeros(model.layer_dims[l + 1]) for l in range(L)]
    task_loss = np.zeros(len(tasks))
    parts_rows, parts_grad = [], []
    for i, t in enumerate(tasks):
        rec = [] if masks_out is not None else None
        pre = [] if pre_out is not None else None
        lq, vW, vb, rows, vE = task_meta_grad(model, params, sup, qry, t, alpha, K, order, full_table, operand,
                                              adapt_rows, relu_masks[t] if isinstance(relu_masks, dict) else relu_masks,
                                              rec, pre)
        if masks_out is not None:
            masks_out[t] = rec
        if pre_out is not None:
            pre_out[t] = pre
        task_loss[i] = lq
        for l in range(L):
            gW[l] += vW[l]
            gb[l] += vb[l]
        parts_rows.append(rows)
        parts_grad.append(vE)
    if parts_rows:
        all_rows = np.concatenate(parts_rows)
        emb_rows, inv = np.unique(all_rows, return_inverse=True)
        emb_grad = np.zeros((len(emb_rows), model.emb_dim))
        np.add.at(emb_grad, inv, np.concatenate(parts_grad))
    else:
        emb_rows, emb_grad = np.zeros(0, np.int64), np.zeros((0, model.emb_dim))
    return dict(loss=float(task_loss.sum()), task_loss=task_loss, dW=gW, db=gb,
                emb_rows=emb_rows, emb_grad=emb_grad)


def meta_train_step(model: Model, params, sup, qry, alpha: float, K: int, order: int, beta: float,
                    operand: str = "fp64", adapt_rows: bool = True, relu_masks=None):
    """One whole iteration of Alg. 1 on one shard: the step above, then the two global back-propagation steps with
    the outer step size beta (plain SGD on the summed meta-gradient): theta <- theta - beta * sum_t grad_theta and,
    for every looked-up row, xi[row] <- xi[row] - beta * sum_t grad_xi[row].

    Returns (new params dict (float64 copies; the input is not modified), loss of the step before the update).
    """
    r = meta_step(model, params, sup, qry, alpha, K, order, operand=operand, adapt_rows=adapt_rows,
                  relu_masks=relu_masks)
    emb = np.array(params["emb"], dtype=np.float64, copy=True)
    emb[r["emb_rows"]] -= beta * r["emb_grad"]
    W = [np.asarray(w, dtype=np.float64) - beta * g for w, g in zip(params["W"], r["dW"])]
    b = [np.asarray(x, dtype=np.float64) - beta * g for x, g in zip(params["b"], r["db"])]
    return dict(emb=emb, W=W, b=b), r["loss"]


# --------------------------------------------------------------------------
# integer side of the step: what the index preparation must produce, exactly
# --------------------------------------------------------------------------
def index_prep(model: Model, sup, qry):
    """The unique integer structures behind the overlap update and the sparse gradient.

    Per (task, field), in task-major then field order:
      slot_counts[T*F]    number of distinct rows the task's SUPPORT lookups touch in the field
      slot_rows           those rows (global ids), ascending within each (task, field)
      sup_slot[nnz_sup]   for every support lookup, the rank of its row in its (task, field) list
      qry_slot[nnz_qry]   for every query lookup, that rank if the row is in the task's
                          support list for the field, else -1   (the overlap join)
    Over the whole batch:
      emb_rows            ascending distinct global rows over all support and query lookups
      seg_counts          number of lookups (support + query, all tasks) of each of them
    """
    F = model.n_fields
    T = len(sup["task_offsets"]) - 1
    sup_slot = np.zeros(len(sup["indices"]), dtype=np.int32)
    qry_slot = np.full(len(qry["indices"]), -1, dtype=np.int32)
    slot_counts = np.zeros(T * F, dtype=np.int64)
    slot_rows = []
    all_rows = []
    for t in range(T):
        s_lo, s_hi = int(sup["task_offsets"][t]), int(sup["task_offsets"][t + 1])
        q_lo, q_hi = int(qry["task_offsets"][t]), int(qry["task_offsets"][t + 1])
        rows_s, bag_s = lookup_rows(model, sup, s_lo, s_hi)
        rows_q, bag_q = lookup_rows(model, qry, q_lo, q_hi)
        all_rows += [rows_s, rows_q]
        ps, pq = int(sup["bag_offsets"][s_lo * F]), int(qry["bag_offsets"][q_lo * F])
        for f in range(F):
            ms, mq = (bag_s % F) == f, (bag_q % F) == f
            u = np.unique(rows_s[ms])
            slot_counts[t * F + f] = len(u)
            slot_rows.append(u)
            sup_slot[ps + np.nonzero(ms)[0]] = np.searchsorted(u, rows_s[ms])
            if len(u):
                pos = np.searchsorted(u, rows_q[mq])
                hit = (pos < len(u)) & (u[np.minimum(pos, len(u) - 1)] == rows_q[mq])
                qry_slot[pq + np.nonzero(mq)[0]] = np.where(hit, pos, -1)
    cat = np.concatenate(all_rows) if all_rows else np.zeros(0, np.int64)
    emb_rows, seg_counts = np.unique(cat, return_counts=True)
    return dict(slot_counts=slot_counts,
                slot_rows=np.concatenate(slot_rows) if slot_rows else np.zeros(0, np.int64),
                sup_slot=sup_slot, qry_slot=qry_slot,
                emb_rows=emb_rows.astype(np.int64), seg_counts=seg_counts.astype(np.int64))


def gather_pool(model: Model, emb: np.ndarray, s) -> np.ndarray:
    """Pooled model input of every sample of a set: [n, F*D + n_dense] (Alg. 1, prefetch step)."""
    n = int(s["task_offsets"][-1])
    rows, bag = lookup_rows(model, s, 0, n)
    x = pool(model, emb.astype(np.float64), rows, bag, n)
    return np.concatenate([x, s["dense"].astype(np.float64)], axis=1)


# --------------------------------------------------------------------------
# the step before the hot path: one-task batches out of a flat record stream (Sec. 2.2.2, Meta I/O pipeline)
# --------------------------------------------------------------------------
def group_batch(n_fields: int, task, batch_id, bag_offsets, indices, dense, labels, support_num: int, support_den: int):
    """Assembles task batches from a flat stream of records: records with equal (task, batch_id) form one batch
    (the paper's GroupBatchOp), and every batch is split into a support and a query set (Alg. 1, "Split T_i").

    Readings where the paper is silent: batches come out in ascending (task, batch_id) order; inside a batch the
    records keep their order in the stream; the first ceil(n * support_num / support_den) records of a batch of n are
    its support set, the rest its query set.

    Returns (support, query): dicts with task_offsets, bag_offsets, indices, dense, labels (the layout of the step).
    """
    task = np.asarray(task, dtype=np.int64)
    batch_id = np.asarray(batch_id, dtype=np.int64)
    bag_offsets = np.asarray(bag_offsets, dtype=np.int64)
    n = task.shape[0]
    order = sorted(range(n), key=lambda i: (int(task[i]), int(batch_id[i]), i))
    groups = []
    for i in order:
        if groups and (task[groups[-1][0]], batch_id[groups[-1][0]]) == (task[i], batch_id[i]):
            groups[-1].append(i)
        else:
            groups.append([i])

    def build(parts):
        toff, boff, idx, dn, lb = [0], [0], [], [], []
        for recs in parts:
            for i in recs:
                for f in range(n_fields):
                    p0, p1 = int(bag_offsets[i * n_fields + f]), int(bag_offsets[i * n_fields + f + 1])
                    idx.extend(int(x) for x in indices[p0:p1])
                    boff.append(len(idx))
                dn.append(np.asarray(dense[i]))
                lb.append(labels[i])
            toff.append(toff[-1] + len(recs))
        nd = np.asarray(dense).shape[1]
        return dict(task_offsets=np.asarray(toff, dtype=np.int64), bag_offsets=np.asarray(boff, dtype=np.int64),
                    indices=np.asarray(idx, dtype=np.int32),
                    dense=np.asarray(dn, dtype=np.float32).reshape(len(dn), nd), labels=np.asarray(lb, dtype=np.float32))

    sup_parts, qry_parts = [], []
    for recs in groups:
        k = (len(recs) * support_num + support_den - 1) // support_den
        sup_parts.append(recs[:k])
        qry_parts.append(recs[k:])
    return build(sup_parts), build(qry_parts)
