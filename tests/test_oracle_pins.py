"""Pins of the CPU oracle against things other than itself (all CPU, float64).

The paper prints no worked numeric example of a MAML step, so the oracle is
pinned by: finite differences, closed forms, identities of the method
(Algorithm 1; Section 2.1.2 overlap update; Section 2.1.3 sum rule), brute
force, pure-Python loops and a library autograd.
"""
import math

import numpy as np
import pytest

from oracle import maml_dlrm as O
from synth import TINY
from tests.autograd_ref import meta_step_autograd
from tests.helpers import oracle_inputs, oracle_model, rel_err, small_cfg


def _full_grad(model, out):
    g = np.zeros((int(model.field_base[-1]), model.emb_dim))
    g[out["emb_rows"]] = out["emb_grad"]
    return g


def _objective(model, params, sup, qry, alpha, K, adapt_rows=True):
    """M(phi) = sum_t L^Query_t(phi_K(phi)): forward value only."""
    return O.meta_step(model, params, sup, qry, alpha, K, 1, adapt_rows=adapt_rows)["loss"]


def _min_hidden_margin(model, params, sup, qry, alpha, K):
    """Smallest |pre-activation| seen at a ReLU on the whole path (kink guard for differences)."""
    m = np.inf
    T = len(sup["task_offsets"]) - 1
    import torch
    # re-run the inner loop with the autograd reference's forward pieces is overkill; use the oracle's
    for t in range(T):
        s_lo, s_hi = int(sup["task_offsets"][t]), int(sup["task_offsets"][t + 1])
        rows, bag = O.lookup_rows(model, sup, s_lo, s_hi)
        x = np.concatenate([O.pool(model, params["emb"].astype(np.float64), rows, bag, s_hi - s_lo),
                            sup["dense"][s_lo:s_hi]], axis=1)
        a = x
        for l in range(model.n_layers - 1):
            z = a @ params["W"][l].astype(np.float64) + params["b"][l]
            m = min(m, np.abs(z).min())
            a = np.maximum(z, 0)
    return m


# ---------------------------------------------------------------- forward value
def test_forward_loss_against_python_loops():
    """Pooling (with a duplicate index and an empty bag), MLP and BCE by scalar loops."""
    model = O.Model(rows_per_field=[5, 4], emb_dim=2, n_dense=1, layer_dims=[5, 3, 1])
    rng = np.random.default_rng(0)
    emb = rng.normal(size=(9, 2))
    W = [rng.normal(size=(5, 3)), rng.normal(size=(3, 1))]
    b = [rng.normal(size=3), rng.normal(size=1)]
    # 3 samples; bags: s0:(f0:[1,1], f1:[]) s1:(f0:[4], f1:[0,3]) s2:(f0:[0,2,4], f1:[2])
    bags = [[[1, 1], []], [[4], [0, 3]], [[0, 2, 4], [2]]]
    indices, offs = [], [0]
    for s in bags:
        for f in s:
            indices += f
            offs.append(len(indices))
    dense = rng.normal(size=(3, 1))
    y = np.array([1.0, 0.0, 1.0])
    st = dict(task_offsets=np.array([0, 3]), bag_offsets=np.array(offs, dtype=np.int64),
              indices=np.array(indices, dtype=np.int32), dense=dense, labels=y)
    x = O.gather_pool(model, emb, st)
    acts, z, _ = O.forward(x, W, b)
    got = O.set_loss(z, y)
    # scalar loops
    total = 0.0
    for s in range(3):
        xin = []
        for f in range(2):
            v = [0.0, 0.0]
            for r in bags[s][f]:
                g = [0, 5][f] + r
                v = [v[0] + emb[g, 0], v[1] + emb[g, 1]]
            xin += v
        xin += [dense[s, 0]]
        assert np.allclose(x[s], xin, rtol=0, atol=1e-15)
        h = [max(0.0, sum(xin[i] * W[0][i, j] for i in range(5)) + b[0][j]) for j in range(3)]
        zz = sum(h[j] * W[1][j, 0] for j in range(3)) + b[1][0]
        p = 1.0 / (1.0 + math.exp(-zz))
        total += -(y[s] * math.log(p) + (1 - y[s]) * math.log(1 - p))
    assert abs(got - total / 3) < 1e-13
    # duplicate index counts twice; empty bag pools to zero
    assert np.allclose(x[0, 0:2], 2 * emb[1]) and np.all(x[0, 2:4] == 0.0)


def test_zero_weights_give_log2():
    model, params, sup, qry = oracle_inputs(small_cfg())
    params["W"] = [np.zeros_like(w) for w in params["W"]]
    params["b"] = [np.zeros_like(x) for x in params["b"]]
    out = O.meta_step(model, params, sup, qry, 0.1, 0, 1)
    assert np.allclose(out["task_loss"], math.log(2.0), atol=1e-15)


# ---------------------------------------------------------------- finite differences
def _fd_check(cfg, K, n_coords=40, eps=1e-5, tol=2e-6, emb_std=0.3, adapt_rows=True):
    model, params, sup, qry = oracle_inputs(cfg, emb_std=emb_std)
    params = {k: ([a.astype(np.float64) for a in v] if isinstance(v, list) else v.astype(np.float64))
              for k, v in params.items()}
    alpha = cfg.inner_lr
    out = O.meta_step(model, params, sup, qry, alpha, K, 2, adapt_rows=adapt_rows)
    gfull = _full_grad(model, out)
    rng = np.random.default_rng(1)
    checks = []
    # dense coordinates
    for l in range(model.n_layers):
        for _ in range(n_coords // model.n_layers):
            i = tuple(rng.integers(0, s) for s in params["W"][l].shape)
            checks.append(("W", l, i, out["dW"][l][i]))
        j = (int(rng.integers(0, params["b"][l].shape[0])),)
        checks.append(("b", l, j, out["db"][l][j]))
    # touched embedding rows: random ones plus every touched row of field 0
    touched = out["emb_rows"]
    f0 = touched[touched < model.field_base[1]]
    pick = np.concatenate([rng.choice(touched, size=min(20, len(touched)), replace=False), f0[:30]])
    for r in pick:
        c = int(rng.integers(0, model.emb_dim))
        checks.append(("emb", None, (int(r), c), gfull[int(r), c]))
    worst = 0.0
    scale = max(np.abs(gfull).max(), max(np.abs(g).max() for g in out["dW"]))
    for kind, l, i, g in checks:
        arr = params["emb"] if kind == "emb" else params[kind][l]
        old = arr[i]
        arr[i] = old + eps
        fp = _objective(model, params, sup, qry, alpha, K, adapt_rows)
        arr[i] = old - eps
        fm = _objective(model, params, sup, qry, alpha, K, adapt_rows)
        arr[i] = old
        fd = (fp - fm) / (2 * eps)
        worst = max(worst, abs(fd - g) / scale)
    assert worst < tol, worst
    # an untouched row has exactly no gradient and is not listed
    untouched = np.setdiff1d(np.arange(model.field_base[-1]), touched)
    if len(untouched):
        assert np.all(gfull[untouched] == 0.0)


def test_plain_gradient_by_central_differences():
    """K = 0: the step is the plain DLRM gradient of the query loss."""
    _fd_check(small_cfg(), K=0)


@pytest.mark.parametrize("K", [1, 2, 3])
def test_meta_gradient_by_central_differences(K):
    """order = 2: d/dphi of sum_t L^Query_t(phi_K(phi)), theta and xi parts."""
    cfg = small_cfg(inner_lr=0.3)
    model, params, sup, qry = oracle_inputs(cfg, emb_std=0.3)
    assert _min_hidden_margin(model, params, sup, qry, cfg.inner_lr, K) > 1e-4
    _fd_check(cfg, K=K)


def test_meta_gradient_fd_tiny_config_shape():
    """Same on the Tiny workload's shape (bag size 1, uniform indices), fewer tasks for speed."""
    _fd_check(TINY.with_(n_tasks=2, n_support=8, n_query=8, inner_lr=0.2), K=1, n_coords=12)


def test_second_order_term_is_not_negligible():
    """The differences above would not notice a dropped Hessian term if it were tiny: it is not."""
    cfg = small_cfg(inner_lr=0.3)
    model, params, sup, qry = oracle_inputs(cfg, emb_std=0.3)
    o1 = O.meta_step(model, params, sup, qry, 0.3, 2, 1)
    o2 = O.meta_step(model, params, sup, qry, 0.3, 2, 2)
    assert rel_err(o1["dW"][0], o2["dW"][0])[0] > 1e-3
    assert rel_err(o1["emb_grad"], o2["emb_grad"])[0] > 1e-3


# ---------------------------------------------------------------- identities of the method
def test_alpha_zero_orders_agree_and_equal_K0():
    model, params, sup, qry = oracle_inputs(small_cfg())
    ref = O.meta_step(model, params, sup, qry, 0.0, 0, 1)
    for K in (1, 3):
        for order in (1, 2):
            out = O.meta_step(model, params, sup, qry, 0.0, K, order)
            assert out["loss"] == pytest.approx(ref["loss"], abs=1e-15)
            for a, b in zip(out["dW"] + out["db"] + [out["emb_grad"]],
                            ref["dW"] + ref["db"] + [ref["emb_grad"]]):
                assert np.allclose(a, b, rtol=0, atol=1e-15)
            assert np.array_equal(out["emb_rows"], ref["emb_rows"])


def test_K0_ignores_support_set():
    cfg = small_cfg()
    model, params, sup, qry = oracle_inputs(cfg)
    _, _, sup2, _ = oracle_inputs(cfg, iteration=5)
    a = O.meta_step(model, params, sup, qry, 0.1, 0, 2)
    b = O.meta_step(model, params, sup2, qry, 0.1, 0, 2)
    assert a["loss"] == b["loss"]
    ga, gb = _full_grad(model, a), _full_grad(model, b)
    assert np.array_equal(ga, gb)          # listed rows differ (support rows), values do not


def test_K1_relation_with_hessian_by_gradient_differences():
    """order2 = order1 - alpha * H^Sup(phi_0) order1, H.v from central differences of the gradient."""
    cfg = small_cfg(n_tasks=1, inner_lr=0.2)
    model, params, sup, qry = oracle_inputs(cfg, emb_std=0.3)
    params = {k: ([a.astype(np.float64) for a in v] if isinstance(v, list) else v.astype(np.float64))
              for k, v in params.items()}
    alpha = 0.2
    o1 = O.meta_step(model, params, sup, qry, alpha, 1, 1)
    o2 = O.meta_step(model, params, sup, qry, alpha, 1, 2)
    v_emb = _full_grad(model, o1)

    def sup_grad(p):
        # plain gradient of the SUPPORT loss: a K=0 step with the support set as the query set
        o = O.meta_step(model, p, sup, sup, 0.0, 0, 1)
        return o["dW"], o["db"], _full_grad(model, o)

    def shifted(sign, eps=1e-5):
        return dict(emb=params["emb"] + sign * eps * v_emb,
                    W=[w + sign * eps * v for w, v in zip(params["W"], o1["dW"])],
                    b=[x + sign * eps * v for x, v in zip(params["b"], o1["db"])])

    gp, gm = sup_grad(shifted(+1)), sup_grad(shifted(-1))
    eps = 1e-5
    HW = [(a - b) / (2 * eps) for a, b in zip(gp[0], gm[0])]
    Hb = [(a - b) / (2 * eps) for a, b in zip(gp[1], gm[1])]
    HE = (gp[2] - gm[2]) / (2 * eps)
    for l in range(model.n_layers):
        assert np.allclose(o2["dW"][l], o1["dW"][l] - alpha * HW[l], rtol=0, atol=2e-7)
        assert np.allclose(o2["db"][l], o1["db"][l] - alpha * Hb[l], rtol=0, atol=2e-7)
    assert np.allclose(_full_grad(model, o2), v_emb - alpha * HE, rtol=0, atol=2e-7)


def test_logistic_regression_closed_form():
    """L = 1, no sparse fields: H = X~^T diag(s(1-s)) X~ / N, meta-grad = (I - alpha H) grad L^Q(phi_1)."""
    rng = np.random.default_rng(7)
    d, ns, nq, alpha = 6, 9, 11, 0.7
    model = O.Model(rows_per_field=[], emb_dim=4, n_dense=d, layer_dims=[d, 1])
    params = dict(emb=np.zeros((0, 4)), W=[rng.normal(size=(d, 1))], b=[rng.normal(size=1)])

    def mkset(n):
        return dict(task_offsets=np.array([0, n]), bag_offsets=np.zeros(1, np.int64),
                    indices=np.zeros(0, np.int32), dense=rng.normal(size=(n, d)),
                    labels=(rng.random(n) < 0.4).astype(np.float64))
    sup, qry = mkset(ns), mkset(nq)
    Xs = np.concatenate([sup["dense"], np.ones((ns, 1))], axis=1)
    Xq = np.concatenate([qry["dense"], np.ones((nq, 1))], axis=1)
    w0 = np.concatenate([params["W"][0][:, 0], params["b"][0]])
    sig = lambda z: 1.0 / (1.0 + np.exp(-z))
    ps = sig(Xs @ w0)
    w1 = w0 - alpha * Xs.T @ (ps - sup["labels"]) / ns
    gq = Xq.T @ (sig(Xq @ w1) - qry["labels"]) / nq
    H = Xs.T @ (Xs * (ps * (1 - ps))[:, None]) / ns
    want2 = gq - alpha * H @ gq
    o1 = O.meta_step(model, params, sup, qry, alpha, 1, 1)
    o2 = O.meta_step(model, params, sup, qry, alpha, 1, 2)
    assert np.allclose(np.concatenate([o1["dW"][0][:, 0], o1["db"][0]]), gq, atol=1e-14)
    assert np.allclose(np.concatenate([o2["dW"][0][:, 0], o2["db"][0]]), want2, atol=1e-14)
    zq = Xq @ w1
    want_loss = np.mean(-(qry["labels"] * np.log(sig(zq)) + (1 - qry["labels"]) * np.log(1 - sig(zq))))
    assert o2["loss"] == pytest.approx(want_loss, abs=1e-14)


@pytest.mark.parametrize("order", [1, 2])
def test_overlap_update_equals_full_table_copy(order):
    """Row dictionaries vs copying the whole table into every task (Section 2.1.2)."""
    cfg = TINY.with_(rows_per_field=30, n_support=16, n_query=16, inner_lr=0.2)  # forces overlap
    model, params, sup, qry = oracle_inputs(cfg, emb_std=0.3)
    a = O.meta_step(model, params, sup, qry, 0.2, 2, order)
    b = O.meta_step(model, params, sup, qry, 0.2, 2, order, full_table=True)
    assert a["loss"] == pytest.approx(b["loss"], abs=1e-14)
    assert np.array_equal(a["emb_rows"], b["emb_rows"])
    assert np.allclose(a["emb_grad"], b["emb_grad"], rtol=0, atol=1e-15)
    for x, y in zip(a["dW"] + a["db"], b["dW"] + b["db"]):
        assert np.allclose(x, y, rtol=0, atol=1e-15)
    # the case really has overlap between support and query rows
    ip = O.index_prep(model, sup, qry)
    assert (ip["qry_slot"] >= 0).sum() > 10 and (ip["qry_slot"] < 0).sum() > 10


def test_disjoint_rows_mean_query_sees_meta_embeddings():
    """No shared row: the query loss equals the one with un-adapted embeddings (theta still adapted)."""
    cfg = small_cfg(rows_per_field=400, zipf_s=0.0, n_tasks=2)
    model, params, sup, qry = oracle_inputs(cfg, emb_std=0.3)
    qry = dict(qry)
    qry["indices"] = (qry["indices"] % 200) + 200      # query rows in the upper half
    sup = dict(sup)
    sup["indices"] = sup["indices"] % 200              # support rows in the lower half
    # one inner step: with more, the adapted SUPPORT rows already change theta' in later steps
    got = O.meta_step(model, params, sup, qry, 0.3, 1, 2)
    ref = meta_step_autograd(model, params, sup, qry, 0.3, 1, 2, adapt_emb=False)
    assert np.allclose(got["task_loss"], ref["task_loss"], rtol=0, atol=1e-14)
    # and with shared rows the two differ
    sup2 = dict(sup)
    sup2["indices"] = sup["indices"] % 3 + 200
    qry2 = dict(qry)
    qry2["indices"] = qry["indices"] % 3 + 200
    g2 = O.meta_step(model, params, sup2, qry2, 0.3, 1, 2)
    r2 = meta_step_autograd(model, params, sup2, qry2, 0.3, 1, 2, adapt_emb=False)
    assert abs(g2["loss"] - r2["loss"]) > 1e-6


def test_task_additivity_and_permutation():
    """Section 2.1.3: the gradient of the sum is the sum of per-task gradients."""
    cfg = small_cfg(n_tasks=4)
    model, params, sup, qry = oracle_inputs(cfg)
    whole = O.meta_step(model, params, sup, qry, 0.1, 2, 2)
    acc = np.zeros((int(model.field_base[-1]), model.emb_dim))
    accW = [np.zeros_like(w, dtype=np.float64) for w in params["W"]]
    for t in range(4):
        m2, p2, s2, q2 = oracle_inputs(cfg, tasks=[t])
        one = O.meta_step(m2, p2, s2, q2, 0.1, 2, 2)
        assert one["loss"] == pytest.approx(whole["task_loss"][t], abs=1e-15)
        acc += _full_grad(model, one)
        for l in range(model.n_layers):
            accW[l] += one["dW"][l]
    assert np.allclose(acc, _full_grad(model, whole), rtol=0, atol=1e-15)
    for l in range(model.n_layers):
        assert np.allclose(accW[l], whole["dW"][l], rtol=0, atol=1e-15)
    # permuting tasks permutes task_loss and leaves the sums unchanged
    _, _, sp, qp = oracle_inputs(cfg, tasks=[2, 0, 3, 1])
    perm = O.meta_step(model, params, sp, qp, 0.1, 2, 2)
    assert np.allclose(perm["task_loss"], whole["task_loss"][[2, 0, 3, 1]], rtol=0, atol=1e-15)
    assert np.allclose(_full_grad(model, perm), _full_grad(model, whole), rtol=0, atol=1e-14)


def test_gradient_mass_conservation_first_order():
    """Sum over rows of field f of the sparse gradient = sum over query samples of len(bag) * dx."""
    cfg = small_cfg()
    model, params, sup, qry = oracle_inputs(cfg, emb_std=0.3)
    out = O.meta_step(model, params, sup, qry, 0.0, 0, 1)       # plain gradient at phi
    import torch
    emb = torch.tensor(params["emb"], dtype=torch.float64)
    D, F = cfg.emb_dim, cfg.n_fields
    n = int(qry["task_offsets"][-1])
    x = torch.tensor(O.gather_pool(model, params["emb"], qry), requires_grad=True)
    a = x
    for l, (w, b) in enumerate(zip(params["W"], params["b"])):
        a = a @ torch.tensor(w, dtype=torch.float64) + torch.tensor(b, dtype=torch.float64)
        if l < len(params["W"]) - 1:
            a = torch.relu(a)
    y = torch.tensor(qry["labels"], dtype=torch.float64)
    tot = 0.0
    for t in range(cfg.n_tasks):
        lo, hi = int(qry["task_offsets"][t]), int(qry["task_offsets"][t + 1])
        tot = tot + torch.nn.functional.binary_cross_entropy_with_logits(a[lo:hi, 0], y[lo:hi])
    tot.backward()
    dx = x.grad.numpy()[:, :F * D].reshape(n, F, D)
    lens = np.diff(qry["bag_offsets"]).reshape(n, F)
    want = (dx * lens[:, :, None]).sum(axis=0)                  # [F, D]
    g = _full_grad(model, out).reshape(F, cfg.rows_per_field, D).sum(axis=1)
    assert np.allclose(g, want, rtol=0, atol=1e-14)


# ---------------------------------------------------------------- library autograd, whole step
@pytest.mark.parametrize("K,order", [(0, 2), (1, 1), (1, 2), (2, 2), (3, 1), (3, 2)])
def test_against_library_double_backward(K, order):
    cfg = small_cfg(inner_lr=0.3)
    model, params, sup, qry = oracle_inputs(cfg, emb_std=0.3)
    got = O.meta_step(model, params, sup, qry, 0.3, K, order)
    ref = meta_step_autograd(model, params, sup, qry, 0.3, K, order)
    assert got["loss"] == pytest.approx(ref["loss"], abs=1e-13)
    assert np.allclose(got["task_loss"], ref["task_loss"], rtol=0, atol=1e-13)
    for l in range(model.n_layers):
        assert np.allclose(got["dW"][l], ref["dW"][l], rtol=0, atol=1e-13)
        assert np.allclose(got["db"][l], ref["db"][l], rtol=0, atol=1e-13)
    assert np.allclose(_full_grad(model, got), ref["emb_grad_full"], rtol=0, atol=1e-13)


def test_against_library_double_backward_tiny_config():
    """The Tiny workload at full size (4 tasks, 8 fields x 1000 rows x 16, MLP 141-64-32-1, K=1, 2nd order)."""
    model, params, sup, qry = oracle_inputs(TINY)
    got = O.meta_step(model, params, sup, qry, TINY.inner_lr, 1, 2)
    ref = meta_step_autograd(model, params, sup, qry, TINY.inner_lr, 1, 2)
    assert got["loss"] == pytest.approx(ref["loss"], abs=1e-13)
    assert np.allclose(_full_grad(model, got), ref["emb_grad_full"], rtol=0, atol=1e-14)
    for l in range(3):
        assert np.allclose(got["dW"][l], ref["dW"][l], rtol=0, atol=1e-14)


# ---------------------------------------------------------------- integer structures
def test_index_prep_against_sets():
    cfg = small_cfg(n_tasks=3, rows_per_field=12, bag_max=5)
    model, params, sup, qry = oracle_inputs(cfg)
    ip = O.index_prep(model, sup, qry)
    F = cfg.n_fields
    base = model.field_base
    pos = 0
    rows_seen = {}
    cursor = 0
    for t in range(cfg.n_tasks):
        for f in range(F):
            want = set()
            for s in range(int(sup["task_offsets"][t]), int(sup["task_offsets"][t + 1])):
                for p in range(int(sup["bag_offsets"][s * F + f]), int(sup["bag_offsets"][s * F + f + 1])):
                    want.add(int(base[f]) + int(sup["indices"][p]))
            lst = sorted(want)
            n = int(ip["slot_counts"][t * F + f])
            assert n == len(lst)
            assert list(ip["slot_rows"][cursor:cursor + n]) == lst
            for s in range(int(sup["task_offsets"][t]), int(sup["task_offsets"][t + 1])):
                for p in range(int(sup["bag_offsets"][s * F + f]), int(sup["bag_offsets"][s * F + f + 1])):
                    assert lst[ip["sup_slot"][p]] == int(base[f]) + int(sup["indices"][p])
            for s in range(int(qry["task_offsets"][t]), int(qry["task_offsets"][t + 1])):
                for p in range(int(qry["bag_offsets"][s * F + f]), int(qry["bag_offsets"][s * F + f + 1])):
                    g = int(base[f]) + int(qry["indices"][p])
                    sl = int(ip["qry_slot"][p])
                    assert (sl == -1 and g not in want) or (sl >= 0 and lst[sl] == g)
            cursor += n
    for st in (sup, qry):
        n = int(st["task_offsets"][-1])
        for bagi in range(n * F):
            for p in range(int(st["bag_offsets"][bagi]), int(st["bag_offsets"][bagi + 1])):
                g = int(base[bagi % F]) + int(st["indices"][p])
                rows_seen[g] = rows_seen.get(g, 0) + 1
    assert list(ip["emb_rows"]) == sorted(rows_seen)
    assert list(ip["seg_counts"]) == [rows_seen[r] for r in sorted(rows_seen)]
    out = O.meta_step(model, params, sup, qry, 0.1, 1, 2)
    assert np.array_equal(out["emb_rows"], ip["emb_rows"])


# ---------------------------------------------------------------- bf16 operand rounding
def test_round_bf16_matches_library_conversion():
    import torch
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.normal(size=4000) * 10.0 ** rng.integers(-20, 20, size=4000),
                        np.array([0.0, -0.0, 1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 3.3895314e38])]).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(O.round_bf16(x), want)
    # ties go to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert O.round_bf16(np.float32(1.0 + 2.0 ** -8)) == 1.0
    assert O.round_bf16(np.float32(1.0 + 3 * 2.0 ** -8)) == 1.0 + 2.0 ** -6


def test_bf16_operands_with_representable_inputs_change_nothing_in_a_linear_model():
    """L = 1 has no rounded operand except x; with x exactly representable the two modes coincide."""
    rng = np.random.default_rng(2)
    d, n = 8, 12
    model = O.Model(rows_per_field=[], emb_dim=4, n_dense=d, layer_dims=[d, 1])
    params = dict(emb=np.zeros((0, 4)), W=[rng.normal(size=(d, 1))], b=[rng.normal(size=1)])

    def mkset():
        return dict(task_offsets=np.array([0, n]), bag_offsets=np.zeros(1, np.int64), indices=np.zeros(0, np.int32),
                    dense=O.round_bf16(rng.normal(size=(n, d))), labels=(rng.random(n) < 0.4).astype(np.float64))
    sup, qry = mkset(), mkset()
    a = O.meta_step(model, params, sup, qry, 0.3, 2, 2, operand="fp64")
    b = O.meta_step(model, params, sup, qry, 0.3, 2, 2, operand="bf16")
    assert a["loss"] == b["loss"] and np.array_equal(a["dW"][0], b["dW"][0])


def test_bf16_operands_stay_close_to_float64_where_no_mask_decides():
    """Loss (no yes/no decision downstream of it that could amplify) moves by rounding noise only."""
    cfg = small_cfg(inner_lr=0.1)
    model, params, sup, qry = oracle_inputs(cfg, emb_std=0.3)
    a = O.meta_step(model, params, sup, qry, 0.1, 2, 2, operand="fp64")
    b = O.meta_step(model, params, sup, qry, 0.1, 2, 2, operand="bf16")
    assert abs(a["loss"] - b["loss"]) / a["loss"] < 5e-3
    assert abs(a["loss"] - b["loss"]) > 0.0
    assert np.array_equal(a["emb_rows"], b["emb_rows"])


# ---------------------------------------------------------------- the outer update (Alg. 1, global back-propagation)
@pytest.mark.parametrize("K", [0, 2])
def test_train_step_descends_the_meta_objective_by_beta_times_the_squared_gradient(K):
    """phi' = phi - beta * g with g the exact (second-order) meta-gradient: for small beta the objective must fall by
    beta * |g|^2 to first order.  A wrong sign, a wrong scale, or an update landing on other rows than the gradient's
    breaks the ratio."""
    cfg = small_cfg(n_tasks=4, inner_lr=0.2)
    model, params, sup, qry = oracle_inputs(cfg, emb_std=0.3)
    alpha = cfg.inner_lr
    g = O.meta_step(model, params, sup, qry, alpha, K, 2)
    g2 = float((g["emb_grad"] ** 2).sum() + sum((w ** 2).sum() for w in g["dW"]) + sum((b ** 2).sum() for b in g["db"]))
    assert g2 > 0
    j0 = _objective(model, params, sup, qry, alpha, K)
    for beta in (1e-5, 1e-6):
        new, loss = O.meta_train_step(model, params, sup, qry, alpha, K, 2, beta)
        assert loss == g["loss"] == j0
        j1 = _objective(model, new, sup, qry, alpha, K)
        ratio = (j0 - j1) / (beta * g2)
        assert abs(ratio - 1.0) < 2e-3, (K, beta, ratio)


def test_train_step_touches_only_looked_up_rows_and_is_the_identity_for_beta_zero():
    cfg = small_cfg(n_tasks=3, rows_per_field=200)
    model, params, sup, qry = oracle_inputs(cfg, emb_std=0.3)
    new, _ = O.meta_train_step(model, params, sup, qry, cfg.inner_lr, 2, 2, 0.05)
    g = O.meta_step(model, params, sup, qry, cfg.inner_lr, 2, 2)
    touched = np.zeros(params["emb"].shape[0], dtype=bool)
    touched[g["emb_rows"]] = True
    assert np.array_equal(new["emb"][~touched], params["emb"][~touched].astype(np.float64))
    moved = np.abs(new["emb"] - params["emb"]).sum(axis=1) > 0
    assert moved[touched].mean() > 0.5 and not moved[~touched].any()
    same, _ = O.meta_train_step(model, params, sup, qry, cfg.inner_lr, 2, 2, 0.0)
    assert np.array_equal(same["emb"], params["emb"].astype(np.float64))
    for a, b in zip(same["W"] + same["b"], list(params["W"]) + list(params["b"])):
        assert np.array_equal(a, np.asarray(b, dtype=np.float64))


# ---------------------------------------------------------------- dense-only adaptation (embeddings read, not updated)
@pytest.mark.parametrize("K", [1, 2])
def test_dense_only_adaptation_by_central_differences(K):
    """adapt_rows=False, order 2: the exact gradient of its own objective, theta and xi parts (the xi part includes
    the path through the adapted theta)."""
    _fd_check(small_cfg(inner_lr=0.3), K=K, adapt_rows=False)


def test_dense_only_adaptation_differs_from_the_full_one_and_agrees_without_sparse_fields_or_steps():
    cfg = small_cfg(inner_lr=0.3)
    model, params, sup, qry = oracle_inputs(cfg, emb_std=0.3)
    full = O.meta_step(model, params, sup, qry, cfg.inner_lr, 2, 2)
    dense = O.meta_step(model, params, sup, qry, cfg.inner_lr, 2, 2, adapt_rows=False)
    assert abs(full["loss"] - dense["loss"]) > 1e-6 * abs(full["loss"])          # the rows' adaptation matters here
    assert np.array_equal(full["emb_rows"], dense["emb_rows"])
    a = O.meta_step(model, params, sup, qry, cfg.inner_lr, 0, 2)
    b = O.meta_step(model, params, sup, qry, cfg.inner_lr, 0, 2, adapt_rows=False)
    assert a["loss"] == b["loss"] and np.array_equal(a["emb_grad"], b["emb_grad"])   # K = 0: nothing is adapted
    # first order: support-only rows get exactly nothing either way, but the query side sees unadapted rows
    d1 = O.meta_step(model, params, sup, qry, cfg.inner_lr, 2, 1, adapt_rows=False)
    assert abs(d1["loss"] - dense["loss"]) == 0.0


# ---------------------------------------------------------------- ReLU gates given from outside (relu_masks)
def _flipped_gates(model, params, sup, qry, alpha, K, share, seed):
    """The gates of a plain run with a share of them flipped at random: gates that no forward pass would choose."""
    rec = {}
    O.meta_step(model, params, sup, qry, alpha, K, 1, masks_out=rec)
    rng = np.random.default_rng(seed)
    return {t: [[np.logical_xor(m, rng.random(m.shape) < share) for m in one_pass] for one_pass in passes]
            for t, passes in rec.items()}


def test_recorded_gates_given_back_reproduce_the_plain_run():
    cfg = small_cfg(inner_lr=0.3)
    model, params, sup, qry = oracle_inputs(cfg, emb_std=0.3)
    rec = {}
    a = O.meta_step(model, params, sup, qry, cfg.inner_lr, 2, 2, masks_out=rec)
    assert sorted(rec) == [0, 1, 2] and all(len(p) == 3 and len(p[0]) == model.n_layers - 1 for p in rec.values())
    b = O.meta_step(model, params, sup, qry, cfg.inner_lr, 2, 2, relu_masks=rec)
    assert a["loss"] == b["loss"] and np.array_equal(a["emb_grad"], b["emb_grad"])
    assert all(np.array_equal(x, y) for x, y in zip(a["dW"] + a["db"], b["dW"] + b["db"]))


@pytest.mark.parametrize("K", [1, 2])
def test_frozen_gate_meta_gradient_by_central_differences(K):
    """With the gates given (here: a plain run's gates with 15 % flipped, so that they really come from outside),
    the step must be the exact gradient of the frozen-gate objective: a_l = z_l * m_l is smooth in the parameters, so
    central differences of that objective pin every place where the backward and tangent passes apply a gate."""
    cfg = small_cfg(inner_lr=0.3)
    model, params, sup, qry = oracle_inputs(cfg, emb_std=0.3)
    params = {k: ([a.astype(np.float64) for a in v] if isinstance(v, list) else v.astype(np.float64))
              for k, v in params.items()}
    alpha = cfg.inner_lr
    gates = _flipped_gates(model, params, sup, qry, alpha, K, 0.15, 5)
    out = O.meta_step(model, params, sup, qry, alpha, K, 2, relu_masks=gates)
    plain = O.meta_step(model, params, sup, qry, alpha, K, 2)
    assert max(rel_err(out["dW"][0], plain["dW"][0])) > 0.05, "the flipped gates must matter"
    gfull = _full_grad(model, out)
    rng = np.random.default_rng(2)
    checks = []
    for l in range(model.n_layers):
        for _ in range(10):
            i = tuple(rng.integers(0, s) for s in params["W"][l].shape)
            checks.append((params["W"][l], i, out["dW"][l][i]))
        j = (int(rng.integers(0, params["b"][l].shape[0])),)
        checks.append((params["b"][l], j, out["db"][l][j]))
    for r in rng.choice(out["emb_rows"], size=25, replace=False):
        c = int(rng.integers(0, model.emb_dim))
        checks.append((params["emb"], (int(r), c), gfull[int(r), c]))
    scale = max(np.abs(gfull).max(), max(np.abs(g).max() for g in out["dW"]))
    eps, worst = 1e-5, 0.0
    for arr, i, g in checks:
        old = arr[i]
        arr[i] = old + eps
        fp = O.meta_step(model, params, sup, qry, alpha, K, 1, relu_masks=gates)["loss"]
        arr[i] = old - eps
        fm = O.meta_step(model, params, sup, qry, alpha, K, 1, relu_masks=gates)["loss"]
        arr[i] = old
        worst = max(worst, abs((fp - fm) / (2 * eps) - g) / scale)
    assert worst < 2e-6, worst


def test_bf16_gates_with_float64_arithmetic_sit_between_the_two_modes():
    """relu_masks="bf16": float64 arithmetic on the gates of the bf16-operand run.  On configs[1]'s model shape with
    small ragged tasks: against the bf16-operand mode only rounding is left (well inside the bf16 tolerance of 2e-2 on
    every output), while against the plain float64 run whole gradient terms differ (gates that fall differently) --
    which is why a reduced-precision path is held against THIS reference and not against the plain one."""
    from synth import SMALL, make_batch, make_params
    cfg = SMALL.with_(n_tasks=6, n_support=50, n_query=37, mlp_dtype=1, rows_per_field=5000, inner_lr=0.05)
    sup, qry = make_batch(cfg, 0, "cpu")
    params, model = make_params(cfg, "cpu").numpy(), oracle_model(cfg)
    sup, qry = sup.numpy(), qry.numpy()
    rounded = O.meta_step(model, params, sup, qry, cfg.inner_lr, 2, 2, operand="bf16")
    gated = O.meta_step(model, params, sup, qry, cfg.inner_lr, 2, 2, relu_masks="bf16")
    plain = O.meta_step(model, params, sup, qry, cfg.inner_lr, 2, 2)

    def dist(a, b):
        e = [abs(a["loss"] - b["loss"]) / abs(b["loss"]), max(rel_err(a["emb_grad"], b["emb_grad"]))]
        e += [max(rel_err(x, y)) for x, y in zip(a["dW"] + a["db"], b["dW"] + b["db"])]
        return max(e)
    assert dist(rounded, gated) < 1e-2, dist(rounded, gated)
    assert dist(gated, plain) > 2e-2, dist(gated, plain)
    assert abs(gated["loss"] - plain["loss"]) / plain["loss"] < 1e-4     # the loss itself hardly feels a gate near zero
