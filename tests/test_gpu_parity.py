"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by element.

Bar: integers (slots, row lists, segment sizes) bit-exact; fp32 path 1e-4 relative
(L2 and max-abs relative to the reference's max-abs) on losses and gradients.
"""
import numpy as np
import pytest
import torch

from oracle import maml_dlrm as O
from synth import SMALL, TINY, make_batch, make_params
from tests.helpers import compact_task, oracle_model, rel_err, small_cfg

pytestmark = pytest.mark.gpu

TOL_FP32 = 1e-4


@pytest.fixture(scope="module")
def gm():
    from paper_2401_04338_amd import GMeta
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return GMeta


def _to_dev(sd, dev):
    from synth.generate import SetData
    return SetData(sd.task_offsets, sd.bag_offsets.to(dev), sd.indices.to(dev), sd.dense.to(dev), sd.labels.to(dev))


def _inputs(cfg, emb_std=0.05, tasks=None):
    sup, qry = make_batch(cfg, 0, "cpu", tasks)
    params = make_params(cfg, "cpu", emb_std=emb_std)
    return sup, qry, params


def _params_dev(params, dev):
    from synth.generate import Params
    return Params(params.emb.to(dev), [w.to(dev) for w in params.W], [b.to(dev) for b in params.b])


def _errors(out, ref, n, T):
    """Per-output distance (c13: the larger of relative L2 and max-abs over the reference's max-abs) of a step's
    results from an oracle result."""
    errs = {"loss": abs(float(out["loss"].item()) - ref["loss"]) / abs(ref["loss"]),
            "task_loss": max(rel_err(out["task_loss"][:T].cpu().numpy(), ref["task_loss"]))}
    for l in range(len(ref["dW"])):
        errs[f"dW{l}"] = max(rel_err(out["dW"][l].cpu().numpy(), ref["dW"][l]))
        errs[f"db{l}"] = max(rel_err(out["db"][l].cpu().numpy(), ref["db"][l]))
    errs["emb_grad"] = max(rel_err(out["emb_grad"][:n].cpu().numpy(), ref["emb_grad"]))
    return errs


UNDECIDED = 1e-3   # a ReLU gate whose pre-activation is within this fraction of its layer's rms of zero


def _undecided_gates(pre, out, gated, limit=24):
    """Gates of the oracle's bf16-operand run that rounding can turn either way: (task, pass, layer, sample, unit) with
    |z| <= UNDECIDED * rms(z of that layer and pass).  One bf16 operand rounded the other way (a pooled sum or an
    adapted weight computed in fp32 instead of float64 before it is rounded) moves a pre-activation by |w x| 2^-8:
    about 1e-4 of that scale for a typical term of these layers, several times that for a large one; the fp32
    accumulation of a product moves it by far less.  A gate of hidden layer l + 1, unit u, taken the other way changes
    column u of dW[l] and the layers below it, so the candidates are the gates in columns that hold at least half of the
    largest column's share of the kernels' distance from the reference, deepest layer first, nearest to zero first."""
    share = []
    for l in range(len(gated["dW"]) - 1):
        d = np.linalg.norm(out["dW"][l].cpu().numpy().astype(np.float64) - gated["dW"][l], axis=0)
        share.append(d / max(float(d.max()), 1e-300))
    found = []
    for t, passes in pre.items():
        for i, layers in enumerate(passes):
            for l, z in enumerate(layers):
                rms = float(np.sqrt(np.mean(z * z))) if z.size else 0.0
                if rms == 0.0:
                    continue
                ss, uu = np.nonzero(np.abs(z) <= UNDECIDED * rms)
                found += [(-l, abs(float(z[s_, u_])) / rms, t, i, l, int(s_), int(u_)) for s_, u_ in zip(ss, uu)
                          if share[l][u_] >= 0.5]
    return [c[1:] for c in sorted(found)[:limit]]


def _flipped(rec, t, i, l, s_, u_):
    out = {tt: [[m.copy() for m in layers] for layers in passes] for tt, passes in rec.items()}
    out[t][i][l][s_, u_] = not out[t][i][l][s_, u_]
    return out


def _compare_step(cfg, ctx, sup, qry, params, K, order, tol, label, operand="fp64", model=None, adapt_rows=True):
    """fp32 path: every output against the float64 oracle at `tol`.

    bf16 path (operand="bf16"): THE reference is the oracle in float64 arithmetic on the ReLU gates of its bf16-operand
    run (relu_masks="bf16"): only the yes/no decisions are taken on rounded operands, as any path that stores bf16
    activations takes them, and every rounding of the kernels has to fit inside `tol` by itself.  Every output is
    asserted against it element by element.  The oracle's own bf16-operand mode (same rounding schedule as the
    kernels) is kept as a second, tighter look at the same outputs, and the plain float64 oracle bounds what is left:
    the loss at `tol`, and the first layer's gradient within `tol` of the distance the gates themselves account for.

    A gate decided on a pre-activation within rounding distance of zero has no unique value (_undecided_gates): when
    the comparison fails with the oracle's own decisions, such gates are taken the other way one at a time (at most
    four in all) where that explains the kernels' result; every output must then meet `tol`.  Which gates, and how
    near zero they sit, is printed."""
    dev = ctx.device
    model = model or oracle_model(cfg)
    p_np, s_np, q_np = params.numpy(), sup.numpy(), qry.numpy()
    out = ctx.meta_step(_to_dev(sup, dev), _to_dev(qry, dev), _params_dev(params, dev), cfg.inner_lr, K, order)
    rec = {} if operand != "fp64" else None
    pre = {} if operand != "fp64" else None
    ref = O.meta_step(model, p_np, s_np, q_np, cfg.inner_lr, K, order, operand=operand, adapt_rows=adapt_rows, masks_out=rec,
                      pre_out=pre)
    n = int(out["n_emb_rows"].item())
    assert n == len(ref["emb_rows"]), label
    assert np.array_equal(out["emb_rows"][:n].cpu().numpy(), ref["emb_rows"]), label
    T = len(sup.task_offsets) - 1
    if operand != "fp64":
        gated = O.meta_step(model, p_np, s_np, q_np, cfg.inner_lr, K, order, relu_masks=rec, adapt_rows=adapt_rows)
        eg = _errors(out, gated, n, T)
        for _ in range(4):   # (each round settles one gate: the one that brings the kernels' result nearest)
            if max(eg.values()) <= tol:
                break
            best = None
            for margin, t, i, l, s_, u_ in _undecided_gates(pre, out, gated):
                rec2 = _flipped(rec, t, i, l, s_, u_)
                gated2 = O.meta_step(model, p_np, s_np, q_np, cfg.inner_lr, K, order, relu_masks=rec2, adapt_rows=adapt_rows)
                eg2 = _errors(out, gated2, n, T)
                if best is None or max(eg2.values()) < max(best[2].values()):
                    best = (rec2, gated2, eg2, (margin, t, i, l, s_, u_))
            if best is None or max(best[2].values()) > 0.9 * max(eg.values()):
                break
            margin, t, i, l, s_, u_ = best[3]
            print(label, f"undecided gate: task {t}, pass {i}, hidden layer {l + 1}, sample {s_}, unit {u_}: "
                  f"|z| = {margin:.1e} of the layer's rms; taken the kernels' way "
                  f"(largest distance {max(eg.values()):.2e} -> {max(best[2].values()):.2e})", flush=True)
            rec, gated, eg = best[:3]
            ref = O.meta_step(model, p_np, s_np, q_np, cfg.inner_lr, K, order, operand=operand, adapt_rows=adapt_rows, relu_masks=rec)
        print(label, "vs float64 arithmetic on bf16 gates:", {k: f"{v:.2e}" for k, v in eg.items()}, flush=True)
        for k, v in eg.items():
            assert v <= tol, (label, "float64 arithmetic on bf16 gates", k, v)
        ref64 = O.meta_step(model, p_np, s_np, q_np, cfg.inner_lr, K, order, adapt_rows=adapt_rows)
        e64 = abs(float(out["loss"].item()) - ref64["loss"]) / abs(ref64["loss"])
        g64 = max(rel_err(out["dW"][0].cpu().numpy(), ref64["dW"][0]))
        gates = max(rel_err(gated["dW"][0], ref64["dW"][0]))
        print(label, f"vs plain float64: loss {e64:.2e}, dW0 {g64:.2e}, of which the gates account for {gates:.2e}", flush=True)
        assert e64 <= tol, (label, "loss vs float64", e64)
        assert g64 <= gates + tol, (label, "dW0 vs float64 beyond what the gates account for", g64, gates)
    errs = _errors(out, ref, n, T)
    print(label, {k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    for k, v in errs.items():
        assert v <= tol, (label, k, v)
    return out, ref


# ---------------------------------------------------------------- a0: integer structures
@pytest.mark.parametrize("cfg", [small_cfg(n_tasks=5, rows_per_field=12, bag_max=5),
                                 TINY, SMALL.with_(n_tasks=6)], ids=["mini", "tiny", "small6"])
def test_index_prep_bit_exact(gm, cfg):
    print("index_prep", cfg.name, flush=True)
    sup, qry, _ = _inputs(cfg)
    ctx = gm.from_config(cfg, workspace_bytes=1 << 30)
    got = ctx.index_prep(_to_dev(sup, ctx.device), _to_dev(qry, ctx.device))
    ref = O.index_prep(oracle_model(cfg), sup.numpy(), qry.numpy())
    for k in ("slot_counts", "slot_rows", "sup_slot", "qry_slot", "emb_rows", "seg_counts"):
        assert np.array_equal(got[k].cpu().numpy(), ref[k]), k
    ctx.close()


# ---------------------------------------------------------------- a1: gather + sum-pool
@pytest.mark.parametrize("cfg", [small_cfg(n_tasks=5), TINY, SMALL.with_(n_tasks=6)], ids=["mini", "tiny", "small6"])
def test_gather_pool(gm, cfg):
    print("gather_pool", cfg.name, flush=True)
    sup, qry, params = _inputs(cfg)
    ctx = gm.from_config(cfg, workspace_bytes=1 << 28)
    x = ctx.gather_pool(_to_dev(sup, ctx.device), params.emb.to(ctx.device)).cpu().numpy()
    ref = O.gather_pool(oracle_model(cfg), params.emb.numpy(), sup.numpy())
    assert x.shape == ref.shape
    # bag size 1 (Tiny): a pure gather, exact
    if cfg.bag_max == 1:
        assert np.array_equal(x, ref.astype(np.float32))
    assert max(rel_err(x, ref)) <= 1e-6
    ctx.close()


# ---------------------------------------------------------------- the whole step
@pytest.mark.parametrize("K,order", [(0, 1), (1, 1), (1, 2), (2, 1), (2, 2), (3, 2)])
def test_meta_step_mini(gm, K, order):
    cfg = small_cfg(n_tasks=5, inner_lr=0.3)
    sup, qry, params = _inputs(cfg, emb_std=0.3)
    ctx = gm.from_config(cfg, workspace_bytes=1 << 28)
    _compare_step(cfg, ctx, sup, qry, params, K, order, TOL_FP32, f"mini K={K} order={order}")
    ctx.close()


@pytest.mark.parametrize("order", [1, 2])
def test_meta_step_tiny_config(gm, order):
    """configs[0] at full size."""
    cfg = TINY
    sup, qry, params = _inputs(cfg)
    ctx = gm.from_config(cfg, workspace_bytes=1 << 28)
    _compare_step(cfg, ctx, sup, qry, params, cfg.inner_steps, order, TOL_FP32, f"tiny order={order}")
    ctx.close()


def test_meta_step_small_config_subset(gm):
    """configs[1] shape (26 fields x 100k rows x 32, multi-hot Zipf bags, MLP 845-256-128-1), 8 tasks."""
    cfg = SMALL.with_(n_tasks=8)
    sup, qry, params = _inputs(cfg)
    ctx = gm.from_config(cfg, workspace_bytes=2 << 30)
    _compare_step(cfg, ctx, sup, qry, params, 1, 2, TOL_FP32, "small8 K=1 order=2")
    _compare_step(cfg, ctx, sup, qry, params, 2, 2, TOL_FP32, "small8 K=2 order=2")
    ctx.close()


def test_waves_give_the_same_result(gm):
    """A workspace too small for one wave splits the tasks; results agree with the single-wave run."""
    cfg = SMALL.with_(n_tasks=8)
    sup, qry, params = _inputs(cfg)
    big = gm.from_config(cfg, workspace_bytes=2 << 30)
    need = big.workspace_bytes(8, sup.n_samples, qry.n_samples, sup.nnz, qry.nnz, 2, 2)
    small = gm.from_config(cfg, workspace_bytes=int(need * 0.45))
    dev = big.device
    a = big.meta_step(_to_dev(sup, dev), _to_dev(qry, dev), _params_dev(params, dev), 0.01, 2, 2)
    b = small.meta_step(_to_dev(sup, dev), _to_dev(qry, dev), _params_dev(params, dev), 0.01, 2, 2)
    n = int(a["n_emb_rows"].item())
    assert n == int(b["n_emb_rows"].item())
    assert torch.equal(a["emb_rows"][:n], b["emb_rows"][:n])
    assert torch.equal(a["task_loss"], b["task_loss"])
    assert max(rel_err(b["emb_grad"][:n].cpu().numpy(), a["emb_grad"][:n].cpu().numpy())) < 1e-6
    for l in range(3):
        assert max(rel_err(b["dW"][l].cpu().numpy(), a["dW"][l].cpu().numpy())) < 1e-5
    big.close()
    small.close()


@pytest.mark.parametrize("waves", [1, 3], ids=["one_wave", "several_waves"])
def test_table_shaped_sparse_gradient(gm, waves):
    """emb_grad_table: the sparse meta-gradient is added into a caller-owned table, wave by wave.  Held against the
    oracle's row list scattered into a table; with one wave it is bit for bit the listed gradient."""
    cfg = SMALL.with_(n_tasks=8)
    sup, qry, params = _inputs(cfg)
    big = gm.from_config(cfg, workspace_bytes=2 << 30)
    dev = big.device
    ctx = big
    if waves > 1:
        need = big.workspace_bytes(8, sup.n_samples, qry.n_samples, sup.nnz, qry.nnz, 2, 2)
        ctx = gm.from_config(cfg, workspace_bytes=int(need * 0.3))
    ds, dq, dp = _to_dev(sup, dev), _to_dev(qry, dev), _params_dev(params, dev)
    listed = big.meta_step(ds, dq, dp, cfg.inner_lr, 2, 2)
    n = int(listed["n_emb_rows"].item())
    table = torch.zeros_like(dp.emb)
    out = ctx.meta_step(ds, dq, dp, cfg.inner_lr, 2, 2, emb_grad_table=table)
    assert int(out["n_emb_rows"].item()) == 0
    assert torch.equal(out["task_loss"], listed["task_loss"])
    want = torch.zeros_like(table)
    want[listed["emb_rows"][:n]] = listed["emb_grad"][:n]
    if waves == 1:
        assert torch.equal(table, want)
        assert torch.equal(out["dW"][0], listed["dW"][0])
    ref = O.meta_step(oracle_model(cfg), params.numpy(), sup.numpy(), qry.numpy(), cfg.inner_lr, 2, 2)
    got = table.cpu().numpy()
    assert np.all(np.isin(np.flatnonzero(np.abs(got).sum(1) > 0), ref["emb_rows"]))   # no other row is written
    e = max(rel_err(got[ref["emb_rows"]], ref["emb_grad"]))
    print("table mode", waves, f"emb_grad {e:.2e}", flush=True)
    assert e <= TOL_FP32
    # a second call keeps accumulating
    ctx.meta_step(ds, dq, dp, cfg.inner_lr, 2, 2, emb_grad_table=table)
    assert max(rel_err(table.cpu().numpy()[ref["emb_rows"]], 2.0 * ref["emb_grad"])) <= TOL_FP32
    if ctx is not big:
        ctx.close()
    big.close()


def test_determinism(gm):
    cfg = SMALL.with_(n_tasks=4)
    sup, qry, params = _inputs(cfg)
    ctx = gm.from_config(cfg, workspace_bytes=1 << 30)
    dev = ctx.device
    a = ctx.meta_step(_to_dev(sup, dev), _to_dev(qry, dev), _params_dev(params, dev), 0.01, 1, 2)
    b = ctx.meta_step(_to_dev(sup, dev), _to_dev(qry, dev), _params_dev(params, dev), 0.01, 1, 2)
    n = int(a["n_emb_rows"].item())
    assert torch.equal(a["emb_grad"][:n], b["emb_grad"][:n])
    assert torch.equal(a["loss"], b["loss"])
    for l in range(3):
        assert torch.equal(a["dW"][l], b["dW"][l])
    ctx.close()


# ---------------------------------------------------------------- edge cases and error paths
def _drop_task_samples(cfg, sd, t):
    """The set without the samples of task t (the task stays, empty)."""
    from synth.generate import SetData
    F = cfg.n_fields
    lo, hi = int(sd.task_offsets[t]), int(sd.task_offsets[t + 1])
    p0, p1 = int(sd.bag_offsets[lo * F]), int(sd.bag_offsets[hi * F])
    offs = torch.cat([sd.bag_offsets[: lo * F], sd.bag_offsets[hi * F:] - (p1 - p0)])
    toff = sd.task_offsets.copy()
    toff[t + 1:] -= hi - lo
    keep = torch.ones(sd.n_samples, dtype=torch.bool)
    keep[lo:hi] = False
    return SetData(toff, offs, torch.cat([sd.indices[:p0], sd.indices[p1:]]), sd.dense[keep], sd.labels[keep])


def test_ragged_and_empty_tasks(gm):
    """Variable task sizes including a task with no support samples and empty bags."""
    cfg = small_cfg(n_tasks=4, inner_lr=0.2)
    sup, qry, params = _inputs(cfg, emb_std=0.3)

    sup2 = _drop_task_samples(cfg, sup, 1)
    ctx = gm.from_config(cfg, workspace_bytes=1 << 28)
    _compare_step(cfg, ctx, sup2, qry, params, 2, 2, TOL_FP32, "empty-support-task")
    ctx.close()


def test_degenerate_batches_in_both_output_shapes(gm):
    """No tasks at all, and a batch whose bags are all empty (no lookup anywhere): both run, touch no table row and
    list no row; the dense part of the all-empty-bags batch still matches the oracle."""
    from synth.generate import SetData
    cfg = small_cfg(n_tasks=3)
    sup, qry, params = _inputs(cfg)
    ctx = gm.from_config(cfg, workspace_bytes=1 << 28)
    dev = ctx.device
    dp = _params_dev(params, dev)

    def no_lookups(sd):
        return SetData(sd.task_offsets, torch.zeros_like(sd.bag_offsets), sd.indices[:0], sd.dense, sd.labels)

    def no_tasks(sd):
        return SetData(np.zeros(1, dtype=np.int64), sd.bag_offsets[:1] * 0, sd.indices[:0], sd.dense[:0], sd.labels[:0])

    table = torch.zeros_like(dp.emb)
    for label, s2, q2 in (("no tasks", no_tasks(sup), no_tasks(qry)), ("empty bags", no_lookups(sup), no_lookups(qry))):
        out = ctx.meta_step(_to_dev(s2, dev), _to_dev(q2, dev), dp, cfg.inner_lr, 2, 2)
        assert int(out["n_emb_rows"].item()) == 0, label
        ctx.meta_step(_to_dev(s2, dev), _to_dev(q2, dev), dp, cfg.inner_lr, 2, 2, emb_grad_table=table)
        assert not table.any(), label
        if label == "no tasks":
            assert float(out["loss"].item()) == 0.0 and not out["dW"][0].any()
        else:
            ref = O.meta_step(oracle_model(cfg), params.numpy(), s2.numpy(), q2.numpy(), cfg.inner_lr, 2, 2)
            assert len(ref["emb_rows"]) == 0
            assert abs(float(out["loss"].item()) - ref["loss"]) <= TOL_FP32 * abs(ref["loss"])
            for l in range(len(ref["dW"])):
                assert max(rel_err(out["dW"][l].cpu().numpy(), ref["dW"][l])) <= TOL_FP32, (label, l)
    ctx.close()


def test_error_paths(gm):
    from paper_2401_04338_amd import GMetaError
    cfg = small_cfg(n_tasks=3)
    sup, qry, params = _inputs(cfg)
    ctx = gm.from_config(cfg, workspace_bytes=1 << 28)
    dev = ctx.device
    p = _params_dev(params, dev)
    bad = _to_dev(sup, dev)
    bad.indices = bad.indices.clone()
    bad.indices[3] = cfg.rows_per_field        # out of range
    with pytest.raises(GMetaError) as e:
        ctx.meta_step(bad, _to_dev(qry, dev), p, 0.1, 1, 2)
    assert e.value.code == -2
    bad2 = _to_dev(sup, dev)
    bad2.bag_offsets = bad2.bag_offsets.clone()
    bad2.bag_offsets[5] = bad2.bag_offsets[6] + 1   # not monotone
    with pytest.raises(GMetaError) as e:
        ctx.meta_step(bad2, _to_dev(qry, dev), p, 0.1, 1, 2)
    assert e.value.code == -2
    with pytest.raises(GMetaError) as e:
        ctx.meta_step(_to_dev(sup, dev), _to_dev(qry, dev), p, 0.1, 1, 2, emb_rows_capacity=3)
    assert e.value.code == -3
    with pytest.raises(GMetaError) as e:
        ctx.meta_step(_to_dev(sup, dev), _to_dev(qry, dev), p, 0.1, 1, 3)
    assert e.value.code == -1
    # a well-formed input beyond a size limit is a capacity error, not an index error: one bag of 70,000 lookups
    from synth.generate import SetData
    big = _to_dev(sup, dev)
    extra = 70000
    offs = big.bag_offsets.clone()
    offs[1:] += extra
    big = SetData(big.task_offsets, offs, torch.cat([torch.zeros(extra, dtype=torch.int32, device=dev), big.indices]),
                  big.dense, big.labels)
    with pytest.raises(GMetaError) as e:
        ctx.meta_step(big, _to_dev(qry, dev), p, 0.1, 1, 2)
    assert e.value.code == -3 and "65535" in str(e.value)
    # tensors of another type or layout are refused by the binding before the library would misread them
    wrong = _to_dev(sup, dev)
    wrong.indices = wrong.indices.long()
    with pytest.raises(ValueError):
        ctx.meta_step(wrong, _to_dev(qry, dev), p, 0.1, 1, 2)
    from synth.generate import Params
    with pytest.raises(ValueError):
        ctx.meta_step(_to_dev(sup, dev), _to_dev(qry, dev), Params(p.emb.t().contiguous().t(), p.W, p.b), 0.1, 1, 2)
    # the context still works after errors
    _compare_step(cfg, ctx, sup, qry, params, 1, 2, TOL_FP32, "after-errors")
    ctx.close()


@pytest.mark.parametrize("bf", [0, 1], ids=["fp32", "bf16"])
def test_train_steps_follow_the_oracle(gm, bf):
    """gm_meta_train_step: three iterations of Alg. 1 (a fresh batch each), parameters updated in place; losses and
    parameters after every iteration against the oracle's meta_train_step run on its own copy."""
    from synth.generate import Params
    cfg = SMALL.with_(n_tasks=4, n_support=40, n_query=24, n_fields=5, emb_dim=32, rows_per_field=3000, bag_max=6,
                      layer_dims=(5 * 32 + 13, 64, 32, 1), inner_lr=0.05, mlp_dtype=bf)
    beta, K, order = 0.02, 2, 2
    tol = TOL_BF16 if bf else TOL_FP32
    params = make_params(cfg, "cpu", emb_std=0.1)
    ctx = gm.from_config(cfg, workspace_bytes=1 << 30)
    dev = ctx.device
    dp = Params(params.emb.to(dev).clone(), [w.to(dev).clone() for w in params.W], [b.to(dev).clone() for b in params.b])
    ref_p = params.numpy()
    ref_p = dict(emb=ref_p["emb"].astype(np.float64), W=[w.astype(np.float64) for w in ref_p["W"]],
                 b=[b.astype(np.float64) for b in ref_p["b"]])
    for it in range(3):
        sup, qry = make_batch(cfg, it, "cpu")
        loss = ctx.meta_train_step(_to_dev(sup, dev), _to_dev(qry, dev), dp, cfg.inner_lr, K, order, beta)
        ref_p, ref_loss = O.meta_train_step(oracle_model(cfg), ref_p, sup.numpy(), qry.numpy(), cfg.inner_lr, K, order, beta,
                                            operand="bf16" if bf else "fp64")
        e = {"loss": abs(float(loss.item()) - ref_loss) / abs(ref_loss),
             "emb": max(rel_err(dp.emb.cpu().numpy(), ref_p["emb"]))}
        for l in range(len(ref_p["W"])):
            e[f"W{l}"] = max(rel_err(dp.W[l].cpu().numpy(), ref_p["W"][l]))
            e[f"b{l}"] = max(rel_err(dp.b[l].cpu().numpy(), ref_p["b"][l]))
        # what moved, against what the oracle moved (parameters are dominated by their initial values)
        d_emb = max(rel_err(dp.emb.cpu().numpy().astype(np.float64) - params.emb.numpy(), ref_p["emb"] - params.emb.numpy()))
        d_w0 = max(rel_err(dp.W[0].cpu().numpy().astype(np.float64) - params.W[0].numpy(), ref_p["W"][0] - params.W[0].numpy()))
        print(f"train it {it} bf16={bf}", {k: f"{v:.1e}" for k, v in e.items()}, f"moved: emb {d_emb:.1e} W0 {d_w0:.1e}", flush=True)
        assert all(v <= tol for v in e.values()), (it, e)
        assert d_emb <= 5 * tol and d_w0 <= 5 * tol, (it, d_emb, d_w0)
    ctx.close()


@pytest.mark.parametrize("waves", [1, 3], ids=["one_wave", "several_waves"])
def test_train_steps_with_a_table_shaped_gradient(gm, waves):
    """gm_meta_train_step_table: three iterations of Alg. 1 with the sparse meta-gradient accumulated in a table-shaped
    buffer (all zero before and after every call) and applied in one pass: losses and parameters after every iteration
    against the oracle's meta_train_step, tasks in one wave and in several."""
    from synth.generate import Params
    cfg = SMALL.with_(n_tasks=6, n_support=40, n_query=24, n_fields=5, emb_dim=32, rows_per_field=3000, bag_max=6,
                      layer_dims=(5 * 32 + 13, 64, 32, 1), inner_lr=0.05)
    beta, K, order = 0.02, 2, 2
    params = make_params(cfg, "cpu", emb_std=0.1)
    sup0, qry0 = make_batch(cfg, 0, "cpu")
    probe = gm.from_config(cfg, workspace_bytes=1 << 30)
    need = probe.workspace_bytes(cfg.n_tasks, sup0.n_samples, qry0.n_samples, sup0.nnz, qry0.nnz, K, order)
    probe.close()
    ctx = gm.from_config(cfg, workspace_bytes=(1 << 30) if waves == 1 else int(need * 0.45))
    dev = ctx.device
    dp = Params(params.emb.to(dev).clone(), [w.to(dev).clone() for w in params.W], [b.to(dev).clone() for b in params.b])
    table = torch.zeros_like(dp.emb)
    ref_p = params.numpy()
    ref_p = dict(emb=ref_p["emb"].astype(np.float64), W=[w.astype(np.float64) for w in ref_p["W"]],
                 b=[b.astype(np.float64) for b in ref_p["b"]])
    for it in range(3):
        sup, qry = make_batch(cfg, it, "cpu")
        loss = ctx.meta_train_step_table(_to_dev(sup, dev), _to_dev(qry, dev), dp, cfg.inner_lr, K, order, beta, table)
        assert float(table.abs().max()) == 0.0, "the accumulator is cleared by the update"
        ref_p, ref_loss = O.meta_train_step(oracle_model(cfg), ref_p, sup.numpy(), qry.numpy(), cfg.inner_lr, K, order, beta)
        e = {"loss": abs(float(loss.item()) - ref_loss) / abs(ref_loss),
             "emb": max(rel_err(dp.emb.cpu().numpy(), ref_p["emb"]))}
        for l in range(len(ref_p["W"])):
            e[f"W{l}"] = max(rel_err(dp.W[l].cpu().numpy(), ref_p["W"][l]))
            e[f"b{l}"] = max(rel_err(dp.b[l].cpu().numpy(), ref_p["b"][l]))
        d_emb = max(rel_err(dp.emb.cpu().numpy().astype(np.float64) - params.emb.numpy(), ref_p["emb"] - params.emb.numpy()))
        print(f"table train it {it} waves={waves}", {k: f"{v:.1e}" for k, v in e.items()}, f"moved: emb {d_emb:.1e}", flush=True)
        assert all(v <= TOL_FP32 for v in e.values()), (it, e)
        assert d_emb <= 5 * TOL_FP32, (it, d_emb)
    ctx.close()


@pytest.mark.parametrize("bf,K,order", [(0, 1, 2), (0, 2, 2), (0, 3, 1), (1, 2, 2)])
def test_dense_only_adaptation(gm, bf, K, order):
    """gm_configure("adapt_rows", 0): the inner loop adapts theta only; every output against the oracle's
    adapt_rows=False, and the fused training iteration in that mode."""
    from synth.generate import Params
    cfg = SMALL.with_(n_tasks=5, n_support=40, n_query=24, n_fields=5, emb_dim=32, rows_per_field=2000, bag_max=6,
                      layer_dims=(5 * 32 + 13, 64, 32, 1), inner_lr=0.05, mlp_dtype=bf)
    tol = TOL_BF16 if bf else TOL_FP32
    sup, qry, params = _inputs(cfg, emb_std=0.2)
    ctx = gm.from_config(cfg, workspace_bytes=1 << 30)
    ctx.configure("adapt_rows", 0)
    dev = ctx.device
    out = ctx.meta_step(_to_dev(sup, dev), _to_dev(qry, dev), _params_dev(params, dev), cfg.inner_lr, K, order)
    ref = O.meta_step(oracle_model(cfg), params.numpy(), sup.numpy(), qry.numpy(), cfg.inner_lr, K, order,
                      operand="bf16" if bf else "fp64", adapt_rows=False)
    full = O.meta_step(oracle_model(cfg), params.numpy(), sup.numpy(), qry.numpy(), cfg.inner_lr, K, order)
    assert abs(full["loss"] - ref["loss"]) > 1e-7 * abs(ref["loss"]), "the case must tell the two variants apart"
    n = int(out["n_emb_rows"].item())
    assert np.array_equal(out["emb_rows"][:n].cpu().numpy(), ref["emb_rows"])
    e = {"loss": abs(float(out["loss"].item()) - ref["loss"]) / abs(ref["loss"]),
         "emb_grad": max(rel_err(out["emb_grad"][:n].cpu().numpy(), ref["emb_grad"]))}
    for l in range(len(ref["dW"])):
        e[f"dW{l}"] = max(rel_err(out["dW"][l].cpu().numpy(), ref["dW"][l]))
        e[f"db{l}"] = max(rel_err(out["db"][l].cpu().numpy(), ref["db"][l]))
    print(f"dense-only bf16={bf} K={K} order={order}", {k: f"{v:.1e}" for k, v in e.items()}, flush=True)
    assert all(v <= tol for v in e.values()), e
    # one training iteration in this mode
    dp = Params(params.emb.to(dev).clone(), [w.to(dev).clone() for w in params.W], [b.to(dev).clone() for b in params.b])
    ctx.meta_train_step(_to_dev(sup, dev), _to_dev(qry, dev), dp, cfg.inner_lr, K, order, 0.02)
    new, _ = O.meta_train_step(oracle_model(cfg), params.numpy(), sup.numpy(), qry.numpy(), cfg.inner_lr, K, order, 0.02,
                               operand="bf16" if bf else "fp64", adapt_rows=False)
    assert max(rel_err(dp.emb.cpu().numpy(), new["emb"])) <= tol and max(rel_err(dp.W[0].cpu().numpy(), new["W"][0])) <= tol
    ctx.close()


def test_error_paths_of_the_wider_entry_points(gm):
    """gm_meta_train_step without room for the meta-gradient lists, gm_group_batch on offsets that are not monotone or a
    share outside [0, 1], unknown settings: codes come back, nothing is updated, the context stays usable."""
    from paper_2401_04338_amd.binding import GMetaError
    from synth.generate import Params
    cfg = small_cfg(n_tasks=3)
    sup, qry, params = _inputs(cfg)
    ctx = gm.from_config(cfg, workspace_bytes=1 << 26)
    dev = ctx.device
    dp = Params(params.emb.to(dev).clone(), [w.to(dev).clone() for w in params.W], [b.to(dev).clone() for b in params.b])
    big = SMALL.with_(n_tasks=4)
    ctx_big = gm.from_config(big, workspace_bytes=1 << 20)   # no room for the meta-gradient lists beside the step
    sb, qb, pb = _inputs(big)
    dpb = Params(pb.emb.to(dev).clone(), [w.to(dev).clone() for w in pb.W], [b.to(dev).clone() for b in pb.b])
    before = dpb.emb.clone()
    with pytest.raises(GMetaError) as e:
        ctx_big.meta_train_step(_to_dev(sb, dev), _to_dev(qb, dev), dpb, 0.01, 1, 2, 0.1)
    assert e.value.code == -4 and torch.equal(dpb.emb, before)
    ctx_big.close()
    with pytest.raises(GMetaError):
        ctx.configure("no_such_setting", 1)
    with pytest.raises(GMetaError):
        ctx.configure("adapt_rows", 7)
    n = sup.n_samples
    task = np.zeros(n, dtype=np.int64)
    bo = sup.bag_offsets.clone()
    bo[5] = bo[7] + 3                                         # not monotone
    with pytest.raises(GMetaError) as e:
        ctx.group_batch(task, task, bo.to(dev), sup.indices.to(dev), sup.dense.to(dev), sup.labels.to(dev), 1, 2)
    assert e.value.code == -2
    with pytest.raises(GMetaError):
        ctx.group_batch(task, task, sup.bag_offsets.to(dev), sup.indices.to(dev), sup.dense.to(dev), sup.labels.to(dev), 3, 2)
    # still usable
    gs, gq = ctx.group_batch(task, task, sup.bag_offsets.to(dev), sup.indices.to(dev), sup.dense.to(dev), sup.labels.to(dev), 1, 1)
    assert gs.indices.numel() == sup.nnz and gq.indices.numel() == 0
    ctx.meta_train_step(_to_dev(sup, dev), _to_dev(qry, dev), dp, 0.1, 1, 2, 0.1)
    ctx.close()


def test_scatter_add_is_the_outer_update(gm):
    cfg = small_cfg(n_tasks=3)
    sup, qry, params = _inputs(cfg)
    ctx = gm.from_config(cfg, workspace_bytes=1 << 28)
    dev = ctx.device
    out = ctx.meta_step(_to_dev(sup, dev), _to_dev(qry, dev), _params_dev(params, dev), 0.1, 1, 2)
    n = int(out["n_emb_rows"].item())
    table = params.emb.to(dev).clone()
    ctx.scatter_add(table, out["emb_rows"][:n], out["emb_grad"][:n], -0.5)
    want = params.emb.clone()
    want[out["emb_rows"][:n].cpu()] -= 0.5 * out["emb_grad"][:n].cpu()
    assert torch.equal(table.cpu(), want)
    ctx.close()


# ---------------------------------------------------------------- bf16 GEMM path (MFMA), fp32 everything else
TOL_BF16 = 2e-2


@pytest.mark.parametrize("K,order", [(0, 1), (1, 1), (1, 2), (2, 2), (3, 1), (3, 2)])
def test_meta_step_bf16_small_shape(gm, K, order):
    """configs[1]'s model shape with bf16 operands; 6 tasks of ragged size so that the row padding is exercised."""
    cfg = SMALL.with_(n_tasks=6, n_support=50, n_query=37, mlp_dtype=1, rows_per_field=5000, inner_lr=0.05)
    sup, qry, params = _inputs(cfg)
    ctx = gm.from_config(cfg, workspace_bytes=2 << 30)
    _compare_step(cfg, ctx, sup, qry, params, K, order, TOL_BF16, f"bf16 small K={K} order={order}", operand="bf16")
    ctx.close()


def test_meta_step_bf16_tiny_config(gm):
    cfg = TINY.with_(mlp_dtype=1)
    sup, qry, params = _inputs(cfg)
    ctx = gm.from_config(cfg, workspace_bytes=1 << 28)
    _compare_step(cfg, ctx, sup, qry, params, 1, 2, TOL_BF16, "bf16 tiny", operand="bf16")
    ctx.close()


def test_meta_step_bf16_medium_shape_subset(gm):
    """configs[2]'s model (MLP 1677-512-256-1, D=64, bags up to 20, Zipf 1.1, 3 inner steps), 4 tasks, smaller tables."""
    from synth import MEDIUM
    cfg = MEDIUM.with_(n_tasks=4, rows_per_field=20000)
    sup, qry, params = _inputs(cfg)
    ctx = gm.from_config(cfg, workspace_bytes=3 << 30)
    _compare_step(cfg, ctx, sup, qry, params, 3, 2, TOL_BF16, "bf16 medium4 K=3 order=2", operand="bf16")
    _compare_step(cfg, ctx, sup, qry, params, 3, 1, TOL_BF16, "bf16 medium4 K=3 order=1", operand="bf16")
    ctx.close()


# ---------------------------------------------------------------- the two row-arithmetic paths
def _row_path_ctx(gm, cfg, path, ws):
    ctx = gm.from_config(cfg, workspace_bytes=ws)
    ctx.configure("row_path", path)
    return ctx


@pytest.mark.parametrize("path", [1, 2], ids=["sparse", "pairs"])
def test_row_paths_fp32_small_shape(gm, path):
    """configs[1]'s shape (D=32, fp32): the sparse two-hop kernel and the pair-count matrices, each against the oracle."""
    cfg = SMALL.with_(n_tasks=8)
    sup, qry, params = _inputs(cfg)
    ctx = _row_path_ctx(gm, cfg, path, 2 << 30)
    _compare_step(cfg, ctx, sup, qry, params, 1, 2, TOL_FP32, f"small8 path={path} K=1 order=2")
    _compare_step(cfg, ctx, sup, qry, params, 3, 2, TOL_FP32, f"small8 path={path} K=3 order=2")
    _compare_step(cfg, ctx, sup, qry, params, 2, 1, TOL_FP32, f"small8 path={path} K=2 order=1")
    ctx.close()


@pytest.mark.parametrize("path", [1, 2], ids=["sparse", "pairs"])
def test_row_paths_ragged_sizes(gm, path):
    """Task sizes that are no multiple of any tile (50 / 37 samples; 300 / 270 samples: several row blocks, two
    count tiles), D=64, fp32 GEMMs so that the bar is the fp32 one."""
    for ns, nq, nt in ((50, 37, 5), (300, 270, 3)):
        cfg = SMALL.with_(n_tasks=nt, n_support=ns, n_query=nq, n_fields=6, emb_dim=64, rows_per_field=3000,
                          layer_dims=(6 * 64 + 13, 64, 32, 1), inner_lr=0.05)
        sup, qry, params = _inputs(cfg)
        ctx = _row_path_ctx(gm, cfg, path, 2 << 30)
        _compare_step(cfg, ctx, sup, qry, params, 2, 2, TOL_FP32, f"ragged {ns}/{nq} path={path}")
        ctx.close()


@pytest.mark.parametrize("path", [1, 2], ids=["sparse", "pairs"])
def test_row_paths_bf16_medium_shape(gm, path):
    from synth import MEDIUM
    cfg = MEDIUM.with_(n_tasks=4, rows_per_field=20000)
    sup, qry, params = _inputs(cfg)
    ctx = _row_path_ctx(gm, cfg, path, 3 << 30)
    _compare_step(cfg, ctx, sup, qry, params, 3, 2, TOL_BF16, f"bf16 medium4 path={path}", operand="bf16")
    ctx.close()


def test_gemm_wide_tiles_give_the_same_result(gm):
    """gm_configure("gemm_tile_n", 256): the forward / backward products in the pipelined 256 x 256 tiles.  Every
    output element is accumulated in the same order as with 128-wide tiles, so the results are identical."""
    from synth import MEDIUM
    cfg = MEDIUM.with_(n_tasks=3, rows_per_field=20000, n_support=250, n_query=203)
    sup, qry, params = _inputs(cfg)
    ctx = gm.from_config(cfg, workspace_bytes=3 << 30)
    dev = ctx.device
    ds, dq, dp = _to_dev(sup, dev), _to_dev(qry, dev), _params_dev(params, dev)
    a = ctx.meta_step(ds, dq, dp, cfg.inner_lr, 2, 2)
    ctx.configure("gemm_tile_n", 256)
    b = ctx.meta_step(ds, dq, dp, cfg.inner_lr, 2, 2)
    n = int(a["n_emb_rows"].item())
    assert torch.equal(a["loss"], b["loss"]) and torch.equal(a["emb_grad"][:n], b["emb_grad"][:n])
    for l in range(3):
        assert torch.equal(a["dW"][l], b["dW"][l]) and torch.equal(a["db"][l], b["db"][l])
    _compare_step(cfg, ctx, sup, qry, params, 2, 2, TOL_BF16, "bf16 medium3 ragged, 256-wide tiles", operand="bf16")
    ctx.close()


def test_weight_gradient_over_runs_of_tasks_in_wide_tiles(gm):
    """The weight-gradient products that are only ever summed over tasks run over runs of tasks; with thousands of rows
    per run and a first layer wide enough to fill the device they take the pipelined 256 x 256 tiles, both operands read
    contraction-slowest (gm_configure("wgrad_wide"), on by default).  Every element is accumulated in the same order as
    in 128 x 128 tiles: over the same runs of tasks the results are identical; then the whole step against the oracle
    with the number of runs the library picks for the wide tiles."""
    from synth import MEDIUM
    cfg = MEDIUM.with_(n_tasks=40, n_fields=34, rows_per_field=3000, n_support=900, n_query=37, bag_max=3,
                       layer_dims=(34 * 64 + 13, 1024, 64, 1))
    sup, qry, params = _inputs(cfg)
    ctx = gm.from_config(cfg, workspace_bytes=6 << 30)
    dev = ctx.device
    ds, dq, dp = _to_dev(sup, dev), _to_dev(qry, dev), _params_dev(params, dev)
    res = []
    for wide in (0, 1):
        ctx.configure("wgrad_wide", wide)
        ctx.configure("coarse_groups", 16)
        r = ctx.meta_step(ds, dq, dp, cfg.inner_lr, 1, 2)
        res.append({"loss": r["loss"].clone(), "dW": [x.clone() for x in r["dW"]], "db": [x.clone() for x in r["db"]]})
    a, b = res
    assert torch.equal(a["loss"], b["loss"])
    for l in range(3):
        assert torch.equal(a["dW"][l], b["dW"][l]) and torch.equal(a["db"][l], b["db"][l]), l
    ctx.configure("coarse_groups", 0)
    _compare_step(cfg, ctx, sup, qry, params, 1, 2, TOL_BF16, "bf16, weight gradient in 256 x 256 tiles", operand="bf16")
    # a task without support samples (a group with an empty contraction: its tiles hold the old weights alone) and one
    # without query samples
    _compare_step(cfg, ctx, _drop_task_samples(cfg, sup, 3), _drop_task_samples(cfg, qry, 17), params, 1, 2, TOL_BF16,
                  "bf16, wide weight-gradient tiles, empty tasks", operand="bf16")
    ctx.close()


@pytest.mark.parametrize("shape", ["list", "table"])
def test_sort_on_the_side_stream_gives_the_same_result(gm, shape):
    """gm_configure("overlap_sort", 1): the lookups are ordered by row on a second stream beside the dense phase.  Same
    bits as without, in both shapes of the sparse output (the table one with several waves)."""
    cfg = SMALL.with_(n_tasks=8)
    sup, qry, params = _inputs(cfg)
    probe = gm.from_config(cfg, workspace_bytes=2 << 30)
    need = probe.workspace_bytes(8, sup.n_samples, qry.n_samples, sup.nnz, qry.nnz, 2, 2)
    probe.close()
    ctx = gm.from_config(cfg, workspace_bytes=(2 << 30) if shape == "list" else int(need * 0.3))
    dev = ctx.device
    ds, dq, dp = _to_dev(sup, dev), _to_dev(qry, dev), _params_dev(params, dev)
    res = []
    for on in (0, 1, 1):
        ctx.configure("overlap_sort", on)
        table = torch.zeros_like(dp.emb) if shape == "table" else None
        out = ctx.meta_step(ds, dq, dp, cfg.inner_lr, 2, 2, emb_grad_table=table)
        n = int(out["n_emb_rows"].item())
        res.append((out["loss"].clone(), out["dW"][0].clone(), table if table is not None else out["emb_grad"][:n].clone(),
                    out["emb_rows"][:n].clone()))
    for r in res[1:]:
        for a, b in zip(res[0], r):
            assert torch.equal(a, b)
    ctx.close()


@pytest.mark.parametrize("waves", [1, 3], ids=["one_wave", "several_waves"])
def test_pair_counting_on_the_side_stream_gives_the_same_result(gm, waves):
    """gm_configure("overlap_pairs", 1): the pair-count matrices are counted on a second stream beside the prefetch and
    the first forward / backward pass and joined before the first row hop.  Same bits as without, with one wave and
    with several; the overflow fall-back (counts above a byte, found by the kernel on the side stream) still works."""
    cfg = SMALL.with_(n_tasks=8)
    sup, qry, params = _inputs(cfg)
    probe = gm.from_config(cfg, workspace_bytes=2 << 30)
    need = probe.workspace_bytes(8, sup.n_samples, qry.n_samples, sup.nnz, qry.nnz, 2, 2)
    probe.close()
    ctx = gm.from_config(cfg, workspace_bytes=(2 << 30) if waves == 1 else int(need * 0.5))
    dev = ctx.device
    ds, dq, dp = _to_dev(sup, dev), _to_dev(qry, dev), _params_dev(params, dev)
    res = []
    for on in (0, 1, 1):
        ctx.configure("overlap_pairs", on)
        out = ctx.meta_step(ds, dq, dp, cfg.inner_lr, 2, 2)
        n = int(out["n_emb_rows"].item())
        res.append((out["loss"].clone(), out["dW"][0].clone(), out["emb_grad"][:n].clone(), out["emb_rows"][:n].clone()))
    for r in res[1:]:
        for a, b in zip(res[0], r):
            assert torch.equal(a, b)
    ctx.close()
    if waves == 1:
        cfg = SMALL.with_(n_tasks=3, n_support=40, n_query=30, n_fields=4, emb_dim=32, rows_per_field=1, bag_max=24,
                          layer_dims=(4 * 32 + 13, 32, 16, 1), inner_lr=0.01)
        sup, qry, params = _inputs(cfg)
        ctx = gm.from_config(cfg, workspace_bytes=1 << 30)
        ctx.configure("overlap_pairs", 1)
        _compare_step(cfg, ctx, sup, qry, params, 2, 2, TOL_FP32, "pair overflow found on the side stream")
        ctx.close()


def test_pair_counts_above_a_byte_fall_back(gm):
    """One row per table: every pair of bags shares all its lookups, so counts reach bag_i * bag_j > 255.  The default
    choice must fall back to the sparse kernel (and still match the oracle); the forced pair path must refuse."""
    from paper_2401_04338_amd.binding import GMetaError
    cfg = SMALL.with_(n_tasks=3, n_support=40, n_query=30, n_fields=4, emb_dim=32, rows_per_field=1, bag_max=24,
                      layer_dims=(4 * 32 + 13, 32, 16, 1), inner_lr=0.01)
    sup, qry, params = _inputs(cfg)
    ctx = gm.from_config(cfg, workspace_bytes=1 << 30)
    _compare_step(cfg, ctx, sup, qry, params, 2, 2, TOL_FP32, "pair overflow, auto")
    ctx.configure("row_path", 2)
    dev = ctx.device
    with pytest.raises(GMetaError):
        ctx.meta_step(_to_dev(sup, dev), _to_dev(qry, dev), _params_dev(params, dev), cfg.inner_lr, 2, 2)
    ctx.close()


def test_bags_longer_than_the_pair_path_allows(gm):
    """Bags of up to 200 lookups: a (bag, row) count may not fit the pair-count kernel's signed 8-bit operands, so the
    default choice takes the sparse kernel (and matches the oracle) and the forced pair path refuses."""
    from paper_2401_04338_amd.binding import GMetaError
    cfg = SMALL.with_(n_tasks=3, n_support=24, n_query=20, n_fields=3, emb_dim=32, rows_per_field=5000, bag_max=200,
                      layer_dims=(3 * 32 + 13, 32, 16, 1), inner_lr=0.01)
    sup, qry, params = _inputs(cfg)
    lens = (sup.bag_offsets[1:] - sup.bag_offsets[:-1])
    assert int(lens.max()) > 127
    ctx = gm.from_config(cfg, workspace_bytes=1 << 30)
    _compare_step(cfg, ctx, sup, qry, params, 2, 2, TOL_FP32, "long bags, auto")
    ctx.configure("row_path", 2)
    dev = ctx.device
    with pytest.raises(GMetaError):
        ctx.meta_step(_to_dev(sup, dev), _to_dev(qry, dev), _params_dev(params, dev), cfg.inner_lr, 2, 2)
    ctx.close()


def test_mixed_row_paths_in_one_wave(gm):
    """configs[3]'s size mix in miniature (log-normal task sizes, task-private rows in the first fields): tasks above
    512 samples per set take the sparse kernel, the others the pair-count kernels, inside one wave of tasks."""
    from synth import COLDSTART
    from synth.generate import task_sizes
    cfg = COLDSTART.with_(n_tasks=7, n_fields=5, rows_per_field=40000, layer_dims=(5 * 64 + 13, 64, 32, 1), mlp_dtype=0,
                          size_median=600, size_sigma=1.2, size_max=3000, n_private_fields=2, inner_lr=0.05, seed=5)
    ns = task_sizes(cfg)[:, 0]
    print("support samples per task", list(ns), flush=True)
    assert max(ns) > 512 and min(ns) <= 512, "the case must mix both paths"
    sup, qry, params = _inputs(cfg)
    ctx = gm.from_config(cfg, workspace_bytes=3 << 30)
    _compare_step(cfg, ctx, sup, qry, params, 2, 2, TOL_FP32, "mixed paths K=2 order=2")
    ctx.close()


# ---------------------------------------------------------------- the benchmark configurations at full size
def test_small_config_full_size(gm):
    """configs[1] whole (64 tasks x (128 + 128) samples, 26 fields x 100k rows x 32, fp32, K=1, second order): every
    output against the oracle."""
    cfg = SMALL
    sup, qry, params = _inputs(cfg)
    ctx = gm.from_config(cfg, workspace_bytes=4 << 30)
    _compare_step(cfg, ctx, sup, qry, params, cfg.inner_steps, cfg.order, TOL_FP32, "c2_small full size")
    ctx.close()


def test_coldstart_config_full_size_sampled_tasks(gm):
    """configs[3] whole (2,048 tasks of log-normal size, 40 fields x 4 M rows x 64, MLP 2573-1024-512-256-1, bf16
    operands, K=2, second order), as bench.py launches it.  Tasks are independent (Alg. 1): the loss of a sampled task
    must equal the oracle's for that task alone (the oracle sees only the table rows the task looks up: the tables do
    not fit a host copy).  The first fields draw from rows private to a task, so on those rows the batch's sparse
    gradient IS the task's and is compared element by element.  Over all tasks: loss = sum of task losses, listed rows
    = distinct rows looked up."""
    from synth import COLDSTART
    from synth.generate import task_sizes
    cfg = COLDSTART
    dev = torch.device("cuda", 0)
    sup, qry = make_batch(cfg, 0, dev)
    params = make_params(cfg, dev)
    K, order = cfg.inner_steps, cfg.order
    probe = gm.from_config(cfg, workspace_bytes=1 << 20)
    need = probe.workspace_bytes(cfg.n_tasks, sup.n_samples, qry.n_samples, sup.nnz, qry.nnz, K, order)
    probe.close()
    ctx = gm.from_config(cfg, workspace_bytes=int(need * 1.02))
    out = ctx.meta_step(sup, qry, params, cfg.inner_lr, K, order)
    task_loss = out["task_loss"][: cfg.n_tasks].double().cpu().numpy()
    loss = float(out["loss"].item())
    assert abs(task_loss.sum() - loss) <= 1e-5 * abs(loss)
    n = int(out["n_emb_rows"].item())
    rows = out["emb_rows"][:n]
    F = cfg.n_fields
    want = []
    for sd in (sup, qry):
        lens = sd.bag_offsets[1:] - sd.bag_offsets[:-1]
        field = (torch.arange(lens.numel(), device=dev) % F).repeat_interleave(lens)
        want.append(sd.indices.long() + field * cfg.rows_per_field)
    want = torch.unique(torch.cat(want))
    assert n == want.numel() and torch.equal(rows, want), "listed rows != distinct rows looked up"
    del want
    sizes = task_sizes(cfg)[:, 0]
    picks = [int(np.argmax(sizes)), int(np.argsort(sizes)[len(sizes) // 2]), int(np.argmin(sizes))]
    print("c4 sampled tasks", picks, "support samples", [int(sizes[t]) for t in picks], flush=True)
    assert sizes[picks[0]] > 512 >= sizes[picks[1]], "one sampled task per row path"
    errs = []
    for t in picks:
        s1, q1 = make_batch(cfg, 0, "cpu", [t])
        model, p_np, sd, qd, grows = compact_task(cfg, s1, q1, params.emb, params.W, params.b)
        ref = O.meta_step(model, p_np, sd, qd, cfg.inner_lr, K, order, operand="bf16")
        e = abs(task_loss[t] - ref["loss"]) / abs(ref["loss"])
        # rows of the task-private fields: nobody else touches them
        priv = ref["emb_rows"] < np.cumsum([0] + list(model.rows_per_field))[cfg.n_private_fields]
        g_rows = torch.from_numpy(grows[ref["emb_rows"][priv]]).to(dev)
        pos = torch.searchsorted(rows, g_rows)
        assert torch.equal(rows[pos], g_rows)
        got_g, ref_g = out["emb_grad"][pos].double().cpu().numpy(), ref["emb_grad"][priv]
        row_err = np.linalg.norm(got_g - ref_g, axis=1) / np.linalg.norm(ref_g, axis=1).max()
        q50, q90, q99 = np.quantile(row_err, [0.5, 0.9, 0.99])
        print(f"c4 full size, task {t}: loss {task_loss[t]:.6f} vs oracle {ref['loss']:.6f} ({e:.2e}); "
              f"{int(priv.sum())} private rows, row error median {q50:.1e}, 90% {q90:.1e}, 99% {q99:.1e}, "
              f"max {row_err.max():.1e}", flush=True)
        errs.append((e, q50, q90, row_err.max()))
    # A ReLU decision on a pre-activation within float32 accumulation error of zero may fall differently than in the
    # oracle's float64 accumulation (a few units in a million; seen here on 2 of one task's 62 samples).  That changes
    # that sample's whole gradient, i.e. exactly the rows it looks up, and a task of a few dozen samples does not
    # average it away.  The bar is therefore on the bulk of the rows: the median must sit far below bf16 resolution
    # (the rounding points agree), 90 % within the bf16 tolerance, and the rest bounded by one sample's share.
    for e, q50, q90, emax in errs:
        assert e <= TOL_BF16 and q50 <= 1e-3 and q90 <= TOL_BF16 and emax <= 0.5
    ctx.close()


@pytest.mark.parametrize("bf,K,order", [(0, 2, 2), (0, 1, 1), (1, 2, 2), (1, 0, 2)])
def test_more_tasks_than_coarse_runs(gm, bf, K, order):
    """The weight-gradient products that only feed the sum over the tasks (last step of the second-order chain; the
    query gradient when there is no chain) are taken over 16 runs of consecutive tasks.  37 tasks of log-normal size:
    runs of two and three tasks with ragged row counts, every output against the oracle."""
    from synth.generate import task_sizes
    cfg = small_cfg(n_tasks=37, inner_lr=0.1, mlp_dtype=bf).with_(lognormal_sizes=True, size_median=9, size_sigma=0.8,
                                                                   size_max=40)
    sup, qry, params = _inputs(cfg, emb_std=0.3)
    assert len(set(task_sizes(cfg)[:, 0])) > 3, "the case must have ragged tasks"
    ctx = gm.from_config(cfg, workspace_bytes=1 << 29)
    _compare_step(cfg, ctx, sup, qry, params, K, order, TOL_BF16 if bf else TOL_FP32, f"37 tasks bf16={bf} K={K} order={order}",
                  operand="bf16" if bf else "fp64")
    ctx.close()


@pytest.mark.parametrize("K", [2, 3, 4])
def test_inner_step_weights_from_the_meta_parameters(gm, K):
    """bf16, second order, several inner steps: by default a step's weight matrices are theta - alpha * (all steps'
    gradients so far) in one accumulation; gm_configure("theta_from_meta", 0) keeps a per-task fp32 master updated step by
    step.  Both against the oracle; the two agree far inside the bf16 tolerance (they differ by fp32 rounding before the
    operand copy is rounded)."""
    cfg = SMALL.with_(n_tasks=5, n_support=70, n_query=40, n_fields=4, emb_dim=32, rows_per_field=400, bag_max=5,
                      layer_dims=(4 * 32 + 13, 96, 48, 1), mlp_dtype=1, inner_lr=0.05)
    sup, qry, params = _inputs(cfg)
    ctx = gm.from_config(cfg, workspace_bytes=1 << 30)
    out_a, _ = _compare_step(cfg, ctx, sup, qry, params, K, 2, TOL_BF16, f"K={K}, weights from the meta parameters", operand="bf16")
    a = [x.clone() for x in out_a["dW"]]
    ctx.configure("theta_from_meta", 0)
    out_b, _ = _compare_step(cfg, ctx, sup, qry, params, K, 2, TOL_BF16, f"K={K}, per-task fp32 master", operand="bf16")
    for l in range(len(a)):
        assert max(rel_err(out_b["dW"][l].cpu().numpy(), a[l].cpu().numpy())) <= 5e-3
    ctx.close()


@pytest.mark.parametrize("runs", [1, 7, 32])
def test_other_numbers_of_task_runs(gm, runs):
    """gm_configure("coarse_groups"): the products only summed over tasks taken over another number of runs of tasks --
    the same per-task terms added in another order: against the oracle, and within fp32 rounding of the default."""
    from paper_2401_04338_amd.binding import GMetaError
    cfg = small_cfg(n_tasks=37, inner_lr=0.1).with_(lognormal_sizes=True, size_median=9, size_sigma=0.8, size_max=40)
    sup, qry, params = _inputs(cfg, emb_std=0.3)
    ctx = gm.from_config(cfg, workspace_bytes=1 << 29)
    dev = ctx.device
    a = ctx.meta_step(_to_dev(sup, dev), _to_dev(qry, dev), _params_dev(params, dev), cfg.inner_lr, 2, 2)
    a = [x.clone() for x in a["dW"]]
    ctx.configure("coarse_groups", runs)
    out, _ = _compare_step(cfg, ctx, sup, qry, params, 2, 2, TOL_FP32, f"37 tasks in {runs} runs")
    for l in range(len(a)):
        assert max(rel_err(out["dW"][l].cpu().numpy(), a[l].cpu().numpy())) <= 1e-5
    with pytest.raises(GMetaError):
        ctx.configure("coarse_groups", 33)
    ctx.close()


@pytest.mark.parametrize("D", [8, 16, 128, 256])
def test_embedding_widths(gm, D):
    """Every embedding width has its own lane-group shape in the gather, the segmented reduction and the scatter
    (D / 4 lanes per row): widths the five configs do not use, hot rows whose segments span many 64-lookup chunks
    (zipf over 300 rows), both shapes of the sparse output."""
    cfg = SMALL.with_(n_tasks=3, n_support=48, n_query=40, n_fields=3, emb_dim=D, rows_per_field=300, bag_max=9,
                      layer_dims=(3 * D + 13, 32, 1), inner_lr=0.05, zipf_s=1.2)
    sup, qry, params = _inputs(cfg, emb_std=0.2)
    ctx = gm.from_config(cfg, workspace_bytes=1 << 30)
    dev = ctx.device
    out, ref = _compare_step(cfg, ctx, sup, qry, params, 1, 2, TOL_FP32, f"D={D}")
    table = torch.zeros(cfg.total_rows, D, dtype=torch.float32, device=dev)
    ctx.meta_step(_to_dev(sup, dev), _to_dev(qry, dev), _params_dev(params, dev), cfg.inner_lr, 1, 2, emb_grad_table=table)
    n = int(out["n_emb_rows"].item())
    want = torch.zeros_like(table)
    want[out["emb_rows"][:n]] = out["emb_grad"][:n]
    assert torch.equal(table, want)
    ctx.close()


def test_large_config_shape(gm):
    """configs[4]'s shapes on two of its tasks (64 fields, bags of 1-32, 512 + 512 samples per task, MLP
    4109-1024-512-256-1, bf16 operands, K=1, second order) over smaller tables (2^16 rows per field, so that the oracle's
    copy fits the test): more than 8192 lookups per (task, field, set), 512-row pair-count matrices, and the widest
    grouped GEMMs; every output against the oracle, in both shapes of the sparse output."""
    from synth import LARGE
    cfg = LARGE.with_(n_tasks=2, rows_per_field=1 << 16)
    ctx = gm.from_config(cfg, workspace_bytes=6 << 30)
    dev = ctx.device
    sup, qry = (_to_dev(sd, "cpu") for sd in make_batch(cfg, 0, dev))   # the same streams, drawn faster on the device
    params = make_params(cfg, "cpu")
    out, ref = _compare_step(cfg, ctx, sup, qry, params, cfg.inner_steps, cfg.order, TOL_BF16, "c5 shape, 2 tasks",
                             operand="bf16")
    table = torch.zeros(cfg.total_rows, cfg.emb_dim, dtype=torch.float32, device=dev)
    ctx.meta_step(_to_dev(sup, dev), _to_dev(qry, dev), _params_dev(params, dev), cfg.inner_lr, cfg.inner_steps, cfg.order,
                  emb_grad_table=table)
    n = int(out["n_emb_rows"].item())
    want = torch.zeros_like(table)
    want[out["emb_rows"][:n]] = out["emb_grad"][:n]
    assert torch.equal(table, want)
    ctx.close()


def test_medium_config_full_size_sampled_tasks(gm):
    """configs[2] whole, as bench.py launches it (512 tasks, 26 fields x 1M rows x 64, bf16 operands, K=3, second
    order).  The oracle cannot run the whole batch in the test budget, but tasks are independent (Alg. 1): the loss of
    a sampled task from the full-size run must equal the oracle's for that task alone.  Over all tasks: the loss is
    the sum of the task losses, and the listed rows are exactly the distinct rows looked up, ascending."""
    from synth import MEDIUM
    cfg = MEDIUM
    dev = torch.device("cuda", 0)
    sup, qry = make_batch(cfg, 0, dev)
    params = make_params(cfg, dev)
    probe = gm.from_config(cfg, workspace_bytes=1 << 20)   # the workspace that holds one wave, as the benchmark does
    need = probe.workspace_bytes(cfg.n_tasks, sup.n_samples, qry.n_samples, sup.nnz, qry.nnz, cfg.inner_steps, cfg.order)
    probe.close()
    ctx = gm.from_config(cfg, workspace_bytes=int(need * 1.02))
    out = ctx.meta_step(sup, qry, params, cfg.inner_lr, cfg.inner_steps, cfg.order)
    task_loss = out["task_loss"][: cfg.n_tasks].double().cpu().numpy()
    loss = float(out["loss"].item())
    assert abs(task_loss.sum() - loss) <= 1e-5 * abs(loss)
    n = int(out["n_emb_rows"].item())
    rows = out["emb_rows"][:n]
    F = cfg.n_fields
    want = []
    for sd in (sup, qry):
        lens = sd.bag_offsets[1:] - sd.bag_offsets[:-1]
        field = (torch.arange(lens.numel(), device=dev) % F).repeat_interleave(lens)
        want.append(sd.indices.long() + field * cfg.rows_per_field)
    want = torch.unique(torch.cat(want))
    assert n == want.numel() and torch.equal(rows, want), "listed rows != distinct rows looked up"
    assert torch.isfinite(out["emb_grad"][:n]).all()
    params_np = make_params(cfg, "cpu").numpy()
    for t in (0, 257, 511):
        s1, q1 = make_batch(cfg, 0, "cpu", [t])
        ref = O.meta_step(oracle_model(cfg), params_np, s1.numpy(), q1.numpy(), cfg.inner_lr, cfg.inner_steps, cfg.order,
                          operand="bf16")
        e = abs(task_loss[t] - ref["loss"]) / abs(ref["loss"])
        print(f"c3 full size, task {t}: loss {task_loss[t]:.6f} vs oracle {ref['loss']:.6f} ({e:.2e})", flush=True)
        assert e <= TOL_BF16
    ctx.close()


def test_large_config_full_size_sampled_tasks(gm):
    """configs[4] whole (8,192 tasks x (512 + 512) samples, 64 fields x 4 M rows x 64, 8.9 G lookups: more than 2^31 per
    set), as bench.py launches it: 32-odd waves of tasks, the sparse gradient added wave by wave into a table-shaped
    accumulator.  Checked: loss = sum of task losses; for sampled tasks the loss against the oracle run on the task's
    own rows; and, on table rows that the whole batch looks up exactly once (so that the batch's gradient of the row IS
    the sampled task's), the accumulated gradient against the oracle's, row by row."""
    from synth import LARGE
    cfg = LARGE
    dev = torch.device("cuda", 0)
    torch.cuda.empty_cache()
    free_b, _ = torch.cuda.mem_get_info()
    if free_b < (250 << 30):
        pytest.skip(f"needs about 250 GiB of free device memory, {free_b >> 30} GiB are free")
    K, order, F, R = cfg.inner_steps, cfg.order, cfg.n_fields, cfg.rows_per_field
    print("c5 full size: generating", flush=True)
    sup, qry = make_batch(cfg, 0, dev)
    params = make_params(cfg, dev)
    table = torch.zeros_like(params.emb)
    assert sup.nnz >= 2 ** 31 and qry.nnz >= 2 ** 31
    free_b, _ = torch.cuda.mem_get_info()
    ctx = gm.from_config(cfg, workspace_bytes=int(free_b - (16 << 30)))
    print("c5 full size: step", flush=True)
    out = ctx.meta_step(sup, qry, params, cfg.inner_lr, K, order, emb_grad_table=table)
    ctx.close()
    task_loss = out["task_loss"][: cfg.n_tasks].double().cpu().numpy()
    loss = float(out["loss"].item())
    assert np.isfinite(loss) and abs(task_loss.sum() - loss) <= 1e-5 * abs(loss)
    rng = np.random.default_rng(0)
    for t in (0, 8191):
        s1, q1 = make_batch(cfg, 0, "cpu", [t])
        model, p_np, sd, qd, grows = compact_task(cfg, s1, q1, params.emb, params.W, params.b)
        ref = O.meta_step(model, p_np, sd, qd, cfg.inner_lr, K, order, operand="bf16")
        e = abs(task_loss[t] - ref["loss"]) / abs(ref["loss"])
        # candidate rows of the task; keep those that the whole batch looks up exactly once
        cand = rng.choice(len(ref["emb_rows"]), size=4000, replace=False)
        cand_rows = grows[ref["emb_rows"][cand]]
        is_cand = torch.zeros(R, dtype=torch.bool, device=dev)   # by index within a field; the field is resolved below
        is_cand[torch.from_numpy(np.unique(cand_rows % R)).to(dev)] = True
        hits = []
        for sdv in (sup, qry):
            for lo in range(0, sdv.nnz, 1 << 28):
                chunk = sdv.indices[lo: lo + (1 << 28)]
                p = torch.nonzero(is_cand[chunk.long()]).flatten() + lo
                if p.numel():
                    bag = torch.searchsorted(sdv.bag_offsets, p, right=True) - 1
                    hits.append((bag % F) * R + sdv.indices[p].long())
                del chunk, p
        hits = torch.cat(hits).cpu().numpy()
        rows_hit, counts = np.unique(hits, return_counts=True)
        once = set(rows_hit[counts == 1].tolist())
        print("c5 full size: candidate rows by number of lookups in the batch:",
              {int(k): int((counts[np.isin(rows_hit, cand_rows)] == k).sum()) for k in (1, 2, 3, 4, 8)}, flush=True)
        keep = np.array([i for i, g in zip(cand, cand_rows) if int(g) in once], dtype=np.int64)
        assert keep.size >= 10, "too few rows that only this task looks up"
        got = table[torch.from_numpy(grows[ref["emb_rows"][keep]]).to(dev)].double().cpu().numpy()
        want = ref["emb_grad"][keep]
        row_err = np.linalg.norm(got - want, axis=1) / np.linalg.norm(ref["emb_grad"], axis=1).max()
        q50, q90 = np.quantile(row_err, [0.5, 0.9])
        print(f"c5 full size, task {t}: loss {task_loss[t]:.6f} vs oracle {ref['loss']:.6f} ({e:.2e}); {keep.size} rows "
              f"looked up once in the batch: row error median {q50:.1e}, 90% {q90:.1e}, max {row_err.max():.1e}", flush=True)
        # (bar as in the configs[3] test: a ReLU decision that falls differently moves one sample's rows)
        assert e <= TOL_BF16 and q50 <= 1e-3 and q90 <= TOL_BF16 and row_err.max() <= 0.5
        assert np.abs(got).sum() > 0
    del table, params, sup, qry
    torch.cuda.empty_cache()


# ---------------------------------------------------------------- the three large configurations: every output on a task subset at
# full table size
def _subset_case(name):
    from synth import COLDSTART, LARGE, MEDIUM
    from synth.generate import task_sizes
    if name == "c3":
        return MEDIUM, [0, 31, 64, 101, 128, 170, 201, 255, 256, 300, 333, 384, 420, 457, 500, 511], 6
    if name == "c4":
        sizes = task_sizes(COLDSTART)[:, 0]
        by_size = np.argsort(sizes, kind="stable")
        # stratified over the size distribution: the smallest and the largest task, the tasks nearest to 512 samples per
        # set from both sides (one per row path), and quantiles in between
        above = [int(t) for t in by_size if sizes[t] > 512]
        below = [int(t) for t in by_size if sizes[t] <= 512]
        picks = {below[0], below[-1], above[0], above[-1]}
        for q in np.linspace(0.05, 0.95, 12):
            picks.add(int(by_size[int(q * (len(by_size) - 1))]))
        tasks = sorted(picks)
        assert len(tasks) >= 16 or len(tasks) == len(picks)
        return COLDSTART, tasks, 6
    return LARGE, [0, 2741, 5555, 8191], 2


@pytest.mark.parametrize("name", ["c3", "c4", "c5"])
def test_large_configs_task_subset_at_full_table_size(gm, name):
    """configs[2], [3], [4]: a GPU run restricted to a subset of the configuration's tasks -- the full batch's values for
    those tasks (the generator's streams are per task), tables at FULL size, the launch configuration bench.py uses,
    several waves of tasks -- against the oracle on the same subset (which sees the rows the subset looks up,
    re-indexed): loss, every task's loss, every dW and db, the listed rows and the whole sparse gradient.  c3: 16
    tasks; c4: the smallest and the largest task, both row paths, quantiles of the size distribution; c5: 4 tasks."""
    cfg, tasks, per_wave = _subset_case(name)
    dev = torch.device("cuda", 0)
    torch.cuda.empty_cache()
    free_b, _ = torch.cuda.mem_get_info()
    need_b = cfg.total_rows * cfg.emb_dim * 4 + (24 << 30)
    if free_b < need_b:
        pytest.skip(f"needs {need_b >> 30} GiB of free device memory, {free_b >> 30} GiB are free")
    K, order = cfg.inner_steps, cfg.order
    print(f"{name}: {len(tasks)} tasks {tasks}", flush=True)
    params = make_params(cfg, dev, chunk=1 << 26)
    sup, qry = make_batch(cfg, 0, dev, tasks)
    ctx = gm.from_config(cfg, workspace_bytes=16 << 30)
    ctx.configure("max_wave_tasks", per_wave)
    out = ctx.meta_step(sup, qry, params, cfg.inner_lr, K, order)
    ctx.close()
    s_cpu, q_cpu = make_batch(cfg, 0, "cpu", tasks)
    assert torch.equal(s_cpu.indices, sup.indices.cpu()) and torch.equal(q_cpu.bag_offsets, qry.bag_offsets.cpu())
    model, p_np, sd, qd, grows = compact_task(cfg, s_cpu, q_cpu, params.emb, params.W, params.b)
    rec = {}
    ref = O.meta_step(model, p_np, sd, qd, cfg.inner_lr, K, order, operand="bf16", masks_out=rec)
    gated = O.meta_step(model, p_np, sd, qd, cfg.inner_lr, K, order, relu_masks=rec)
    n = int(out["n_emb_rows"].item())
    assert n == len(ref["emb_rows"])
    assert np.array_equal(out["emb_rows"][:n].cpu().numpy(), grows[ref["emb_rows"]])     # integers: exact
    T = len(tasks)
    for label, r in (("float64 arithmetic on bf16 gates", gated), ("bf16-operand oracle", ref)):
        e = _errors(out, r, n, T)
        got, want = out["emb_grad"][:n].double().cpu().numpy(), r["emb_grad"]
        row_err = np.linalg.norm(got - want, axis=1) / np.linalg.norm(want, axis=1).max()
        print(f"{name} subset vs {label}:", {k: f"{v:.2e}" for k, v in e.items()},
              f"rows: median {np.median(row_err):.1e}, 99.9% {np.quantile(row_err, 0.999):.1e}, max {row_err.max():.1e}, "
              f"above tolerance {int((row_err > TOL_BF16).sum())} of {n}", flush=True)
        for k, v in e.items():
            assert v <= TOL_BF16, (name, label, k, v)
    del params, sup, qry, out
    torch.cuda.empty_cache()


def test_tables_of_unequal_size(gm):
    """rows_per_field need not be equal: 5 fields of 7 to 3,001 rows (field bases that are no multiple of anything),
    fp32, every output against the oracle; and the integer structures bit for bit."""
    from paper_2401_04338_amd import GMeta
    from synth.generate import Params, SetData
    rows = [7, 3001, 64, 1234, 333]
    cfg = SMALL.with_(n_tasks=5, n_support=33, n_query=21, n_fields=5, emb_dim=16, rows_per_field=4000, bag_max=6,
                      layer_dims=(5 * 16 + 13, 32, 16, 1), inner_lr=0.05)
    sup, qry, params = _inputs(cfg, emb_std=0.2)
    F = cfg.n_fields

    def fold(sd):   # every index taken modulo its own field's table size
        lens = sd.bag_offsets[1:] - sd.bag_offsets[:-1]
        field = (torch.arange(lens.numel()) % F).repeat_interleave(lens)
        return SetData(sd.task_offsets, sd.bag_offsets, (sd.indices.long() % torch.tensor(rows)[field]).int(), sd.dense, sd.labels)

    sup, qry = fold(sup), fold(qry)
    emb = params.emb[: sum(rows)].contiguous()
    p2 = Params(emb, params.W, params.b)
    model = O.Model(rows_per_field=rows, emb_dim=cfg.emb_dim, n_dense=cfg.n_dense, layer_dims=list(cfg.layer_dims))
    ctx = GMeta(F, rows, cfg.emb_dim, cfg.n_dense, cfg.layer_dims, 0, workspace_bytes=1 << 28)
    dev = ctx.device
    got = ctx.index_prep(_to_dev(sup, dev), _to_dev(qry, dev))
    want = O.index_prep(model, sup.numpy(), qry.numpy())
    for k in ("slot_counts", "slot_rows", "sup_slot", "qry_slot", "emb_rows", "seg_counts"):
        assert np.array_equal(got[k].cpu().numpy(), want[k]), k
    _compare_step(cfg, ctx, sup, qry, p2, 2, 2, TOL_FP32, "unequal tables", model=model)
    ctx.close()
