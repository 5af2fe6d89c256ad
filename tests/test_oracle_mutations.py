"""Planted mistakes in the ORACLE (CPU only) must be caught by the pins' machinery.

Each case breaks one term of the oracle and checks that the finite-difference
pin then fails: evidence that the pins are sensitive to that term.
"""
import numpy as np
import pytest

from oracle import maml_dlrm as O
from tests.helpers import small_cfg
from tests.test_oracle_pins import _fd_check


def _drop_cross_term(acts, z, y, W, deltas, masks, vW, vb, vx, q=None):
    hW, hb, hx = _ORIG(acts, z, y, W, deltas, masks, vW, vb, vx)
    return hW, hb, hx * 0.0 + (hx - deltas[0] @ vW[0].T)      # drop delta * vW^T at the input


def _wrong_sign(acts, z, y, W, deltas, masks, vW, vb, vx, q=None):
    hW, hb, hx = _ORIG(acts, z, y, W, deltas, masks, vW, vb, vx)
    return [-h for h in hW], hb, hx


def _no_bias_tangent(acts, z, y, W, deltas, masks, vW, vb, vx, q=None):
    return _ORIG(acts, z, y, W, deltas, masks, vW, [np.zeros_like(v) for v in vb], vx)


_ORIG = O.hvp


@pytest.mark.parametrize("bad", [_drop_cross_term, _wrong_sign, _no_bias_tangent])
def test_broken_hvp_is_caught(monkeypatch, bad):
    monkeypatch.setattr(O, "hvp", bad)
    with pytest.raises(AssertionError):
        _fd_check(small_cfg(inner_lr=0.3), K=2)


def test_transposed_pool_is_caught(monkeypatch):
    orig = O.pool

    def no_multiplicity(model, E, loc, bag, n):
        out = np.zeros((n * model.n_fields, model.emb_dim))
        out[bag] = E[loc]                      # last write wins: multiplicity lost
        return out.reshape(n, model.n_fields * model.emb_dim)
    monkeypatch.setattr(O, "pool", no_multiplicity)
    with pytest.raises(AssertionError):
        from tests.test_oracle_pins import test_against_library_double_backward
        test_against_library_double_backward(2, 2)


def test_dense_only_chain_without_its_cross_term_is_caught(monkeypatch):
    """adapt_rows=False: dropping the path from the adapted theta back to the embeddings (the input part of the
    Hessian-vector product) must break the finite-difference pin of that variant."""
    def no_input_part(acts, z, y, W, deltas, masks, vW, vb, vx, q=None):
        hW, hb, hx = _ORIG(acts, z, y, W, deltas, masks, vW, vb, vx)
        return hW, hb, hx * 0.0
    monkeypatch.setattr(O, "hvp", no_input_part)
    with pytest.raises(AssertionError):
        _fd_check(small_cfg(inner_lr=0.3), K=2, adapt_rows=False)


def test_outer_update_with_the_wrong_sign_or_rows_is_caught(monkeypatch):
    """The descent pin of meta_train_step must fail for an ascent step and for an update that lands one row off."""
    from tests.test_oracle_pins import test_train_step_descends_the_meta_objective_by_beta_times_the_squared_gradient as pin
    orig = O.meta_step

    def negated(*a, **k):
        r = orig(*a, **k)
        r = dict(r)
        r["emb_grad"] = -r["emb_grad"]
        r["dW"] = [-w for w in r["dW"]]
        r["db"] = [-b for b in r["db"]]
        return r

    def shifted(*a, **k):
        r = dict(orig(*a, **k))
        r["emb_rows"] = np.roll(r["emb_rows"], 1)
        return r

    import inspect
    src_step = O.meta_train_step

    for bad in (negated, shifted):
        def train(model, params, sup, qry, alpha, K, order, beta, operand="fp64", adapt_rows=True, _bad=bad):
            monkeypatch.setattr(O, "meta_step", _bad)
            try:
                return src_step(model, params, sup, qry, alpha, K, order, beta, operand, adapt_rows)
            finally:
                monkeypatch.setattr(O, "meta_step", orig)
        monkeypatch.setattr(O, "meta_train_step", train)
        with pytest.raises(AssertionError):
            pin(2)
        monkeypatch.setattr(O, "meta_train_step", src_step)


def test_grouping_with_a_wrong_split_or_order_is_caught(monkeypatch):
    """The hand-written stream must fail for a split at another share, the generator round trip for a reversed order
    inside a batch."""
    from tests import test_group_batch as G
    orig = O.group_batch

    def other_share(F, task, batch_id, bo, idx, dn, lb, num, den):
        return orig(F, task, batch_id, bo, idx, dn, lb, 1, 2)

    def reversed_inside(F, task, batch_id, bo, idx, dn, lb, num, den):
        n = len(task)
        rev = list(range(n))[::-1]
        bo = np.asarray(bo)
        lens = np.diff(bo).reshape(n, F)[rev]
        starts = bo[:-1].reshape(n, F)[rev]
        idx = np.asarray(idx)
        idx2 = np.concatenate([idx[a:a + l] for a, l in zip(starts.ravel(), lens.ravel())]) if lens.sum() else idx[:0]
        bo2 = np.concatenate([[0], np.cumsum(lens.ravel())])
        return orig(F, np.asarray(task)[rev], np.asarray(batch_id)[rev], bo2, idx2, np.asarray(dn)[rev], np.asarray(lb)[rev], num, den)

    monkeypatch.setattr(O, "group_batch", other_share)
    with pytest.raises(AssertionError):
        G.test_grouping_by_hand_on_a_tiny_stream()
    monkeypatch.setattr(O, "group_batch", reversed_inside)
    with pytest.raises(AssertionError):
        G.test_grouping_recovers_the_generators_sets()


@pytest.mark.parametrize("where", ["backward", "hvp"])
def test_given_gates_ignored_by_a_pass_is_caught(monkeypatch, where):
    """A backward or tangent pass that re-derives its gates from the activations instead of applying the given ones
    must break the frozen-gate finite-difference pin."""
    from tests.test_oracle_pins import test_frozen_gate_meta_gradient_by_central_differences as pin
    if where == "backward":
        orig = O.backward
        monkeypatch.setattr(O, "backward", lambda acts, z, y, W, masks, q=O._identity:
                            orig(acts, z, y, W, [a > 0.0 for a in acts[1:]], q))
    else:
        monkeypatch.setattr(O, "hvp", lambda acts, z, y, W, deltas, masks, vW, vb, vx, q=O._identity:
                            _ORIG(acts, z, y, W, deltas, [a > 0.0 for a in acts[1:]], vW, vb, vx, q))
    with pytest.raises(AssertionError):
        pin(2)
