"""Planted mistakes in the ORACLE (CPU only) must be caught by the pins' machinery.

Each case breaks one term of the oracle and checks that the finite-difference
pin then fails: evidence that the pins are sensitive to that term.
"""
import numpy as np
import pytest

from oracle import maml_dlrm as O
from tests.helpers import small_cfg
from tests.test_oracle_pins import _fd_check


def _drop_cross_term(acts, z, y, W, deltas, vW, vb, vx, q=None):
    hW, hb, hx = _ORIG(acts, z, y, W, deltas, vW, vb, vx)
    return hW, hb, hx * 0.0 + (hx - deltas[0] @ vW[0].T)      # drop delta * vW^T at the input


def _wrong_sign(acts, z, y, W, deltas, vW, vb, vx, q=None):
    hW, hb, hx = _ORIG(acts, z, y, W, deltas, vW, vb, vx)
    return [-h for h in hW], hb, hx


def _no_bias_tangent(acts, z, y, W, deltas, vW, vb, vx, q=None):
    return _ORIG(acts, z, y, W, deltas, vW, [np.zeros_like(v) for v in vb], vx)


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
