"""Stored oracle outputs (tests/golden/mini_step.json, written by tests/golden/write_mini_step.py from oracle/ alone).

CPU: the oracle still reproduces them (an unintended change of its arithmetic or of the input recipe shows here).
GPU: the HIP path, through the C ABI, against the stored values."""
import json
import os

import numpy as np
import pytest
import torch

from tests.golden.write_mini_step import compute
from tests.helpers import small_cfg

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "mini_step.json")


def _stored():
    with open(GOLDEN) as f:
        return json.load(f)


def test_oracle_reproduces_the_stored_values():
    stored, now = _stored(), compute()
    assert stored["cases"].keys() == now["cases"].keys()
    for name, s in stored["cases"].items():
        n = now["cases"][name]
        assert s["emb_rows"] == n["emb_rows"], name
        for key in ("loss", "task_loss", "emb_grad_row_sums", "dW_sums", "dW_abs_sums"):
            assert np.allclose(np.asarray(s[key]), np.asarray(n[key]), rtol=1e-12, atol=1e-15), (name, key)
        for a, b in zip(s["db"], n["db"]):
            assert np.allclose(a, b, rtol=1e-12, atol=1e-15), name


@pytest.mark.gpu
def test_hip_path_against_the_stored_values():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2401_04338_amd import GMeta
    from synth import make_batch, make_params
    from synth.generate import Params, SetData
    cfg = small_cfg(n_tasks=5, inner_lr=0.3)
    sup, qry = make_batch(cfg, 0, "cpu")
    params = make_params(cfg, "cpu", emb_std=0.3)
    ctx = GMeta.from_config(cfg, workspace_bytes=1 << 28)
    dev = ctx.device
    to_dev = lambda s: SetData(s.task_offsets, s.bag_offsets.to(dev), s.indices.to(dev), s.dense.to(dev), s.labels.to(dev))
    pd = Params(params.emb.to(dev), [w.to(dev) for w in params.W], [b.to(dev) for b in params.b])
    for name, s in _stored()["cases"].items():
        K, order = int(name[1]), int(name[-1])
        out = ctx.meta_step(to_dev(sup), to_dev(qry), pd, cfg.inner_lr, K, order)
        n = int(out["n_emb_rows"].item())
        assert out["emb_rows"][:n].cpu().tolist() == s["emb_rows"], name
        assert abs(float(out["loss"].item()) - s["loss"]) <= 1e-4 * abs(s["loss"]), name
        assert np.allclose(out["task_loss"][:5].cpu().numpy(), s["task_loss"], rtol=1e-4), name
        got_rows = out["emb_grad"][:n].double().sum(dim=1).cpu().numpy()
        scale = np.abs(s["emb_grad_row_sums"]).max()
        assert np.abs(got_rows - np.asarray(s["emb_grad_row_sums"])).max() <= 1e-4 * scale, name
        for l, (ws, was) in enumerate(zip(s["dW_sums"], s["dW_abs_sums"])):
            w = out["dW"][l].double()
            assert abs(float(w.sum()) - ws) <= 1e-4 * was and abs(float(w.abs().sum()) - was) <= 1e-4 * was, (name, l)
            assert np.allclose(out["db"][l].cpu().numpy(), s["db"][l], rtol=1e-3, atol=1e-4 * max(1e-30, np.abs(s["db"][l]).max())), (name, l)
    ctx.close()
