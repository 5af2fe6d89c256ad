"""The row compaction that lets the oracle check one task of a configuration with very large tables."""
import numpy as np

from oracle import maml_dlrm as O
from synth import make_batch, make_params
from tests.helpers import compact_task, oracle_model, small_cfg


def test_compacted_task_gives_the_same_oracle_result():
    cfg = small_cfg(n_tasks=4, rows_per_field=500, n_fields=3, bag_max=5)
    params = make_params(cfg, "cpu", emb_std=0.3)
    for t in (0, 3):
        s1, q1 = make_batch(cfg, 0, "cpu", [t])
        full = O.meta_step(oracle_model(cfg), params.numpy(), s1.numpy(), q1.numpy(), cfg.inner_lr, 2, 2)
        model, p_np, sd, qd, grows = compact_task(cfg, s1, q1, params.emb, params.W, params.b)
        assert sum(model.rows_per_field) < cfg.total_rows
        comp = O.meta_step(model, p_np, sd, qd, cfg.inner_lr, 2, 2)
        assert np.isclose(comp["loss"], full["loss"], rtol=1e-12)
        assert np.array_equal(grows[comp["emb_rows"]], full["emb_rows"])
        assert np.allclose(comp["emb_grad"], full["emb_grad"], rtol=1e-12, atol=0)
        for a, b in zip(comp["dW"], full["dW"]):
            assert np.allclose(a, b, rtol=1e-12, atol=1e-300)
