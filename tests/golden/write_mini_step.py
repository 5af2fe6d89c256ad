"""Writes tests/golden/mini_step.json: the oracle's outputs on the miniature configuration of the tests.

Calls only oracle/ and the seeded input generator.  The paper prints no numeric worked example of the method (its
tables are throughput and AUC on its own data), so this fixture is not a pin of the oracle: it detects an unintended
change of the oracle's arithmetic or of the input recipe, and gives the GPU tests a stored target that no GPU code
produced.  Run from the repository root:  python tests/golden/write_mini_step.py
"""
import json
import os
import sys

sys.path.insert(0, os.path.join(os.path.dirname(os.path.abspath(__file__)), "..", ".."))

from oracle import maml_dlrm as O  # noqa: E402
from tests.helpers import oracle_inputs, small_cfg  # noqa: E402


def compute():
    cfg = small_cfg(n_tasks=5, inner_lr=0.3)
    model, params, sup, qry = oracle_inputs(cfg, emb_std=0.3)
    cases = {}
    for K, order in ((0, 1), (1, 2), (2, 1), (2, 2)):
        r = O.meta_step(model, params, sup, qry, cfg.inner_lr, K, order)
        cases[f"K{K}_order{order}"] = dict(
            loss=float(r["loss"]), task_loss=[float(x) for x in r["task_loss"]],
            emb_rows=[int(x) for x in r["emb_rows"]],
            emb_grad_row_sums=[float(x) for x in r["emb_grad"].sum(axis=1)],
            dW_sums=[float(w.sum()) for w in r["dW"]], dW_abs_sums=[float(abs(w).sum()) for w in r["dW"]],
            db=[[float(x) for x in b] for b in r["db"]])
    return dict(config="tests.helpers.small_cfg(n_tasks=5, inner_lr=0.3), emb_std=0.3, iteration 0", cases=cases)


if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "mini_step.json")
    with open(out, "w") as f:
        json.dump(compute(), f, indent=1)
    print("wrote", out)
