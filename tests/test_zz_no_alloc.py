"""gm_meta_step_static: the step with its intermediate buffers in the library's static scratch array (for callers that
cannot allocate device memory), through the C ABI, against gm_meta_step on the same inputs: two calls in a row, the
second with a smaller input, then a call that does not fit."""
import numpy as np
import pytest
import torch

from synth import SMALL, make_batch, make_params

pytestmark = pytest.mark.gpu


def _same(a, b, n_tasks):
    n = int(a["n_emb_rows"].item())
    assert n == int(b["n_emb_rows"].item()) and n > 0
    assert torch.equal(a["emb_rows"][:n], b["emb_rows"][:n])            # integers: bit-exact
    # same kernels, same launch shapes, one wave of tasks in both: the floats agree bit for bit as well
    assert torch.equal(a["loss"], b["loss"]) and torch.equal(a["task_loss"][:n_tasks], b["task_loss"][:n_tasks])
    assert torch.equal(a["emb_grad"][:n], b["emb_grad"][:n])
    for x, y in zip(a["dW"] + a["db"], b["dW"] + b["db"]):
        assert torch.equal(x, y)


@pytest.mark.parametrize("bf", [0, 1], ids=["fp32", "bf16"])
def test_static_scratch_step_matches_the_workspace_step(bf):
    from paper_2401_04338_amd import GMeta, GMetaError
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    dev = torch.device("cuda", 0)
    big = SMALL.with_(n_tasks=3, mlp_dtype=bf)
    small = SMALL.with_(n_tasks=2, n_support=40, n_query=24, mlp_dtype=bf)
    params = make_params(big, dev)
    ctx = GMeta.from_config(big, workspace_bytes=1 << 30)
    for cfg in (big, small):                       # the second call is smaller and sees the first call's leftovers
        print("static scratch:", cfg.n_tasks, "tasks, bf16 =", bf, flush=True)
        sup, qry = make_batch(cfg, 0, dev)
        assert ctx.workspace_bytes(cfg.n_tasks, sup.n_samples, qry.n_samples, sup.nnz, qry.nnz, 2, 2) < (64 << 20)
        want = ctx.meta_step(sup, qry, params, cfg.inner_lr, 2, 2)
        out = ctx.alloc_outputs(cfg.n_tasks, int(want["capacity"]))
        got = ctx.meta_step(sup, qry, params, cfg.inner_lr, 2, 2, out=out, static_scratch=True)
        _same(got, want, cfg.n_tasks)
    # a batch whose batch-level buffers exceed the array is refused, and the context keeps working
    sup, qry = make_batch(SMALL, 0, dev)
    with pytest.raises(GMetaError) as e:
        ctx.meta_step(sup, qry, params, 0.01, 1, 2, static_scratch=True)
    assert e.value.code == -4 and "static scratch" in str(e.value)
    sup, qry = make_batch(small, 0, dev)
    _same(ctx.meta_step(sup, qry, params, small.inner_lr, 1, 2, static_scratch=True),
          ctx.meta_step(sup, qry, params, small.inner_lr, 1, 2), small.n_tasks)
    ctx.close()
