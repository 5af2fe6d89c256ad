"""gm_meta_train: several iterations of Alg. 1 in one call, the index side of batch i+1 prepared on the second stream
while batch i computes.  Through the C ABI: parameters after n iterations equal n calls of gm_meta_train_step bit for
bit (overlapped path and the one-after-the-other fall-back), and follow the oracle's meta_train_step."""
import numpy as np
import pytest
import torch

from oracle import maml_dlrm as O
from synth import SMALL, make_batch, make_params
from synth.generate import Params, SetData
from tests.helpers import oracle_model, rel_err

pytestmark = pytest.mark.gpu


def _clone(p, dev):
    return Params(p.emb.to(dev).clone(), [w.to(dev).clone() for w in p.W], [b.to(dev).clone() for b in p.b])


def _same_params(a, b):
    assert torch.equal(a.emb, b.emb)
    for x, y in zip(a.W + a.b, b.W + b.b):
        assert torch.equal(x, y)


@pytest.mark.parametrize("bf", [0, 1], ids=["fp32", "bf16"])
@pytest.mark.parametrize("mode", ["overlapped", "fallback"])
def test_train_loop_equals_single_iterations(bf, mode):
    from paper_2401_04338_amd import GMeta
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    cfg = SMALL.with_(n_tasks=5, n_support=40, n_query=24, n_fields=6, emb_dim=32, rows_per_field=3000, bag_max=6,
                      layer_dims=(6 * 32 + 13, 64, 32, 1), inner_lr=0.05, mlp_dtype=bf)
    beta, K, order, n = 0.02, 2, 2, 5
    dev = torch.device("cuda", 0)
    params = make_params(cfg, "cpu", emb_std=0.1)
    # batches of different sizes, so that the two index arenas are reused with different layouts
    batches = []
    for it in range(n):
        c_it = cfg.with_(n_tasks=5 - (it % 3))
        s, q = make_batch(c_it, it, dev)
        batches.append((s, q))
    probe = GMeta.from_config(cfg, workspace_bytes=1 << 20)
    need = max(probe.workspace_bytes(len(s.task_offsets) - 1, s.n_samples, q.n_samples, s.nnz, q.nnz, K, order) for s, q in batches)
    probe.close()
    # overlapped: room for two index arenas; fall-back: a workspace that holds one batch and the lists only
    ws = (1 << 30) if mode == "overlapped" else int(need * 1.15) + (4 << 20)
    ctx = GMeta.from_config(cfg, workspace_bytes=ws)
    one = _clone(params, dev)
    want_losses = [float(ctx.meta_train_step(s, q, one, cfg.inner_lr, K, order, beta).item()) for s, q in batches]
    loop = _clone(params, dev)
    ctx.profile(True)
    losses = ctx.meta_train(batches, loop, cfg.inner_lr, K, order, beta)
    ctx.profile(False)
    assert ctx.iterations_done == n
    assert [float(x) for x in losses.cpu()] == want_losses
    _same_params(loop, one)
    # the oracle's training loop on its own copy (fp32 only: the bf16 reference is covered by the single-step tests)
    if not bf:
        ref = params.numpy()
        ref = dict(emb=ref["emb"].astype(np.float64), W=[w.astype(np.float64) for w in ref["W"]], b=[b.astype(np.float64) for b in ref["b"]])
        for (s, q), got in zip(batches, want_losses):
            c_it = cfg.with_(n_tasks=len(s.task_offsets) - 1)
            ref, ref_loss = O.meta_train_step(oracle_model(c_it), ref, s.numpy(), q.numpy(), cfg.inner_lr, K, order, beta)
            assert abs(got - ref_loss) <= 1e-4 * abs(ref_loss)
        moved = max(rel_err(loop.emb.cpu().numpy().astype(np.float64) - params.emb.numpy(), ref["emb"] - params.emb.numpy()))
        assert moved <= 5e-4, moved
    ctx.close()


def test_train_loop_stops_at_a_bad_batch():
    """A batch with an index outside its table in the middle of the loop: the iterations before it are applied (and
    reported), the bad one and the ones after it are not, and the error names the index."""
    from paper_2401_04338_amd import GMeta, GMetaError
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    cfg = SMALL.with_(n_tasks=4, n_support=30, n_query=20, n_fields=4, emb_dim=16, rows_per_field=500, bag_max=5,
                      layer_dims=(4 * 16 + 13, 32, 16, 1), inner_lr=0.05)
    dev = torch.device("cuda", 0)
    params = make_params(cfg, "cpu", emb_std=0.1)
    batches = [make_batch(cfg, it, dev) for it in range(4)]
    s, q = batches[2]
    bad = s.indices.clone()
    bad[7] = cfg.rows_per_field
    batches[2] = (SetData(s.task_offsets, s.bag_offsets, bad, s.dense, s.labels), q)
    ctx = GMeta.from_config(cfg, workspace_bytes=1 << 29)
    one, loop = _clone(params, dev), _clone(params, dev)
    for sb, qb in batches[:2]:
        ctx.meta_train_step(sb, qb, one, cfg.inner_lr, 1, 2, 0.05)
    with pytest.raises(GMetaError) as e:
        ctx.meta_train(batches, loop, cfg.inner_lr, 1, 2, 0.05)
    assert e.value.code == -2 and ctx.iterations_done == 2
    _same_params(loop, one)
    # the context keeps working
    ctx.meta_train(batches[:2], loop, cfg.inner_lr, 1, 2, 0.05)
    ctx.close()
