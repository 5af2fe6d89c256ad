"""The record-grouping step before the hot path (Sec. 2.2.2): oracle pins (CPU) and the C-ABI op against it (GPU)."""
import numpy as np
import pytest
import torch

from oracle import maml_dlrm as O
from synth import make_batch
from tests.helpers import small_cfg


def _stream_from_batch(cfg, it, rng, tasks=None):
    """A flat record stream whose grouping is known: the generator's (support, query) sets, task by task (support
    records first), with the batches then shuffled as a whole (Sec. 2.2.2: shuffling at batch level)."""
    sup, qry = make_batch(cfg, it, "cpu", tasks)
    s, q = sup.numpy(), qry.numpy()
    F = cfg.n_fields
    T = len(s["task_offsets"]) - 1
    recs = []   # (task, source dict, sample)
    for t in rng.permutation(T):
        for d in (s, q):
            for i in range(int(d["task_offsets"][t]), int(d["task_offsets"][t + 1])):
                recs.append((int(t), d, i))
    task = np.array([r[0] * 7 + 3 for r in recs], dtype=np.int64)          # arbitrary increasing ids
    batch_id = np.array([11 for _ in recs], dtype=np.int64)
    boff, idx, dn, lb = [0], [], [], []
    for _, d, i in recs:
        for f in range(F):
            p0, p1 = int(d["bag_offsets"][i * F + f]), int(d["bag_offsets"][i * F + f + 1])
            idx.extend(d["indices"][p0:p1].tolist())
            boff.append(len(idx))
        dn.append(d["dense"][i])
        lb.append(d["labels"][i])
    stream = dict(task=task, batch_id=batch_id, bag_offsets=np.array(boff, dtype=np.int64),
                  indices=np.array(idx, dtype=np.int32), dense=np.array(dn, dtype=np.float32), labels=np.array(lb, dtype=np.float32))
    return stream, s, q


def _same(a, b):
    for k in ("task_offsets", "bag_offsets", "indices", "dense", "labels"):
        assert np.array_equal(np.asarray(a[k]), np.asarray(b[k])), k


def test_grouping_recovers_the_generators_sets():
    """The generator's batch, flattened and shuffled at batch level, must come back exactly (tasks ascending, records in
    stream order, support first): checks keys, order, the split rule and the CSR assembly at once."""
    cfg = small_cfg(n_tasks=5, n_support=6, n_query=6)
    stream, s, q = _stream_from_batch(cfg, 0, np.random.default_rng(0))
    gs, gq = O.group_batch(cfg.n_fields, stream["task"], stream["batch_id"], stream["bag_offsets"], stream["indices"],
                           stream["dense"], stream["labels"], 1, 2)
    _same(gs, s)
    _same(gq, q)


def test_grouping_by_hand_on_a_tiny_stream():
    """Six records, one field, written out by hand: two tasks, task 5 in two batches; uneven split 2/3 -> ceil."""
    task = [5, 2, 5, 5, 2, 5]
    batch = [1, 0, 0, 1, 0, 1]
    bag_offsets = [0, 1, 3, 3, 4, 6, 7]          # bag lengths 1, 2, 0, 1, 2, 1
    indices = [10, 20, 21, 40, 50, 51, 60]
    dense = [[0.0], [1.0], [2.0], [3.0], [4.0], [5.0]]
    labels = [0, 1, 0, 1, 0, 1]
    s, q = O.group_batch(1, task, batch, bag_offsets, indices, dense, labels, 2, 3)
    # groups in (task, batch) order: (2,0): records 1,4 ; (5,0): record 2 ; (5,1): records 0,3,5
    # support sizes ceil(2*2/3)=2, ceil(1*2/3)=1, ceil(3*2/3)=2
    assert s["task_offsets"].tolist() == [0, 2, 3, 5] and q["task_offsets"].tolist() == [0, 0, 0, 1]
    assert s["bag_offsets"].tolist() == [0, 2, 4, 4, 5, 6] and s["indices"].tolist() == [20, 21, 50, 51, 10, 40]
    assert s["dense"][:, 0].tolist() == [1.0, 4.0, 2.0, 0.0, 3.0] and s["labels"].tolist() == [1, 0, 0, 0, 1]
    assert q["bag_offsets"].tolist() == [0, 1] and q["indices"].tolist() == [60] and q["labels"].tolist() == [1]


@pytest.mark.gpu
@pytest.mark.parametrize("case", ["mini", "ragged"])
def test_group_batch_op_bit_exact(case):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2401_04338_amd import GMeta
    rng = np.random.default_rng(1)
    if case == "mini":
        cfg = small_cfg(n_tasks=6, n_support=9, n_query=7, bag_max=5)
        stream, _, _ = _stream_from_batch(cfg, 0, rng)
        num, den = 9, 16
    else:
        cfg = small_cfg(n_tasks=40, n_support=33, n_query=20, n_fields=4, bag_max=7, rows_per_field=500)
        stream, _, _ = _stream_from_batch(cfg, 1, rng)
        stream["batch_id"] = rng.integers(0, 3, size=stream["task"].shape[0]).astype(np.int64)   # several batches per task
        perm = rng.permutation(stream["task"].shape[0])                                          # and no order at all
        F = cfg.n_fields
        lens = np.diff(stream["bag_offsets"]).reshape(-1, F)[perm]
        starts = stream["bag_offsets"][:-1].reshape(-1, F)[perm]
        idx = np.concatenate([stream["indices"][a:a + l] for a, l in zip(starts.ravel(), lens.ravel())]) if lens.sum() else stream["indices"][:0]
        stream = dict(task=stream["task"][perm], batch_id=stream["batch_id"][perm],
                      bag_offsets=np.concatenate([[0], np.cumsum(lens.ravel())]).astype(np.int64), indices=idx.astype(np.int32),
                      dense=stream["dense"][perm], labels=stream["labels"][perm])
        num, den = 2, 3
    ref_s, ref_q = O.group_batch(cfg.n_fields, stream["task"], stream["batch_id"], stream["bag_offsets"], stream["indices"],
                                 stream["dense"], stream["labels"], num, den)
    ctx = GMeta.from_config(cfg, workspace_bytes=1 << 28)
    dev = ctx.device
    got_s, got_q = ctx.group_batch(stream["task"], stream["batch_id"], torch.from_numpy(stream["bag_offsets"]).to(dev),
                                   torch.from_numpy(stream["indices"]).to(dev), torch.from_numpy(stream["dense"]).to(dev),
                                   torch.from_numpy(stream["labels"]).to(dev), num, den)
    _same(got_s.numpy(), ref_s)
    _same(got_q.numpy(), ref_q)
    ctx.close()
