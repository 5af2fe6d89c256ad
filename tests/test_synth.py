"""The seeded generator: layout, determinism, task-subset reproducibility, distribution shape."""
import numpy as np
import torch

from synth import COLDSTART, SMALL, TINY, make_batch, make_params, task_sizes
from synth.generate import zipf_cdf


def test_layout_and_ranges():
    for cfg in (TINY, SMALL.with_(n_tasks=4)):
        sup, qry = make_batch(cfg)
        for st in (sup, qry):
            F = cfg.n_fields
            assert st.bag_offsets.numel() == st.n_samples * F + 1
            assert int(st.bag_offsets[0]) == 0 and int(st.bag_offsets[-1]) == st.nnz
            lens = torch.diff(st.bag_offsets)
            assert int(lens.min()) >= 1 and int(lens.max()) <= cfg.bag_max
            assert int(st.indices.min()) >= 0 and int(st.indices.max()) < cfg.rows_per_field
            assert st.dense.shape == (st.n_samples, cfg.n_dense)
            assert set(np.unique(st.labels.numpy())) <= {0.0, 1.0}
            assert st.indices.dtype == torch.int32 and st.bag_offsets.dtype == torch.int64


def test_deterministic_and_iteration_dependent():
    a, _ = make_batch(SMALL.with_(n_tasks=3))
    b, _ = make_batch(SMALL.with_(n_tasks=3))
    c, _ = make_batch(SMALL.with_(n_tasks=3), iteration=1)
    assert torch.equal(a.indices, b.indices) and torch.equal(a.dense, b.dense)
    assert not torch.equal(a.bag_offsets, c.bag_offsets)


def test_task_subset_reproduces_full_batch():
    cfg = SMALL.with_(n_tasks=6)
    full_s, full_q = make_batch(cfg)
    sub_s, sub_q = make_batch(cfg, tasks=[4, 1])
    F = cfg.n_fields
    for full, sub in ((full_s, sub_s), (full_q, sub_q)):
        for k, t in enumerate([4, 1]):
            lo, hi = int(full.task_offsets[t]), int(full.task_offsets[t + 1])
            slo, shi = int(sub.task_offsets[k]), int(sub.task_offsets[k + 1])
            a = full.bag_offsets[lo * F: hi * F + 1]
            b = sub.bag_offsets[slo * F: shi * F + 1]
            assert torch.equal(a - a[0], b - b[0])
            assert torch.equal(full.indices[a[0]:a[-1]], sub.indices[b[0]:b[-1]])
            assert torch.equal(full.dense[lo:hi], sub.dense[slo:shi])
            assert torch.equal(full.labels[lo:hi], sub.labels[slo:shi])


def test_chunked_generation_is_identical():
    cfg = SMALL.with_(n_tasks=5)
    a, _ = make_batch(cfg)
    b, _ = make_batch(cfg, chunk_lookups=30_000)
    assert torch.equal(a.indices, b.indices) and torch.equal(a.bag_offsets, b.bag_offsets)
    assert torch.equal(a.labels, b.labels)


def test_zipf_head_mass_and_label_rate():
    cfg = SMALL.with_(n_tasks=16)
    sup, _ = make_batch(cfg)
    cdf = zipf_cdf(cfg.rows_per_field, cfg.zipf_s)
    # field 0's lookups: share of the 100 hottest ranks close to the law's
    F = cfg.n_fields
    lens = torch.diff(sup.bag_offsets)
    field = torch.repeat_interleave(torch.arange(sup.n_samples * F) % F, lens)
    idx0 = sup.indices[field == 0].numpy()
    counts = np.sort(np.bincount(idx0, minlength=cfg.rows_per_field))[::-1]
    assert abs(counts[:100].sum() / len(idx0) - cdf[99]) < 0.03
    assert abs(float(sup.labels.mean()) - 0.2) < 0.03


def test_coldstart_sizes_and_private_rows():
    sizes = task_sizes(COLDSTART)
    tot = sizes.sum(axis=1)
    assert tot.min() >= 2 and tot.max() <= 2048 and np.all(tot % 2 == 0)
    assert 48 <= np.median(tot) <= 80
    cfg = COLDSTART.with_(rows_per_field=4096 * 16)
    sup, _ = make_batch(cfg, tasks=[5, 9])
    F = cfg.n_fields
    B = cfg.rows_per_field // cfg.n_tasks
    lens = torch.diff(sup.bag_offsets)
    bag = torch.repeat_interleave(torch.arange(sup.n_samples * F), lens)
    n5 = int(sup.task_offsets[1])
    priv = (bag % F) < cfg.n_private_fields
    rows5 = sup.indices[priv & (bag // F < n5)]
    assert int(rows5.min()) >= 5 * B and int(rows5.max()) < 6 * B


def test_params_statistics():
    p = make_params(TINY)
    assert abs(float(p.emb.std()) - 0.05) < 0.002
    assert abs(float(p.W[0].std()) * 141 ** 0.5 - 1.0) < 0.05
    assert float(p.b[0].min()) >= -0.1 and float(p.b[0].max()) <= 0.1
