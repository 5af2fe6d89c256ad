"""The five synthetic MAML-DLRM workloads (click-log shaped), as plain data.

Nothing here computes anything of the method: this module only names shapes,
sizes and distributions.  Both the CPU oracle's tests and the HIP path's tests
and benchmark build their inputs from these descriptions.

Model shape follows the paper's description of a Meta DLRM (Section 2.1: a huge
embedding layer xi plus small dense layers theta); the concrete sizes are the
benchmark's, not the paper's (the paper gives none for its in-house model).
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Tuple


@dataclass(frozen=True)
class Config:
    name: str
    n_tasks: int
    n_fields: int
    rows_per_field: int          # every table of a config has the same row count
    emb_dim: int
    layer_dims: Tuple[int, ...]  # d_0 .. d_L with d_0 = F*D + n_dense, d_L = 1
    bag_max: int                 # bag lengths uniform in 1..bag_max
    zipf_s: float                # 0.0 -> uniform indices
    n_support: int               # fixed per-task size; ignored when lognormal
    n_query: int
    inner_steps: int
    order: int
    inner_lr: float = 0.01
    n_dense: int = 13
    mlp_dtype: int = 0           # 0 = fp32 GEMMs, 1 = bf16 operands + fp32 accumulate
    lognormal_sizes: bool = False  # task sizes ~ logN(median, sigma), support:query 1:1
    size_median: int = 64
    size_sigma: float = 1.0
    size_max: int = 2048
    n_private_fields: int = 0    # first fields draw uniformly from a per-task row block
    label_rate: float = 0.2
    seed: int = 0

    def __post_init__(self):
        assert self.layer_dims[0] == self.n_fields * self.emb_dim + self.n_dense
        assert self.layer_dims[-1] == 1

    @property
    def total_rows(self) -> int:
        return self.n_fields * self.rows_per_field

    def with_(self, **kw) -> "Config":
        return replace(self, **kw)


TINY = Config(
    name="c1_tiny", n_tasks=4, n_fields=8, rows_per_field=1000, emb_dim=16,
    layer_dims=(141, 64, 32, 1), bag_max=1, zipf_s=0.0, n_support=32, n_query=32,
    inner_steps=1, order=2)

SMALL = Config(
    name="c2_small", n_tasks=64, n_fields=26, rows_per_field=100_000, emb_dim=32,
    layer_dims=(845, 256, 128, 1), bag_max=8, zipf_s=1.05, n_support=128, n_query=128,
    inner_steps=1, order=2)

MEDIUM = Config(
    name="c3_medium", n_tasks=512, n_fields=26, rows_per_field=1_000_000, emb_dim=64,
    layer_dims=(1677, 512, 256, 1), bag_max=20, zipf_s=1.1, n_support=256, n_query=256,
    inner_steps=3, order=2, mlp_dtype=1)

COLDSTART = Config(
    name="c4_coldstart", n_tasks=2048, n_fields=40, rows_per_field=4_000_000, emb_dim=64,
    layer_dims=(2573, 1024, 512, 256, 1), bag_max=10, zipf_s=1.2, n_support=32, n_query=32,
    inner_steps=2, order=2, mlp_dtype=1, lognormal_sizes=True, size_median=64,
    size_sigma=1.0, size_max=2048, n_private_fields=4)

LARGE = Config(
    name="c5_large", n_tasks=8192, n_fields=64, rows_per_field=1 << 22, emb_dim=64,
    layer_dims=(4109, 1024, 512, 256, 1), bag_max=32, zipf_s=1.05, n_support=512, n_query=512,
    inner_steps=1, order=2, mlp_dtype=1)

CONFIGS = {c.name: c for c in (TINY, SMALL, MEDIUM, COLDSTART, LARGE)}
# short aliases
for _c in (TINY, SMALL, MEDIUM, COLDSTART, LARGE):
    CONFIGS[_c.name.split("_")[0]] = _c
