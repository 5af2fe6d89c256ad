"""Seeded, counter-based generator of synthetic click-log-shaped MAML batches.

Serves both the CPU oracle's tests and the HIP path's tests/benchmark; holds
none of the method's arithmetic (no pooling, no MLP, no gradients).  Every
random value is a pure function of (seed, stream name, iteration, element
counter), so a subset of tasks regenerates exactly the values the full batch
holds for those tasks, and integer outputs are identical on CPU and GPU
tensors (all integer decisions are taken on exact integers or on float64
values that are products of exact integers and powers of two, compared against
a cumulative table that is always built on the host).

Layout produced (the boundary's layout): per set (support / query)
  task_offsets [T+1]            int64, host (numpy)   sample range of each task
  bag_offsets  [n_samples*F+1]  int64   lookups of bag (sample s, field f) are
                                        indices[bag_offsets[s*F+f] : bag_offsets[s*F+f+1]]
  indices      [nnz]            int32   row within its field's table
  dense        [n_samples, 13]  float32
  labels       [n_samples]      float32 in {0,1}
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

from .configs import Config

_M64 = (1 << 64) - 1
_GOLD = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB
_UID_STRIDE = 1 << 16          # max samples of one task in one set


def _s64(x: int) -> int:
    """Unsigned 64-bit constant as the signed Python int torch.int64 wants."""
    x &= _M64
    return x - (1 << 64) if x >= (1 << 63) else x


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical right shift of an int64 tensor."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def mix64(c: torch.Tensor) -> torch.Tensor:
    """A 64-bit finalizer (xor-shift-multiply) on wrapping int64 arithmetic."""
    z = c
    z = (z ^ _lsr(z, 30)) * _s64(_C1)
    z = (z ^ _lsr(z, 27)) * _s64(_C2)
    return z ^ _lsr(z, 31)


def _mix64_py(z: int) -> int:
    z &= _M64
    z = ((z ^ (z >> 30)) * _C1) & _M64
    z = ((z ^ (z >> 27)) * _C2) & _M64
    return z ^ (z >> 31)


def stream_key(seed: int, name: str, iteration: int = 0) -> int:
    """Key of an independent random stream."""
    k = _mix64_py(seed * _GOLD + 0x243F6A8885A308D3)
    for ch in name.encode():
        k = _mix64_py(k * 31 + ch + 1)
    k = _mix64_py(k ^ ((iteration + 1) * _GOLD))
    return k


def bits(key: int, counters: torch.Tensor) -> torch.Tensor:
    return mix64(counters * _s64(_GOLD) + _s64(key))


def uniform(key: int, counters: torch.Tensor) -> torch.Tensor:
    """float64 in [0,1), exact (53 random bits times 2^-53)."""
    return _lsr(bits(key, counters), 11).to(torch.float64) * (2.0 ** -53)


def normal(key: int, counters: torch.Tensor) -> torch.Tensor:
    """Standard normal (Box-Muller on two uniforms of the same stream), float64."""
    u1 = uniform(key, counters * 2)
    u2 = uniform(key, counters * 2 + 1)
    r = torch.sqrt(-2.0 * torch.log(1.0 - u1))
    return r * torch.cos((2.0 * math.pi) * u2)


# ----------------------------------------------------------------------------
# task sizes
# ----------------------------------------------------------------------------
def task_sizes(cfg: Config) -> np.ndarray:
    """[T, 2] int64: (support, query) samples of every task (iteration independent)."""
    T = cfg.n_tasks
    if not cfg.lognormal_sizes:
        return np.tile(np.array([[cfg.n_support, cfg.n_query]], dtype=np.int64), (T, 1))
    z = normal(stream_key(cfg.seed, "task_size"), torch.arange(T, dtype=torch.int64)).numpy()
    n = np.exp(math.log(cfg.size_median) + cfg.size_sigma * z)
    n = 2 * np.rint(n / 2.0).astype(np.int64)          # even, split 1:1
    n = np.clip(n, 2, cfg.size_max)
    half = n // 2
    return np.stack([half, half], axis=1).astype(np.int64)


# ----------------------------------------------------------------------------
# index distributions
# ----------------------------------------------------------------------------
_CDF_CACHE: Dict[tuple, np.ndarray] = {}


def zipf_cdf(R: int, s: float) -> np.ndarray:
    """Cumulative table of the bounded Zipf law P(rank k) ~ k^-s, k = 1..R (host, float64)."""
    key = (R, s)
    if key not in _CDF_CACHE:
        w = np.arange(1, R + 1, dtype=np.float64) ** (-s)
        c = np.cumsum(w)
        c /= c[-1]
        _CDF_CACHE[key] = c
    return _CDF_CACHE[key]


def field_multipliers(cfg: Config) -> np.ndarray:
    """Odd-ish multipliers A_f coprime to R: row = (rank * A_f) mod R spreads hot ranks."""
    R = cfg.rows_per_field
    out = np.zeros(cfg.n_fields, dtype=np.int64)
    for f in range(cfg.n_fields):
        a = (_mix64_py(stream_key(cfg.seed, "field_mult") + f) % max(R - 1, 1)) + 1
        while math.gcd(a, R) != 1:
            a += 1
        out[f] = a % R if R > 1 else 0
    return out


@dataclass
class SetData:
    task_offsets: np.ndarray       # host int64 [T+1]
    bag_offsets: torch.Tensor      # int64 [n_samples*F+1]
    indices: torch.Tensor          # int32 [nnz]
    dense: torch.Tensor            # float32 [n_samples, n_dense]
    labels: torch.Tensor           # float32 [n_samples]

    @property
    def n_samples(self) -> int:
        return int(self.task_offsets[-1])

    @property
    def nnz(self) -> int:
        return int(self.indices.numel())

    def numpy(self) -> Dict[str, np.ndarray]:
        return dict(task_offsets=np.asarray(self.task_offsets, dtype=np.int64),
                    bag_offsets=self.bag_offsets.cpu().numpy(),
                    indices=self.indices.cpu().numpy(),
                    dense=self.dense.cpu().numpy(),
                    labels=self.labels.cpu().numpy())


def _gen_set(cfg: Config, set_id: int, tasks: np.ndarray, sizes: np.ndarray, iteration: int,
             device, cdf_dev: Optional[torch.Tensor], mult_dev: torch.Tensor,
             chunk_lookups: int) -> SetData:
    F, Lmax, R = cfg.n_fields, cfg.bag_max, cfg.rows_per_field
    k_len = stream_key(cfg.seed, "bag_len", iteration)
    k_idx = stream_key(cfg.seed, "index", iteration)
    k_dense = stream_key(cfg.seed, "dense", iteration)
    k_lab = stream_key(cfg.seed, "label", iteration)
    n_per_task = sizes[:, set_id]
    task_offsets = np.zeros(len(tasks) + 1, dtype=np.int64)
    np.cumsum(n_per_task, out=task_offsets[1:])
    assert n_per_task.max(initial=0) <= _UID_STRIDE

    # chunk tasks so that a chunk holds at most ~chunk_lookups lookups (upper bound)
    bounds = [0]
    acc = 0
    for i, n in enumerate(n_per_task):
        acc += int(n) * F * Lmax
        if acc > chunk_lookups and i + 1 > bounds[-1]:
            bounds.append(i + 1)
            acc = 0
    if bounds[-1] != len(tasks):
        bounds.append(len(tasks))

    offs_parts: List[torch.Tensor] = []
    idx_parts: List[torch.Tensor] = []
    dense_parts: List[torch.Tensor] = []
    lab_parts: List[torch.Tensor] = []
    base = 0
    B_priv = R // cfg.n_tasks if cfg.n_private_fields else 0
    for lo, hi in zip(bounds[:-1], bounds[1:]):
        n_t = torch.as_tensor(n_per_task[lo:hi], device=device)
        t_id = torch.as_tensor(tasks[lo:hi], device=device, dtype=torch.int64)
        n_s = int(n_t.sum())
        if n_s == 0:
            continue
        task_of_s = torch.repeat_interleave(t_id, n_t)                      # [n_s]
        first = torch.repeat_interleave(torch.cumsum(n_t, 0) - n_t, n_t)
        local = torch.arange(n_s, device=device, dtype=torch.int64) - first
        uid = (task_of_s * 2 + set_id) * _UID_STRIDE + local                # [n_s]
        f_ar = torch.arange(F, device=device, dtype=torch.int64)
        bag_ctr = uid[:, None] * F + f_ar[None, :]                          # [n_s, F]
        lens = 1 + torch.floor(uniform(k_len, bag_ctr) * Lmax).to(torch.int64)
        lens = lens.clamp_(max=Lmax).reshape(-1)
        ends = torch.cumsum(lens, 0)
        nnz = int(ends[-1])
        starts = ends - lens
        bag_of = torch.repeat_interleave(torch.arange(n_s * F, device=device), lens)
        j = torch.arange(nnz, device=device, dtype=torch.int64) - starts[bag_of]
        ctr = bag_ctr.reshape(-1)[bag_of] * Lmax + j
        u = uniform(k_idx, ctr)
        f_of = bag_of % F
        if cfg.zipf_s > 0.0:
            rank = torch.searchsorted(cdf_dev, u, right=True).clamp_(max=R - 1)
            row = (rank * mult_dev[f_of]) % R
        else:
            row = torch.floor(u * R).to(torch.int64).clamp_(max=R - 1)
        if cfg.n_private_fields:
            t_of = task_of_s[bag_of // F]
            priv = t_of * B_priv + torch.floor(u * B_priv).to(torch.int64).clamp_(max=B_priv - 1)
            row = torch.where(f_of < cfg.n_private_fields, priv, row)
        idx_parts.append(row.to(torch.int32))
        offs_parts.append(starts + base)
        base += nnz
        d_ctr = uid[:, None] * cfg.n_dense + torch.arange(cfg.n_dense, device=device)[None, :]
        dense_parts.append(normal(k_dense, d_ctr).to(torch.float32))
        lab_parts.append((uniform(k_lab, uid) < cfg.label_rate).to(torch.float32))
        del bag_of, j, ctr, u, f_of, row, lens, ends, starts

    def _cat(parts, dtype, shape_tail=()):
        if not parts:
            return torch.zeros((0,) + shape_tail, dtype=dtype, device=device)
        return torch.cat(parts)

    offs = _cat(offs_parts, torch.int64)
    offs = torch.cat([offs, torch.tensor([base], dtype=torch.int64, device=device)])
    return SetData(task_offsets=task_offsets, bag_offsets=offs,
                   indices=_cat(idx_parts, torch.int32),
                   dense=_cat(dense_parts, torch.float32, (cfg.n_dense,)),
                   labels=_cat(lab_parts, torch.float32))


def make_batch(cfg: Config, iteration: int = 0, device="cpu",
               tasks: Optional[Sequence[int]] = None, chunk_lookups: int = 1 << 25):
    """(support, query) SetData for the given task ids (default: all tasks of cfg).

    Tasks are independent streams: make_batch(tasks=[3, 7]) holds exactly the
    samples tasks 3 and 7 have in the full batch of the same iteration.
    """
    device = torch.device(device)
    sizes_all = task_sizes(cfg)
    tasks_np = np.arange(cfg.n_tasks, dtype=np.int64) if tasks is None else np.asarray(tasks, dtype=np.int64)
    sizes = sizes_all[tasks_np]
    cdf_dev = None
    if cfg.zipf_s > 0.0:
        cdf_dev = torch.from_numpy(zipf_cdf(cfg.rows_per_field, cfg.zipf_s)).to(device)
    mult_dev = torch.from_numpy(field_multipliers(cfg)).to(device)
    sup = _gen_set(cfg, 0, tasks_np, sizes, iteration, device, cdf_dev, mult_dev, chunk_lookups)
    qry = _gen_set(cfg, 1, tasks_np, sizes, iteration, device, cdf_dev, mult_dev, chunk_lookups)
    return sup, qry


@dataclass
class Params:
    emb: torch.Tensor              # float32 [F*R, D], field-major
    W: List[torch.Tensor]          # W_l float32 [d_{l-1}, d_l], row-major
    b: List[torch.Tensor]          # b_l float32 [d_l]

    def numpy(self):
        return dict(emb=self.emb.cpu().numpy(), W=[w.cpu().numpy() for w in self.W],
                    b=[x.cpu().numpy() for x in self.b])


def make_params(cfg: Config, device="cpu", chunk: int = 1 << 24, emb_std: float = 0.05) -> Params:
    """Meta-parameters: xi ~ N(0, emb_std^2), W_l ~ N(0, 1/d_{l-1}), b_l ~ U(-0.1, 0.1)."""
    device = torch.device(device)
    n = cfg.total_rows * cfg.emb_dim
    emb = torch.empty(n, dtype=torch.float32, device=device)
    k = stream_key(cfg.seed, "emb")
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        c = torch.arange(lo, hi, device=device, dtype=torch.int64)
        emb[lo:hi] = (normal(k, c) * emb_std).to(torch.float32)
    W, b = [], []
    for l in range(1, len(cfg.layer_dims)):
        din, dout = cfg.layer_dims[l - 1], cfg.layer_dims[l]
        c = torch.arange(din * dout, device=device, dtype=torch.int64)
        W.append((normal(stream_key(cfg.seed, f"W{l}"), c) / math.sqrt(din)).to(torch.float32).reshape(din, dout))
        c = torch.arange(dout, device=device, dtype=torch.int64)
        b.append(((uniform(stream_key(cfg.seed, f"b{l}"), c) * 0.2) - 0.1).to(torch.float32))
    return Params(emb=emb.reshape(cfg.total_rows, cfg.emb_dim), W=W, b=b)
