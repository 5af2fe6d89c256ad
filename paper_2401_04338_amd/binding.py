"""ctypes binding of libgmeta.so: argument marshalling only.

Every step of the MAML-DLRM path runs inside the library's HIP kernels; PyTorch
is used here for device memory (torch.empty on the GPU) and nothing else.
There is no CPU fallback: if the shared library is missing, loading fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgmeta.so")

GM_OK, GM_ERR_ARG, GM_ERR_INDEX, GM_ERR_CAPACITY, GM_ERR_WORKSPACE, GM_ERR_HIP = 0, -1, -2, -3, -4, -5

EXPORTS = ["gm_create", "gm_destroy", "gm_last_error", "gm_workspace_bytes", "gm_meta_step", "gm_meta_step_static",
           "gm_meta_train_step", "gm_meta_train_step_table", "gm_meta_train", "gm_group_batch", "gm_scatter_add", "gm_gather_pool", "gm_index_prep", "gm_configure", "gm_profile", "gm_profile_report", "gm_ceilings"]


class gm_model_desc(C.Structure):
    _fields_ = [("n_fields", C.c_int32), ("rows_per_field", C.POINTER(C.c_int64)),
                ("emb_dim", C.c_int32), ("n_dense", C.c_int32), ("n_layers", C.c_int32),
                ("layer_dims", C.POINTER(C.c_int32)), ("mlp_dtype", C.c_int32)]


class gm_set(C.Structure):
    _fields_ = [("n_samples", C.c_int64), ("nnz", C.c_int64), ("task_offsets", C.POINTER(C.c_int64)),
                ("bag_offsets", C.c_void_p), ("indices", C.c_void_p), ("dense", C.c_void_p),
                ("labels", C.c_void_p)]


class gm_params(C.Structure):
    _fields_ = [("emb", C.c_void_p), ("W", C.POINTER(C.c_void_p)), ("b", C.POINTER(C.c_void_p))]


class gm_grads(C.Structure):
    _fields_ = [("dW", C.POINTER(C.c_void_p)), ("db", C.POINTER(C.c_void_p)), ("emb_rows", C.c_void_p),
                ("emb_grad", C.c_void_p), ("n_emb_rows", C.c_void_p), ("emb_rows_capacity", C.c_int64),
                ("task_loss", C.c_void_p), ("emb_grad_table", C.c_void_p)]


class gm_set_buffers(C.Structure):
    _fields_ = [("n_samples", C.c_int64), ("nnz", C.c_int64), ("task_offsets", C.POINTER(C.c_int64)),
                ("bag_offsets", C.c_void_p), ("indices", C.c_void_p), ("dense", C.c_void_p), ("labels", C.c_void_p)]


class GMetaError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"gmeta error {code}: {msg}")
        self.code = code


_lib = None


def load_library() -> C.CDLL:
    """Loads libgmeta.so (built in-tree by paper_2401_04338_amd.build); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is not built; run `python -m paper_2401_04338_amd.build` (there is no fallback path)")
    lib = C.CDLL(LIB_PATH)
    lib.gm_create.restype = C.c_int
    lib.gm_create.argtypes = [C.POINTER(C.c_void_p), C.POINTER(gm_model_desc), C.c_int, C.c_void_p, C.c_size_t]
    lib.gm_destroy.restype = None
    lib.gm_destroy.argtypes = [C.c_void_p]
    lib.gm_last_error.restype = C.c_char_p
    lib.gm_last_error.argtypes = [C.c_void_p]
    lib.gm_workspace_bytes.restype = C.c_size_t
    lib.gm_workspace_bytes.argtypes = [C.POINTER(gm_model_desc), C.c_int32, C.c_int64, C.c_int64, C.c_int64,
                                       C.c_int64, C.c_int32, C.c_int32]
    lib.gm_group_batch.restype = C.c_int
    lib.gm_group_batch.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.c_void_p,
                                   C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.POINTER(gm_set_buffers),
                                   C.POINTER(gm_set_buffers), C.POINTER(C.c_int32)]
    lib.gm_meta_train_step.restype = C.c_int
    lib.gm_meta_train_step.argtypes = [C.c_void_p, C.c_int32, C.POINTER(gm_set), C.POINTER(gm_set), C.POINTER(gm_params),
                                       C.c_float, C.c_int32, C.c_int32, C.c_float, C.c_void_p, C.c_void_p]
    lib.gm_meta_train_step_table.restype = C.c_int
    lib.gm_meta_train_step_table.argtypes = [C.c_void_p, C.c_int32, C.POINTER(gm_set), C.POINTER(gm_set), C.POINTER(gm_params),
                                             C.c_float, C.c_int32, C.c_int32, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.gm_meta_train.restype = C.c_int
    lib.gm_meta_train.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.POINTER(gm_set), C.POINTER(gm_set),
                                  C.POINTER(gm_params), C.c_float, C.c_int32, C.c_int32, C.c_float, C.c_void_p,
                                  C.POINTER(C.c_int32)]
    lib.gm_meta_step.restype = C.c_int
    lib.gm_meta_step.argtypes = [C.c_void_p, C.c_int32, C.POINTER(gm_set), C.POINTER(gm_set),
                                 C.POINTER(gm_params), C.c_float, C.c_int32, C.c_int32, C.c_void_p,
                                 C.POINTER(gm_grads)]
    lib.gm_meta_step_static.restype = C.c_int
    lib.gm_meta_step_static.argtypes = lib.gm_meta_step.argtypes
    lib.gm_scatter_add.restype = C.c_int
    lib.gm_scatter_add.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_float]
    lib.gm_gather_pool.restype = C.c_int
    lib.gm_gather_pool.argtypes = [C.c_void_p, C.c_int32, C.POINTER(gm_set), C.c_void_p, C.c_void_p]
    lib.gm_index_prep.restype = C.c_int
    lib.gm_index_prep.argtypes = [C.c_void_p, C.c_int32, C.POINTER(gm_set), C.POINTER(gm_set)] + [C.c_void_p] * 7 + [C.c_int64]
    lib.gm_configure.restype = C.c_int
    lib.gm_configure.argtypes = [C.c_void_p, C.c_char_p, C.c_int64]
    lib.gm_profile.restype = C.c_int
    lib.gm_profile.argtypes = [C.c_void_p, C.c_int]
    lib.gm_profile_report.restype = C.c_char_p
    lib.gm_profile_report.argtypes = [C.c_void_p]
    lib.gm_ceilings.restype = C.c_int
    lib.gm_ceilings.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_double),
                                C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    _lib = lib
    return lib


def _model_desc(n_fields, rows_per_field, emb_dim, n_dense, layer_dims, mlp_dtype):
    rows = (C.c_int64 * max(n_fields, 1))(*[int(r) for r in rows_per_field])
    dims = (C.c_int32 * len(layer_dims))(*[int(d) for d in layer_dims])
    m = gm_model_desc(n_fields, rows, emb_dim, n_dense, len(layer_dims) - 1, dims, mlp_dtype)
    m._keep = (rows, dims)
    return m


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _checked(t: torch.Tensor, dtype, name: str, device=None) -> torch.Tensor:
    """The library reads raw pointers: a tensor of another type, layout or device would be misread silently."""
    if t.dtype != dtype or not t.is_contiguous() or not t.is_cuda or (device is not None and t.device != device):
        raise ValueError(f"{name} must be a contiguous {dtype} tensor on {device or 'the GPU'} "
                         f"(got {t.dtype}, contiguous={t.is_contiguous()}, device={t.device})")
    return t


def _set_struct(s, device=None) -> gm_set:
    """s: an object with task_offsets (host numpy int64), bag_offsets, indices, dense, labels (device tensors)."""
    _checked(s.bag_offsets, torch.int64, "bag_offsets", device)
    _checked(s.indices, torch.int32, "indices", device)
    _checked(s.dense, torch.float32, "dense", device)
    _checked(s.labels, torch.float32, "labels", device)
    toff = np.ascontiguousarray(np.asarray(s.task_offsets, dtype=np.int64))
    st = gm_set(int(toff[-1]), int(s.indices.numel()), toff.ctypes.data_as(C.POINTER(C.c_int64)),
                _ptr(s.bag_offsets), _ptr(s.indices), _ptr(s.dense), _ptr(s.labels))
    st._keep = (toff, s)
    return st


class GMeta:
    """One context of the library: model shape + workspace on one GPU."""

    def __init__(self, n_fields: int, rows_per_field: Sequence[int], emb_dim: int, n_dense: int,
                 layer_dims: Sequence[int], mlp_dtype: int = 0, device: int = 0,
                 workspace_bytes: int = 1 << 30, stream: Optional[int] = None):
        self.lib = load_library()
        self.n_fields, self.emb_dim, self.n_dense = n_fields, emb_dim, n_dense
        self.layer_dims = list(layer_dims)
        self.rows_per_field = list(rows_per_field)
        self.device = torch.device("cuda", device)
        self._desc = _model_desc(n_fields, rows_per_field, emb_dim, n_dense, layer_dims, mlp_dtype)
        self._ctx = C.c_void_p()
        rc = self.lib.gm_create(C.byref(self._ctx), C.byref(self._desc), device,
                                C.c_void_p(stream) if stream else None, workspace_bytes)
        if rc != GM_OK:
            msg = self.lib.gm_last_error(self._ctx).decode() if self._ctx else "gm_create failed"
            if self._ctx:
                self.lib.gm_destroy(self._ctx)
                self._ctx = C.c_void_p()
            raise GMetaError(rc, msg)

    @classmethod
    def from_config(cls, cfg, device: int = 0, workspace_bytes: int = 1 << 30, stream=None, mlp_dtype=None):
        return cls(cfg.n_fields, [cfg.rows_per_field] * cfg.n_fields, cfg.emb_dim, cfg.n_dense, cfg.layer_dims,
                   cfg.mlp_dtype if mlp_dtype is None else mlp_dtype, device, workspace_bytes, stream)

    def workspace_bytes(self, n_tasks, n_support, n_query, nnz_support, nnz_query, inner_steps, order) -> int:
        return int(self.lib.gm_workspace_bytes(C.byref(self._desc), n_tasks, n_support, n_query, nnz_support,
                                               nnz_query, inner_steps, order))

    def close(self):
        if getattr(self, "_ctx", None):
            self.lib.gm_destroy(self._ctx)
            self._ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int):
        if rc != GM_OK:
            raise GMetaError(rc, self.lib.gm_last_error(self._ctx).decode())

    def _check_params(self, params):
        L = len(self.layer_dims) - 1
        if self.n_fields > 0:
            _checked(params.emb, torch.float32, "params.emb", self.device)
            if tuple(params.emb.shape) != (int(sum(self.rows_per_field)), self.emb_dim):
                raise ValueError("params.emb must be [sum rows_per_field, emb_dim]")
        if len(params.W) != L or len(params.b) != L:
            raise ValueError("params.W / params.b must hold one tensor per layer")
        for l in range(L):
            _checked(params.W[l], torch.float32, f"params.W[{l}]", self.device)
            _checked(params.b[l], torch.float32, f"params.b[{l}]", self.device)
            if tuple(params.W[l].shape) != (self.layer_dims[l], self.layer_dims[l + 1]) or params.b[l].numel() != self.layer_dims[l + 1]:
                raise ValueError(f"layer {l}: W must be [{self.layer_dims[l]}, {self.layer_dims[l + 1]}] and b [{self.layer_dims[l + 1]}]")

    # ------------------------------------------------------------------ entry points
    def alloc_outputs(self, n_tasks: int, emb_rows_capacity: int) -> Dict[str, object]:
        dev, L = self.device, len(self.layer_dims) - 1
        return dict(
            loss=torch.empty(1, dtype=torch.float32, device=dev),
            task_loss=torch.empty(max(n_tasks, 1), dtype=torch.float32, device=dev),
            dW=[torch.empty(self.layer_dims[l], self.layer_dims[l + 1], dtype=torch.float32, device=dev) for l in range(L)],
            db=[torch.empty(self.layer_dims[l + 1], dtype=torch.float32, device=dev) for l in range(L)],
            emb_rows=torch.empty(max(emb_rows_capacity, 1), dtype=torch.int64, device=dev),
            emb_grad=torch.empty(max(emb_rows_capacity, 1), self.emb_dim, dtype=torch.float32, device=dev),
            n_emb_rows=torch.zeros(1, dtype=torch.int64, device=dev),
            capacity=emb_rows_capacity)

    def meta_step(self, support, query, params, inner_lr: float, inner_steps: int, order: int,
                  out: Optional[Dict[str, object]] = None, emb_rows_capacity: Optional[int] = None,
                  emb_grad_table: Optional[torch.Tensor] = None, static_scratch: bool = False):
        """gm_meta_step.  support/query: SetData-like; params: object with emb, W[], b[] device tensors.
        emb_grad_table: a float32 device tensor shaped like params.emb that the sparse gradient is added to
        (then no row list is produced).  static_scratch: call gm_meta_step_static instead (the library's static
        scratch array in place of the context's workspace; pass `out` to keep the call itself free of allocations)."""
        n_tasks = len(support.task_offsets) - 1
        if emb_grad_table is not None:
            if (emb_grad_table.dtype != torch.float32 or not emb_grad_table.is_contiguous()
                    or tuple(emb_grad_table.shape) != (int(sum(self.rows_per_field)), self.emb_dim)
                    or emb_grad_table.device != params.emb.device):
                raise ValueError("emb_grad_table must be a contiguous float32 [sum rows_per_field, emb_dim] device tensor")
        if out is None:
            cap = emb_rows_capacity
            if emb_grad_table is not None:
                cap = 0
            elif cap is None:
                cap = min(int(support.indices.numel() + query.indices.numel()), int(sum(self.rows_per_field)))
            out = self.alloc_outputs(n_tasks, cap)
        L = len(self.layer_dims) - 1
        ss, qs = _set_struct(support, self.device), _set_struct(query, self.device)
        self._check_params(params)
        Wp = (C.c_void_p * L)(*[w.data_ptr() for w in params.W])
        bp = (C.c_void_p * L)(*[x.data_ptr() for x in params.b])
        ps = gm_params(_ptr(params.emb), Wp, bp)
        dWp = (C.c_void_p * L)(*[w.data_ptr() for w in out["dW"]])
        dbp = (C.c_void_p * L)(*[x.data_ptr() for x in out["db"]])
        gs = gm_grads(dWp, dbp, _ptr(out["emb_rows"]), _ptr(out["emb_grad"]), _ptr(out["n_emb_rows"]),
                      int(out["capacity"]), _ptr(out["task_loss"]),
                      _ptr(emb_grad_table) if emb_grad_table is not None else None)
        entry = self.lib.gm_meta_step_static if static_scratch else self.lib.gm_meta_step
        rc = entry(self._ctx, n_tasks, C.byref(ss), C.byref(qs), C.byref(ps), float(inner_lr),
                   int(inner_steps), int(order), _ptr(out["loss"]), C.byref(gs))
        self._check(rc)
        return out

    def meta_train_step(self, support, query, params, inner_lr: float, inner_steps: int, order: int, outer_lr: float,
                        loss: Optional[torch.Tensor] = None, task_loss: Optional[torch.Tensor] = None):
        """gm_meta_train_step: the step and the outer update; params.emb / W[] / b[] are updated in place.
        Returns the device scalar holding the step's loss."""
        n_tasks = len(support.task_offsets) - 1
        L = len(self.layer_dims) - 1
        if loss is None:
            loss = torch.empty(1, dtype=torch.float32, device=self.device)
        ss, qs = _set_struct(support, self.device), _set_struct(query, self.device)
        self._check_params(params)
        Wp = (C.c_void_p * L)(*[w.data_ptr() for w in params.W])
        bp = (C.c_void_p * L)(*[x.data_ptr() for x in params.b])
        ps = gm_params(_ptr(params.emb), Wp, bp)
        rc = self.lib.gm_meta_train_step(self._ctx, n_tasks, C.byref(ss), C.byref(qs), C.byref(ps), float(inner_lr),
                                         int(inner_steps), int(order), float(outer_lr), _ptr(loss), _ptr(task_loss))
        self._check(rc)
        return loss

    def meta_train_step_table(self, support, query, params, inner_lr: float, inner_steps: int, order: int, outer_lr: float,
                              emb_grad_table: torch.Tensor, loss: Optional[torch.Tensor] = None,
                              task_loss: Optional[torch.Tensor] = None):
        """gm_meta_train_step_table: the step with the table-shaped sparse meta-gradient (all zero on entry and again on
        return) and the outer update; params.emb / W[] / b[] are updated in place.  Returns the device scalar of the loss."""
        n_tasks = len(support.task_offsets) - 1
        L = len(self.layer_dims) - 1
        if loss is None:
            loss = torch.empty(1, dtype=torch.float32, device=self.device)
        ss, qs = _set_struct(support, self.device), _set_struct(query, self.device)
        self._check_params(params)
        assert emb_grad_table.dtype == torch.float32 and emb_grad_table.is_contiguous() and emb_grad_table.shape == params.emb.shape
        Wp = (C.c_void_p * L)(*[w.data_ptr() for w in params.W])
        bp = (C.c_void_p * L)(*[x.data_ptr() for x in params.b])
        ps = gm_params(_ptr(params.emb), Wp, bp)
        rc = self.lib.gm_meta_train_step_table(self._ctx, n_tasks, C.byref(ss), C.byref(qs), C.byref(ps), float(inner_lr),
                                               int(inner_steps), int(order), float(outer_lr), _ptr(loss), _ptr(task_loss),
                                               _ptr(emb_grad_table))
        self._check(rc)
        return loss

    def meta_train(self, batches, params, inner_lr: float, inner_steps: int, order: int, outer_lr: float,
                   losses: Optional[torch.Tensor] = None):
        """gm_meta_train: one iteration per (support, query) pair of `batches`, parameters updated in place, the index
        side of each batch prepared while the previous one computes.  Returns the device tensor of the steps' losses."""
        n = len(batches)
        L = len(self.layer_dims) - 1
        if losses is None:
            losses = torch.empty(max(n, 1), dtype=torch.float32, device=self.device)
        self._check_params(params)
        sup = (gm_set * max(n, 1))()
        qry = (gm_set * max(n, 1))()
        keep = []
        nt = (C.c_int32 * max(n, 1))()
        for i, (s, q) in enumerate(batches):
            ss, qs = _set_struct(s, self.device), _set_struct(q, self.device)
            keep.append((ss, qs))
            for f, _t in gm_set._fields_:
                setattr(sup[i], f, getattr(ss, f))
                setattr(qry[i], f, getattr(qs, f))
            nt[i] = len(s.task_offsets) - 1
        Wp = (C.c_void_p * L)(*[w.data_ptr() for w in params.W])
        bp = (C.c_void_p * L)(*[x.data_ptr() for x in params.b])
        ps = gm_params(_ptr(params.emb), Wp, bp)
        done = C.c_int32(0)
        rc = self.lib.gm_meta_train(self._ctx, n, nt, sup, qry, C.byref(ps), float(inner_lr), int(inner_steps), int(order),
                                    float(outer_lr), _ptr(losses), C.byref(done))
        self.iterations_done = int(done.value)
        self._check(rc)
        return losses[:n]

    def group_batch(self, task, batch_id, bag_offsets: torch.Tensor, indices: torch.Tensor, dense: torch.Tensor,
                    labels: torch.Tensor, support_num: int, support_den: int):
        """gm_group_batch: task / batch_id host int64 arrays, the other arrays device tensors of the flat stream.
        Returns (support, query) as SetData-like objects (host task_offsets, device tensors)."""
        from types import SimpleNamespace
        task = np.ascontiguousarray(np.asarray(task, dtype=np.int64))
        batch_id = np.ascontiguousarray(np.asarray(batch_id, dtype=np.int64))
        n, nnz, F, nd = int(task.shape[0]), int(indices.numel()), self.n_fields, self.n_dense
        dev = self.device
        outs, structs, toffs = [], [], []
        for _ in range(2):
            o = dict(bag_offsets=torch.empty(n * F + 1, dtype=torch.int64, device=dev),
                     indices=torch.empty(max(nnz, 1), dtype=torch.int32, device=dev),
                     dense=torch.empty(max(n, 1), max(nd, 1), dtype=torch.float32, device=dev),
                     labels=torch.empty(max(n, 1), dtype=torch.float32, device=dev))
            toff = np.zeros(n + 1, dtype=np.int64)
            st = gm_set_buffers(0, 0, toff.ctypes.data_as(C.POINTER(C.c_int64)), _ptr(o["bag_offsets"]), _ptr(o["indices"]),
                                _ptr(o["dense"]), _ptr(o["labels"]))
            outs.append(o); structs.append(st); toffs.append(toff)
        n_tasks = C.c_int32(0)
        rc = self.lib.gm_group_batch(self._ctx, n, nnz, task.ctypes.data_as(C.POINTER(C.c_int64)),
                                     batch_id.ctypes.data_as(C.POINTER(C.c_int64)), _ptr(bag_offsets), _ptr(indices), _ptr(dense),
                                     _ptr(labels), int(support_num), int(support_den), C.byref(structs[0]), C.byref(structs[1]),
                                     C.byref(n_tasks))
        self._check(rc)
        res = []
        for o, st, toff in zip(outs, structs, toffs):
            ns, nz, T = int(st.n_samples), int(st.nnz), int(n_tasks.value)
            sd = SimpleNamespace(task_offsets=toff[: T + 1].copy(), bag_offsets=o["bag_offsets"][: ns * F + 1],
                                 indices=o["indices"][:nz], dense=o["dense"][:ns, :nd], labels=o["labels"][:ns])
            sd.numpy = (lambda d=sd: dict(task_offsets=d.task_offsets, bag_offsets=d.bag_offsets.cpu().numpy(),
                                          indices=d.indices.cpu().numpy(), dense=d.dense.cpu().numpy(),
                                          labels=d.labels.cpu().numpy()))
            res.append(sd)
        return res[0], res[1]

    def gather_pool(self, set_, emb: torch.Tensor) -> torch.Tensor:
        n_tasks = len(set_.task_offsets) - 1
        st = _set_struct(set_, self.device)
        _checked(emb, torch.float32, "emb", self.device)
        x = torch.empty(max(st.n_samples, 1), self.layer_dims[0], dtype=torch.float32, device=self.device)
        self._check(self.lib.gm_gather_pool(self._ctx, n_tasks, C.byref(st), _ptr(emb), _ptr(x)))
        return x[: st.n_samples]

    def index_prep(self, support, query, emb_rows_capacity: Optional[int] = None):
        n_tasks = len(support.task_offsets) - 1
        ss, qs = _set_struct(support, self.device), _set_struct(query, self.device)
        dev, F = self.device, self.n_fields
        cap = emb_rows_capacity
        if cap is None:
            cap = min(ss.nnz + qs.nnz, int(sum(self.rows_per_field)))
        o = dict(slot_counts=torch.zeros(max(n_tasks * F, 1), dtype=torch.int64, device=dev),
                 slot_rows=torch.zeros(max(ss.nnz, 1), dtype=torch.int64, device=dev),
                 sup_slot=torch.zeros(max(ss.nnz, 1), dtype=torch.int32, device=dev),
                 qry_slot=torch.zeros(max(qs.nnz, 1), dtype=torch.int32, device=dev),
                 emb_rows=torch.zeros(max(cap, 1), dtype=torch.int64, device=dev),
                 seg_counts=torch.zeros(max(cap, 1), dtype=torch.int64, device=dev),
                 n_emb_rows=torch.zeros(1, dtype=torch.int64, device=dev))
        rc = self.lib.gm_index_prep(self._ctx, n_tasks, C.byref(ss), C.byref(qs), _ptr(o["slot_counts"]),
                                    _ptr(o["slot_rows"]), _ptr(o["sup_slot"]), _ptr(o["qry_slot"]),
                                    _ptr(o["emb_rows"]), _ptr(o["seg_counts"]), _ptr(o["n_emb_rows"]), cap)
        self._check(rc)
        n = int(o["n_emb_rows"].item())
        ns = int(o["slot_counts"][: n_tasks * F].sum().item())
        return dict(slot_counts=o["slot_counts"][: n_tasks * F], slot_rows=o["slot_rows"][:ns],
                    sup_slot=o["sup_slot"][: ss.nnz], qry_slot=o["qry_slot"][: qs.nnz],
                    emb_rows=o["emb_rows"][:n], seg_counts=o["seg_counts"][:n])

    def configure(self, key: str, value: int):
        self._check(self.lib.gm_configure(self._ctx, key.encode(), int(value)))

    def profile(self, enable: bool):
        self._check(self.lib.gm_profile(self._ctx, 1 if enable else 0))

    def profile_report(self) -> Dict[str, Dict[str, float]]:
        """{family: {launches, ms, bytes, flops}} accumulated since profile(True)."""
        out = {}
        for line in self.lib.gm_profile_report(self._ctx).decode().splitlines():
            name, n, ms, by, fl = line.split()
            out[name] = dict(launches=int(n), ms=float(ms), bytes=float(by), flops=float(fl))
        return out

    def ceilings(self) -> Dict[str, float]:
        """gm_ceilings: streaming copy / read rates and the register-resident bf16 MFMA rate (constant operands, and
        operands that toggle like real data) measured on this GPU with the library's own kernels."""
        a, b, m, r, n = C.c_double(0), C.c_double(0), C.c_double(0), C.c_double(0), C.c_int64(0)
        self._check(self.lib.gm_ceilings(self._ctx, C.byref(a), C.byref(b), C.byref(m), C.byref(r), C.byref(n)))
        return {"copy_GBps": a.value, "read_GBps": b.value, "mfma_bf16_TFLOPs": m.value,
                "mfma_bf16_TFLOPs_toggling_operands": r.value, "copy_buffer_bytes": n.value}

    def scatter_add(self, table: torch.Tensor, rows: torch.Tensor, grad: torch.Tensor, scale: float):
        self._check(self.lib.gm_scatter_add(self._ctx, _ptr(table), _ptr(rows), _ptr(grad), int(rows.numel()),
                                            float(scale)))
