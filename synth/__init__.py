"""Seeded synthetic inputs shared by the oracle's tests and the HIP path's tests."""
from .configs import CONFIGS, Config, TINY, SMALL, MEDIUM, COLDSTART, LARGE
from .generate import make_batch, make_params, task_sizes, SetData, Params
from .compact import compact_tasks

__all__ = ["CONFIGS", "Config", "TINY", "SMALL", "MEDIUM", "COLDSTART", "LARGE",
           "make_batch", "make_params", "task_sizes", "SetData", "Params", "compact_tasks"]
