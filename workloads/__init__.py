"""Seeded synthetic inputs shared by the tests, the oracle runs and the bench.

Holds no arithmetic of the attention method itself.
"""
from .synth import (WORKLOADS, Workload, make_qkv, make_qkv_batched, sweep_points,
                    torch_dtype)

__all__ = ["WORKLOADS", "Workload", "make_qkv", "make_qkv_batched", "sweep_points",
           "torch_dtype"]
