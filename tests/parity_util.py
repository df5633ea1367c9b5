"""Helpers for the GPU-vs-oracle parity tests (error metrics, oracle drivers)."""
from __future__ import annotations

import numpy as np
import torch

from oracle import pisa_oracle as po

# Tolerances of the benchmark spec: fp32 build 1e-4, bf16 build 2e-2 with
# per-row cosine >= 0.999.  "Relative" is taken per output row, normalised by the
# row's largest reference magnitude (an elementwise ratio is unbounded near zeros).
TOL = {torch.float32: 1e-4, torch.bfloat16: 2e-2}
COS_MIN = 0.999
GAP_TOL = 1e-6          # index rows may differ only where the oracle's k-th gap is below this


def row_errors(out: np.ndarray, ref: np.ndarray):
    """(max over rows of ||d||_inf / ||ref||_inf, min over rows of cosine)."""
    out = np.asarray(out, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    num = np.abs(out - ref).max(axis=-1)
    den = np.abs(ref).max(axis=-1)
    rel = num / np.maximum(den, 1e-30)
    cos = (out * ref).sum(-1) / np.maximum(np.linalg.norm(out, axis=-1) * np.linalg.norm(ref, axis=-1), 1e-30)
    return float(rel.max()), float(cos.min())


def head_np(t: torch.Tensor, b: int, h: int) -> np.ndarray:
    return t[b, h].detach().to("cpu", torch.float64).numpy()


def compare_index_rows(idx_gpu: np.ndarray, idx_ref: np.ndarray, gap_ref: np.ndarray):
    """Returns (rows that differ at a gap >= GAP_TOL, rows that differ at a tiny gap)."""
    diff = np.any(idx_gpu != idx_ref, axis=1) if idx_ref.shape[1] else np.zeros(len(idx_ref), bool)
    hard = np.nonzero(diff & (gap_ref >= GAP_TOL))[0]
    soft = np.nonzero(diff & (gap_ref < GAP_TOL))[0]
    return hard, soft


def check_index_rows_valid(idx_gpu: np.ndarray, N: int):
    """Every row in range, strictly ascending (hence unique)."""
    if idx_gpu.shape[1] == 0:
        return
    assert idx_gpu.min() >= 0 and idx_gpu.max() < N
    assert np.all(np.diff(idx_gpu, axis=1) > 0)


def oracle_blocks(q, k, v, b, h, block, idx_row_source, scale, blocks, mode="hybrid", stats=None):
    """Oracle output rows (and lse) of the listed query blocks of one head.
    idx_row_source: [N, k] int array of selected blocks (ignored for dense)."""
    Q, K, V = head_np(q, b, h), head_np(k, b, h), head_np(v, b, h)
    return po.attention_head(Q, K, V, block, idx_row_source, scale, mode, blocks=blocks, stats=stats)


def rows_of_blocks(blocks, block, L):
    return np.concatenate([np.arange(i * block, min((i + 1) * block, L)) for i in blocks])
