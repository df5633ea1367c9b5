"""Python binding of libpisa (piecewise sparse attention forward pass, MI355X).

Argument marshalling only: every step runs in the HIP kernels of libpisa.so.
torch supplies device memory and the stream.  Importing this package loads the
shared library and raises if it has not been built (`python -m
paper_2602_01077_amd.build`); there is no fallback path of any kind.
"""
from __future__ import annotations

import ctypes
import math
import os
from typing import Optional, Tuple

import torch

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG_DIR, "libpisa.so")

PISA_OK, PISA_INVALID_ARG, PISA_UNSUPPORTED, PISA_WORKSPACE_TOO_SMALL, PISA_HIP_ERROR = range(5)
PISA_FP32, PISA_BF16 = 0, 1
PISA_NORM_SPECTRAL, PISA_NORM_FROBENIUS, PISA_NORM_FROBENIUS_FAST = 0, 1, 2

EXPORTS = ("pisa_num_blocks", "pisa_topk_count", "pisa_workspace_bytes", "pisa_block_stats",
           "pisa_block_heterogeneity", "pisa_select", "pisa_attention", "pisa_attention_static",
           "pisa_forward_workspace_bytes", "pisa_forward", "dense_attention",
           "pisa_probe_mfma_rate", "pisa_probe_shader_clock", "pisa_last_error")


class PisaShape(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("heads", ctypes.c_int32), ("seq_len", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("block", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("scale", ctypes.c_float)]


class PisaError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"libpisa error {code}: {message}")
        self.code = code
        self.message = message


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python paper_2602_01077_amd/build.py` "
            "(there is no fallback implementation)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    shp = ctypes.POINTER(PisaShape)
    lib.pisa_num_blocks.argtypes = [i32, i32]
    lib.pisa_num_blocks.restype = i32
    lib.pisa_topk_count.argtypes = [i32, ctypes.c_double]
    lib.pisa_topk_count.restype = i32
    lib.pisa_workspace_bytes.argtypes = [shp]
    lib.pisa_workspace_bytes.restype = sz
    lib.pisa_block_stats.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.pisa_block_stats.restype = i32
    lib.pisa_block_heterogeneity.argtypes = [shp, vp, vp, vp, vp, i32, ctypes.c_double, vp, vp, sz, vp]
    lib.pisa_block_heterogeneity.restype = i32
    lib.pisa_select.argtypes = [shp, vp, vp, vp, i32, vp, vp, vp, sz, vp]
    lib.pisa_select.restype = i32
    lib.pisa_attention.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, sz, vp]
    lib.pisa_attention.restype = i32
    lib.pisa_attention_static.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp]
    lib.pisa_attention_static.restype = i32
    lib.pisa_forward_workspace_bytes.argtypes = [shp, i32]
    lib.pisa_forward_workspace_bytes.restype = sz
    lib.pisa_forward.argtypes = [shp, vp, vp, vp, i32, vp, vp, vp, sz, vp]
    lib.pisa_forward.restype = i32
    lib.dense_attention.argtypes = [shp, vp, vp, vp, vp, vp, vp]
    lib.dense_attention.restype = i32
    lib.pisa_probe_mfma_rate.argtypes = [i32, vp, sz, ctypes.POINTER(ctypes.c_double), vp]
    lib.pisa_probe_mfma_rate.restype = i32
    lib.pisa_probe_shader_clock.argtypes = [ctypes.c_double, vp, ctypes.POINTER(ctypes.c_double), vp]
    lib.pisa_probe_shader_clock.restype = i32
    lib.pisa_last_error.argtypes = []
    lib.pisa_last_error.restype = ctypes.c_char_p
    return lib


_lib = _load()


def raw() -> ctypes.CDLL:
    """The ctypes handle, for tests that call the C ABI with hand-made arguments."""
    return _lib


def last_error() -> str:
    return _lib.pisa_last_error().decode()


def _check(code: int) -> None:
    if code != PISA_OK:
        raise PisaError(code, last_error())


def num_blocks(seq_len: int, block: int) -> int:
    return _lib.pisa_num_blocks(seq_len, block)


def topk_count(n_blocks: int, sparsity: float) -> int:
    return _lib.pisa_topk_count(n_blocks, float(sparsity))


def resolved_scale(head_dim: int, scale: Optional[float] = None) -> float:
    """The fp32 softmax scale the library uses (as a Python float)."""
    s = 1.0 / math.sqrt(head_dim) if scale is None or scale <= 0 else scale
    return float(torch.tensor(s, dtype=torch.float32).item())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return PISA_FP32
    if t.dtype == torch.bfloat16:
        return PISA_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def make_shape(q: torch.Tensor, block: int, scale: Optional[float] = None) -> PisaShape:
    if q.dim() != 4:
        raise ValueError("expected [batch, heads, seq_len, head_dim]")
    b, h, L, d = q.shape
    return PisaShape(b, h, L, d, block, _dtype_code(q), 0.0 if scale is None else float(scale))


def _dev(t: Optional[torch.Tensor], name: str, dtype=None, like: Optional[torch.Tensor] = None):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    if like is not None and (t.dtype != like.dtype or t.shape != like.shape or t.device != like.device):
        raise ValueError(f"{name} must match q in shape, dtype and device")
    return ctypes.c_void_p(t.data_ptr())


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def workspace_bytes(shape: PisaShape) -> int:
    return int(_lib.pisa_workspace_bytes(ctypes.byref(shape)))


def alloc_workspace(shape: PisaShape, device) -> torch.Tensor:
    return torch.empty(max(1, workspace_bytes(shape)), dtype=torch.uint8, device=device)


def block_stats(q, k, v, block: int, workspace: Optional[torch.Tensor] = None):
    """pisa_block_stats.  Returns dict(qbar, kbar, vsum, hsum, qbar64, kbar64)."""
    shape = make_shape(q, block)
    b, h, L, d = q.shape
    n = num_blocks(L, block)
    dev = q.device
    out = dict(
        qbar=torch.empty(b, h, n, d, dtype=torch.float32, device=dev),
        kbar=torch.empty(b, h, n, d, dtype=torch.float32, device=dev),
        vsum=torch.empty(b, h, n, d, dtype=torch.float32, device=dev),
        hsum=torch.empty(b, h, d, d, dtype=torch.float32, device=dev),
        qbar64=torch.empty(b, h, n, d, dtype=torch.float64, device=dev),
        kbar64=torch.empty(b, h, n, d, dtype=torch.float64, device=dev),
    )
    ws = alloc_workspace(shape, dev) if workspace is None else workspace
    block_stats_into(shape, q, k, v, out, ws)
    return out


def block_stats_into(shape, q, k, v, out: dict, workspace: torch.Tensor) -> None:
    _check(_lib.pisa_block_stats(
        ctypes.byref(shape), _dev(q, "q"), _dev(k, "k", like=q), _dev(v, "v", like=q),
        _dev(out["qbar"], "qbar", torch.float32), _dev(out["kbar"], "kbar", torch.float32),
        _dev(out["vsum"], "vsum", torch.float32), _dev(out["hsum"], "hsum", torch.float32),
        _dev(out["qbar64"], "qbar64", torch.float64), _dev(out["kbar64"], "kbar64", torch.float64),
        _dev(workspace, "workspace"), workspace.numel() * workspace.element_size(), _stream()))


def block_heterogeneity(shape: PisaShape, k, v, kbar64, norm: int = PISA_NORM_SPECTRAL, eps: float = 1e-6,
                        workspace: Optional[torch.Tensor] = None, hsum: Optional[torch.Tensor] = None
                        ) -> torch.Tensor:
    """pisa_block_heterogeneity.  Returns log(M_j + eps), fp64 [b,h,N].  hsum (fp32, from
    block_stats) lets the library take Hbar from it instead of accumulating it again in fp64."""
    b, h = k.shape[0], k.shape[1]
    n = num_blocks(shape.seq_len, shape.block)
    log_m = torch.empty(b, h, n, dtype=torch.float64, device=k.device)
    ws = alloc_workspace(shape, k.device) if workspace is None else workspace
    _check(_lib.pisa_block_heterogeneity(
        ctypes.byref(shape), _dev(k, "k"), _dev(v, "v", like=k), _dev(kbar64, "kbar64", torch.float64),
        _dev(hsum, "hsum", torch.float32), norm, float(eps), _dev(log_m, "log_m", torch.float64),
        _dev(ws, "workspace"), ws.numel() * ws.element_size(), _stream()))
    return log_m


def select(shape: PisaShape, qbar64, kbar64, k_top: int, workspace: Optional[torch.Tensor] = None,
           want_gap: bool = True, col_bias: Optional[torch.Tensor] = None
           ) -> Tuple[torch.Tensor, Optional[torch.Tensor]]:
    """pisa_select.  Returns (idx int32 [b,h,N,k_top], kth_gap fp32 [b,h,N] or None)."""
    b, h, n, _ = qbar64.shape
    dev = qbar64.device
    idx = torch.empty(b, h, n, k_top, dtype=torch.int32, device=dev)
    gap = torch.empty(b, h, n, dtype=torch.float32, device=dev) if want_gap else None
    ws = alloc_workspace(shape, dev) if workspace is None else workspace
    select_into(shape, qbar64, kbar64, k_top, idx, gap, ws, col_bias)
    return idx, gap


def select_into(shape, qbar64, kbar64, k_top: int, idx, gap, workspace, col_bias=None) -> None:
    _check(_lib.pisa_select(
        ctypes.byref(shape), _dev(qbar64, "qbar64", torch.float64), _dev(kbar64, "kbar64", torch.float64),
        _dev(col_bias, "col_bias", torch.float64), k_top, _dev(idx, "idx", torch.int32) if k_top > 0 else None, _dev(gap, "kth_gap", torch.float32),
        _dev(workspace, "workspace"), workspace.numel() * workspace.element_size(), _stream()))


def attention(shape: PisaShape, q, k, v, kbar, vsum, hsum, idx, k_top: int,
              out: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None,
              want_lse: bool = False, workspace: Optional[torch.Tensor] = None):
    """pisa_attention.  Returns (out, lse or None)."""
    if workspace is None:
        workspace = alloc_workspace(shape, q.device)
    if out is None:
        out = torch.empty_like(q)
    if lse is None and want_lse:
        lse = torch.empty(q.shape[:3], dtype=torch.float32, device=q.device)
    _check(_lib.pisa_attention(
        ctypes.byref(shape), _dev(q, "q"), _dev(k, "k", like=q), _dev(v, "v", like=q),
        _dev(kbar, "kbar", torch.float32), _dev(vsum, "vsum", torch.float32),
        _dev(hsum, "hsum", torch.float32),
        _dev(idx, "idx", torch.int32) if k_top > 0 else None, k_top,
        _dev(out, "out", like=q), _dev(lse, "lse", torch.float32),
        _dev(workspace, "workspace"), workspace.numel() * workspace.element_size(), _stream()))
    return out, lse


STATIC_SCRATCH_BYTES = 40 << 20


def attention_static(shape: PisaShape, q, k, v, kbar, vsum, hsum, idx, k_top: int,
                     out: torch.Tensor, lse: Optional[torch.Tensor] = None):
    """pisa_attention_static: pisa_attention on the library's built-in scratch array; the
    caller passes every buffer (nothing is allocated here either).  Returns (out, lse)."""
    _check(_lib.pisa_attention_static(
        ctypes.byref(shape), _dev(q, "q"), _dev(k, "k", like=q), _dev(v, "v", like=q),
        _dev(kbar, "kbar", torch.float32), _dev(vsum, "vsum", torch.float32),
        _dev(hsum, "hsum", torch.float32),
        _dev(idx, "idx", torch.int32) if k_top > 0 else None, k_top,
        _dev(out, "out", like=q), _dev(lse, "lse", torch.float32), _stream()))
    return out, lse


def dense_attention(q, k, v, block: int = 64, scale: Optional[float] = None,
                    out: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None,
                    want_lse: bool = False):
    """dense_attention.  Returns (out, lse or None)."""
    shape = make_shape(q, block, scale)
    if out is None:
        out = torch.empty_like(q)
    if lse is None and want_lse:
        lse = torch.empty(q.shape[:3], dtype=torch.float32, device=q.device)
    _check(_lib.dense_attention(
        ctypes.byref(shape), _dev(q, "q"), _dev(k, "k", like=q), _dev(v, "v", like=q),
        _dev(out, "out", like=q), _dev(lse, "lse", torch.float32), _stream()))
    return out, lse


def probe_mfma_rate(iters: int, sink: torch.Tensor) -> float:
    """pisa_probe_mfma_rate: enqueues the matrix-instruction loop; returns its flop count
    (the caller times the launch)."""
    flop = ctypes.c_double(0.0)
    _check(_lib.pisa_probe_mfma_rate(iters, _dev(sink, "sink", torch.float32), sink.numel(), ctypes.byref(flop),
                                     _stream()))
    return flop.value


def probe_shader_clock(window_ms: float, counts: torch.Tensor) -> float:
    """pisa_probe_shader_clock: enqueues the clock probe on the current stream; `counts` is an
    int64 device tensor of two entries.  Returns the wall clock's rate in Hz; once the stream
    has drained, counts[0] / counts[1] * rate is the shader clock held during the window."""
    hz = ctypes.c_double(0.0)
    _check(_lib.pisa_probe_shader_clock(float(window_ms), _dev(counts, "counts", torch.int64), ctypes.byref(hz),
                                        _stream()))
    return hz.value


def forward_workspace_bytes(shape: PisaShape, k_top: int) -> int:
    return _lib.pisa_forward_workspace_bytes(ctypes.byref(shape), k_top)


def forward(shape: PisaShape, q, k, v, k_top: int, out: Optional[torch.Tensor] = None,
            lse: Optional[torch.Tensor] = None, want_lse: bool = False,
            workspace: Optional[torch.Tensor] = None):
    """pisa_forward: statistics, selection and attention in one library call (three launches on
    the bf16 path for short sequences).  Returns (out, lse or None)."""
    if out is None:
        out = torch.empty_like(q)
    if lse is None and want_lse:
        lse = torch.empty(q.shape[:3], dtype=torch.float32, device=q.device)
    if workspace is None:
        workspace = torch.empty(forward_workspace_bytes(shape, k_top), dtype=torch.uint8, device=q.device)
    _check(_lib.pisa_forward(
        ctypes.byref(shape), _dev(q, "q"), _dev(k, "k", like=q), _dev(v, "v", like=q), k_top,
        _dev(out, "out", like=q), _dev(lse, "lse", torch.float32),
        _dev(workspace, "workspace", torch.uint8), workspace.numel(), _stream()))
    return out, lse


def forward_in_steps(q, k, v, block: int = 64, sparsity: float = 0.85, first_order: bool = True,
                 want_lse: bool = False, approximate: bool = True, covariance_aware: bool = False,
                 norm: int = PISA_NORM_SPECTRAL, eps: float = 1e-6, scale: Optional[float] = None,
                 hbar_from_stats: bool = False):
    """The whole hot path as separate library calls: block_stats -> select -> attention (the
    variants and the covariance-aware score are options of those calls; `forward` is the one-call
    form of the default configuration).

    first_order=False gives the zeroth-order variant, approximate=False plain block-sparse
    attention over the selected blocks, covariance_aware=True adds log(M_j + eps) to the
    selection score (hbar_from_stats=True: with Hbar from the statistics' fp32 hsum).  Returns dict(out, lse, idx, kth_gap, stats, k_top, log_m).
    """
    shape = make_shape(q, block, scale)
    n = num_blocks(q.shape[2], block)
    k_top = topk_count(n, sparsity)
    ws = alloc_workspace(shape, q.device)
    stats = block_stats(q, k, v, block, ws)
    log_m = block_heterogeneity(shape, k, v, stats["kbar64"], norm, eps, ws,
                                hsum=stats["hsum"] if (hbar_from_stats or norm == PISA_NORM_FROBENIUS_FAST) else None
                                ) if covariance_aware else None
    idx, gap = select(shape, stats["qbar64"], stats["kbar64"], k_top, ws, col_bias=log_m)
    out, lse = attention(shape, q, k, v, stats["kbar"] if approximate else None,
                         stats["vsum"] if approximate else None,
                         stats["hsum"] if (first_order and approximate) else None, idx, k_top,
                         want_lse=want_lse, workspace=ws)
    return dict(out=out, lse=lse, idx=idx, kth_gap=gap, stats=stats, k_top=k_top, log_m=log_m)
