"""Seeded synthetic Q/K/V for the PISA forward pass.

This module only *draws inputs*.  It holds none of the method's arithmetic (no
block statistics, no scores, no softmax): the CPU oracle and the HIP library
both receive the tensors made here, and share nothing else.

Every element is a pure function of (seed, tensor id, head, token, channel)
through a counter-based generator (the splitmix64 finaliser applied to a
mixed counter, then Box-Muller), so any subset of heads can be produced on its
own and equals the same heads of the full tensor.  The arithmetic is written
with torch integer / fp64 ops so it runs on the host or on a device; the
transcendental functions may round differently on different devices, so a
parity test always hands the *same generated tensor* to both sides.

Workloads stand in for attention layers of the models the paper evaluates
(Experimental Setup, "Models"): FLUX.1-dev at 1024x1024, Wan2.1-14B 720p and
Hunyuan-Video 720p.  The real activations are not available; the recipe is
q,k = N(0,1) noise plus a smooth spatial(-temporal) field shared by q and k,
v = N(0,1).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Optional, Sequence, Tuple

import torch

_MASK64 = (1 << 64) - 1


def _s64(x: int) -> int:
    """Python int (mod 2^64) -> the signed value torch.int64 stores."""
    x &= _MASK64
    return x - (1 << 64) if x >= (1 << 63) else x


_C1 = _s64(0xBF58476D1CE4E5B9)
_C2 = _s64(0x94D049BB133111EB)
_GOLD = _s64(0x9E3779B97F4A7C15)


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical right shift of int64 lanes."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix(x: torch.Tensor) -> torch.Tensor:
    """splitmix64 finaliser on int64 lanes (arithmetic wraps mod 2^64)."""
    x = (x ^ _lsr(x, 30)) * _C1
    x = (x ^ _lsr(x, 27)) * _C2
    return x ^ _lsr(x, 31)


def _stream_key(seed: int, tensor_id: int, head: int) -> int:
    """Host-side 64-bit key for one (seed, tensor, head) stream."""
    def mix_int(z: int) -> int:
        z &= _MASK64
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
        return z ^ (z >> 31)
    z = mix_int(seed * 0x9E3779B97F4A7C15 + 0x1234567)
    z = mix_int(z ^ (tensor_id * 0xD1B54A32D192ED03))
    z = mix_int(z ^ (head * 0x8CB92BA72F3D8DD7))
    return z


def _uniform(key: int, counter: torch.Tensor) -> torch.Tensor:
    """fp64 uniforms in (0,1), one per int64 counter, from stream `key`."""
    bits = _mix(counter * _GOLD + _s64(key))
    return (_lsr(bits, 11).to(torch.float64) + 0.5) * (1.0 / 9007199254740992.0)


def _normal(key: int, n: int, device) -> torch.Tensor:
    """n standard normals (fp64) from stream `key` by Box-Muller on counters 2e, 2e+1."""
    e = torch.arange(n, dtype=torch.int64, device=device)
    u1 = _uniform(key, 2 * e)
    u2 = _uniform(key, 2 * e + 1)
    return torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)


# tensor ids of the independent streams
_TID_Q, _TID_K, _TID_V, _TID_FIELD, _TID_OFFSET, _TID_VFIELD = 1, 2, 3, 4, 5, 6


@dataclass(frozen=True)
class Workload:
    """One attention-layer shape plus the recipe for its inputs."""
    name: str
    batch: int
    heads: int
    seq_len: int
    head_dim: int
    dtype: str                      # "fp32" | "bf16"
    block: int
    sparsity: float
    seed: int
    grid: Optional[Tuple[int, ...]] = None   # latent grid of the field-carrying tokens
    grid_start: int = 0             # first token of the grid; others are plain N(0,1)
    block_offset_std: float = 0.0   # config "tiny": shared per-block offset on q and k
    field_terms: int = 4
    field_fmax: float = 0.2
    value_field: float = 0.0        # > 0: v also carries a smooth field of its own, scaled by this (error studies)

    def with_(self, **kw) -> "Workload":
        d = dict(self.__dict__)
        d.update(kw)
        return Workload(**d)


WORKLOADS = {
    # small case the oracle finishes in seconds
    "tiny": Workload("tiny", 1, 2, 1024, 64, "fp32", 64, 0.75, seed=0, block_offset_std=0.5),
    # 512 text tokens, then 64x64 image latents (row-major)
    "flux": Workload("flux", 1, 24, 4608, 128, "bf16", 64, 0.85, seed=1,
                     grid=(64, 64), grid_start=512),
    # 21x45x80 video latents, t-major (headline)
    "wan": Workload("wan", 1, 40, 75600, 128, "bf16", 64, 0.85, seed=2,
                    grid=(21, 45, 80), grid_start=0),
    # 33x45x80 video latents, then 256 text tokens
    "hunyuan": Workload("hunyuan", 1, 24, 119056, 128, "bf16", 64, 0.90, seed=3,
                        grid=(33, 45, 80), grid_start=0),
}


def torch_dtype(name: str) -> torch.dtype:
    return {"fp32": torch.float32, "bf16": torch.bfloat16}[name]


def _field(w: Workload, head: int, device, tid: int = _TID_FIELD) -> Optional[torch.Tensor]:
    """[L, d] fp64 smooth field for one head (zero on non-grid tokens), or None."""
    if w.grid is None:
        return None
    d, L = w.head_dim, w.seq_len
    n_grid = 1
    for g in w.grid:
        n_grid *= g
    assert w.grid_start + n_grid <= L
    naxes = len(w.grid)
    key = _stream_key(w.seed, tid, head)
    # per (channel, term): naxes frequencies then one phase
    per = naxes + 1
    cnt = torch.arange(d * w.field_terms * per, dtype=torch.int64, device=device)
    u = _uniform(key, cnt).reshape(d, w.field_terms, per)
    freq = u[..., :naxes] * w.field_fmax          # cycles per grid step, per axis
    phase = u[..., naxes] * (2.0 * math.pi)
    t = torch.arange(n_grid, dtype=torch.int64, device=device)
    coords = []
    rem = t
    for g in reversed(w.grid):                    # last axis varies fastest
        coords.append((rem % g).to(torch.float64))
        rem = rem // g
    coords = coords[::-1]
    out = torch.zeros(L, d, dtype=torch.float64, device=device)
    acc = torch.zeros(n_grid, d, dtype=torch.float64, device=device)
    for m in range(w.field_terms):
        arg = phase[:, m].unsqueeze(0).expand(n_grid, d).clone()
        for a in range(naxes):
            arg += (2.0 * math.pi) * coords[a].unsqueeze(1) * freq[:, m, a].unsqueeze(0)
        acc += torch.sin(arg)
    out[w.grid_start:w.grid_start + n_grid] = acc
    return out


def _block_offsets(w: Workload, head: int, device) -> Optional[torch.Tensor]:
    if w.block_offset_std <= 0.0:
        return None
    n, d = -(-w.seq_len // w.block), w.head_dim      # one offset vector per run of `block` tokens
    key = _stream_key(w.seed, _TID_OFFSET, head)
    off = _normal(key, n * d, device).reshape(n, d) * w.block_offset_std
    return off.repeat_interleave(w.block, dim=0)[: w.seq_len]


def make_qkv(w: Workload, device="cpu", heads: Optional[Sequence[int]] = None,
             batch_index: int = 0):
    """Return (q, k, v), each [1, len(heads), L, d] in the workload's dtype.

    `heads` selects global head numbers (default: all); `batch_index` offsets
    the stream so that different batch entries differ.
    """
    heads = list(range(w.heads)) if heads is None else list(heads)
    dt = torch_dtype(w.dtype)
    L, d = w.seq_len, w.head_dim
    q = torch.empty(1, len(heads), L, d, dtype=dt, device=device)
    k = torch.empty_like(q)
    v = torch.empty_like(q)
    for slot, h in enumerate(heads):
        hh = h + batch_index * w.heads
        shared = _field(w, hh, device)
        off = _block_offsets(w, hh, device)
        vfield = _field(w, hh, device, _TID_VFIELD) if w.value_field > 0.0 else None
        for tid, dst in ((_TID_Q, q), (_TID_K, k), (_TID_V, v)):
            x = _normal(_stream_key(w.seed, tid, hh), L * d, device).reshape(L, d)
            if tid != _TID_V:
                if shared is not None:
                    x = x + shared
                if off is not None:
                    x = x + off
            elif vfield is not None:
                x = x + w.value_field * vfield
            dst[0, slot] = x.to(dt)
    return q, k, v


def make_qkv_batched(w: Workload, device="cpu"):
    """Full [batch, heads, L, d] tensors for workloads with batch > 1."""
    parts = [make_qkv(w, device=device, batch_index=b) for b in range(w.batch)]
    return tuple(torch.cat([p[i] for p in parts], dim=0) for i in range(3))


def sweep_points():
    """(block, sparsity) points of the sparsity / block-size sweep at the Wan shape."""
    return [(64, 0.0), (64, 0.5), (64, 0.75), (64, 0.85), (64, 0.95), (128, 0.85)]
