"""Host-side checks of the C ABI: the library loads, exports every declared symbol,
and rejects bad arguments before touching a device.  No GPU needed."""
import ctypes
import os
import re

import pytest

import paper_2602_01077_amd as pisa

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "pisa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pisa_[a-z_0-9]+|dense_attention)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    syms = declared_symbols()
    assert set(syms) == set(pisa.EXPORTS)
    lib = ctypes.CDLL(pisa.LIB_PATH)
    for s in syms:
        assert hasattr(lib, s), s


def test_block_and_topk_arithmetic():
    assert pisa.num_blocks(75600, 64) == 1182
    assert pisa.num_blocks(75600, 128) == 591
    assert pisa.num_blocks(0, 64) == -1
    # sparsity -> exact blocks (Implementation Details), at the benchmark shapes
    assert [pisa.topk_count(n, r) for n, r in ((16, .75), (72, .85), (1182, .85), (1861, .9), (591, .85))] \
        == [4, 11, 178, 187, 89]
    assert pisa.topk_count(16, 0.0) == 16 and pisa.topk_count(16, 1.0) == 0
    assert pisa.topk_count(16, 0.875) == 2        # 12.5 % density
    assert pisa.topk_count(-1, 0.5) == -1
    from oracle import pisa_oracle as po
    for n in (1, 7, 72, 1182, 1861):
        for r in (0, .1, .5, .75, .85, .9, .95, 1):
            assert pisa.topk_count(n, r) == po.topk_count(n, r)


def shape(**kw):
    d = dict(batch=1, heads=2, seq_len=1024, head_dim=64, block=64, dtype=pisa.PISA_FP32, scale=0.0)
    d.update(kw)
    return pisa.PisaShape(**d)


def test_workspace_bytes():
    s = shape()
    assert pisa.workspace_bytes(s) >= 2 * 16 * 16 * 8
    assert pisa.workspace_bytes(shape(head_dim=96)) == 0
    wan = shape(heads=40, seq_len=75600, head_dim=128, dtype=pisa.PISA_BF16)
    assert pisa.workspace_bytes(wan) >= 40 * 1182 * 1182 * 8


FAKE = ctypes.c_void_p(0x1000)   # never dereferenced: validation fails first


@pytest.mark.parametrize("kw,code", [
    (dict(batch=0), pisa.PISA_INVALID_ARG),
    (dict(seq_len=0), pisa.PISA_INVALID_ARG),
    (dict(block=32), pisa.PISA_INVALID_ARG),
    (dict(head_dim=96), pisa.PISA_INVALID_ARG),
    (dict(dtype=7), pisa.PISA_INVALID_ARG),
    (dict(scale=float("nan")), pisa.PISA_INVALID_ARG),
    (dict(batch=300, heads=300), pisa.PISA_UNSUPPORTED),
])
def test_bad_shapes_are_rejected(kw, code):
    lib = pisa.raw()
    s = shape(**kw)
    assert lib.dense_attention(ctypes.byref(s), FAKE, FAKE, FAKE, FAKE, None, None) == code
    assert pisa.last_error() != ""
    assert lib.pisa_attention(ctypes.byref(s), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 1, FAKE, None, FAKE, 1 << 40, None) == code
    assert lib.pisa_select(ctypes.byref(s), FAKE, FAKE, None, 1, FAKE, None, FAKE, 1 << 40, None) == code
    assert lib.pisa_block_heterogeneity(ctypes.byref(s), FAKE, FAKE, FAKE, None, 0, 1e-6, FAKE, FAKE, 1 << 40, None) == code
    assert lib.pisa_block_stats(ctypes.byref(s), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE,
                                FAKE, 1 << 40, None) == code


def test_fast_frobenius_kind_is_validated():
    lib = pisa.raw()
    bf = shape(dtype=pisa.PISA_BF16, head_dim=128)
    call = lambda s, hsum, kind: lib.pisa_block_heterogeneity(ctypes.byref(s), FAKE, FAKE, None, hsum, kind, 1e-6,
                                                              FAKE, None, 0, None)
    assert call(shape(), FAKE, pisa.PISA_NORM_FROBENIUS_FAST) == pisa.PISA_UNSUPPORTED      # fp32 inputs
    assert call(bf, None, pisa.PISA_NORM_FROBENIUS_FAST) == pisa.PISA_INVALID_ARG           # needs hsum
    assert call(bf, FAKE, 3) == pisa.PISA_INVALID_ARG
    assert call(bf, FAKE, pisa.PISA_NORM_FROBENIUS) == pisa.PISA_INVALID_ARG                # the fp64 kinds need kbar64


def test_forward_validation():
    lib = pisa.raw()
    s = shape(dtype=pisa.PISA_BF16, head_dim=128)
    need = pisa.forward_workspace_bytes(s, 4)
    # at least the intermediates of the three stages: fp32 and fp64 block means, the index rows
    assert need >= 2 * 16 * 128 * (3 * 4 + 2 * 8) + 2 * 16 * 4 * 4
    assert pisa.forward_workspace_bytes(s, 17) == 0 and pisa.forward_workspace_bytes(s, -1) == 0
    assert pisa.forward_workspace_bytes(shape(head_dim=96), 4) == 0
    assert lib.pisa_forward(ctypes.byref(s), FAKE, FAKE, FAKE, 4, FAKE, None, None, 0, None) == pisa.PISA_INVALID_ARG
    assert lib.pisa_forward(ctypes.byref(s), FAKE, FAKE, FAKE, 4, FAKE, None, FAKE, need - 1, None) \
        == pisa.PISA_WORKSPACE_TOO_SMALL
    assert lib.pisa_forward(ctypes.byref(s), FAKE, FAKE, FAKE, 17, FAKE, None, FAKE, 1 << 40, None) \
        == pisa.PISA_INVALID_ARG
    assert lib.pisa_forward(ctypes.byref(s), None, FAKE, FAKE, 4, FAKE, None, FAKE, 1 << 40, None) \
        == pisa.PISA_INVALID_ARG


def test_heads_of_two_gib_are_refused_by_the_bf16_attention():
    # the bf16 kernels address the tiles of one head with 32-bit byte offsets
    lib = pisa.raw()
    s = shape(seq_len=9_000_000, head_dim=128, dtype=pisa.PISA_BF16)
    assert lib.dense_attention(ctypes.byref(s), FAKE, FAKE, FAKE, FAKE, None, None) == pisa.PISA_UNSUPPORTED
    assert "2 GiB" in pisa.last_error()


def test_null_and_range_arguments():
    lib = pisa.raw()
    s = shape()
    assert lib.dense_attention(None, FAKE, FAKE, FAKE, FAKE, None, None) == pisa.PISA_INVALID_ARG
    assert lib.dense_attention(ctypes.byref(s), None, FAKE, FAKE, FAKE, None, None) == pisa.PISA_INVALID_ARG
    assert lib.pisa_attention(ctypes.byref(s), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 17, FAKE, None, FAKE, 1 << 40, None) \
        == pisa.PISA_INVALID_ARG
    assert "k_top" in pisa.last_error()
    assert lib.pisa_attention(ctypes.byref(s), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, 4, FAKE, None, FAKE, 1 << 40, None) \
        == pisa.PISA_INVALID_ARG
    assert lib.pisa_attention(ctypes.byref(s), FAKE, FAKE, FAKE, None, FAKE, FAKE, FAKE, 4, FAKE, None, FAKE, 1 << 40, None) \
        == pisa.PISA_INVALID_ARG          # kbar without vsum
    assert lib.pisa_attention(ctypes.byref(s), FAKE, FAKE, FAKE, None, None, None, None, 0, FAKE, None, FAKE, 1 << 40, None) \
        == pisa.PISA_INVALID_ARG          # keep-or-drop with no block kept
    assert lib.pisa_select(ctypes.byref(s), FAKE, FAKE, None, -1, FAKE, None, FAKE, 1 << 40, None) == pisa.PISA_INVALID_ARG
    assert lib.pisa_select(ctypes.byref(s), FAKE, FAKE, None, 4, FAKE, None, FAKE, 8, None) == pisa.PISA_WORKSPACE_TOO_SMALL
    assert lib.pisa_select(ctypes.byref(s), FAKE, FAKE, None, 4, FAKE, None, None, 0, None) == pisa.PISA_INVALID_ARG
    assert lib.pisa_block_stats(ctypes.byref(s), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE,
                                FAKE, 16, None) == pisa.PISA_WORKSPACE_TOO_SMALL
    assert "workspace" in pisa.last_error()
    assert lib.pisa_block_stats(ctypes.byref(s), FAKE, FAKE, FAKE, None, FAKE, FAKE, FAKE, FAKE, FAKE,
                                FAKE, 1 << 40, None) == pisa.PISA_INVALID_ARG
    assert lib.pisa_block_heterogeneity(ctypes.byref(s), FAKE, FAKE, FAKE, None, 5, 1e-6, FAKE, FAKE, 1 << 40, None) \
        == pisa.PISA_INVALID_ARG
    assert lib.pisa_block_heterogeneity(ctypes.byref(s), FAKE, FAKE, FAKE, None, 0, -1.0, FAKE, FAKE, 1 << 40, None) \
        == pisa.PISA_INVALID_ARG
    assert lib.pisa_block_heterogeneity(ctypes.byref(s), FAKE, FAKE, FAKE, FAKE, 1, 1e-6, FAKE, FAKE, 64, None) \
        == pisa.PISA_WORKSPACE_TOO_SMALL
    big = shape(seq_len=64 * 5000)
    assert lib.pisa_select(ctypes.byref(big), FAKE, FAKE, None, 4, FAKE, None, FAKE, 1 << 60, None) == pisa.PISA_UNSUPPORTED


def test_misaligned_pointers_are_rejected():
    """The kernels move 16 bytes per lane; a pointer off a 16-byte boundary is refused on the
    host, before any launch."""
    lib = pisa.raw()
    s = shape()
    odd = ctypes.c_void_p(FAKE.value + 2)
    assert lib.dense_attention(ctypes.byref(s), FAKE, odd, FAKE, FAKE, None, None) == pisa.PISA_INVALID_ARG
    assert "aligned" in pisa.last_error()
    assert lib.pisa_attention(ctypes.byref(s), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 4, odd, None, FAKE, 1 << 40,
                              None) == pisa.PISA_INVALID_ARG
    assert "aligned" in pisa.last_error()
    assert lib.pisa_select(ctypes.byref(s), FAKE, FAKE, None, 4, FAKE, None, odd, 1 << 40, None) == pisa.PISA_INVALID_ARG
    assert lib.pisa_block_stats(ctypes.byref(s), odd, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 40,
                                None) == pisa.PISA_INVALID_ARG
    assert lib.pisa_block_heterogeneity(ctypes.byref(s), FAKE, FAKE, FAKE, None, 1, 1e-6, odd, FAKE, 1 << 40, None) \
        == pisa.PISA_INVALID_ARG


def test_probe_arguments_are_checked():
    lib = pisa.raw()
    hz = ctypes.c_double(0.0)
    flop = ctypes.c_double(0.0)
    assert lib.pisa_probe_shader_clock(0.0, FAKE, ctypes.byref(hz), None) == pisa.PISA_INVALID_ARG
    assert lib.pisa_probe_shader_clock(51.0, FAKE, ctypes.byref(hz), None) == pisa.PISA_INVALID_ARG
    assert lib.pisa_probe_shader_clock(float("nan"), FAKE, ctypes.byref(hz), None) == pisa.PISA_INVALID_ARG
    assert lib.pisa_probe_shader_clock(1.0, None, ctypes.byref(hz), None) == pisa.PISA_INVALID_ARG
    assert lib.pisa_probe_shader_clock(1.0, FAKE, None, None) == pisa.PISA_INVALID_ARG
    assert lib.pisa_probe_mfma_rate(0, FAKE, 1 << 20, ctypes.byref(flop), None) == pisa.PISA_INVALID_ARG
    assert lib.pisa_probe_mfma_rate(8, FAKE, 16, ctypes.byref(flop), None) == pisa.PISA_WORKSPACE_TOO_SMALL


def test_binding_refuses_host_tensors():
    import torch
    q = torch.zeros(1, 2, 128, 64)
    with pytest.raises(ValueError):
        pisa.dense_attention(q, q, q)
