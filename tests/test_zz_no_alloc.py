"""pisa_attention_static (the entry point for callers that cannot allocate): same output as
pisa_attention, bit for bit, on two calls in a row that share the built-in scratch array, the
second on a smaller input; and shapes beyond the array are refused before any device work."""
import ctypes

import pytest
import torch

import paper_2602_01077_amd as pisa
from workloads import WORKLOADS, make_qkv

DEV = "cuda:0"
FAKE = ctypes.c_void_p(0x1000)   # never dereferenced: validation fails first


def test_static_scratch_limit_is_enforced_on_the_host():
    lib = pisa.raw()
    big = pisa.PisaShape(batch=1, heads=64, seq_len=4096 * 64, head_dim=128, block=64, dtype=pisa.PISA_BF16,
                         scale=0.0)
    rc = lib.pisa_attention_static(ctypes.byref(big), FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 100, FAKE, None,
                                   None)
    assert rc == pisa.PISA_WORKSPACE_TOO_SMALL
    assert "pisa_attention" in pisa.last_error()
    # the paper's three bf16 shapes fit
    for name in ("flux", "wan", "hunyuan"):
        w = WORKLOADS[name]
        n = -(-w.seq_len // w.block)
        npad = -(-n // 64) * 64
        need = w.batch * w.heads * (4 * npad * w.head_dim + 4 * w.head_dim ** 2)
        if w.block == 64 and n >= 256:                   # scratch of the query-block pairing
            need += w.batch * w.heads * (4 * n * -(-n // 32) + 32 * n + 8 * -(-n // 2))
        assert need <= pisa.STATIC_SCRATCH_BYTES, name


def _case(lib, L, heads, d, block, r, dtype):
    w = WORKLOADS["flux"].with_(seq_len=L, heads=heads, head_dim=d, block=block, sparsity=r, grid=None,
                                dtype=dtype)
    q, k, v = (x.to(DEV) for x in make_qkv(w, device="cpu"))
    shape = lib.make_shape(q, block)
    ws = lib.alloc_workspace(shape, DEV)
    st = lib.block_stats(q, k, v, block, ws)
    k_top = lib.topk_count(lib.num_blocks(L, block), r)
    idx, _ = lib.select(shape, st["qbar64"], st["kbar64"], k_top, ws, want_gap=False)
    ref = torch.empty_like(q)
    ref_lse = torch.empty(q.shape[:3], dtype=torch.float32, device=DEV)
    lib.attention(shape, q, k, v, st["kbar"], st["vsum"], st["hsum"], idx, k_top, out=ref, lse=ref_lse,
                  workspace=ws)
    out = torch.full_like(q, float("nan"))
    lse = torch.full_like(ref_lse, float("nan"))
    lib.attention_static(shape, q, k, v, st["kbar"], st["vsum"], st["hsum"], idx, k_top, out=out, lse=lse)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16) if out.dtype == torch.bfloat16 else out.view(torch.int32),
                       ref.view(torch.int16) if ref.dtype == torch.bfloat16 else ref.view(torch.int32)), \
        f"L={L} d={d} block={block}: outputs differ"
    assert torch.equal(lse.view(torch.int32), ref_lse.view(torch.int32))


@pytest.mark.gpu
def test_static_scratch_matches_workspace_call_twice(lib):
    # two calls in a row on the same device array, the second with a smaller input
    _case(lib, L=5000, heads=3, d=128, block=64, r=0.8, dtype="bf16")
    _case(lib, L=1111, heads=2, d=128, block=64, r=0.7, dtype="bf16")
    # other instantiations that use the scratch, and the fp32 path (needs none)
    _case(lib, L=2000, heads=2, d=64, block=128, r=0.75, dtype="bf16")
    _case(lib, L=700, heads=2, d=64, block=64, r=0.75, dtype="fp32")
