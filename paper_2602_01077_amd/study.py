"""Measurement sweeps on synthetic inputs (run on the GPU machine):

    python -m paper_2602_01077_amd.study error  [--workload wan] [--heads 8]
    python -m paper_2602_01077_amd.study speed  [--lengths 4096 8192 ...]
    python -m paper_2602_01077_amd.study l2-miss-cost

`error`  normalised L1 error against the library's dense_attention,
         sum|O - O_dense| / sum|O_dense|, for the keep-or-drop, zeroth-order and hybrid
         variants over a range of densities (the quantity of the paper's ablation figure
         "Relative error with respect to dense attention", here on synthetic inputs).
`error --lengths L1 L2 ...`  the same three errors at ONE density over sequence lengths (the
         length axis of that figure): the Wan-style generator on a t x 45 x 80 latent grid cut
         to the length asked for.
`l2-miss-cost`  pisa_attention at the Wan shape on the real index sets and on lists that make
         every tile load hit L2, with the shader clock held under each.
`speed`  ms per call of dense_attention and of the whole PISA path over sequence lengths
         and densities at the paper's kernel-study shape B2-H16-D128 ("Kernel Efficiency
         Evaluation").
All print one JSON line per point.
"""
from __future__ import annotations

import argparse
import os
import json

import torch

import paper_2602_01077_amd as pisa
from workloads import WORKLOADS, make_qkv


def _time_ms(fn, iters):
    fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


def _error_row(w, q, k, v, r, row):
    dense, _ = pisa.dense_attention(q, k, v, w.block)
    den = dense.float().abs().sum().item()
    n = pisa.num_blocks(w.seq_len, w.block)
    for name, kw in (("keep_or_drop", dict(approximate=False)),
                     ("zeroth_order", dict(first_order=False)),
                     ("hybrid", dict())):
        if name == "keep_or_drop" and pisa.topk_count(n, r) == 0:
            row[name] = None
            continue
        out = pisa.forward_in_steps(q, k, v, w.block, r, **kw)["out"]
        row[name] = (out.float() - dense.float()).abs().sum().item() / den
    print(json.dumps(row), flush=True)


def error_vs_length(args):
    """Fixed density, growing length (the paper's second error plot: 20 % density).  --style wan: the
    first L tokens of a video-shaped latent grid; --style flux: 512 text tokens and a square image
    grid of about L latents."""
    r = args.sparsity[0]
    for L in args.lengths:
        if args.style == "flux":
            base = WORKLOADS["flux"]
            g = max(8, int(round(L ** 0.5)))
            w = base.with_(name=f"flux-{g}x{g}", seq_len=512 + g * g, grid=(g, g),
                           block_offset_std=args.block_offset_std, value_field=args.value_field)
            heads = list(range(0, base.heads, max(1, base.heads // args.heads)))[: args.heads]
            q, k, v = make_qkv(w, device="cuda:0", heads=heads)
        else:
            base = WORKLOADS["wan"]
            heads = list(range(0, base.heads, max(1, base.heads // args.heads)))[: args.heads]
            frames = -(-L // (45 * 80))
            w = base.with_(name=f"wan-L{L}" + ("-clustered" if args.block_offset_std > 0 else "")
                           + ("-vfield" if args.value_field > 0 else ""), seq_len=L,
                           grid=(frames, 45, 80), block_offset_std=args.block_offset_std,
                           value_field=args.value_field)
            # the generator lays the field over whole frames; the sequence is its first L tokens
            full = w.with_(seq_len=frames * 45 * 80)
            q, k, v = (x[:, :, :L].contiguous() for x in make_qkv(full, device="cuda:0", heads=heads))
        _error_row(w, q, k, v, r, {"workload": w.name, "heads": len(heads), "seq_len": w.seq_len, "block": w.block,
                                   "sparsity": r, "density": round(1 - r, 4)})


def error_study(args):
    if args.lengths:
        return error_vs_length(args)
    w = WORKLOADS[args.workload]
    heads = list(range(0, w.heads, max(1, w.heads // args.heads)))[: args.heads]
    q, k, v = make_qkv(w, device="cuda:0", heads=heads)
    dense, _ = pisa.dense_attention(q, k, v, w.block)
    den = dense.float().abs().sum().item()
    for r in args.sparsity:
        row = {"workload": w.name, "heads": len(heads), "seq_len": w.seq_len, "block": w.block,
               "sparsity": r, "density": round(1 - r, 4)}
        for name, kw in (("keep_or_drop", dict(approximate=False)),
                         ("zeroth_order", dict(first_order=False)),
                         ("hybrid", dict())):
            if name == "keep_or_drop" and pisa.topk_count(pisa.num_blocks(w.seq_len, w.block), r) == 0:
                row[name] = None
                continue
            out = pisa.forward_in_steps(q, k, v, w.block, r, **kw)["out"]
            row[name] = (out.float() - dense.float()).abs().sum().item() / den
        print(json.dumps(row), flush=True)


def speed_study(args):
    dev = torch.device("cuda:0")
    base = WORKLOADS["wan"]
    for L in args.lengths:
        w = base.with_(name=f"B2-H16-D128-L{L}", heads=16, seq_len=L, grid=None, block_offset_std=0.5)
        parts = [make_qkv(w, device=dev, batch_index=b) for b in range(2)]
        q, k, v = (torch.cat([p[i] for p in parts], dim=0).contiguous() for i in range(3))
        shape = pisa.make_shape(q, w.block)
        ws = pisa.alloc_workspace(shape, dev)
        out = torch.empty_like(q)
        dense_ms = _time_ms(lambda: pisa.dense_attention(q, k, v, w.block, out=out), args.iters)
        st = pisa.block_stats(q, k, v, w.block, ws)          # allocates the statistics tensors once
        for r in args.sparsity:
            k_top = pisa.topk_count(pisa.num_blocks(w.seq_len, w.block), r)
            idx = torch.empty(q.shape[0], q.shape[1], pisa.num_blocks(w.seq_len, w.block), k_top, dtype=torch.int32, device=dev)

            def path():
                pisa.block_stats_into(shape, q, k, v, st, ws)
                pisa.select_into(shape, st["qbar64"], st["kbar64"], k_top, idx, None, ws)
                pisa.attention(shape, q, k, v, st["kbar"], st["vsum"], st["hsum"], idx, k_top, out=out,
                               workspace=ws)

            ms = _time_ms(path, args.iters)
            fws = torch.empty(pisa.forward_workspace_bytes(shape, k_top), dtype=torch.uint8, device=dev)
            one_ms = _time_ms(lambda: pisa.forward(shape, q, k, v, k_top, out=out, workspace=fws), args.iters)
            del fws
            row = {"shape": "B2-H16-D128", "seq_len": L, "density": round(1 - r, 4), "k_top": k_top,
                   "dense_ms": round(dense_ms, 4), "pisa_ms": round(ms, 4), "speedup": round(dense_ms / ms, 3),
                   "one_call_ms": round(one_ms, 4), "one_call_speedup": round(dense_ms / one_ms, 3)}
            if args.graph:                                   # the same six launches replayed from a HIP graph
                graph = torch.cuda.CUDAGraph()
                side = torch.cuda.Stream()
                side.wait_stream(torch.cuda.current_stream())
                with torch.cuda.stream(side):
                    with torch.cuda.graph(graph, stream=side):
                        path()
                torch.cuda.current_stream().wait_stream(side)
                row["pisa_graph_ms"] = round(_time_ms(graph.replay, args.iters), 4)
            print(json.dumps(row), flush=True)


def l2_miss_cost_study(args):
    """What the L2 misses of the exact phase cost at the Wan shape: pisa_attention on the real index sets
    against the same trip mix with every workgroup on one pair of rows (the same tiles for everybody, so all
    tile loads hit L2), each with the shader clock the chip holds meanwhile (the library's clock probe on a
    second stream).  Under rocprofv3 --pmc the launches come in this order: real x (2 + reps), all-hit x (2 + reps).
    The pairing of query blocks by row overlap is switched off for this process (it would put the identical rows
    of the all-hit lists together), so both launches walk neighbour pairs."""
    os.environ["PISA_NO_PAIRING"] = "1"            # read by the library at its first attention call
    dev = torch.device("cuda:0")
    w = WORKLOADS["wan"]
    q, k, v = make_qkv(w, device=dev)
    shape = pisa.make_shape(q, w.block)
    ws = pisa.alloc_workspace(shape, dev)
    st = pisa.block_stats(q, k, v, w.block, ws)
    n = pisa.num_blocks(w.seq_len, w.block)
    k_top = pisa.topk_count(n, w.sparsity)
    idx, _ = pisa.select(shape, st["qbar64"], st["kbar64"], k_top, ws, want_gap=False)
    # mean overlap of two neighbouring rows of the real index sets -> number of unshared tiles per row
    a, b = idx[0, :, 0:n - 1:2].long(), idx[0, :, 1:n:2].long()
    hit = torch.zeros(a.shape[0], a.shape[1], n, dtype=torch.bool, device=dev).scatter_(2, a, True)
    shared = hit.gather(2, b).float().sum(dim=2).mean().item()
    pairs = int(round(k_top - shared))
    g = torch.Generator(device="cpu")
    g.manual_seed(0)
    perm = torch.randperm(n - 1, generator=g)
    row_a = torch.sort(perm[:k_top]).values
    row_b = torch.sort(torch.cat([perm[pairs:k_top], perm[k_top:k_top + pairs]])).values
    same = torch.empty(1, w.heads, n, k_top, dtype=torch.int64)
    same[:, :, 0::2] = row_a
    same[:, :, 1::2] = row_b
    same = same.to(dev).to(torch.int32).contiguous()
    out = torch.empty_like(q)
    for name, lists in (("real index sets", idx), ("same two rows for every workgroup", same)):
        run = lambda: pisa.attention(shape, q, k, v, st["kbar"], st["vsum"], st["hsum"], lists, k_top, out=out,
                                     workspace=ws)
        run()
        run()
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        counts = torch.zeros(2, dtype=torch.int64, device=dev)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.reps):
            run()
        e1.record()
        with torch.cuda.stream(side):
            hz = pisa.probe_shader_clock(8.0, counts)
        torch.cuda.synchronize()
        cyc, ticks = (int(x) for x in counts.cpu())
        ms = e0.elapsed_time(e1) / args.reps
        ghz = cyc / ticks * hz / 1e9
        print(json.dumps({"lists": name, "shared_tiles_per_pair_of_rows": round(k_top - pairs if lists is same else shared, 1),
                          "pisa_attention_ms": round(ms, 3), "shader_clock_GHz": round(ghz, 3),
                          "ms_x_GHz": round(ms * ghz, 2)}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="cmd", required=True)
    e = sub.add_parser("error")
    e.add_argument("--workload", default="wan", choices=list(WORKLOADS))
    e.add_argument("--heads", type=int, default=8)
    e.add_argument("--sparsity", type=float, nargs="+", default=[0.5, 0.75, 0.8, 0.85, 0.875, 0.9, 0.95])
    e.add_argument("--block-offset-std", type=float, default=0.0,
                   help="with --lengths: add one N(0, std^2) offset per 64-token block to q and k (the tiny "
                        "configuration's clustered keys), so that the blocks differ and the approximation terms show")
    e.add_argument("--style", choices=["wan", "flux"], default="wan",
                   help="with --lengths: which model's token layout the sequences of growing length follow")
    e.add_argument("--value-field", type=float, default=0.0,
                   help="with --lengths: v = N(0,1) + this x a smooth field of its own over the latent grid "
                        "(values that vary slowly with position, as real activations do; the default values are "
                        "pure noise, whose block means carry nothing for the approximation terms to recover)")
    e.add_argument("--lengths", type=int, nargs="+", default=None,
                   help="sweep the sequence length at the first --sparsity instead of sweeping the density")
    s = sub.add_parser("speed")
    s.add_argument("--lengths", type=int, nargs="+", default=[4096, 8192, 16384, 32768, 65536])
    s.add_argument("--sparsity", type=float, nargs="+", default=[0.3, 0.5, 0.7, 0.875])
    s.add_argument("--iters", type=int, default=5)
    s.add_argument("--graph", action="store_true", help="also time the path replayed from a captured HIP graph")
    m = sub.add_parser("l2-miss-cost")
    m.add_argument("--reps", type=int, default=6)
    args = ap.parse_args()
    {"error": error_study, "speed": speed_study, "l2-miss-cost": l2_miss_cost_study}[args.cmd](args)


if __name__ == "__main__":
    main()
