"""Operation-level scaling of the two batched primitives of Diagonal Batching (paper Section 4.1-4.2,
the figures on grouped-GEMM FLOPS vs group size and attention vs batch size), on synthetic data.

    python -m paper_2506_05229_amd.microbench gemm      [--workload 1b_128k] [--data randn|zeros] [--iters 30]
    python -m paper_2506_05229_amd.microbench attention [--workload 1b_128k] [--iters 30]
    python -m paper_2506_05229_amd.microbench head      [--workload 1b_128k] [--iters 10]
    python -m paper_2506_05229_amd.microbench orders    [--workload 1b_8k]   [--iters 5]

`gemm` times the four big linear shapes of one cell (QKV, attention output, gate/up as one N = 2 d_ff problem,
down) as one grouped launch of g = 1, 2, 4, 8, n_layers groups, every group with its own weight, through the
library's armt_grouped_gemm entry point (plain store epilogue).  `--data zeros` multiplies zero matrices:
the arithmetic is the same but nothing toggles, which shows how much of the rate the chip's power limit takes
(the sustained clock under random data is lower than under constant data).
`attention` times the fused segment attention (RoPE + GQA + causal softmax) for g = 1 ... n_layers cells.

`head` times the final RMSNorm + linear head over the LLaMA-3 vocabulary (128256) for 1, 4 and 16 segments of rows.

`orders` is the short-input comparison behind armt_forward_auto (the 4096 - 16384-token columns of the paper's timing
tables, where its implementation is slower than its baseline): the widths of the workload with segments of 512 ...
4096 tokens and 16 or 128 memory tokens, both orders, the order the library picks, and the split-group hybrid with
groups of at most 1, 2 and 4 cells launched cell by cell; one markdown table row per case.

Everything is timed with device events after a warm-up in the same process; one JSON line per measurement.
"""
from __future__ import annotations

import argparse
import json
import sys


def _time(torch, fn, iters: int, warmup: int) -> float:
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


def _groups(n_layers: int):
    gs = [g for g in (1, 2, 4, 8) if g < n_layers]
    return gs + [n_layers]


def bench_gemm(shape, data: str, iters: int, warmup: int):
    import torch
    from . import grouped_gemm

    s = shape
    qkv = (s.n_heads + 2 * s.n_kv_heads) * s.head_dim
    kinds = [("qkv", qkv, s.d_model), ("attn_out", s.d_model, s.n_heads * s.head_dim),
             ("gate_up", 2 * s.d_ff, s.d_model), ("down", s.d_model, s.d_ff)]
    gen = torch.Generator(device="cuda").manual_seed(0)

    def mat(r, c, std):
        if data == "zeros":
            return torch.zeros(r, c, device="cuda", dtype=torch.bfloat16)
        return (torch.randn(r, c, device="cuda", generator=gen) * std).to(torch.bfloat16)

    for name, N, K in kinds:
        for g in _groups(s.n_layers):
            a = [mat(s.T, K, 1.0) for _ in range(g)]
            b = [mat(N, K, 0.02) for _ in range(g)]
            out = [torch.empty(s.T, N, device="cuda", dtype=torch.bfloat16) for _ in range(g)]
            ws = torch.empty(max(256, g * 128), dtype=torch.uint8, device="cuda")
            ms = _time(torch, lambda: grouped_gemm(a, b, out, ws), iters, warmup)
            print(json.dumps({"op": "grouped_gemm", "kind": name, "data": data, "groups": g, "M": s.T, "N": N, "K": K,
                              "ms": round(ms, 4), "tflops": round(2.0 * g * s.T * N * K / ms / 1e9, 1)}), flush=True)
            del a, b, out


def bench_attention(shape, iters: int, warmup: int):
    import torch
    from . import ArmtSteps

    s = shape
    steps = ArmtSteps(s)
    width = (s.n_heads + 2 * s.n_kv_heads) * s.head_dim
    gen = torch.Generator(device="cuda").manual_seed(0)
    for g in _groups(s.n_layers):
        src = torch.randn(g, s.T, width, device="cuda", generator=gen).to(steps.act_dtype)
        qkv = src.clone()

        def run():
            qkv.copy_(src)          # the kernel rotates q and k in place
            steps.segment_attention(qkv)

        ms_copy = _time(torch, lambda: qkv.copy_(src), iters, warmup)
        ms = _time(torch, run, iters, warmup) - ms_copy
        # causal: T (T + 1) / 2 score pairs per head, 2 matmuls of 2 dh flops each
        flops = g * s.n_heads * (s.T * (s.T + 1) / 2) * 4.0 * s.head_dim
        print(json.dumps({"op": "segment_attention", "groups": g, "T": s.T, "heads": s.n_heads, "kv_heads": s.n_kv_heads,
                          "head_dim": s.head_dim, "ms": round(ms, 4), "tflops": round(flops / ms / 1e9, 1)}), flush=True)


def bench_head(shape, iters: int, warmup: int):
    import torch
    import armt_synth as S
    from . import TokenEnds

    s = shape
    ids, E, gf, W = S.make_token_ends(s, vocab=S.LLAMA3_VOCAB, seed=0, n_tokens=s.seg_len)
    te = TokenEnds(s, E, gf, W)
    gen = torch.Generator(device="cuda").manual_seed(0)
    for segs in (1, 4, 16):
        rows = segs * s.seg_len
        h = torch.randn(rows, s.d_model, device="cuda", generator=gen).to(te.dt)
        out = torch.empty((rows, S.LLAMA3_VOCAB), dtype=torch.float32, device="cuda")
        ms = _time(torch, lambda: te.logits(h, out=out), iters, min(warmup, 5))
        print(json.dumps({"op": "lm_head", "rows": rows, "vocab": S.LLAMA3_VOCAB, "d_model": s.d_model, "ms": round(ms, 4),
                          "tflops": round(2.0 * rows * S.LLAMA3_VOCAB * s.d_model / ms / 1e9, 1)}), flush=True)
        del h, out


def bench_orders(shape, iters: int):
    import numpy as np
    import torch
    import armt_synth as S
    from . import Armt
    layers, _ = S.make_weights(shape, seed=0)
    print("| tokens | segment + memory | segments | diagonal ms | sequential ms | seq / diag | auto picks | split<=1 ms | split<=2 ms | split<=4 ms |")
    print("|---|---|---|---|---|---|---|---|---|---|")
    for n_mem in (16, 128):
        for tokens in (4096, 8192, 16384):
            for seg in (512, 1024, 2048, 4096):
                sh = shape.replace(seg_len=seg, n_mem=n_mem, n_tokens=tokens)
                model = Armt(sh, layers, S.make_weights(sh, seed=0, n_layers=0)[1])
                xd = model.embed(S.make_embeddings(sh, seed=0))
                out = model.forward(xd, diagonal=True)
                t = lambda **kw: _time(torch, lambda: model.forward(xd, out=out, **kw), iters, 1)
                d, q = t(diagonal=True), t(diagonal=False)
                model.forward(xd, diagonal="auto", out=out)
                sp = [t(split_upto=k) for k in (1, 2, 4)]
                print(f"| {tokens} | {seg} + {n_mem} | {tokens // seg} | {d:.2f} | {q:.2f} | {q / d:.2f} | "
                      f"{'diagonal' if model.order_used else 'sequential'} | " + " | ".join(f"{v:.2f}" for v in sp) + " |", flush=True)
                del model, xd, out
                torch.cuda.empty_cache()


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("op", choices=["gemm", "attention", "head", "orders"])
    ap.add_argument("--workload", default="1b_128k")
    ap.add_argument("--data", choices=["randn", "zeros"], default="randn")
    ap.add_argument("--iters", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=100)
    args = ap.parse_args(argv)
    import torch
    from armt_synth import CONFIGS

    if not torch.cuda.is_available():
        print("microbench needs the GPU: the library has no CPU path", file=sys.stderr)
        return 2
    shape = CONFIGS[args.workload]
    if shape.dtype != "bf16":
        print("microbench times the bf16 path", file=sys.stderr)
        return 2
    if args.op == "gemm":
        bench_gemm(shape, args.data, args.iters, args.warmup)
    elif args.op == "attention":
        bench_attention(shape, args.iters, args.warmup)
    elif args.op == "orders":
        bench_orders(shape, min(args.iters, 5))
    else:
        bench_head(shape, min(args.iters, 10), args.warmup)
    return 0


if __name__ == "__main__":
    sys.exit(main())
