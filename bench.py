#!/usr/bin/env python3
"""Headline benchmark: ARMT forward with Diagonal Batching on one MI355X.

One "step" is one whole forward pass (every cell of every segment: associative read, decoder block,
memory update) over one synthetic sequence that is already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 1b_128k] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_PEAK_TFLOPS = 2500.0          # MI355X dense bf16 matrix-core peak (published)
HBM_PEAK_GBPS = 8000.0             # MI355X HBM3E peak (published)
# HBM traffic of the gate/up GEMM comes from the rocprofv3 --pmc summary of this kernel build, if one is committed:
# a line "hbm_bytes_per_cell = <number>" in this file (FETCH_SIZE + WRITE_SIZE per dispatch, each scaled by what the
# same counter reads for a plain copy kernel of known size, divided by the cells of the dispatch).
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "gate_up_gemm_1b_128k_hbm_traffic.md")
# the other configurations the benchmark spec names, reported in `configs` next to the headline workload
OTHER_CONFIGS = ("1b_8k", "1b_32k", "1b_128k_s512", "1b_128k_s2048", "3b_128k")


def measured_traffic_per_cell():
    """(bytes per cell, kernel build tag) from the committed counter summary, or (None, None)."""
    import re
    try:
        text = open(TRAFFIC_PROFILE).read()
    except OSError:
        return None, None
    m = re.search(r"hbm_bytes_per_cell\s*=\s*([0-9.eE+]+)", text)
    t = re.search(r"kernel_build\s*=\s*(\S+)", text)
    return (float(m.group(1)) if m else None), (t.group(1) if t else None)


def cpu_baseline(shape, layers, mem_emb, x, n_seg):
    """The oracle as it stands, timed on this machine's host cores on the first n_seg segments."""
    import numpy as np
    from oracle import armt_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count() or 1])
    except Exception:
        cores = os.cpu_count() or 1
    n_tok = n_seg * shape.seg_len
    t0 = time.perf_counter()
    O.armt_forward_sequential(shape, layers, mem_emb, x[:n_tok])
    dt = time.perf_counter() - t0
    return {"value": n_tok / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"first {n_seg} segments ({n_tok} tokens) of the same workload, float64 numpy, {dt:.1f} s"}


def memory_op_bytes(shape):
    """Algorithmic bytes per cell of the kernels of the associative memory (Eq. 3-6): every operand read or written once."""
    d, P, T, dm, m = shape.d_model, shape.phi, shape.T, shape.d_mem, shape.n_mem
    e = 2 if shape.dtype == "bf16" else 4
    shadow = d * P * 2 if shape.dtype == "bf16" else 0
    return {
        "delta_rule": ("delta rule, one pass over A (Eq. 5): A read and written in fp32, its bf16 copy written, "
                       "values v and features phi(k) read", 2 * d * P * 4 + shadow + m * (d + dm) * 4 + m * P * 4),
        "dpfp_read": ("phi(W_Q x) and 1 / (z.phi + eps) of the T rows (Eq. 6): q read (or produced in the same kernel), "
                      "phi and the row scale written", T * dm * 4 + T * P * e + T * 4 + P * 4),
        "mem_q": ("W_Q projection of the T rows: x and W_Q read, q written", T * d * e + dm * d * e + T * dm * 4),
        "mem_q_fused": ("W_Q projection of the T rows with phi(q) and 1 / (z.phi + eps) as its epilogue (Eq. 6): x and W_Q "
                        "read, phi and the row scale written", T * d * e + dm * d * e + T * P * e + T * 4 + P * 4),
        "mem_read": ("read GEMM A phi with residual epilogue: phi, A (bf16 copy) and the fp32 residual stream read; residual "
                     "stream and the operand of the next norm written", T * P * e + d * P * e + 2 * T * d * 4 + T * d * e),
        "mem_kv": ("W_K | W_V projections of the memory rows: rows and weights read, k | v written",
                   m * d * e + (dm + d) * d * e + m * (dm + d) * 4),
        "update_prep": ("phi(k), beta, gamma, 1 / (z.phi + eps) of the memory rows (Eq. 3-4)",
                        m * (dm + d) * 4 + m * d * e + d * e + P * 4 + m * P * 4 + m * 16),
    }


def other_config(name, base_shape, base_layers, steps=2):
    """Diagonal and sequential tokens/s and the matrix-core fractions of another named workload.  The 1B workloads share
    their weights with the headline one (same seed, same widths) up to the power of two on W_K^mem."""
    import numpy as np
    import torch
    import armt_synth as S
    import paper_2506_05229_amd as P
    shape = S.get_shape(name)
    same = all(getattr(shape, f) == getattr(base_shape, f) for f in
               ("n_layers", "d_model", "n_heads", "n_kv_heads", "head_dim", "d_ff", "n_mem", "d_mem", "mem_v_scale", "dtype"))
    if same:
        ratio = np.float32(shape.mem_k_scale / base_shape.mem_k_scale)
        layers = [dict(lw, wm_k=lw["wm_k"] * ratio) for lw in base_layers] if ratio != 1.0 else base_layers
        mem_emb = S.make_weights(shape, seed=0, n_layers=0)[1]
    else:
        layers, mem_emb = S.make_weights(shape, seed=0)
    model = P.Armt(shape, layers, mem_emb)
    xd = model.embed(S.make_embeddings(shape, seed=0))
    out = model.forward(xd, diagonal=True)
    torch.cuda.synchronize()

    def run(diagonal, n, profile=None):
        model.forward(xd, diagonal=diagonal, out=out)
        torch.cuda.synchronize()
        if profile:
            P.profile_begin(profile, n * (shape.n_layers + shape.n_segments))
        t0 = time.perf_counter()
        for _ in range(n):
            model.forward(xd, diagonal=diagonal, out=out)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / n
        return dt, (P.profile_end() if profile else None)

    dt, (k_ms, k_launches, k_groups) = run(True, steps, "gate_up")
    dts, _ = run(False, 1)
    finite = bool(torch.isfinite(out[0].float()).all())
    flops = shape.flops_total()
    gu = 2.0 * shape.T * shape.d_model * 2 * shape.d_ff * k_groups / (k_ms / 1e3) / 1e12 if k_launches else None
    del model, xd, out
    torch.cuda.empty_cache()
    return {"workload": S.describe_workload(shape), "tokens": shape.n_tokens, "steps": steps,
            "diagonal_tokens_per_s": shape.n_tokens / dt, "sequential_tokens_per_s": shape.n_tokens / dts,
            "speedup_vs_sequential": dts / dt, "mfma_fraction_end_to_end": flops / dt / 1e12 / MFMA_PEAK_TFLOPS,
            "gate_up_gemm_tflops": gu, "gate_up_gemm_frac": None if gu is None else gu / MFMA_PEAK_TFLOPS,
            "outputs_finite": finite}


def C_byref(x):
    import ctypes
    return ctypes.byref(x)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="1b_128k")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sequential", action="store_true")
    ap.add_argument("--batch", type=int, default=1,
                    help="B independent sequences per call (default 1 = the headline metric); tokens/s counts all B")
    ap.add_argument("--no-lm-head", action="store_true",
                    help="skip the extra timing of the token-level ends (embedding gather, final norm + head)")
    ap.add_argument("--cpu-segments", type=int, default=4)
    ap.add_argument("--no-train", action="store_true",
                    help="skip the training leg (forward with tape + backward pass; reported under `training`, not in `value`)")
    ap.add_argument("--no-memory-ops", action="store_true",
                    help="skip the per-kernel timing passes of the associative-memory kernels (reported under `memory_ops`)")
    ap.add_argument("--no-configs", action="store_true",
                    help="skip the short runs of the other named configurations (reported under `configs`)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain device copy of known size (the memory-state carry-in copy), so that a "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE run can be scaled against it")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import armt_synth as S
    import paper_2506_05229_amd as P

    shape = S.get_shape(args.workload)
    t_gen = time.perf_counter()
    layers, mem_emb = S.make_weights(shape, seed=0)
    x = S.make_embeddings(shape, seed=0)
    t_gen = time.perf_counter() - t_gen
    model = P.Armt(shape, layers, mem_emb)
    B = max(1, args.batch)
    if B == 1:
        xd = model.embed(x)
        fwd = model.forward
    else:       # sequence b = the embeddings of seed b
        xd = model.embed(np.stack([x] + [S.make_embeddings(shape, seed=b) for b in range(1, B)]))
        fwd = model.forward_batched
    out = fwd(xd, diagonal=True)            # allocates the outputs once
    torch.cuda.synchronize()

    def timed(diagonal, steps, warmup, profile=None):
        for _ in range(warmup):
            fwd(xd, diagonal=diagonal, out=out)
        torch.cuda.synchronize()
        if profile:
            P.profile_begin(profile, steps * (shape.n_layers + shape.n_segments))
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for _ in range(steps):
            fwd(xd, diagonal=diagonal, out=out)
        e1.record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) / steps
        prof = P.profile_end() if profile else None
        return e0.elapsed_time(e1) / steps, wall * 1e3, prof

    ms, wall_ms, prof = timed(True, args.steps, args.warmup, profile="gate_up")
    n_tok = shape.n_tokens * B
    total_flops = shape.flops_total() * B
    res = {
        "metric": "ARMT forward tokens/s, Diagonal Batching, 131072 tokens" if (n_tok == 131072 and B == 1)
                  else f"ARMT forward tokens/s, Diagonal Batching, {B} x {shape.n_tokens} tokens",
        "value": n_tok / (wall_ms / 1e3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall_ms, "gpu_ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": shape.dtype, "data": "synthetic",
        "config": {"workload": S.describe_workload(shape, batch=B, seed=0),
                   "mem_k_scale": shape.mem_k_scale, "mem_v_scale": shape.mem_v_scale,
                   "cells": shape.n_layers * shape.n_segments * B,
                   "diagonal_steps": shape.n_layers + shape.n_segments - 1,
                   "algorithmic_tflop": total_flops / 1e12},
        "mfma_fraction_end_to_end": total_flops / (ms / 1e3) / 1e12 / MFMA_PEAK_TFLOPS,
        "outputs_finite": bool(torch.isfinite(out[0].float()).all() and torch.isfinite(out[1]).all()),
        "hidden_rms_first_last_segment": [float(out[0][..., :shape.seg_len, :].float().pow(2).mean().sqrt()),
                                          float(out[0][..., -shape.seg_len:, :].float().pow(2).mean().sqrt())],
    }
    # roofline of the dominant kernel: the gate/up grouped GEMM with the SwiGLU epilogue
    k_ms, k_launches, k_groups = prof
    traffic_cell, traffic_build = measured_traffic_per_cell()
    if k_launches:
        flops_per_cell = 2.0 * shape.T * shape.d_model * 2 * shape.d_ff
        per_launch = flops_per_cell * k_groups / k_launches
        achieved = per_launch / (k_ms / k_launches / 1e3) / 1e12
        res["roofline"] = {"kernel": "gemm_mfma_kernel<..., EPI_SWIGLU> (gate/up grouped GEMM + SiLU*up)",
                           "bound": "mfma", "achieved": achieved, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                           "frac": achieved / MFMA_PEAK_TFLOPS,
                           "traffic": (traffic_cell * k_groups / k_launches
                                       if traffic_cell and shape.name.startswith("1b_") and shape.seg_len == 1024 else None),
                           "traffic_unit": "bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE per dispatch, calibrated "
                                           f"against a copy kernel; from profiles/{os.path.basename(TRAFFIC_PROFILE)}, "
                                           f"kernel build {traffic_build})",
                           "algorithmic_bytes_per_launch": (2 * shape.d_ff * shape.d_model * 2 + shape.T * shape.d_model * 2
                                                            + shape.T * shape.d_ff * 2) * k_groups / k_launches,
                           "avg_launch_ms": k_ms / k_launches, "launches": k_launches,
                           "avg_groups_per_launch": k_groups / k_launches,
                           "algorithmic_gflop_per_launch": per_launch / 1e9}
    if not args.no_sequential:
        sms, swall, _ = timed(False, max(1, min(args.steps, 2)), 1)      # one warm-up pass: one-off costs of its tile configurations
        res["sequential_tokens_per_s"] = n_tok / (swall / 1e3)
        res["speedup_vs_sequential"] = swall / wall_ms
    if B == 1 and not args.no_memory_ops:
        # Kernels of the associative memory: HIP-event time of each over one more pass (one kind per pass), against the
        # bytes each must move at least.  The 16 A matrices of the 1B shape (50 MB) fit the chip's last-level cache, so
        # "achieved" is a rate against the HBM peak, not a claim that the bytes came from HBM.
        mem = {}
        op_bytes = memory_op_bytes(shape)
        for kind in ("dpfp_read", "mem_q", "mem_read", "mem_kv", "update_prep", "delta_rule"):
            what, cell_bytes = op_bytes[kind]
            if kind == "mem_q" and "dpfp_read" not in mem:       # no separate feature-map launch: it is the epilogue
                what, cell_bytes = op_bytes["mem_q_fused"]
            try:
                P.profile_begin(kind, 2 * (shape.n_layers + shape.n_segments))
            except Exception:
                continue
            fwd(xd, diagonal=True, out=out)
            torch.cuda.synchronize()
            m_ms, m_launches, m_groups = P.profile_end()
            if not m_launches:
                continue
            per_launch = cell_bytes * m_groups / m_launches
            gbps = per_launch / (m_ms / m_launches / 1e3) / 1e9
            mem[kind] = {"what": what, "algorithmic_bytes_per_launch": per_launch, "avg_us": 1e3 * m_ms / m_launches,
                         "launches": m_launches, "avg_cells_per_launch": m_groups / m_launches,
                         "achieved_GBps": gbps, "frac_of_hbm_peak": gbps / HBM_PEAK_GBPS,
                         "share_of_pass": m_ms / ms}
        res["memory_ops"] = mem
    if not args.no_lm_head and B == 1:
        # Token-level ends of Algorithm 1 (not part of `value`, which is the headline metric on hidden states):
        # embedding gather for the whole sequence, final norm + LLaMA-3-sized head on the last segment and on
        # 16 segments, the latter extrapolated to all rows (the head's cost is linear in the rows).
        ids, E, gf, Wlm = S.make_token_ends(shape, vocab=S.LLAMA3_VOCAB, seed=0)
        te = P.TokenEnds(shape, E, gf, Wlm)
        ids_d = torch.from_numpy(ids).cuda()
        hid = out[0]

        def ev(fn, reps=3):
            fn()
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(reps):
                fn()
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) / reps

        ms_embed = ev(lambda: te.embed(ids_d))
        rows_big = min(16 * shape.seg_len, n_tok)
        lg_last = torch.empty((shape.seg_len, S.LLAMA3_VOCAB), dtype=torch.float32, device="cuda")
        lg_big = torch.empty((rows_big, S.LLAMA3_VOCAB), dtype=torch.float32, device="cuda")
        ms_last = ev(lambda: te.logits(hid[-shape.seg_len:], out=lg_last))
        ms_big = ev(lambda: te.logits(hid[:rows_big], out=lg_big))
        fl = lambda r: 2.0 * r * S.LLAMA3_VOCAB * shape.d_model
        ms_all = ms_big * n_tok / rows_big
        res["token_ends"] = {
            "vocab": S.LLAMA3_VOCAB, "embed_ms_all_tokens": ms_embed,
            "lm_head_last_segment_ms": ms_last, "lm_head_last_segment_tflops": fl(shape.seg_len) / ms_last / 1e9,
            "lm_head_rows_timed": rows_big, "lm_head_ms": ms_big, "lm_head_tflops": fl(rows_big) / ms_big / 1e9,
            "tokens_per_s_ids_to_last_segment_logits": n_tok / ((wall_ms + ms_embed + ms_last) / 1e3),
            "tokens_per_s_ids_to_all_logits_extrapolated": n_tok / ((wall_ms + ms_embed + ms_all) / 1e3)}
        if not args.no_train:
            # backward of the head on the same 16 segments: d_hidden, d_gain, d_W_lm from an upstream gradient of the logits
            dl = torch.randn(lg_big.shape, device="cuda", generator=torch.Generator(device="cuda").manual_seed(2))
            grads = None
            def head_bwd():
                nonlocal grads
                out_b = te.logits_backward(hid[:rows_big], dl, grads=grads)
                grads = (out_b[1], out_b[2])
            ms_bwd = ev(head_bwd, reps=2)
            res["token_ends"]["lm_head_backward_ms"] = ms_bwd
            res["token_ends"]["lm_head_backward_tflops"] = 2.0 * fl(rows_big) / ms_bwd / 1e9
            del dl, grads
            te.bws = None
        del lg_last, lg_big, te
    if not args.no_train and P.load_library().armt_backward_workspace_bytes_batched(C_byref(model.cfg), B) > 0:
        # Training leg (outside `value`): forward that records the tape, then the backward pass in reverse diagonal
        # order, for an upstream gradient on every hidden state; one warm-up, one timed pass of each.
        gh = torch.randn(tuple(xd.shape), device="cuda", generator=torch.Generator(device="cuda").manual_seed(1)).to(model.act_dtype)
        grads, t_f, t_b, t_bs = None, 0.0, 0.0, None
        for rep in range(2):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            _, _, _, tape = model.forward_train(xd, diagonal=True)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            grads = model.backward(tape, shape.n_tokens, gh, diagonal=True, want_dx=False, grads=grads)
            torch.cuda.synchronize()
            t_f, t_b = t1 - t0, time.perf_counter() - t1
        if not args.no_sequential:
            t0 = time.perf_counter()
            model.backward(tape, shape.n_tokens, gh, diagonal=False, want_dx=False, grads=grads)
            torch.cuda.synchronize()
            t_bs = time.perf_counter() - t0
        res["training"] = {
            "forward_with_tape_ms": t_f * 1e3, "backward_ms": t_b * 1e3,
            "tokens_per_s_forward_backward": n_tok / (t_f + t_b),
            "backward_over_forward": t_b / (wall_ms / 1e3),
            "mfma_fraction_forward_backward": 4.0 * total_flops / (t_f + t_b) / 1e12 / MFMA_PEAK_TFLOPS,
            "flops_counted": "forward + recomputed forward + 2 x forward for the gradients = 4 x algorithmic forward FLOPs",
            "sequential_backward_ms": None if t_bs is None else t_bs * 1e3,
            "backward_speedup_vs_sequential": None if t_bs is None else t_bs / t_b,
            "tape_gb": tape.numel() / 1e9, "backward_workspace_gb": model.bwd_workspace.numel() / 1e9}
        del tape, grads, gh
        model.bwd_workspace = None
    if args.calibrate_copy:
        # copy_f32_kernel moves the whole memory state A_in -> A_out: n_layers * d_model * Phi floats read and written
        A_src, z_src = out[1].clone(), out[2].clone()
        model.forward(xd[:shape.seg_len].contiguous(), diagonal=True, A_in=A_src, z_in=z_src)
        torch.cuda.synchronize()
        res["calibration_copy_bytes"] = int(A_src.numel() * 4)
    if not args.no_cpu_baseline and B == 1:
        res["cpu_baseline"] = cpu_baseline(shape, layers, mem_emb, x, min(args.cpu_segments, shape.n_segments))
    if B == 1 and not args.no_configs and args.workload == "1b_128k":
        # the other named configurations, two timed passes each (not part of `value`)
        del out, xd, model, x
        torch.cuda.empty_cache()
        res["configs"] = [other_config(name, shape, layers) for name in OTHER_CONFIGS]
    res["input_generation_s"] = t_gen
    print(json.dumps(res))


if __name__ == "__main__":
    main()
