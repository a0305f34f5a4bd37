"""Conditioning of the delta rule (Eq. 3-5) on a synthetic workload -- TEST INFRASTRUCTURE, calls only the oracle.

For a LLaMA-shaped workload this script runs the float64 oracle over the first segments with the key weights
W_K^mem scaled by 2^-p, p = p_min .. p_max, and prints, per p: whether every denominator z.phi (read side and update
side) stays positive, the range of gamma (Eq. 4), the ratio |v_bar| / |v| (Eq. 4: how much of the written value
is the correction by what the memory already holds), the ratio |phi(k)|^2 / assoc_eps, the size of the memory
read relative to the row it is added to, and the rms of the hidden states per segment.  The largest scale that
keeps the recurrence well conditioned (all denominators positive, hidden rms not growing) is what the workload
table of the input generators uses; the table printed here is quoted in the design notes.

    python -m oracle.key_scale_search --workload 1b_8k --segments 8 --p-min 4 --p-max 8 [--layers 16]

Everything is computed with the oracle's own functions (dpfp, assoc_read, llama_block, assoc_update) in the
order of Section 3.1; the loop below repeats the oracle's sequential driver only to look at intermediate values.
"""
from __future__ import annotations

import argparse
import json
import sys
import time

import numpy as np

import armt_synth as S
from oracle import armt_oracle as O


def run(shape, n_segments: int, verbose: bool = True):
    """Sequential ARMT over n_segments segments with per-cell conditioning figures."""
    layers, mem_emb = S.make_weights(shape, seed=0)
    x = S.make_embeddings(shape, seed=0, n_tokens=n_segments * shape.seg_len).astype(np.float64)
    W = [{k: np.asarray(v, dtype=np.float64) for k, v in lw.items()} for lw in layers]
    mem_emb = np.asarray(mem_emb, dtype=np.float64)
    L, d, P, Sg = shape.n_layers, shape.d_model, shape.phi, shape.seg_len
    A = [np.zeros((d, P)) for _ in range(L)]
    z = [np.zeros(P) for _ in range(L)]
    empty = [True] * L
    eps, nu = shape.assoc_eps, shape.dpfp_nu
    rec = dict(min_den_read=np.inf, min_den_upd=np.inf, gamma_min=np.inf, gamma_max=-np.inf, vbar_over_v=[],
               f2_over_eps=[], read_over_x=[], hidden_rms=[], ok=True)
    for s in range(n_segments):
        U = np.concatenate([x[s * Sg:(s + 1) * Sg], mem_emb], axis=0)
        for l in range(L):
            w = W[l]
            if not empty[l]:
                f = O.dpfp(U @ w["wm_q"].T, nu)
                den = f @ z[l]
                rec["min_den_read"] = min(rec["min_den_read"], float(den.min()))
                U2 = O.assoc_read(U, A[l], z[l], w["wm_q"], eps, nu)
                rec["read_over_x"].append(float(np.linalg.norm(U2 - U) / np.linalg.norm(U)))
                U = U2
            Y = O.llama_block(U, w, shape)
            Ym = Y[Sg:]
            fk = O.dpfp(Ym @ w["wm_k"].T, nu)
            zf = fk @ z[l]
            f2 = np.sum(fk * fk, axis=-1)
            rec["f2_over_eps"].append(float(np.median(f2) / eps) if eps > 0 else float("inf"))
            if not empty[l]:
                rec["min_den_upd"] = min(rec["min_den_upd"], float(zf.min()))
                gamma = 1.0 - zf / (f2 + eps)
                rec["gamma_min"] = min(rec["gamma_min"], float(gamma.min()))
                rec["gamma_max"] = max(rec["gamma_max"], float(gamma.max()))
                v = Ym @ w["wm_v"].T
                vbar = (fk @ A[l].T) / (zf + eps)[:, None]
                rec["vbar_over_v"].append(float(np.linalg.norm(vbar) / np.linalg.norm(v)))
            A[l], z[l] = O.assoc_update(Ym, A[l], z[l], empty[l], w, eps, nu)
            empty[l] = False
            U = Y
        rms = float(np.sqrt(np.mean(U[:Sg] ** 2)))
        rec["hidden_rms"].append(rms)
        if verbose:
            print(f"    segment {s}: hidden rms {rms:.4g}, min z.phi read {rec['min_den_read']:.3g} update "
                  f"{rec['min_den_upd']:.3g}, gamma [{rec['gamma_min']:.4g}, {rec['gamma_max']:.4g}]", flush=True)
        if not np.isfinite(rms) or rms > 1e3 or rec["min_den_read"] <= 0.0 or rec["min_den_upd"] <= 0.0:
            rec["ok"] = False
            break
    return rec


def summarise(rec):
    q = lambda a: (float(np.min(a)), float(np.median(a)), float(np.max(a))) if len(a) else (None, None, None)
    return dict(ok=rec["ok"], min_den_read=rec["min_den_read"], min_den_upd=rec["min_den_upd"],
                gamma=(rec["gamma_min"], rec["gamma_max"]), vbar_over_v_min_med_max=q(rec["vbar_over_v"]),
                f2_over_eps_min_med_max=q(rec["f2_over_eps"]), read_over_x_min_med_max=q(rec["read_over_x"]),
                hidden_rms=rec["hidden_rms"])


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--workload", default="1b_8k")
    ap.add_argument("--segments", type=int, default=8)
    ap.add_argument("--layers", type=int, default=None, help="use only the first layers of the shape")
    ap.add_argument("--p-min", type=int, default=4)
    ap.add_argument("--p-max", type=int, default=8)
    ap.add_argument("--v-log2", type=int, default=None, help="log2 of the W_V^mem scale (default: the workload's)")
    ap.add_argument("--json", default=None, help="also write the table here")
    a = ap.parse_args(argv)
    shape = S.get_shape(a.workload)
    if a.layers:
        shape = shape.replace(n_layers=a.layers)
    if a.v_log2 is not None:
        shape = shape.replace(mem_v_scale=2.0 ** a.v_log2)
    table = {}
    for p in range(a.p_min, a.p_max + 1):
        t0 = time.time()
        print(f"key scale 2^-{p} (value scale {shape.mem_v_scale:g}), {shape.n_layers} layers, {a.segments} segments",
              flush=True)
        rec = summarise(run(shape.replace(mem_k_scale=2.0 ** -p), a.segments))
        rec["seconds"] = time.time() - t0
        table[p] = rec
        print(f"  -> {json.dumps(rec)}", flush=True)
    good = [p for p, r in table.items() if r["ok"]]
    print("largest well-conditioned key scale: " + (f"2^-{min(good)}" if good else "none in range"), flush=True)
    if a.json:
        with open(a.json, "w") as f:
            json.dump(table, f, indent=1)
    return 0


if __name__ == "__main__":
    sys.exit(main())
