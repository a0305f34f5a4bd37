"""Writes tests/golden/1b_32k_oracle_samples.npz: the float64 oracle on ALL 32 segments of the `1b_32k` workload
(16 layers at LLaMA-3.2-1B width, 32768 tokens), reduced to what a parity test at that length needs.

Calls only `oracle/` and the seeded input generators; nothing here comes from the HIP path.  About 12 minutes on 8
cores (68 TFLOP in float64), which is why the result is stored instead of recomputed by the GPU tests.

    python tests/golden/make_1b_32k_oracle_samples.py

Stored, per segment s = 0..31: the hidden states of the last layer at ROWS_PER_SEGMENT sampled token rows (the first,
the last and seeded random ones; float32), and the Frobenius norm of the whole segment's hidden states; after segments
8, 16 and 32: z of every layer (full) and A at sampled rows of every layer.  The segments are run one at a time with
the memory state carried over, which the oracle's pins show to be bit-identical to one long run.
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import armt_synth as S                      # noqa: E402
from oracle import armt_oracle as O         # noqa: E402

WORKLOAD = "1b_32k"
ROWS_PER_SEGMENT = 16
A_ROWS_PER_LAYER = 16
STATE_AFTER = (8, 16, 32)
OUT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "1b_32k_oracle_samples.npz")


def sample_rows(shape, s):
    """Token rows of segment s whose hidden states are stored: 0, seg_len - 1 and seeded random ones."""
    rng = np.random.default_rng([32768, 7, s])
    extra = rng.choice(np.arange(1, shape.seg_len - 1), size=ROWS_PER_SEGMENT - 2, replace=False)
    return np.sort(np.concatenate([[0, shape.seg_len - 1], extra])).astype(np.int32)


def sample_a_rows(shape):
    rng = np.random.default_rng([32768, 8])
    return np.sort(rng.choice(shape.d_model, size=A_ROWS_PER_LAYER, replace=False)).astype(np.int32)


def main():
    shape = S.get_shape(WORKLOAD)
    layers, mem_emb = S.make_weights(shape, seed=0)
    layers = [{k: v.astype(np.float64) for k, v in lw.items()} for lw in layers]
    Sg, N = shape.seg_len, shape.n_segments
    a_rows = sample_a_rows(shape)
    out = {"rows": np.stack([sample_rows(shape, s) for s in range(N)]), "a_rows": a_rows,
           "mem_k_scale": np.float64(shape.mem_k_scale), "mem_v_scale": np.float64(shape.mem_v_scale),
           "hidden_rows": np.empty((N, ROWS_PER_SEGMENT, shape.d_model), np.float32),
           "hidden_fro": np.empty(N, np.float64)}
    A = z = None
    t0 = time.time()
    for s in range(N):
        xs = S.make_embeddings(shape, seed=0, n_tokens=(s + 1) * Sg)[s * Sg:]
        h, A, z = O.armt_forward_sequential(shape, layers, mem_emb, xs, A_in=A, z_in=z)
        out["hidden_rows"][s] = h[out["rows"][s]].astype(np.float32)
        out["hidden_fro"][s] = np.linalg.norm(h)
        if s + 1 in STATE_AFTER:
            out[f"z_after_{s + 1}"] = z.astype(np.float32)
            out[f"A_rows_after_{s + 1}"] = A[:, a_rows, :].astype(np.float32)
        print(f"segment {s}: hidden rms {np.sqrt(np.mean(h * h)):.4f}, |A| {np.linalg.norm(A):.4g}, "
              f"|z| {np.linalg.norm(z):.4g}, {time.time() - t0:.0f} s", flush=True)
    np.savez_compressed(OUT, **out)
    print("wrote", OUT, os.path.getsize(OUT), "bytes")


if __name__ == "__main__":
    main()
