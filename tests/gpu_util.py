"""Helpers shared by the GPU parity tests: run the HIP path and the oracle on the same seeded inputs."""
import numpy as np

import armt_synth as S
from oracle import armt_oracle as O


def rel_fro(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def bf16_errors(got, want):
    """The three error figures of a bf16 hidden-state comparison: relative Frobenius error (the paper's Section 4.4
    metric), the largest relative error of a single row, and the largest element error in units of the rms of `want`."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    diff = got - want
    rows = np.linalg.norm(diff, axis=-1) / np.maximum(np.linalg.norm(want, axis=-1), 1e-300)
    rms = float(np.sqrt(np.mean(want * want)))
    return rel_fro(got, want), float(rows.max()), float(np.abs(diff).max() / max(rms, 1e-300))


# Companion bounds of the bf16 Frobenius tolerance e (2e-2), so that a defect confined to a few rows or elements cannot
# hide inside a norm over millions of elements:
#  * per row: a row's error is the sum of d_model element errors of comparable variance, so its norm concentrates
#    around the global figure; what varies between rows is the error level itself (late rows of a segment attend to
#    more keys, memory rows go through one more projection).  Bound: 2 e.  A row that is wrong in more than
#    (2e)^2 = 0.16 % of its energy fails it, whatever the number of rows.
#  * per element: if the relative Frobenius error is e, the element errors have rms e * rms(want); the largest of n
#    Gaussian errors is sqrt(2 ln n) sigma = 6.1 sigma for n = 1.3e8 (131072 x 2048 elements), and bf16 rounding of the
#    output adds at most 2^-9 |x| <= 0.012 rms(want) for |x| <= 6 rms.  Bound: 8 e * rms(want).
BF16_ROW_FACTOR, BF16_ELEM_FACTOR = 2.0, 8.0


def assert_bf16_close(got, want, tol, what):
    fro, row, elem = bf16_errors(got, want)
    print(f"{what}: rel. Frobenius {fro:.3e}, worst row {row:.3e}, worst element {elem:.3e} x rms", flush=True)
    assert fro <= tol, (what, "Frobenius", fro)
    assert row <= BF16_ROW_FACTOR * tol, (what, "row", row)
    assert elem <= BF16_ELEM_FACTOR * tol, (what, "element", elem)
    return fro, row, elem


def make_problem(shape, seed=0, std=0.02, gain_std=0.0, mem_std=None, x_std=1.0, v_scale=1.0):
    """v_scale (a power of two) multiplies W_V of the associative block: it makes the values read back
    from memory large (a strong memory effect on the hidden states) without touching the keys, so the
    denominators z.phi keep the sign and size they have on the paper-style N(0, 0.02) workload."""
    layers, mem_emb = S.make_weights(shape, seed=seed, std=std, gain_std=gain_std)
    if v_scale != 1.0:
        for lw in layers:
            lw["wm_v"] = (lw["wm_v"] * np.float32(v_scale)).astype(np.float32)
    if mem_std is not None:
        rng = np.random.default_rng([seed, 9])
        mem_emb = (rng.standard_normal(mem_emb.shape) * mem_std).astype(np.float32)
        if shape.dtype == "bf16":
            mem_emb = S.round_to_bf16(mem_emb)
    x = S.make_embeddings(shape, seed=seed)
    if x_std != 1.0:
        x = x * np.float32(x_std)
        if shape.dtype == "bf16":
            x = S.round_to_bf16(x)
    return layers, mem_emb, x


def run_hip(shape, layers, mem_emb, x, diagonal, A_in=None, z_in=None, model=None):
    import torch
    import paper_2506_05229_amd as P
    model = model or P.Armt(shape, layers, mem_emb)
    xd = model.embed(x)
    if A_in is not None:
        A_in = torch.as_tensor(A_in, dtype=torch.float32).cuda().contiguous()
        z_in = torch.as_tensor(z_in, dtype=torch.float32).cuda().contiguous()
    h, A, z = model.forward(xd, diagonal=diagonal, A_in=A_in, z_in=z_in)
    torch.cuda.synchronize()
    return h.float().cpu().numpy(), A.cpu().numpy(), z.cpu().numpy()


def run_oracle(shape, layers, mem_emb, x, A_in=None, z_in=None):
    return O.armt_forward_sequential(shape, layers, mem_emb, x, A_in=A_in, z_in=z_in)


def largest_stable_key_scale(shape, make_inputs, p_range, max_rms=50.0):
    """Largest key scale 2^-p (p taken from p_range in order) for which the float64 oracle keeps every denominator
    z.phi positive (read and update side) and the hidden states bounded: the recurrence of Eq. 4-5 is only
    well-conditioned there (below it z.phi crosses zero and the values read back grow without bound, a property of the
    equations and not of any kernel).  The oracle runs segment by segment with the memory state carried over
    (bit-identical to one run, see the oracle's pins), so that a diverging scale is given up early.
    make_inputs(shape) -> (layers, mem_emb, x).  Returns (p, shape, inputs, (hidden, A, z), stats) or None."""
    Sg = shape.seg_len
    for p in p_range:
        sh = shape.replace(mem_k_scale=2.0 ** -p)
        layers, mem_emb, x = make_inputs(sh)
        L64 = [{k: np.asarray(v, dtype=np.float64) for k, v in lw.items()} for lw in layers]
        A = z = None
        hs, stats, ok = [], [], True
        for s in range(x.shape[0] // Sg):
            st = []
            h, A, z = O.armt_forward_sequential(sh, L64, mem_emb, x[s * Sg:(s + 1) * Sg], A_in=A, z_in=z, stats=st)
            stats += [dict(e, s=s) for e in st]
            hs.append(h)
            if (not np.isfinite(h).all() or np.abs(h).max() > max_rms
                    or any(e["min_den"] <= 0.0 or e.get("min_zf", 1.0) <= 0.0 for e in st)):
                ok = False
                break
        if ok:
            return p, sh, (layers, mem_emb, x), (np.concatenate(hs), A, z), stats
    return None
