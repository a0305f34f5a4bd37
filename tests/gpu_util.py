"""Helpers shared by the GPU parity tests: run the HIP path and the oracle on the same seeded inputs."""
import numpy as np

import armt_synth as S
from oracle import armt_oracle as O


def rel_fro(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


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
