"""Seeded sweep of the backward pass over random small configurations inside the supported range (the generator of the
forward sweep: both dtypes, odd row counts, head_dim 64 / 128 and arbitrary even ones in fp32, n_mem from 1 to 48, fewer
segments than layers and the other way round), a random batch and a random order; parity of every gradient with the
autograd oracle on well-conditioned inputs."""
import numpy as np
import pytest
import torch

import armt_synth as S
from oracle import armt_oracle as O
from oracle import armt_oracle_grad as G
from test_gpu_backward import BF16_REL, BF16_REL_MEM, F32_REL, compare, upstream
from test_gpu_random_shapes import _random_shape

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("case", range(12))
def test_random_configuration_backward(case):
    import paper_2506_05229_amd as P
    rng = np.random.default_rng([2506, 77, case])
    bf16 = case % 2 == 1
    shape = _random_shape(rng, bf16)
    if shape.n_segments * shape.n_layers > 12:                 # keep the float64 autograd of the oracle to seconds
        shape = shape.replace(n_tokens=shape.seg_len * max(1, 12 // shape.n_layers))
    B = int(rng.integers(1, 3))
    diagonal = bool(rng.integers(0, 2))
    xs = [S.make_embeddings(shape, seed=100 * case + b) for b in range(B)]
    for p in (0, 2, 4, 6, 8, 10, 12):                          # largest key scale with positive denominators and modest reads
        shape = shape.replace(mem_k_scale=2.0 ** -p, mem_v_scale=16.0)
        layers, mem_emb = S.make_weights(shape, seed=case, gain_std=0.1)
        stats = []
        for x in xs:
            O.armt_forward_sequential(shape, layers, mem_emb, x, stats=stats)
        # z . phi(q) = 0 exactly is as good as positive: with few features (nu = 1, d_mem of a dozen) a query's active
        # features may share no support with any stored key, and its read is 0 / eps = 0 on both sides
        if not stats or (all(r["min_den"] >= 0.0 for r in stats) and max(r["max_abs_read"] for r in stats) < 2.0):
            break
    else:
        pytest.skip("no well-conditioned key scale found")
    print(f"case {case}: {shape} batch {B} diagonal {diagonal} key scale 2^-{p}", flush=True)
    Gss = [upstream(shape, 1000 * case + b, with_state=True) for b in range(B)]
    wants = [G.armt_grad(shape, layers, mem_emb, xs[b], *Gss[b]) for b in range(B)]
    model = P.Armt(shape, layers, mem_emb)
    dev = lambda a: torch.as_tensor(np.stack(a), dtype=torch.float32).cuda().contiguous()
    hidden, A, z, tape = model.forward_train(model.embed(np.stack(xs)), diagonal=diagonal)
    g = model.backward(tape, shape.n_tokens, model.embed(np.stack([q[0] for q in Gss])), dev([q[1] for q in Gss]),
                       dev([q[2] for q in Gss]), diagonal=diagonal)
    torch.cuda.synchronize()
    np_ = lambda t: None if t is None else t.float().cpu().numpy()
    got = {"layers": [{k: np_(v) for k, v in lw.items()} for lw in g["layers"]], "mem_emb": np_(g["mem_emb"]), "x": np_(g["x"]),
           "A_in": None, "z_in": None, "hidden": np_(hidden), "A": np_(A), "z": np_(z)}
    want = {"layers": [{k: sum(w["layers"][l][k] for w in wants) for k in G.WEIGHT_KEYS} for l in range(shape.n_layers)],
            "mem_emb": sum(w["mem_emb"] for w in wants), "A_in": None, "z_in": None}
    for k in ("x", "hidden", "A", "z"):
        want[k] = np.stack([w[k] for w in wants])
    if bf16:
        compare(got, want, BF16_REL, f"random case {case}", tol_mem=BF16_REL_MEM)
    else:
        compare(got, want, F32_REL, f"random case {case}")
