"""The forward calls can be recorded into a HIP graph and replayed: they allocate nothing, never wait for the stream,
copy nothing from host memory (the pointer tables travel as kernel arguments) and clear memory with kernels.

Every replay is checked against the eager result, bit for bit, with the program's own eager work between the replays:
another forward call of the same model on other input, which overwrites the whole workspace and the pointer tables
the recorded kernels read, and a clearing of the outputs."""
import numpy as np
import pytest
import torch

import armt_synth as S
from gpu_util import make_problem

pytestmark = pytest.mark.gpu

SMALL_BF16 = dict(n_layers=3, d_model=256, n_heads=4, n_kv_heads=2, head_dim=64, d_ff=512, seg_len=144,
                  n_mem=16, d_mem=32, n_tokens=144 * 5, dtype="bf16")


@pytest.mark.parametrize("diagonal", [True, False])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_forward_replays_from_a_graph(dtype, diagonal):
    import paper_2506_05229_amd as P
    shape = S.get_shape("tiny") if dtype == "f32" else S.get_shape("tiny").replace(**SMALL_BF16)
    layers, mem_emb, x = make_problem(shape, seed=5, gain_std=0.1, v_scale=16.0)
    model = P.Armt(shape, layers, mem_emb)
    xd = model.embed(x)
    other = model.embed(S.make_embeddings(shape, seed=6))
    want = [t.clone() for t in model.forward(xd, diagonal=diagonal)]            # eager (also the warm-up of every kernel)
    scratch = [t.clone() for t in model.forward(other, diagonal=diagonal)]
    torch.cuda.synchronize()
    assert not torch.equal(want[0], scratch[0])
    out = tuple(torch.empty_like(t) for t in want)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        model.forward(xd, diagonal=diagonal, out=out)
    torch.cuda.synchronize()
    for rep in range(3):
        for t in out:
            t.zero_()
        model.forward(other, diagonal=diagonal, out=tuple(scratch))            # eager work on the same workspace
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref, name in zip(out, want, ("hidden", "A", "z")):
            assert torch.equal(got, ref), (dtype, diagonal, rep, name)


def test_static_head_replays_from_a_graph():
    """armt_lm_head_static is the entry point for callers under graph capture: record it, replay it."""
    import paper_2506_05229_amd as P
    shape = S.get_shape("tiny").replace(**SMALL_BF16)
    vocab, rows = 1000, 200
    rng = np.random.default_rng(3)
    E = S.round_to_bf16(rng.standard_normal((vocab, shape.d_model)).astype(np.float32))
    gain = S.round_to_bf16((1.0 + 0.1 * rng.standard_normal(shape.d_model)).astype(np.float32))
    W = S.round_to_bf16((0.02 * rng.standard_normal((vocab, shape.d_model))).astype(np.float32))
    ends = P.TokenEnds(shape, E, gain, W)
    hidden = torch.from_numpy(rng.standard_normal((rows, shape.d_model)).astype(np.float32)).to("cuda:0", torch.bfloat16)
    other = torch.from_numpy(rng.standard_normal((rows, shape.d_model)).astype(np.float32)).to("cuda:0", torch.bfloat16)
    want = torch.empty((rows, vocab), dtype=torch.float32, device="cuda:0")
    spare = torch.empty_like(want)
    ends.logits_static(hidden, want)
    torch.cuda.synchronize()
    assert torch.equal(want, ends.logits(hidden))
    out = torch.empty_like(want)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ends.logits_static(hidden, out)
    torch.cuda.synchronize()
    for rep in range(3):
        out.zero_()
        ends.logits_static(other, spare)                                        # eager call on the same fixed scratch array
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want), rep
