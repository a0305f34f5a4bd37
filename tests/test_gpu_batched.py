"""Batched forward (B independent sequences, the paper's batched setting): every sequence of a batched call
must get the bits of a call on that sequence alone, in both orders, and match the oracle."""
import numpy as np
import pytest
import torch

import armt_synth as S
from gpu_util import rel_fro

pytestmark = pytest.mark.gpu


def _seqs(shape, B, n_seg, seed0=10):
    return np.stack([S.make_embeddings(shape, seed=seed0 + b, n_tokens=n_seg * shape.seg_len) for b in range(B)])


@pytest.mark.parametrize("name,kw,B,n_seg", [
    ("tiny", dict(), 3, 6),                                             # fp32, more segments than layers
    ("tiny", dict(n_layers=5), 2, 3),                                   # fp32, fewer segments than layers
    ("1b_8k", dict(n_layers=3, d_ff=1024, seg_len=240), 4, 4),          # bf16 MFMA path, T = 256
])
def test_batched_equals_single_and_oracle(name, kw, B, n_seg):
    import paper_2506_05229_amd as P
    from oracle import armt_oracle as O
    shape = S.get_shape(name).replace(**kw) if kw else S.get_shape(name)
    layers, mem_emb = S.make_weights(shape, seed=3, gain_std=0.1)
    model = P.Armt(shape, layers, mem_emb)
    x = _seqs(shape, B, n_seg)
    xd = model.embed(x)
    hd, Ad, zd = model.forward_batched(xd, diagonal=True)
    hs, As, zs = model.forward_batched(xd, diagonal=False)
    torch.cuda.synchronize()
    assert torch.equal(hd, hs) and torch.equal(Ad, As) and torch.equal(zd, zs)      # exact recurrence, both orders
    for b in range(B):
        h1, A1, z1 = model.forward(xd[b].contiguous(), diagonal=True)
        torch.cuda.synchronize()
        assert torch.equal(h1, hd[b]) and torch.equal(A1, Ad[b]) and torch.equal(z1, zd[b]), b
    oh, oA, oz = O.armt_forward_batched(shape, layers, mem_emb, x)
    if shape.dtype == "f32":
        assert np.abs(hd.cpu().numpy() - oh).max() <= 1e-4
        assert np.abs(Ad.cpu().numpy() - oA).max() <= 1e-4 and np.abs(zd.cpu().numpy() - oz).max() <= 1e-4
    else:
        assert rel_fro(hd.float().cpu().numpy(), oh) <= 2e-2
        assert rel_fro(Ad.cpu().numpy(), oA) <= 8e-2 and rel_fro(zd.cpu().numpy(), oz) <= 4e-2


def test_batched_carry_in_splits_exactly():
    import paper_2506_05229_amd as P
    shape = S.get_shape("tiny")
    layers, mem_emb = S.make_weights(shape, seed=4)
    model = P.Armt(shape, layers, mem_emb)
    xd = model.embed(_seqs(shape, 2, 5))
    h, A, z = model.forward_batched(xd, diagonal=True)
    cut = 2 * shape.seg_len
    h1, A1, z1 = model.forward_batched(xd[:, :cut].contiguous(), diagonal=True)
    h2, A2, z2 = model.forward_batched(xd[:, cut:].contiguous(), diagonal=True, A_in=A1, z_in=z1)
    torch.cuda.synchronize()
    assert torch.equal(torch.cat([h1, h2], dim=1), h) and torch.equal(A2, A) and torch.equal(z2, z)
