"""Seeded sweep over random small configurations inside the supported range: both dtypes, both orders, a
random batch, shapes that switch the epilogue fusions and tile paths on and off (rows not a multiple of 8,
head_dim 64 / 128, v columns on / off a tile boundary, n_mem in several delta-rule chunks, fewer segments than
layers and the other way round).  Every case: diagonal == sequential bit for bit, and parity with the oracle."""
import numpy as np
import pytest
import torch

import armt_synth as S
from gpu_util import rel_fro

pytestmark = pytest.mark.gpu


def _random_shape(rng, bf16):
    if bf16:
        dh = int(rng.choice([64, 128]))
        hkv = int(rng.choice([1, 2, 4]))
        group = int(rng.choice([1, 2, 4]))
        H = hkv * group
        d = H * dh
        while d % 64:
            H += hkv
            d = H * dh
        d_ff = 64 * int(rng.integers(2, 9))
        n_mem = 16 * int(rng.choice([1, 1, 2, 3]))
        seg_len = int(rng.choice([48, 100, 112, 240, 253, 300]))
        d_mem = int(rng.choice([32, 64]))
        nu = int(rng.choice([1, 2, 3])) if d_mem == 64 else int(rng.choice([1, 2]))
        while (2 * nu * d_mem) % 64 or 2 * nu * d_mem > 512:
            nu = nu % 3 + 1
    else:
        dh = 2 * int(rng.integers(4, 21))
        hkv = int(rng.choice([1, 2, 3]))
        H = hkv * int(rng.choice([1, 2, 3]))
        d = H * dh
        d_ff = int(rng.integers(40, 300))
        n_mem = int(rng.integers(1, 45))
        seg_len = int(rng.integers(5, 90))
        d_mem = int(rng.integers(4, 33))
        nu = int(rng.integers(1, 4))
    L = int(rng.integers(1, 5))
    n_seg = int(rng.integers(1, 6))
    return S.get_shape("tiny").replace(n_layers=L, d_model=d, n_heads=H, n_kv_heads=hkv, head_dim=dh, d_ff=d_ff,
                                       seg_len=seg_len, n_mem=n_mem, d_mem=d_mem, dpfp_nu=nu,
                                       n_tokens=seg_len * n_seg, dtype="bf16" if bf16 else "f32")


@pytest.mark.parametrize("case", range(16))
def test_random_configuration(case):
    import paper_2506_05229_amd as P
    from oracle import armt_oracle as O
    rng = np.random.default_rng([2506, case])
    bf16 = case % 2 == 1
    shape = _random_shape(rng, bf16)
    B = int(rng.integers(1, 4))
    print(f"case {case}: {shape} batch {B}", flush=True)
    # Well-conditioned inputs only: with many memory tokens the recurrence of Eq. 4-5 can drive z.phi through zero
    # (a property of the equations, the oracle shows it), and parity on such inputs is void.  Take the largest key
    # scale 2^-p (from 2^8 down) for which the oracle keeps every z.phi positive and the hidden states bounded: at the
    # edge of that range gamma and v_bar of Eq. 4 are far from their trivial values 1 and 0.
    x = np.stack([S.make_embeddings(shape, seed=100 * case + b) for b in range(B)])
    for p in (-8, -6, -4, -2, 0, 2, 4, 6, 8, 10):
        shape = shape.replace(mem_k_scale=2.0 ** -p, mem_v_scale=16.0)
        layers, mem_emb = S.make_weights(shape, seed=case, gain_std=0.1)
        stats, ref = [], []
        for b in range(B):
            ref.append(O.armt_forward_sequential(shape, layers, mem_emb, x[b], stats=stats))
        if (all(r["min_den"] > 0.0 and r["min_zf"] > 0.0 for r in stats)
                and max(np.abs(r[0]).max() for r in ref) < 50.0):
            break
    else:
        pytest.skip("no well-conditioned key scale found")
    if stats:
        print(f"  key scale 2^{-p}: gamma in [{min(r['gamma_min'] for r in stats):.3f}, {max(r['gamma_max'] for r in stats):.3f}], "
              f"median |v_bar|/|v| {np.median([r['vbar_over_v'] for r in stats]):.3f}", flush=True)
    oh, oA, oz = (np.stack([r[i] for r in ref]) for i in range(3))
    model = P.Armt(shape, layers, mem_emb)
    xd = model.embed(x)
    hd, Ad, zd = model.forward_batched(xd, diagonal=True)
    hs, As, zs = model.forward_batched(xd, diagonal=False)
    torch.cuda.synchronize()
    assert torch.equal(hd, hs) and torch.equal(Ad, As) and torch.equal(zd, zs)
    h = hd.float().cpu().numpy()
    assert np.isfinite(h).all()
    if bf16:
        err = rel_fro(h, oh)
        print(f"  rel. Frobenius error {err:.3e}", flush=True)
        assert err <= 2e-2
        assert rel_fro(zd.cpu().numpy(), oz) <= 4e-2 and rel_fro(Ad.cpu().numpy(), oA) <= 8e-2
    else:
        err = np.abs(h - oh).max()
        print(f"  max abs error {err:.3e}", flush=True)
        assert err <= 1e-4
        assert rel_fro(Ad.cpu().numpy(), oA) <= 1e-4 and rel_fro(zd.cpu().numpy(), oz) <= 1e-4
