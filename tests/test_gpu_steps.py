"""Parity of the single steps of the path (through the C ABI) against the oracle's functions.

fp32: element-wise max-abs tolerances; bf16: relative Frobenius error, operands rounded to bf16 before
both sides see them (the oracle computes in float64 from the same rounded values)."""
import numpy as np
import pytest
import torch

import armt_synth as S
from gpu_util import rel_fro
from oracle import armt_oracle as O

pytestmark = pytest.mark.gpu


def _dev(a, dtype):
    return torch.as_tensor(np.ascontiguousarray(a)).to(device="cuda", dtype=dtype).contiguous()


def _rand(rng, shape, std, bf16):
    a = (rng.standard_normal(shape) * std).astype(np.float32)
    return S.round_to_bf16(a) if bf16 else a


# ---------------------------------------------------------------- grouped GEMM (Section 3.3 item 1)
@pytest.mark.parametrize("g,M,N,K", [
    (1, 16, 64, 64),          # one memory-row tile
    (3, 72, 200, 128),        # ragged M and N
    (2, 1040, 512, 256),      # the real cell height: 4 full 256-row tiles and a 16-row tail
    (5, 300, 2112, 192),      # N = d_mem + d of the update projections, several tiles and a tail
    (16, 130, 96, 64),        # group = number of layers
    # 256 x 256 tiles for whole rounds of the 256 CUs, the rest of the launch as 128 x 128 tiles: 9 x 4 x 8 = 288 tiles
    # (a round and 32 tiles = one group), 7 x 4 x 12 = 336 (the cut falls inside a group), 66 x 1 x 4 = 264 (one M-tile)
    (9, 1040, 2048, 128),
    (7, 1040, 3072, 64),
    (66, 256, 1024, 64),
])
# tile configurations only exist for the bf16 MFMA kernel; -1 = the library's own choice
@pytest.mark.parametrize("dtype,tile_cfg", [("f32", -1)] + [("bf16", c) for c in (-1, 1, 2, 3, 4, 5, 6)])
def test_grouped_gemm(dtype, g, M, N, K, tile_cfg):
    import paper_2506_05229_amd as P
    bf = dtype == "bf16"
    rng = np.random.default_rng(g * 1000 + M)
    a = [_rand(rng, (M, K), 1.0, bf) for _ in range(g)]
    b = [_rand(rng, (N, K), 0.05, bf) for _ in range(g)]
    td = torch.bfloat16 if bf else torch.float32
    old = P.set_gemm_tile_config(tile_cfg)
    try:
        out = P.grouped_gemm([_dev(x, td) for x in a], [_dev(x, td) for x in b])
        torch.cuda.synchronize()
    finally:
        P.set_gemm_tile_config(old)
    for i in range(g):
        want = a[i].astype(np.float64) @ b[i].astype(np.float64).T      # every group with its own weights
        got = out[i].float().cpu().numpy()
        if bf:
            assert rel_fro(got, want) <= 4e-3, (i, rel_fro(got, want))   # output rounded to bf16: 2^-9 per element
            assert np.abs(got - want).max() <= 2e-2 * np.abs(want).max()
        else:
            assert np.abs(got - want).max() <= 1e-5 * max(1.0, np.abs(want).max())


# ---------------------------------------------------------------- segment attention (Section 4.2)
@pytest.mark.parametrize("dtype,kw", [
    ("f32", {}),
    ("f32", dict(n_heads=6, n_kv_heads=3, head_dim=20, d_model=120, seg_len=37, n_mem=5)),
    ("bf16", dict(n_heads=4, n_kv_heads=2, head_dim=64, d_model=256, d_ff=512, seg_len=144, n_mem=16, d_mem=32)),
    ("bf16", dict(n_heads=8, n_kv_heads=2, head_dim=64, d_model=512, d_ff=512, seg_len=1024, n_mem=16, d_mem=32)),
    ("bf16", dict(n_heads=3, n_kv_heads=1, head_dim=128, d_model=384, d_ff=512, seg_len=200, n_mem=16, d_mem=32)),
    # one query head per KV head: four row tiles per workgroup, the last workgroup only partly inside the cell
    ("bf16", dict(n_heads=4, n_kv_heads=4, head_dim=64, d_model=256, d_ff=512, seg_len=200, n_mem=16, d_mem=32)),
    ("bf16", dict(n_heads=2, n_kv_heads=2, head_dim=128, d_model=256, d_ff=512, seg_len=1024, n_mem=16, d_mem=32)),
    # the software-pipelined kernel (head_dim 64, 4 or 8 query heads per KV head) at its edges: a cell of one half-tile
    # (T = 20: only the masked last step), of two (T = 33 + 16) and three half-tiles (T = 80 + 16, ragged last tile), an
    # even and an odd number of half-tiles over several tiles, eight waves per workgroup
    ("bf16", dict(n_heads=4, n_kv_heads=1, head_dim=64, d_model=256, d_ff=512, seg_len=4, n_mem=16, d_mem=32)),
    ("bf16", dict(n_heads=4, n_kv_heads=1, head_dim=64, d_model=256, d_ff=512, seg_len=33, n_mem=16, d_mem=32)),
    ("bf16", dict(n_heads=8, n_kv_heads=2, head_dim=64, d_model=512, d_ff=512, seg_len=80, n_mem=16, d_mem=32)),
    ("bf16", dict(n_heads=8, n_kv_heads=2, head_dim=64, d_model=512, d_ff=512, seg_len=240, n_mem=16, d_mem=32)),
    ("bf16", dict(n_heads=4, n_kv_heads=1, head_dim=64, d_model=256, d_ff=512, seg_len=300, n_mem=16, d_mem=32)),
    ("bf16", dict(n_heads=8, n_kv_heads=1, head_dim=64, d_model=512, d_ff=512, seg_len=333, n_mem=16, d_mem=32)),
    ("bf16", dict(n_heads=16, n_kv_heads=2, head_dim=64, d_model=1024, d_ff=512, seg_len=1024, n_mem=16, d_mem=32)),
])
def test_segment_attention(dtype, kw):
    import paper_2506_05229_amd as P
    shape = S.get_shape("tiny").replace(dtype=dtype, n_layers=3, rope_theta=1000.0, **kw)
    bf = dtype == "bf16"
    g, T, H, Hkv, dh = 3, shape.T, shape.n_heads, shape.n_kv_heads, shape.head_dim
    rng = np.random.default_rng(T)
    qkv = _rand(rng, (g, T, (H + 2 * Hkv) * dh), 1.0, bf)
    steps = P.ArmtSteps(shape)
    out = steps.segment_attention(_dev(qkv, steps.act_dtype))
    torch.cuda.synchronize()
    got = out.float().cpu().numpy()
    for i in range(g):
        q = qkv[i, :, :H * dh].reshape(T, H, dh).astype(np.float64)
        k = qkv[i, :, H * dh:(H + Hkv) * dh].reshape(T, Hkv, dh).astype(np.float64)
        v = qkv[i, :, (H + Hkv) * dh:].reshape(T, Hkv, dh).astype(np.float64)
        want = O.causal_gqa_attention(O.rope(q, shape.rope_theta), O.rope(k, shape.rope_theta), v).reshape(T, H * dh)
        if bf:
            assert rel_fro(got[i], want) <= 1e-2, rel_fro(got[i], want)
            # per query row as well: a wrong half-tile of one row tile hides in the norm over the cell
            row_err = np.linalg.norm(got[i] - want, axis=1) / np.linalg.norm(want, axis=1)
            assert row_err.max() <= 3e-2, (int(row_err.argmax()), float(row_err.max()))
        else:
            assert np.abs(got[i] - want).max() <= 2e-5


@pytest.mark.parametrize("n_kv_heads", [2, 1])     # two / four query heads per KV head: the two kernels for head_dim 64
@pytest.mark.parametrize("kind", ["growing", "huge", "tiny_then_huge"])
def test_segment_attention_moving_maximum(kind, n_kv_heads):
    """The matrix-core attention kernel keeps a reference exponent per query that it only moves when the unnormalised
    probabilities of a half-tile get large.  Inputs that make it move all the time, or by a lot: keys whose scores grow
    along the sequence (every later tile beats the reference), scores of magnitude 10^2 - 10^3 (exp2 of the difference
    overflows unless the reference moves first), and a sequence whose first keys are tiny and whose later ones are huge."""
    import paper_2506_05229_amd as P
    kw = dict(n_heads=4, n_kv_heads=n_kv_heads, head_dim=64, d_model=256, d_ff=512, seg_len=400, n_mem=16, d_mem=32)
    shape = S.get_shape("tiny").replace(dtype="bf16", n_layers=2, rope_theta=1000.0, **kw)
    g, T, H, Hkv, dh = 2, shape.T, shape.n_heads, shape.n_kv_heads, shape.head_dim
    rng = np.random.default_rng(7)
    qkv = rng.standard_normal((g, T, (H + 2 * Hkv) * dh)).astype(np.float32)
    ramp = np.ones(T, np.float32)
    if kind == "growing":
        ramp = 1.0 + np.arange(T, dtype=np.float32) / 16.0           # |k_j| grows 26-fold over the cell
    elif kind == "huge":
        ramp = np.full(T, 12.0, np.float32)                             # scores of a few hundred
        qkv[:, :, :H * dh] *= 4.0
    else:
        ramp = np.where(np.arange(T) < 200, 1e-3, 30.0).astype(np.float32)
    qkv[:, :, H * dh:(H + Hkv) * dh] *= ramp[None, :, None]
    qkv = S.round_to_bf16(qkv)
    steps = P.ArmtSteps(shape)
    out = steps.segment_attention(_dev(qkv, steps.act_dtype))
    torch.cuda.synchronize()
    got = out.float().cpu().numpy()
    assert np.isfinite(got).all()
    for i in range(g):
        q = qkv[i, :, :H * dh].reshape(T, H, dh).astype(np.float64)
        k = qkv[i, :, H * dh:(H + Hkv) * dh].reshape(T, Hkv, dh).astype(np.float64)
        v = qkv[i, :, (H + Hkv) * dh:].reshape(T, Hkv, dh).astype(np.float64)
        # the entry point rotates q and k and rounds them to bf16 again before the kernel under test sees them; with scores
        # of 10^2 - 10^3 that rounding alone changes the softmax, so the oracle gets the same rotated, rounded operands
        qr = S.round_to_bf16(O.rope(q, shape.rope_theta).astype(np.float32)).astype(np.float64)
        kr = S.round_to_bf16(O.rope(k, shape.rope_theta).astype(np.float32)).astype(np.float64)
        want = O.causal_gqa_attention(qr, kr, v).reshape(T, H * dh)
        err = rel_fro(got[i], want)
        print(f"attention, {kind}: rel. Frobenius {err:.3e}", flush=True)
        assert err <= 1e-2, (kind, err)


# ---------------------------------------------------------------- associative read / update (Eq. 3-6)
def _memory_problem(shape, g, rng, bf):
    d, dm, P_, m, T = shape.d_model, shape.d_mem, shape.phi, shape.n_mem, shape.T
    w = [dict(wm_q=_rand(rng, (dm, d), 0.1, bf), wm_k=_rand(rng, (dm, d), 0.1, bf),
              wm_v=_rand(rng, (d, d), 0.1, bf), wm_b=_rand(rng, (1, d), 0.1, bf)) for _ in range(g)]
    x = (rng.standard_normal((g, T, d))).astype(np.float32)
    ym = (rng.standard_normal((g, m, d))).astype(np.float32)
    if bf:      # the bf16 path rounds these operands; give both sides the rounded values
        x, ym = S.round_to_bf16(x), S.round_to_bf16(ym)
    # a non-trivial but positive previous state: written by an earlier update of the oracle
    A = np.zeros((g, d, P_))
    z = np.zeros((g, P_))
    for i in range(g):
        A[i], z[i] = O.assoc_update(rng.standard_normal((m, d)), A[i], z[i], True, w[i], shape.assoc_eps, shape.dpfp_nu)
    return w, x, ym, A.astype(np.float32), z.astype(np.float32)


MEM_SHAPES = [
    ("f32", dict()),
    ("f32", dict(d_model=120, n_heads=6, head_dim=20, n_kv_heads=3, seg_len=37, n_mem=5, d_mem=12, dpfp_nu=2)),
    ("bf16", dict(d_model=256, n_heads=4, head_dim=64, n_kv_heads=2, d_ff=512, seg_len=144, n_mem=16, d_mem=32)),
    ("bf16", dict(d_model=512, n_heads=8, head_dim=64, n_kv_heads=2, d_ff=512, seg_len=1024, n_mem=16, d_mem=64)),
    # memory tokens in several LDS chunks of the generic delta rule: 32 + 8, and the 128 of the paper's tables
    ("f32", dict(n_mem=40)),
    ("bf16", dict(d_model=256, n_heads=4, head_dim=64, n_kv_heads=2, d_ff=512, seg_len=128, n_mem=128, d_mem=64)),
]


@pytest.mark.parametrize("dtype,kw", MEM_SHAPES)
def test_assoc_read(dtype, kw):
    import paper_2506_05229_amd as P
    shape = S.get_shape("tiny").replace(dtype=dtype, n_layers=3, **kw)
    bf, g = dtype == "bf16", 3
    rng = np.random.default_rng(17)
    w, x, ym, A, z = _memory_problem(shape, g, rng, bf)
    steps = P.ArmtSteps(shape)
    xd = _dev(x, torch.float32)
    steps.assoc_read(xd, [_dev(w[i]["wm_q"], steps.act_dtype) for i in range(g)], _dev(A, torch.float32), _dev(z, torch.float32))
    torch.cuda.synchronize()
    got = xd.cpu().numpy()
    for i in range(g):
        want = O.assoc_read(x[i].astype(np.float64), A[i].astype(np.float64), z[i].astype(np.float64),
                            w[i]["wm_q"].astype(np.float64), shape.assoc_eps, shape.dpfp_nu)
        delta_want, delta_got = want - x[i], got[i] - x[i]
        assert np.abs(delta_want).max() > 1e-2          # the read is not a rounding-level effect here
        if bf:
            assert rel_fro(delta_got, delta_want) <= 1.5e-2, rel_fro(delta_got, delta_want)
        else:
            assert np.abs(got[i] - want).max() <= 1e-4 * max(1.0, np.abs(want).max())


@pytest.mark.parametrize("dtype,kw", MEM_SHAPES)
@pytest.mark.parametrize("empty_group", [-1, 1])
def test_assoc_update(dtype, kw, empty_group):
    import paper_2506_05229_amd as P
    shape = S.get_shape("tiny").replace(dtype=dtype, n_layers=3, **kw)
    bf, g = dtype == "bf16", 3
    rng = np.random.default_rng(23)
    w, x, ym, A, z = _memory_problem(shape, g, rng, bf)
    if empty_group >= 0:
        A[empty_group], z[empty_group] = 0.0, 0.0
    steps = P.ArmtSteps(shape)
    Ad, zd = _dev(A, torch.float32), _dev(z, torch.float32)
    lists = [[_dev(w[i][f], steps.act_dtype) for i in range(g)] for f in ("wm_k", "wm_v", "wm_b")]
    steps.assoc_update(_dev(ym, torch.float32), *lists, Ad, zd, empty_group=empty_group)
    torch.cuda.synchronize()
    gA, gz = Ad.cpu().numpy(), zd.cpu().numpy()
    for i in range(g):
        wi = {k: v.astype(np.float64) for k, v in w[i].items()}
        wA, wz = O.assoc_update(ym[i].astype(np.float64), A[i].astype(np.float64), z[i].astype(np.float64),
                                i == empty_group, wi, shape.assoc_eps, shape.dpfp_nu)
        dA, dz = wA - A[i], wz - z[i]
        assert np.abs(dA).max() > 0 and np.abs(dz).max() > 0
        if bf:
            assert rel_fro(gA[i] - A[i], dA) <= 1.5e-2 and rel_fro(gz[i] - z[i], dz) <= 1.5e-2
        else:
            assert rel_fro(gA[i] - A[i], dA) <= 1e-5 and rel_fro(gz[i] - z[i], dz) <= 1e-5
