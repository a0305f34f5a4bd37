"""End-to-end parity of the HIP path (through the C ABI) against the CPU oracle.

Tolerances: fp32 configurations max |hidden - oracle| <= 1e-4; bf16 configurations relative
Frobenius error of the final hidden states <= 2e-2 (the error metric of the paper's Section 4.4)."""
import numpy as np
import pytest

import armt_synth as S
from gpu_util import make_problem, rel_fro, run_hip, run_oracle

pytestmark = pytest.mark.gpu

F32_ABS = 1e-4
BF16_REL = 2e-2


def _check_f32(got, want, what):
    h, A, z = got
    oh, oA, oz = want
    err = np.abs(h - oh).max()
    print(f"{what}: max|dh|={err:.3e} relA={rel_fro(A, oA):.3e} relz={rel_fro(z, oz):.3e}", flush=True)
    assert np.isfinite(h).all()
    assert err <= F32_ABS, what
    assert rel_fro(A, oA) <= 1e-4 and rel_fro(z, oz) <= 1e-4, what


@pytest.mark.parametrize("diagonal", [False, True])
def test_tiny_f32_matches_oracle(diagonal):
    """The tiny configuration: 4 layers, d=128, 4/2 heads, 8 segments of 64 + 8 memory tokens."""
    shape = S.get_shape("tiny")
    prob = make_problem(shape, seed=0)
    _check_f32(run_hip(shape, *prob, diagonal=diagonal), run_oracle(shape, *prob), f"tiny diag={diagonal}")


@pytest.mark.parametrize("diagonal", [False, True])
@pytest.mark.parametrize("case", ["strong_memory", "ragged", "one_segment", "more_segments_than_layers",
                                  "one_layer"])
def test_f32_variants_match_oracle(case, diagonal):
    base = S.get_shape("tiny")
    kw = dict(std=0.02, gain_std=0.1)
    if case == "strong_memory":      # memory values large enough to change the hidden states by ~20 %
        shape, kw = base.replace(n_tokens=5 * 64), dict(std=0.02, gain_std=0.1, v_scale=64.0)
    elif case == "ragged":           # nothing is a multiple of a tile
        shape = base.replace(n_layers=3, d_model=120, n_heads=6, n_kv_heads=3, head_dim=20, d_ff=200,
                             seg_len=37, n_mem=5, d_mem=12, n_tokens=37 * 4, dpfp_nu=2)
    elif case == "one_segment":
        shape = base.replace(n_tokens=64)
    elif case == "more_segments_than_layers":
        shape = base.replace(n_layers=2, n_tokens=64 * 7)
    else:
        shape = base.replace(n_layers=1, n_tokens=64 * 3)
    prob = make_problem(shape, seed=3, **kw)
    _check_f32(run_hip(shape, *prob, diagonal=diagonal), run_oracle(shape, *prob), f"{case} diag={diagonal}")


def test_f32_carry_in_and_prefix():
    """[0, k) then [k, N) with the exported memory state equals one full run (dependency rule of
    Section 3.1), and both match the oracle."""
    shape = S.get_shape("tiny")
    layers, mem_emb, x = make_problem(shape, seed=5, gain_std=0.1, v_scale=64.0)
    oh, oA, oz = run_oracle(shape, layers, mem_emb, x)
    k = 3 * shape.seg_len
    h1, A1, z1 = run_hip(shape, layers, mem_emb, x[:k], diagonal=True)
    assert np.abs(h1 - oh[:k]).max() <= F32_ABS
    h2, A2, z2 = run_hip(shape, layers, mem_emb, x[k:], diagonal=True, A_in=A1, z_in=z1)
    assert np.abs(h2 - oh[k:]).max() <= F32_ABS
    assert rel_fro(A2, oA) <= 1e-4 and rel_fro(z2, oz) <= 1e-4


def test_diagonal_equals_sequential_on_gpu():
    shape = S.get_shape("tiny")
    prob = make_problem(shape, seed=7, gain_std=0.1, v_scale=64.0)
    a = run_hip(shape, *prob, diagonal=False)
    b = run_hip(shape, *prob, diagonal=True)
    for u, v in zip(a, b):
        assert np.array_equal(u, v)         # same kernels, same per-cell arithmetic: bit-identical


SMALL_BF16 = dict(n_layers=3, d_model=256, n_heads=4, n_kv_heads=2, head_dim=64, d_ff=512, seg_len=144,
                  n_mem=16, d_mem=32, n_tokens=144 * 5, dtype="bf16")


@pytest.mark.parametrize("diagonal", [False, True])
@pytest.mark.parametrize("case", ["paper_init", "strong_memory"])
def test_small_bf16_matches_oracle(case, diagonal):
    shape = S.get_shape("tiny").replace(**SMALL_BF16)
    kw = dict(std=0.02) if case == "paper_init" else dict(std=0.02, gain_std=0.1, v_scale=16.0)
    prob = make_problem(shape, seed=11, **kw)
    h, A, z = run_hip(shape, *prob, diagonal=diagonal)
    oh, oA, oz = run_oracle(shape, *prob)
    e = rel_fro(h, oh), rel_fro(A, oA), rel_fro(z, oz)
    print(f"small bf16 {case} diag={diagonal}: rel hidden={e[0]:.3e} A={e[1]:.3e} z={e[2]:.3e}", flush=True)
    assert np.isfinite(h).all()
    assert e[0] <= BF16_REL and e[1] <= 5e-2 and e[2] <= 5e-2


# a cell of 1024 + 16 rows and widths that are multiples of 256: the shapes on which the forced tile configurations take
# their own code paths (256-row tiles with the strip of memory rows, scalar-addressed copies, fused epilogues)
TILED_BF16 = dict(n_layers=3, d_model=512, n_heads=8, n_kv_heads=2, head_dim=64, d_ff=1024, seg_len=1024,
                  n_mem=16, d_mem=32, n_tokens=1024 * 3, dtype="bf16")


@pytest.mark.parametrize("rows", ["1024+16", "300+16"])
def test_tile_configurations_give_the_same_bits(rows):
    """Every tile configuration of the grouped GEMM accumulates a result element in the same order (k ascending, fp32),
    so forcing one for all GEMMs of a pass must not change a single bit of the outputs.  300 + 16 rows: a ragged last
    M-tile, read as a whole tile from the padded operand buffers by the configurations with scalar-addressed copies."""
    import paper_2506_05229_amd as P
    shape = S.get_shape("tiny").replace(**TILED_BF16)
    if rows == "300+16":
        shape = shape.replace(seg_len=300, n_tokens=300 * 3)
    prob = make_problem(shape, seed=3, std=0.02, gain_std=0.1, v_scale=16.0)
    model = P.Armt(shape, prob[0], prob[1])
    want = run_hip(shape, *prob, diagonal=True, model=model)
    assert np.isfinite(want[0]).all()
    for cfg in range(9):
        old = P.set_gemm_tile_config(cfg)
        try:
            got = run_hip(shape, *prob, diagonal=True, model=model)
        finally:
            P.set_gemm_tile_config(old)
        for u, v in zip(got, want):
            assert np.array_equal(u, v), cfg
