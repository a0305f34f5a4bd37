"""What the synthetic workloads exercise (no GPU): conditioning of the associative memory on them, and proof that the
parity tolerances of the GPU tests would catch a delta-rule kernel that drops a term of Eq. 4.

The mistakes are planted in copies of the ORACLE's update, on the CPU; the deviation they cause is measured with the
metrics and tolerances the GPU parity tests use.
"""
import numpy as np
import pytest

import armt_synth as S
from oracle import armt_oracle as O

# tolerances of tests/test_gpu_fullsize.py and tests/test_gpu_forward.py on bf16 configurations
BF16_REL, MEM_Z_REL, MEM_A_REL = 2e-2, 4e-2, 8e-2


def rel_fro(a, b):
    return float(np.linalg.norm(a - b) / np.linalg.norm(b))


# ------------------------------------------------------------------ role of assoc_eps on the tiny configuration
def test_eps_decides_the_result_on_the_tiny_configuration_and_is_placed_identically():
    """On the tiny fp32 configuration exactly as specified (N(0, 0.02) weights) the denominators z.phi are far below
    assoc_eps = 1e-5, so the printed equations (eps = 0) and the eps = 1e-5 reading give different results: the
    configuration does NOT satisfy "eps = 0 and eps = 1e-5 agree".  What is well posed, and what both sides of the
    parity tests implement, is the reading with eps inside both denominators: there the result is a smooth function of
    eps (relative sensitivity at most 1, no cancellation), which is what this test pins."""
    cfg = S.get_shape("tiny")
    layers, mem_emb = S.make_weights(cfg, seed=0)
    x = S.make_embeddings(cfg, seed=0)
    st = []
    h, A, z = O.armt_forward_sequential(cfg, layers, mem_emb, x, stats=st)
    assert 0.0 < min(e["min_den"] for e in st) and max(e["max_den"] for e in st) < 1e3 * cfg.assoc_eps
    h0, A0, z0 = O.armt_forward_sequential(cfg.replace(assoc_eps=0.0), layers, mem_emb, x)
    assert rel_fro(h0, h) > 1e-2                       # eps = 0 is another (ill-conditioned) computation here
    # sensitivity to eps: a relative change t of eps changes the memory read by at most t, the hidden states by less
    t = 1e-3
    h1, A1, z1 = O.armt_forward_sequential(cfg.replace(assoc_eps=cfg.assoc_eps * (1 + t)), layers, mem_emb, x)
    assert rel_fro(h1, h) <= t and rel_fro(A1, A) <= 2 * t and rel_fro(z1, z) <= 2 * t


def test_eps_zero_and_default_agree_where_the_memory_is_well_filled():
    """The printed equations (eps = 0) and the eps = 1e-5 reading agree to 1e-5 once |z.phi| >> eps: the tiny
    configuration with two memory tokens per segment and the key / query projections of the memory scaled by 2^8, so
    that every denominator is at least 10^6 eps in size (gamma then leaves [0, 1] and z.phi(q) takes both signs: the
    reading "no clamp" is what runs here, and the hidden states stay bounded)."""
    cfg = S.get_shape("tiny").replace(n_mem=2, mem_k_scale=2.0 ** 8, mem_v_scale=1.0)
    layers, mem_emb = S.make_weights(cfg, seed=0)
    for lw in layers:
        lw["wm_q"] = lw["wm_q"] * np.float32(2.0 ** 8)
    x = S.make_embeddings(cfg, seed=0)
    st = []
    h, A, z = O.armt_forward_sequential(cfg, layers, mem_emb, x, stats=st)
    assert min(e["min_abs_den"] for e in st) > 10.0 and min(e["min_zf"] for e in st) > 10.0
    assert min(e["gamma_min"] for e in st) < 0.0 < max(e["gamma_max"] for e in st)
    assert np.isfinite(h).all() and np.abs(h).max() < 50.0
    h0, A0, z0 = O.armt_forward_sequential(cfg.replace(assoc_eps=0.0), layers, mem_emb, x)
    assert rel_fro(h, h0) <= 1e-5 and rel_fro(A, A0) <= 1e-5 and rel_fro(z, z0) <= 1e-5


# ------------------------------------------------------------------ Eq. 4 is live on the LLaMA-width parity case
def _planted_update(kind):
    """The oracle's delta-rule update with one term of Eq. 4 dropped."""
    def update(Ym, A, z, empty, w, eps, nu):
        k = Ym @ w["wm_k"].T
        v = Ym @ w["wm_v"].T
        beta = 1.0 / (1.0 + np.exp(-(Ym @ w["wm_b"].T)[:, 0]))
        f = O.dpfp(k, nu)
        zf = f @ z
        vbar = np.zeros_like(v) if (empty or kind == "no_vbar") else (f @ A.T) / (zf + eps)[:, None]
        gamma = np.ones_like(zf) if kind == "gamma_one" else 1.0 - zf / (np.sum(f * f, axis=-1) + eps)
        return A + (beta[:, None] * (v - vbar)).T @ f, z + gamma @ f
    return update


LIVE_1B_WIDTH = dict(n_layers=4, n_tokens=3 * 1024, mem_k_scale=2.0 ** -6)


@pytest.mark.timeout(600)
def test_dropped_terms_of_eq4_exceed_the_gpu_tolerances_at_1b_width(monkeypatch):
    """Four layers of the 1B width over three segments with the largest stable key scale for that depth (2^-6, the
    case tests/test_gpu_forward.py::test_1b_width_live_delta_rule runs on the GPU): gamma reaches well below 1 and
    v_bar is a visible part of v.  A delta rule without v_bar, or with gamma = 1, deviates from the definition by more
    than the tolerances the GPU test holds the kernels to."""
    shape = S.get_shape("1b_8k").replace(**LIVE_1B_WIDTH)
    layers, mem_emb = S.make_weights(shape, seed=0, gain_std=0.1)
    layers = [{k: v.astype(np.float64) for k, v in lw.items()} for lw in layers]
    x = S.make_embeddings(shape, seed=0)
    st = []
    h, A, z = O.armt_forward_sequential(shape, layers, mem_emb, x, stats=st)
    assert all(e["min_den"] > 0.0 and e["min_zf"] > 0.0 for e in st)
    g_lo, g_hi = min(e["gamma_min"] for e in st), max(e["gamma_max"] for e in st)
    vb = [e["vbar_over_v"] for e in st]
    print(f"gamma in [{g_lo:.3f}, {g_hi:.3f}], |v_bar|/|v| min {min(vb):.3f} median {np.median(vb):.3f} max {max(vb):.3f}")
    assert g_lo < 0.0 and g_hi < 1.0 and np.median(vb) > 0.1
    worst = lambda a, b: max(rel_fro(a[l], b[l]) for l in range(a.shape[0]))
    monkeypatch.setattr(O, "assoc_update", _planted_update("no_vbar"))
    h1, A1, z1 = O.armt_forward_sequential(shape, layers, mem_emb, x)
    print(f"without v_bar: hidden {rel_fro(h1, h):.3e}, A worst layer {worst(A1, A):.3e}, z worst layer {worst(z1, z):.3e}")
    assert worst(A1, A) > MEM_A_REL
    monkeypatch.setattr(O, "assoc_update", _planted_update("gamma_one"))
    h2, A2, z2 = O.armt_forward_sequential(shape, layers, mem_emb, x)
    print(f"gamma = 1: hidden {rel_fro(h2, h):.3e}, A worst layer {worst(A2, A):.3e}, z worst layer {worst(z2, z):.3e}")
    assert worst(z2, z) > MEM_Z_REL


def test_named_workloads_carry_their_memory_scales():
    """Every LLaMA-shaped workload states the scales of its memory projections (they are part of the input recipe)."""
    for name, shape in S.CONFIGS.items():
        if name == "tiny":
            assert shape.mem_k_scale == 1.0 and shape.mem_v_scale == 1.0
        else:
            assert 0.0 < shape.mem_k_scale < 1.0 and 0.0 < shape.mem_v_scale <= 1.0, name
            assert f"2^{int(np.log2(shape.mem_k_scale))}" in S.describe_workload(shape)
