"""Pins of the backward oracle (oracle/armt_oracle_grad.py) to things other than itself; no GPU.

What fixes the expected values: the NUMPY forward oracle (which has its own pins) differentiated by
central finite differences, a decoder block built from library routines and differentiated by the
library, and properties any gradient of this forward must have (linearity in the upstream gradients,
causality over segments)."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import armt_synth as S
from oracle import armt_oracle as O
from oracle import armt_oracle_grad as G


def tiny_cfg(**kw):
    base = dict(name="t", n_layers=2, d_model=8, n_heads=2, n_kv_heads=1, head_dim=4, d_ff=12,
                seg_len=3, n_mem=2, d_mem=2, n_tokens=9, dtype="f32")
    base.update(kw)
    return S.ArmtShape(**base)


def rand_problem(cfg, seed=0, std=0.5, gain_std=0.2):
    layers, _ = S.make_weights(cfg, seed=seed, std=std, gain_std=gain_std)
    layers = [{k: np.asarray(v, dtype=np.float64) for k, v in lw.items()} for lw in layers]
    rng = np.random.default_rng(seed + 100)
    mem_emb = rng.standard_normal((cfg.n_mem, cfg.d_model))
    x = np.asarray(S.make_embeddings(cfg, seed=seed), dtype=np.float64)
    return layers, mem_emb, x


def upstream(cfg, seed):
    rng = np.random.default_rng(seed + 7)
    return (rng.standard_normal((cfg.n_tokens, cfg.d_model)),
            rng.standard_normal((cfg.n_layers, cfg.d_model, cfg.phi)) * 0.3,
            rng.standard_normal((cfg.n_layers, cfg.phi)) * 0.3)


def carried_state(cfg, layers, mem_emb, seed):
    """A dense carried-in state with a positive normaliser, as many segments leave behind (the features are
    non-negative, so every denominator z.phi + eps stays away from a sign change)."""
    rng = np.random.default_rng(seed + 50)
    return (rng.standard_normal((cfg.n_layers, cfg.d_model, cfg.phi)) * 0.5,
            rng.uniform(0.5, 1.5, (cfg.n_layers, cfg.phi)))


def J_numpy(cfg, layers, mem_emb, x, Gs, A_in=None, z_in=None):
    h, A, z = O.armt_forward_sequential(cfg, layers, mem_emb, x, A_in=A_in, z_in=z_in)
    return float((h * Gs[0]).sum() + (A * Gs[1]).sum() + (z * Gs[2]).sum())


@pytest.mark.parametrize("carry", [False, True])
def test_restated_forward_equals_numpy_oracle(carry):
    cfg = tiny_cfg(n_layers=3, n_tokens=12)
    layers, mem_emb, x = rand_problem(cfg, seed=1)
    A_in, z_in = carried_state(cfg, layers, mem_emb, 1) if carry else (None, None)
    want = O.armt_forward_sequential(cfg, layers, mem_emb, x, A_in=A_in, z_in=z_in)
    W = [{k: torch.tensor(v) for k, v in lw.items()} for lw in layers]
    t = lambda a: None if a is None else torch.tensor(a)
    got = G.armt_forward_torch(cfg, W, torch.tensor(mem_emb), torch.tensor(x), t(A_in), t(z_in))
    for a, b in zip(got, want):
        assert np.abs(a.numpy() - b).max() <= 1e-9 * max(1.0, np.abs(b).max())


def _fd_entries(arr, rng, n):
    idx = [tuple(rng.integers(0, s) for s in arr.shape) for _ in range(n)]
    return list(dict.fromkeys(idx))


@pytest.mark.parametrize("carry", [False, True])
def test_gradient_matches_finite_differences_of_numpy_forward(carry):
    """Every input tensor, a handful of entries each: (J(p + h) - J(p - h)) / 2h of the numpy oracle."""
    cfg = tiny_cfg(n_layers=2, n_tokens=9)
    # std 0.3, seed 7: reads of a few units and no denominator near a sign change (checked with the forward
    # oracle's conditioning figures), so that a step of 1e-5 stays in the smooth regime
    layers, mem_emb, x = rand_problem(cfg, seed=7, std=0.3)
    Gs = upstream(cfg, 2)
    A_in, z_in = carried_state(cfg, layers, mem_emb, 7) if carry else (None, None)
    grads = G.armt_grad(cfg, layers, mem_emb, x, *Gs, A_in=A_in, z_in=z_in)
    assert abs(grads["J"] - J_numpy(cfg, layers, mem_emb, x, Gs, A_in, z_in)) <= 1e-9 * abs(grads["J"])
    rng = np.random.default_rng(0)
    h = 1e-5
    # round-off of the two evaluations of J: a few ulps of the sum of the magnitudes of its terms, divided by 2h
    jscale = sum(float(np.abs(a * b).sum()) for a, b in zip((grads["hidden"], grads["A"], grads["z"]), Gs))
    noise = 1e-13 * jscale / h
    worst = 0.0

    def check(arr, grad, label, n=4):
        nonlocal worst
        for idx in _fd_entries(arr, rng, n):
            keep = arr[idx]
            arr[idx] = keep + h
            jp = J_numpy(cfg, layers, mem_emb, x, Gs, A_in, z_in)
            arr[idx] = keep - h
            jm = J_numpy(cfg, layers, mem_emb, x, Gs, A_in, z_in)
            arr[idx] = keep
            fd = (jp - jm) / (2 * h)
            err = max(0.0, abs(fd - grad[idx]) - noise) / max(abs(fd), abs(grad[idx]), 1e-6)
            worst = max(worst, err)
            assert err <= 2e-5, (label, idx, fd, grad[idx], noise)

    for l in range(cfg.n_layers):
        for k in G.WEIGHT_KEYS:
            check(layers[l][k], grads["layers"][l][k], f"layer {l} {k}")
    check(mem_emb, grads["mem_emb"], "mem_emb", 6)
    check(x, grads["x"], "x", 8)
    if carry:
        check(A_in, grads["A_in"], "A_in", 8)
        check(z_in, grads["z_in"], "z_in", 6)
    else:
        assert grads["A_in"] is None and grads["z_in"] is None
    print("worst relative deviation from finite differences:", worst)


def _library_block(U, w, cfg):
    """LLaMA decoder block from library routines (rms_norm, scaled_dot_product_attention, silu);
    rotary embedding as a complex multiplication."""
    T = U.shape[0]
    H, Hkv, dh = cfg.n_heads, cfg.n_kv_heads, cfg.head_dim

    def rot(t):                      # [T, heads, dh], pairs (j, j + dh/2)
        half = dh // 2
        ang = torch.arange(T, dtype=torch.float64)[:, None] * cfg.rope_theta ** (
            -2.0 * torch.arange(half, dtype=torch.float64) / dh)[None, :]
        c = torch.complex(t[..., :half], t[..., half:]) * torch.polar(torch.ones_like(ang), ang)[:, None, :]
        return torch.cat([c.real, c.imag], dim=-1)

    n = F.rms_norm(U, (cfg.d_model,), w["rms1"], cfg.rms_eps)
    q = rot(F.linear(n, w["wq"]).view(T, H, dh)).transpose(0, 1)
    k = rot(F.linear(n, w["wk"]).view(T, Hkv, dh)).transpose(0, 1).repeat_interleave(H // Hkv, dim=0)
    v = F.linear(n, w["wv"]).view(T, Hkv, dh).transpose(0, 1).repeat_interleave(H // Hkv, dim=0)
    a = F.scaled_dot_product_attention(q[None], k[None], v[None], is_causal=True)[0].transpose(0, 1).reshape(T, H * dh)
    h = U + F.linear(a, w["wo"])
    n2 = F.rms_norm(h, (cfg.d_model,), w["rms2"], cfg.rms_eps)
    return h + F.linear(F.silu(F.linear(n2, w["wgate"])) * F.linear(n2, w["wup"]), w["wdown"])


def test_one_segment_empty_memory_is_the_library_block_gradient():
    """One segment, one layer, no carried state, no gradient into the final memory: the ARMT reduces to
    the decoder block on [tokens; memory embeddings], so the gradients of the block's weights, of x and
    of mem_emb are the library's."""
    cfg = tiny_cfg(n_layers=1, n_tokens=3, seg_len=3, n_heads=4, n_kv_heads=2, head_dim=2)
    layers, mem_emb, x = rand_problem(cfg, seed=3)
    Gh = np.random.default_rng(3).standard_normal((cfg.n_tokens, cfg.d_model))
    got = G.armt_grad(cfg, layers, mem_emb, x, Gh)
    w = {k: torch.tensor(v, requires_grad=True) for k, v in layers[0].items()}
    xt, mt = torch.tensor(x, requires_grad=True), torch.tensor(mem_emb, requires_grad=True)
    Y = _library_block(torch.cat([xt, mt]), w, cfg)
    (Y[:cfg.seg_len] * torch.tensor(Gh)).sum().backward()
    assert np.allclose(got["x"], xt.grad.numpy(), rtol=1e-9, atol=1e-12)
    assert np.allclose(got["mem_emb"], mt.grad.numpy(), rtol=1e-9, atol=1e-12)
    for k in ("rms1", "wq", "wk", "wv", "wo", "rms2", "wgate", "wup", "wdown"):
        assert np.allclose(got["layers"][0][k], w[k].grad.numpy(), rtol=1e-9, atol=1e-12), k
    for k in ("wm_q", "wm_k", "wm_v", "wm_b"):      # the memory is written but never read or scored
        assert not got["layers"][0][k].any(), k


def test_gradient_is_linear_in_the_upstream_gradients():
    cfg = tiny_cfg(n_layers=2, n_tokens=9)
    layers, mem_emb, x = rand_problem(cfg, seed=4)
    G1, G2 = upstream(cfg, 4), upstream(cfg, 5)
    mix = tuple(a + 2.0 * b for a, b in zip(G1, G2))
    g1, g2, gm = (G.armt_grad(cfg, layers, mem_emb, x, *g) for g in (G1, G2, mix))
    assert np.allclose(gm["x"], g1["x"] + 2.0 * g2["x"], rtol=1e-9, atol=1e-11)
    for l in range(cfg.n_layers):
        for k in G.WEIGHT_KEYS:
            assert np.allclose(gm["layers"][l][k], g1["layers"][l][k] + 2.0 * g2["layers"][l][k], rtol=1e-9, atol=1e-11)


def test_gradient_respects_causality_over_segments():
    """Upstream gradient on segment 0 only: later segments' embeddings get no gradient, and every gradient
    equals the one of a run over segment 0 alone (dependency rule of Section 3.1)."""
    cfg = tiny_cfg(n_layers=2, n_tokens=9)
    layers, mem_emb, x = rand_problem(cfg, seed=6)
    Gh = np.zeros((cfg.n_tokens, cfg.d_model))
    Gh[:cfg.seg_len] = np.random.default_rng(6).standard_normal((cfg.seg_len, cfg.d_model))
    full = G.armt_grad(cfg, layers, mem_emb, x, Gh)
    one = G.armt_grad(cfg.replace(n_tokens=cfg.seg_len), layers, mem_emb, x[:cfg.seg_len], Gh[:cfg.seg_len])
    assert not full["x"][cfg.seg_len:].any()
    assert np.allclose(full["x"][:cfg.seg_len], one["x"], rtol=1e-10, atol=1e-13)
    assert np.allclose(full["mem_emb"], one["mem_emb"], rtol=1e-10, atol=1e-13)
    for l in range(cfg.n_layers):
        for k in G.WEIGHT_KEYS:
            assert np.allclose(full["layers"][l][k], one["layers"][l][k], rtol=1e-10, atol=1e-13), k


# ------------------------------------------------------------------ token-level ends
def test_lm_head_gradient_matches_finite_differences_and_library():
    rng = np.random.default_rng(8)
    n, d, V, eps = 5, 8, 11, 1e-5
    h, g, w = rng.standard_normal((n, d)), 1.0 + 0.2 * rng.standard_normal(d), rng.standard_normal((V, d)) * 0.5
    Gl = rng.standard_normal((n, V))
    dh, dg, dw = G.lm_head_grad(h, g, w, eps, Gl)
    J = lambda: float((O.lm_head(h, g, w, eps) * Gl).sum())
    step = 1e-6
    for arr, grad in ((h, dh), (g, dg), (w, dw)):
        for idx in _fd_entries(arr, rng, 6):
            keep = arr[idx]
            arr[idx] = keep + step
            jp = J()
            arr[idx] = keep - step
            jm = J()
            arr[idx] = keep
            assert abs((jp - jm) / (2 * step) - grad[idx]) <= 1e-6 * max(1.0, abs(grad[idx]))
    ht, gt, wt = (torch.tensor(a, requires_grad=True) for a in (h, g, w))
    (F.linear(F.rms_norm(ht, (d,), gt, eps), wt) * torch.tensor(Gl)).sum().backward()
    for a, b in ((dh, ht.grad), (dg, gt.grad), (dw, wt.grad)):
        assert np.allclose(a, b.numpy(), rtol=1e-10, atol=1e-12)


def test_embedding_gradient_adds_rows_per_occurrence():
    ids = np.array([3, 0, 3, 3, 1], dtype=np.int32)
    dx = np.arange(10, dtype=np.float64).reshape(5, 2) + 1.0
    got = G.embed_tokens_grad(ids, dx, vocab=5)
    want = np.zeros((5, 2))
    for i, t in enumerate(ids):
        for c in range(2):
            want[t, c] += dx[i, c]
    assert np.array_equal(got, want) and not got[2].any() and not got[4].any()
    assert np.array_equal(G.embed_tokens_grad(ids, np.ones((5, 2)), 5)[:, 0], np.array([1.0, 1.0, 0.0, 3.0, 0.0]))

