"""Pins of the oracle's token-level ends (Algorithm 1: token ids in, logits out): the embedding gather
and the final RMSNorm + linear head. Each check compares against something the oracle does not compute
itself: the table's own rows, a closed form, a library routine, or pure-python loops."""
import math

import numpy as np
import pytest
import torch

import armt_synth as S
from oracle import armt_oracle as O


def test_embed_rows_are_table_rows_and_bad_ids_raise():
    rng = np.random.default_rng(0)
    E = rng.standard_normal((11, 5))
    ids = np.array([3, 0, 10, 3, 7])
    x = O.embed_tokens(ids, E)
    assert x.shape == (5, 5) and x.dtype == np.float64
    for i, t in enumerate(ids):
        assert np.array_equal(x[i], E[t])
    for bad in ([11], [-1]):
        with pytest.raises(ValueError):
            O.embed_tokens(np.array(bad), E)


def test_identity_head_closed_form():
    # W = I, eps = 0: logits = g * h / rms(h); sum((logits / g)^2) = d
    rng = np.random.default_rng(1)
    d = 12
    h = rng.standard_normal((4, d)) * 3.0
    g = 1.0 + 0.1 * rng.standard_normal(d)
    out = O.lm_head(h, g, np.eye(d), 0.0)
    for i in range(4):
        rms = math.sqrt(sum(v * v for v in h[i]) / d)
        assert np.allclose(out[i], g * h[i] / rms, rtol=1e-13, atol=0)
        assert abs(np.sum((out[i] / g) ** 2) - d) < 1e-10


def test_head_invariants():
    rng = np.random.default_rng(2)
    d, V = 16, 23
    h = rng.standard_normal((6, d))
    g = 1.0 + 0.2 * rng.standard_normal(d)
    W1, W2 = rng.standard_normal((V, d)), rng.standard_normal((V, d))
    a = O.lm_head(h, g, W1, 0.0)
    assert np.allclose(O.lm_head(7.5 * h, g, W1, 0.0), a, rtol=1e-12)                 # RMSNorm forgets the scale
    assert np.allclose(O.lm_head(h, g, W1 + W2, 1e-5), O.lm_head(h, g, W1, 1e-5) + O.lm_head(h, g, W2, 1e-5), rtol=1e-12, atol=1e-12)
    # a row of W orthogonal to g * h gives a zero logit; the row parallel to it gives |g * h| / rms(h)
    u = g * h[0]
    w_par = u / np.linalg.norm(u)
    w_orth = rng.standard_normal(d)
    w_orth -= (w_orth @ w_par) * w_par
    out = O.lm_head(h[:1], g, np.stack([w_par, w_orth]), 0.0)[0]
    assert abs(out[1]) < 1e-12
    assert abs(out[0] - np.linalg.norm(u) / math.sqrt(np.mean(h[0] ** 2))) < 1e-12


def test_head_against_library_routines():
    rng = np.random.default_rng(3)
    d, V, eps = 32, 50, 1e-5
    h = rng.standard_normal((9, d))
    g = 1.0 + 0.1 * rng.standard_normal(d)
    W = rng.standard_normal((V, d)) * 0.1
    want = torch.nn.functional.linear(
        torch.nn.functional.rms_norm(torch.from_numpy(h), (d,), torch.from_numpy(g), eps), torch.from_numpy(W)).numpy()
    assert np.allclose(O.lm_head(h, g, W, eps), want, rtol=1e-12, atol=1e-13)


def test_head_brute_force_python():
    rng = np.random.default_rng(4)
    d, V, eps = 5, 4, 1e-5
    h = rng.standard_normal((3, d)).tolist()
    g = (1.0 + 0.3 * rng.standard_normal(d)).tolist()
    W = rng.standard_normal((V, d)).tolist()
    got = O.lm_head(np.array(h), np.array(g), np.array(W), eps)
    for i in range(3):
        ms = sum(v * v for v in h[i]) / d
        n = [h[i][k] / math.sqrt(ms + eps) * g[k] for k in range(d)]
        for v in range(V):
            assert abs(got[i][v] - sum(n[k] * W[v][k] for k in range(d))) < 1e-13


def test_forward_tokens_is_the_composition():
    shape = S.get_shape("tiny")
    layers, mem_emb = S.make_weights(shape, seed=1, gain_std=0.1)
    ids, E, gf, Wlm = S.make_token_ends(shape, vocab=37, seed=1, n_tokens=2 * shape.seg_len, gain_std=0.1)
    logits, hidden, A, z = O.armt_forward_tokens(shape, layers, mem_emb, E, ids, gf, Wlm)
    h2, A2, z2 = O.armt_forward_sequential(shape, layers, mem_emb, E[ids].astype(np.float64))
    assert np.array_equal(hidden, h2) and np.array_equal(A, A2) and np.array_equal(z, z2)
    assert logits.shape == (2 * shape.seg_len, 37)
    assert np.array_equal(logits, O.lm_head(h2, gf, Wlm, shape.rms_eps))
    last, _, _, _ = O.armt_forward_tokens(shape, layers, mem_emb, E, ids, gf, Wlm, last_rows=5)
    assert np.allclose(last, logits[-5:], rtol=1e-13, atol=1e-13)       # a slice may take another BLAS path
    # ids are a prefix-stable stream and lie in the vocabulary
    ids_long = S.make_token_ends(shape, vocab=37, seed=1, n_tokens=4 * shape.seg_len)[0]
    assert np.array_equal(ids_long[:ids.size], ids) and ids_long.min() >= 0 and ids_long.max() < 37
