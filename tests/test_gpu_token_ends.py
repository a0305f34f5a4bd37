"""Parity of the token-level ends of Algorithm 1 (embedding gather; final RMSNorm + linear head) against
the oracle, through the C-ABI entry points armt_embed_tokens / armt_lm_head."""
import numpy as np
import pytest
import torch

import armt_synth as S
from gpu_util import rel_fro

pytestmark = pytest.mark.gpu


def _ends(shape, vocab, seed, n_tokens):
    import paper_2506_05229_amd as P
    ids, E, gf, W = S.make_token_ends(shape, vocab=vocab, seed=seed, n_tokens=n_tokens, gain_std=0.1)
    return ids, E, gf, W, P.TokenEnds(shape, E, gf, W)


@pytest.mark.parametrize("name,vocab", [("tiny", 301), ("1b_8k", 1000)])
def test_embedding_gather_is_exact(name, vocab):
    shape = S.get_shape(name)
    ids, E, gf, W, te = _ends(shape, vocab, 3, 2 * shape.seg_len)
    from oracle import armt_oracle as O
    x = te.embed(torch.from_numpy(ids).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(x.float().cpu().numpy().astype(np.float64), O.embed_tokens(ids, E))      # a copy: bit-exact


@pytest.mark.parametrize("name,vocab,rows,tol", [
    ("tiny", 301, 72, None),          # fp32: ragged vocabulary, fewer rows than one group
    ("tiny", 64, 2500, None),         # fp32: two groups of 1024 rows and a remainder
    ("1b_8k", 1000, 1040, 2e-2),      # bf16: one group + 16 rows, vocabulary not a multiple of the tile
    ("1b_8k", 2048, 2048, 2e-2),      # bf16: regular shape (scalar-addressed tiles)
])
def test_lm_head_matches_oracle(name, vocab, rows, tol):
    from oracle import armt_oracle as O
    shape = S.get_shape(name)
    ids, E, gf, W, te = _ends(shape, vocab, 4, shape.seg_len)
    rng = np.random.default_rng(5)
    h = (rng.standard_normal((rows, shape.d_model)) * 2.0).astype(np.float32)
    if shape.dtype == "bf16":
        h = S.round_to_bf16(h)
    got = te.logits(torch.from_numpy(h).to("cuda", te.dt))
    torch.cuda.synchronize()
    got = got.cpu().numpy().astype(np.float64)
    want = O.lm_head(h, gf, W, shape.rms_eps)
    assert got.shape == want.shape
    if tol is None:
        assert np.abs(got - want).max() <= 1e-4 * max(1.0, np.abs(want).max())
    else:
        assert rel_fro(got, want) <= tol, rel_fro(got, want)
        assert np.abs(got - want).max() <= 5e-2 * np.abs(want).max()


def test_tokens_to_logits_tiny_end_to_end():
    """ids -> embeddings -> diagonal forward -> logits of the last rows, all through the library, vs the oracle."""
    import paper_2506_05229_amd as P
    from oracle import armt_oracle as O
    shape = S.get_shape("tiny")
    layers, mem_emb = S.make_weights(shape, seed=2, gain_std=0.1)
    n_tok = 3 * shape.seg_len
    ids, E, gf, W, te = _ends(shape, 97, 2, n_tok)
    model = P.Armt(shape, layers, mem_emb)
    x = te.embed(torch.from_numpy(ids).cuda())
    hidden, A, z = model.forward(x, diagonal=True)
    got = te.logits(hidden[-shape.seg_len:].contiguous())
    torch.cuda.synchronize()
    want, h_ref, _, _ = O.armt_forward_tokens(shape, layers, mem_emb, E, ids, gf, W, last_rows=shape.seg_len)
    assert np.abs(hidden.cpu().numpy() - h_ref).max() <= 1e-4
    assert np.abs(got.cpu().numpy() - want).max() <= 1e-4 * max(1.0, np.abs(want).max())


def test_lm_head_full_vocabulary_sampled():
    """LLaMA-3 vocabulary (128256 = 501 tiles of 256) on the last segment of the 1B shape: sampled logits,
    each recomputed by the oracle from its own row and weight row."""
    from oracle import armt_oracle as O
    shape = S.get_shape("1b_128k")
    V = S.LLAMA3_VOCAB
    ids, E, gf, W, te = _ends(shape, V, 6, shape.seg_len)
    rng = np.random.default_rng(7)
    rows = shape.seg_len
    h = S.round_to_bf16(rng.standard_normal((rows, shape.d_model)).astype(np.float32))
    got = te.logits(torch.from_numpy(h).to("cuda", te.dt))
    torch.cuda.synchronize()
    r = np.concatenate([[0, rows - 1], rng.integers(0, rows, 30)])
    c = np.concatenate([[0, V - 1, 255, 256], rng.integers(0, V, 60)])
    sub = got[torch.from_numpy(r).cuda()][:, torch.from_numpy(c).cuda()].cpu().numpy().astype(np.float64)
    want = O.lm_head(h[r], gf, W[c], shape.rms_eps)
    assert rel_fro(sub, want) <= 2e-2, rel_fro(sub, want)
    assert np.isfinite(got.sum().item())


# ------------------------------------------------------------------ backward of the token-level ends
@pytest.mark.parametrize("name,vocab,rows,tol", [
    ("tiny", 301, 72, 2e-5),          # fp32: ragged vocabulary (reduction padded to 320), one pass
    ("tiny", 64, 9000, 2e-5),         # fp32: two passes of rows (8192 + 808)
    ("1b_8k", 1000, 1040, 2e-2),      # bf16: vocabulary padded to 1024, rows not a multiple of the tile
    ("1b_8k", 2048, 8200, 2e-2),      # bf16: a full pass and a short one
])
def test_lm_head_backward_matches_oracle(name, vocab, rows, tol):
    """Relative Frobenius error of d_hidden, d_final_gain, d_W_lm against the autograd oracle; bf16: the upstream
    gradient, the normalised rows and the weight are bf16 operands of the two gradient GEMMs."""
    from oracle import armt_oracle_grad as OG
    shape = S.get_shape(name)
    ids, E, gf, W, te = _ends(shape, vocab, 4, shape.seg_len)
    rng = np.random.default_rng(6)
    h = (rng.standard_normal((rows, shape.d_model)) * 2.0).astype(np.float32)
    Gl = rng.standard_normal((rows, vocab)).astype(np.float32)
    if shape.dtype == "bf16":
        h = S.round_to_bf16(h)
    want = OG.lm_head_grad(h, gf, W, shape.rms_eps, Gl)
    hd = torch.from_numpy(h).cuda().to(te.dt)
    got = te.logits_backward(hd, torch.from_numpy(Gl).cuda())
    torch.cuda.synchronize()
    errs = [rel_fro(a.cpu().numpy(), b) for a, b in zip(got, want)]
    print(f"{name} vocab {vocab} rows {rows}: d_hidden {errs[0]:.2e} d_gain {errs[1]:.2e} d_W {errs[2]:.2e}", flush=True)
    assert max(errs) <= tol
    # accumulation: a second call adds to the weight and gain gradients and rewrites d_hidden
    got2 = te.logits_backward(hd, torch.from_numpy(Gl).cuda(), grads=(got[1], got[2]))
    torch.cuda.synchronize()
    assert rel_fro(got2[2].cpu().numpy(), 2.0 * want[2]) <= tol and rel_fro(got2[0].cpu().numpy(), want[0]) <= tol


def test_embedding_backward_matches_oracle():
    from oracle import armt_oracle_grad as OG
    shape = S.get_shape("tiny")
    ids, E, gf, W, te = _ends(shape, 50, 7, 4 * shape.seg_len)       # 256 tokens over 50 ids: every id repeats
    dx = np.random.default_rng(7).standard_normal((ids.size, shape.d_model)).astype(np.float32)
    got = te.embed_backward(torch.from_numpy(ids).cuda(), torch.from_numpy(dx).cuda())
    torch.cuda.synchronize()
    want = OG.embed_tokens_grad(ids, dx, 50)
    assert np.abs(got.cpu().numpy() - want).max() <= 1e-5 * np.abs(want).max()      # atomics: order of the additions varies
    unique = np.arange(40, dtype=np.int32)[::-1].copy()                             # no repeats: a permuted copy, exact
    got = te.embed_backward(torch.from_numpy(unique).cuda(), torch.from_numpy(dx[:40].copy()).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy().astype(np.float64), OG.embed_tokens_grad(unique, dx[:40], 50))


def test_training_step_from_token_ids_matches_autograd():
    """One whole training step on the tiny configuration, every piece through the C ABI: ids -> embedding gather ->
    forward with tape -> final norm + head -> (cross-entropy of the next token, formed by the caller) -> head backward ->
    ARMT backward in reverse diagonal order -> embedding scatter-add.  The oracle differentiates the same chain in float64."""
    import torch.nn.functional as F
    import paper_2506_05229_amd as P
    from oracle import armt_oracle_grad as OG
    shape = S.get_shape("tiny").replace(n_tokens=3 * 64)
    vocab = 97
    layers, mem_emb = S.make_weights(shape, seed=1, gain_std=0.1)
    ids, E, gf, W = S.make_token_ends(shape, vocab=vocab, seed=1, n_tokens=shape.n_tokens, gain_std=0.1)
    targets = np.roll(ids, -1).astype(np.int64)
    # ---- oracle: autograd through gather, sequential forward, head and loss
    f64 = lambda a: torch.tensor(np.asarray(a, dtype=np.float64), requires_grad=True)
    Wt = [{k: f64(lw[k]) for k in OG.WEIGHT_KEYS} for lw in layers]
    met, Et, gft, Wlt = f64(mem_emb), f64(E), f64(gf), f64(W)
    hid, _, _ = OG.armt_forward_torch(shape, Wt, met, Et[torch.from_numpy(ids.astype(np.int64))])
    loss = F.cross_entropy(OG.rmsnorm(hid, gft, shape.rms_eps) @ Wlt.T, torch.from_numpy(targets))
    loss.backward()
    # ---- library
    model = P.Armt(shape, layers, mem_emb)
    te = P.TokenEnds(shape, E, gf, W)
    ids_d = torch.from_numpy(ids).cuda()
    x = te.embed(ids_d)
    hidden, _, _, tape = model.forward_train(x, diagonal=True)
    logits = te.logits(hidden)
    p = torch.softmax(logits, dim=-1)                        # the loss is the caller's: mean cross-entropy
    got_loss = -torch.log(p[torch.arange(shape.n_tokens), torch.from_numpy(targets).cuda()]).mean().item()
    p[torch.arange(shape.n_tokens), torch.from_numpy(targets).cuda()] -= 1.0
    d_hidden, d_gain, d_wlm = te.logits_backward(hidden, (p / shape.n_tokens).contiguous())
    g = model.backward(tape, shape.n_tokens, d_hidden.to(model.act_dtype).contiguous(), diagonal=True)
    d_table = te.embed_backward(ids_d, g["x"])
    torch.cuda.synchronize()
    assert abs(got_loss - loss.item()) <= 1e-5 * abs(loss.item())
    worst = ("", 0.0)
    def check(name, a, b):
        nonlocal worst
        e = rel_fro(a.cpu().numpy().reshape(b.shape), b.grad.numpy())
        worst = max(worst, (name, e), key=lambda t: t[1])
        assert e <= 2e-4, (name, e)
    check("emb_table", d_table, Et)
    check("final_gain", d_gain, gft)
    check("w_lm", d_wlm, Wlt)
    check("mem_emb", g["mem_emb"], met)
    for l in range(shape.n_layers):
        for k in OG.WEIGHT_KEYS:
            check(f"layer {l} {k}", g["layers"][l][k], Wt[l][k])
    print(f"training step: loss {got_loss:.6f}; worst relative gradient error {worst[1]:.2e} ({worst[0]})", flush=True)
