"""CPU oracle for the ARMT forward pass -- TEST INFRASTRUCTURE, NOT THE PRODUCT.

A plain, slow, float64 numpy statement of what an Associative Recurrent Memory
Transformer computes over a long input: segment by segment, layer by layer, as the
paper defines it (Section 2.1, Eq. 2-6; Section 3.1 for the order of the cells).
Diagonal Batching only reorders independent (layer, segment) cells (Lemma 3.1), so
the sequential definition below is the exact result both GPU entry points must match.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
module. It shares no code with the HIP path and imports nothing but numpy. There is
no blocking, fusion or reordering here beyond what the definition states.

Parity status of each function (what pins it, in tests/test_oracle_*.py):
  dpfp                     hand-worked values, non-negativity, width 2*nu*d_mem, sparsity pattern
  rmsnorm                  unit-RMS invariant, scale invariance
  rope                     identity at position 0, norm preservation, relative-position invariant,
                           complex-multiplication form
  causal_gqa_attention     library scaled-dot-product attention, single-key case, row-stochastic
  llama_block              fp64 library-built decoder block (degenerate ARMT with W_V^mem = 0)
  assoc_read/assoc_update  closed forms (first write, overwrite / delta-rule interpolation,
                           orthogonal keys), brute-force rebuild of A from stored outer products
  armt_forward_sequential  brute-force pure-python recomputation on tiny sizes, prefix and
                           carry-in invariants, perturbation (causality over segments)
  armt_forward_diagonal_order   bit-identical to the sequential order (exact recurrence)
  embed_tokens             row identity with the table, error on ids outside the vocabulary
  lm_head                  identity head (logits = g * h / rms(h)), scale invariance, library
                           rms_norm + matmul, pure-python loops on tiny sizes
  armt_forward_tokens      composition of the three (no arithmetic of its own)
  armt_forward_batched     a loop over the sequences (no arithmetic of its own)
Absolute values of the hidden states on the LLaMA-shaped workloads are not printed
anywhere in the paper; they are pinned only through the checks above.

Readings of the paper taken here (each is listed with its reason in the design notes):
  * the associative read is added to its input (x <- x + read(x)); Algorithm 1 skips the
    read for an empty memory, which is only consistent with adding zero;
  * an empty memory (A = z = 0, first segment without carry-in) skips the read and uses
    v_bar = 0; otherwise denominators are z.f + eps and |f|^2 + eps, eps = assoc_eps;
  * all n_mem memory tokens of a segment see the memory state from before the update
    (Eq. 4 is written with A_{s-1}, z_{s-1});
  * the memory tokens are the last n_mem rows of the cell, the update uses the layer's
    OUTPUT at those rows (Algorithm 1, UpdateMem(G, Y[:, -num_mem_tokens:]));
  * gamma is not clamped;
  * positions restart at 0 in every segment; the transformer layer is a LLaMA-3 decoder
    block (pre-norm RMSNorm, GQA, rotate-half RoPE, SwiGLU, no biases);
  * the result is the last layer's hidden state at the token rows (no final norm, no
    LM head), plus the final memory state of every layer;
  * the token-level ends of Algorithm 1 (token ids in, logits out) are the LLaMA ones: a
    row gather from the embedding table in front, a final RMSNorm (same eps as the
    block's) and a bias-free linear head behind; the head may share the table.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------- feature map
def dpfp(x: np.ndarray, nu: int = 3) -> np.ndarray:
    """DPFP-nu feature map (the untrained nonlinearity phi of Section 2.1; defined by
    Schlag et al. 2021): r = [relu(x), relu(-x)] in R^{2 d_mem};
    phi[(j-1)*2*d_mem + i] = r[i] * r[(i - j) mod 2*d_mem], j = 1..nu."""
    x = np.asarray(x, dtype=F64)
    r = np.concatenate([np.maximum(x, 0.0), np.maximum(-x, 0.0)], axis=-1)
    return np.concatenate([r * np.roll(r, j, axis=-1) for j in range(1, nu + 1)], axis=-1)


# --------------------------------------------------------------------------- LLaMA block
def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * gain


def rope(x: np.ndarray, theta: float) -> np.ndarray:
    """Rotary embedding, rotate-half pairing (j, j + dh/2), angle p * theta^(-2j/dh);
    x is [T, n_heads, dh], position p = row index."""
    T, _, dh = x.shape
    half = dh // 2
    inv_freq = theta ** (-2.0 * np.arange(half, dtype=F64) / dh)
    ang = np.arange(T, dtype=F64)[:, None] * inv_freq[None, :]          # [T, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def causal_gqa_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray) -> np.ndarray:
    """softmax(q k^T / sqrt(dh)) v with a causal mask over the T rows of the cell;
    q [T, H, dh], k, v [T, Hkv, dh]; query head h uses kv head h // (H / Hkv)."""
    T, H, dh = q.shape
    Hkv = k.shape[1]
    rep = H // Hkv
    out = np.empty_like(q)
    mask = np.tril(np.ones((T, T), dtype=bool))
    for h in range(H):
        g = h // rep
        sc = (q[:, h, :] @ k[:, g, :].T) / np.sqrt(F64(dh))
        sc = np.where(mask, sc, -np.inf)
        sc = sc - sc.max(axis=-1, keepdims=True)
        p = np.exp(sc)
        p = p / p.sum(axis=-1, keepdims=True)
        out[:, h, :] = p @ v[:, g, :]
    return out


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def llama_block(U: np.ndarray, w: dict, cfg) -> np.ndarray:
    """One LLaMA-3 decoder block on the T rows of a cell (the TransformerLayer of Eq. 2)."""
    T = U.shape[0]
    H, Hkv, dh = cfg.n_heads, cfg.n_kv_heads, cfg.head_dim
    n = rmsnorm(U, w["rms1"], cfg.rms_eps)
    q = (n @ w["wq"].T).reshape(T, H, dh)
    k = (n @ w["wk"].T).reshape(T, Hkv, dh)
    v = (n @ w["wv"].T).reshape(T, Hkv, dh)
    q, k = rope(q, cfg.rope_theta), rope(k, cfg.rope_theta)
    a = causal_gqa_attention(q, k, v).reshape(T, H * dh)
    h = U + a @ w["wo"].T
    n2 = rmsnorm(h, w["rms2"], cfg.rms_eps)
    return h + (silu(n2 @ w["wgate"].T) * (n2 @ w["wup"].T)) @ w["wdown"].T


# --------------------------------------------------------------------------- associative memory
def assoc_read(U: np.ndarray, A: np.ndarray, z: np.ndarray, wm_q: np.ndarray,
               eps: float, nu: int) -> np.ndarray:
    """AssociativeLayer (Eq. 6) applied to every row of the cell, added to its input:
    x_i <- x_i + A phi(W_Q x_i) / (z^T phi(W_Q x_i) + eps)."""
    f = dpfp(U @ wm_q.T, nu)                       # [T, Phi]
    num = f @ A.T                                  # [T, d]
    den = f @ z + eps                              # [T]
    return U + num / den[:, None]


def assoc_update(Ym: np.ndarray, A: np.ndarray, z: np.ndarray, empty: bool, w: dict,
                 eps: float, nu: int):
    """Delta-rule memory update (Eq. 3-5) from the n_mem memory-token outputs Ym [m, d].
    Every memory token uses the state from before the update. Returns new (A, z)."""
    k = Ym @ w["wm_k"].T                           # [m, d_mem]
    v = Ym @ w["wm_v"].T                           # [m, d]
    beta = 1.0 / (1.0 + np.exp(-(Ym @ w["wm_b"].T)[:, 0]))   # [m]
    f = dpfp(k, nu)                                # [m, Phi]
    zf = f @ z                                     # [m]
    if empty:
        vbar = np.zeros_like(v)
    else:
        vbar = (f @ A.T) / (zf + eps)[:, None]     # [m, d]
    gamma = 1.0 - zf / (np.sum(f * f, axis=-1) + eps)
    A_new = A + (beta[:, None] * (v - vbar)).T @ f           # sum_i beta_i (v_i - vbar_i) (x) phi(k_i)
    z_new = z + gamma @ f                                    # sum_i gamma_i phi(k_i)
    return A_new, z_new


def update_conditioning(Ym: np.ndarray, A: np.ndarray, z: np.ndarray, w: dict, eps: float, nu: int) -> dict:
    """Diagnostics of one delta-rule update on a non-empty memory (no arithmetic of the method depends on them):
    smallest z.phi(k), range of gamma (Eq. 4), |v_bar| / |v| (how much of the written value is the correction by what
    the memory already holds) and the median of |phi(k)|^2 / eps."""
    f = dpfp(Ym @ w["wm_k"].T, nu)
    zf = f @ z
    f2 = np.sum(f * f, axis=-1)
    gamma = 1.0 - zf / (f2 + eps)
    v = Ym @ w["wm_v"].T
    vbar = (f @ A.T) / (zf + eps)[:, None]
    return dict(min_zf=float(zf.min()), gamma_min=float(gamma.min()), gamma_max=float(gamma.max()),
                vbar_over_v=float(np.linalg.norm(vbar) / max(np.linalg.norm(v), 1e-300)),
                f2_over_eps=float(np.median(f2) / eps) if eps > 0 else float("inf"))


# --------------------------------------------------------------------------- one (layer, segment) cell
def armt_cell(U: np.ndarray, A: np.ndarray, z: np.ndarray, empty: bool, w: dict, cfg):
    """Cell (l, s): read from layer l's memory, run the decoder block, update the memory
    from the block's output at the memory rows (Eq. 2). Returns (Y, A_new, z_new)."""
    if not empty:
        U = assoc_read(U, A, z, w["wm_q"], cfg.assoc_eps, cfg.dpfp_nu)
    Y = llama_block(U, w, cfg)
    A_new, z_new = assoc_update(Y[cfg.seg_len:], A, z, empty, w, cfg.assoc_eps, cfg.dpfp_nu)
    return Y, A_new, z_new


def _prepare(cfg, layers, mem_emb, x, A_in, z_in):
    L, d, P = cfg.n_layers, cfg.d_model, 2 * cfg.dpfp_nu * cfg.d_mem
    x = np.asarray(x, dtype=F64)
    assert x.ndim == 2 and x.shape[1] == d and x.shape[0] % cfg.seg_len == 0 and x.shape[0] > 0
    W = [{k: np.asarray(v, dtype=F64) for k, v in lw.items()} for lw in layers]
    assert len(W) == L
    mem_emb = np.asarray(mem_emb, dtype=F64)
    assert mem_emb.shape == (cfg.n_mem, d)
    if A_in is None:
        assert z_in is None
        A = [np.zeros((d, P), dtype=F64) for _ in range(L)]
        z = [np.zeros(P, dtype=F64) for _ in range(L)]
        empty = [True] * L
    else:
        A = [np.array(A_in[l], dtype=F64) for l in range(L)]
        z = [np.array(z_in[l], dtype=F64) for l in range(L)]
        empty = [False] * L
    return x, W, mem_emb, A, z, empty


def armt_forward_sequential(cfg, layers, mem_emb, x, A_in=None, z_in=None, stats=None, trace=None):
    """Sequential ARMT forward: for each segment, for each layer (Section 3.1).
    x [n_tokens, d] token embeddings; returns (hidden [n_tokens, d], A [L, d, Phi], z [L, Phi]).
    stats, if a list, receives per-cell conditioning figures of the associative read and update; trace, if a list,
    receives per cell (s, l, cell input [T, d] before the read, A^l and z^l before the update): what a backward pass has
    to be given about the forward pass."""
    x, W, mem_emb, A, z, empty = _prepare(cfg, layers, mem_emb, x, A_in, z_in)
    S = cfg.seg_len
    N = x.shape[0] // S
    hidden = np.empty_like(x)
    for s in range(N):
        U = np.concatenate([x[s * S:(s + 1) * S], mem_emb], axis=0)     # [H_s, M]
        for l in range(cfg.n_layers):
            if stats is not None and not empty[l]:
                f = dpfp(U @ W[l]["wm_q"].T, cfg.dpfp_nu)
                den = f @ z[l]
                stats.append(dict(s=s, l=l, min_abs_den=float(np.abs(den).min()),
                                  min_den=float(den.min()), max_den=float(den.max()),
                                  max_abs_read=float(np.abs((f @ A[l].T) / (den + cfg.assoc_eps)[:, None]).max()),
                                  max_abs_A=float(np.abs(A[l]).max()), max_abs_z=float(np.abs(z[l]).max())))
            was_empty, A_old, z_old = empty[l], A[l], z[l]
            if trace is not None:
                trace.append((s, l, U, A_old, z_old))
            U, A[l], z[l] = armt_cell(U, A[l], z[l], empty[l], W[l], cfg)
            if stats is not None and not was_empty:      # the update side of the same cell (U is the cell's output here)
                stats[-1].update(update_conditioning(U[S:], A_old, z_old, W[l], cfg.assoc_eps, cfg.dpfp_nu))
            empty[l] = False
        hidden[s * S:(s + 1) * S] = U[:S]
    return hidden, np.stack(A), np.stack(z)


def diagonal_groups(n_layers: int, n_segments: int):
    """Anti-diagonal schedule of Lemma 3.1: group t holds every cell (l, s) with l + s = t."""
    return [[(l, t - l) for l in range(max(0, t - n_segments + 1), min(n_layers - 1, t) + 1)]
            for t in range(n_layers + n_segments - 1)]


def armt_forward_diagonal_order(cfg, layers, mem_emb, x, A_in=None, z_in=None):
    """The same cells visited group by group in anti-diagonal order (Algorithm 1).
    Every cell of a group reads only results of earlier groups, so the outputs must be
    bit-identical to armt_forward_sequential."""
    x, W, mem_emb, A, z, empty = _prepare(cfg, layers, mem_emb, x, A_in, z_in)
    S = cfg.seg_len
    N = x.shape[0] // S
    hidden = np.empty_like(x)
    cell_in = {}                                    # layer -> input of the cell it runs next
    for t, group in enumerate(diagonal_groups(cfg.n_layers, N)):
        if t < N:                                   # ingest a new segment at layer 0
            cell_in[0] = np.concatenate([x[t * S:(t + 1) * S], mem_emb], axis=0)
        results = {}
        for (l, s) in group:                        # independent cells: any order within the group
            results[l] = armt_cell(cell_in[l], A[l], z[l], empty[l], W[l], cfg)
        nxt = {}
        for (l, s) in group:
            Y, A[l], z[l] = results[l]
            empty[l] = False
            if l + 1 < cfg.n_layers:
                nxt[l + 1] = Y                      # same segment, one layer deeper, next group
            else:
                hidden[s * S:(s + 1) * S] = Y[:S]   # segment went through all layers
        cell_in = nxt
    return hidden, np.stack(A), np.stack(z)


# --------------------------------------------------------------------------- token-level ends (Algorithm 1)
def embed_tokens(ids: np.ndarray, emb_table: np.ndarray) -> np.ndarray:
    """x[i] = emb_table[ids[i]]: Algorithm 1 starts from token ids, the cells from embeddings."""
    ids = np.asarray(ids)
    E = np.asarray(emb_table, dtype=F64)
    if ids.size and (ids.min() < 0 or ids.max() >= E.shape[0]):
        raise ValueError("token id outside the vocabulary")
    return E[ids]


def lm_head(hidden: np.ndarray, final_gain: np.ndarray, w_lm: np.ndarray, eps: float) -> np.ndarray:
    """logits = rmsnorm(hidden, final_gain) W_lm^T, W_lm [vocab, d] (Algorithm 1 returns logits)."""
    return rmsnorm(hidden, final_gain, eps) @ np.asarray(w_lm, dtype=F64).T


def armt_forward_tokens(cfg, layers, mem_emb, emb_table, ids, final_gain, w_lm, last_rows=None):
    """Token ids -> logits: gather, the ARMT forward, final norm + head on all rows or on the last
    `last_rows` rows. Returns (logits, hidden, A, z)."""
    x = embed_tokens(ids, emb_table)
    hidden, A, z = armt_forward_sequential(cfg, layers, mem_emb, x)
    rows = hidden if last_rows is None else hidden[-last_rows:]
    return lm_head(rows, final_gain, w_lm, cfg.rms_eps), hidden, A, z


# --------------------------------------------------------------------------- batch (Section 4.3)
def armt_forward_batched(cfg, layers, mem_emb, x):
    """B independent sequences x [B, n_tokens, d]: by definition each one's own sequential result.
    Returns (hidden [B, n_tokens, d], A [B, L, d, Phi], z [B, L, Phi])."""
    outs = [armt_forward_sequential(cfg, layers, mem_emb, xb) for xb in x]
    return tuple(np.stack([o[i] for o in outs]) for i in range(3))
