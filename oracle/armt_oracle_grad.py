"""CPU oracle for the ARMT backward pass -- TEST INFRASTRUCTURE, NOT THE PRODUCT.

The paper states only that a backward pass of the diagonal schedule exists (appendix on
implementation notes); what it must compute is fixed by the forward: the gradient of a
scalar J = <hidden, G_h> + <A_out, G_A> + <z_out, G_z> with respect to every input of the
sequential ARMT forward (Section 2.1, Eq. 2-6; Section 3.1), for given upstream gradients
G_h, G_A, G_z.  Diagonal order only reorders independent cells, so its gradients are the
same numbers.

The oracle is that definition written out: the forward restated in float64 torch CPU ops in
the sequential order (segment by segment, layer by layer), differentiated by the library's
reverse-mode autograd.  Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline
leg may import this module; it shares no code with the HIP path.

Parity status (tests/test_oracle_grad.py):
  forward restated here     equals oracle/armt_oracle.py (numpy) to 1e-9 of the largest value, tiny shapes
  armt_grad                 central finite differences of the NUMPY forward in every input
                            (weights, memory embeddings, token embeddings, carried-in A, z);
                            closed forms: d<hidden,G>/dx for a one-segment, empty-memory run
                            equals the decoder block's library gradient; linearity in (G_h, G_A, G_z);
                            zero gradient of earlier hidden states with respect to later segments

  lm_head_grad              finite differences of the numpy lm_head; library rms_norm + linear differentiated by the library
  embed_tokens_grad         a table of ones-hot rows (each row's gradient counts its occurrences); pure-python loop

Readings taken here: the same as in the forward oracle; in addition the decision "memory
empty -> skip the read and use v_bar = 0" is a constant of the run (not differentiated), and
the gradient with respect to A_in, z_in is reported only when a state was carried in.
"""
from __future__ import annotations

import numpy as np
import torch

F64 = torch.float64
WEIGHT_KEYS = ("rms1", "wq", "wk", "wv", "wo", "rms2", "wgate", "wup", "wdown", "wm_q", "wm_k", "wm_v", "wm_b")


def dpfp(x: torch.Tensor, nu: int) -> torch.Tensor:
    r = torch.cat([torch.relu(x), torch.relu(-x)], dim=-1)
    return torch.cat([r * torch.roll(r, j, dims=-1) for j in range(1, nu + 1)], dim=-1)


def rmsnorm(x, gain, eps):
    return x / torch.sqrt(torch.mean(x * x, dim=-1, keepdim=True) + eps) * gain


def rope(x, theta):
    T, _, dh = x.shape
    half = dh // 2
    inv_freq = theta ** (-2.0 * torch.arange(half, dtype=F64) / dh)
    ang = torch.arange(T, dtype=F64)[:, None] * inv_freq[None, :]
    c, s = torch.cos(ang)[:, None, :], torch.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return torch.cat([x1 * c - x2 * s, x2 * c + x1 * s], dim=-1)


def causal_gqa_attention(q, k, v):
    T, H, dh = q.shape
    rep = H // k.shape[1]
    mask = torch.tril(torch.ones(T, T, dtype=torch.bool))
    outs = []
    for h in range(H):
        g = h // rep
        sc = (q[:, h, :] @ k[:, g, :].T) / float(np.sqrt(dh))
        sc = sc.masked_fill(~mask, float("-inf"))
        outs.append(torch.softmax(sc, dim=-1) @ v[:, g, :])
    return torch.stack(outs, dim=1)


def llama_block(U, w, cfg):
    T = U.shape[0]
    H, Hkv, dh = cfg.n_heads, cfg.n_kv_heads, cfg.head_dim
    n = rmsnorm(U, w["rms1"], cfg.rms_eps)
    q = rope((n @ w["wq"].T).reshape(T, H, dh), cfg.rope_theta)
    k = rope((n @ w["wk"].T).reshape(T, Hkv, dh), cfg.rope_theta)
    v = (n @ w["wv"].T).reshape(T, Hkv, dh)
    a = causal_gqa_attention(q, k, v).reshape(T, H * dh)
    h = U + a @ w["wo"].T
    n2 = rmsnorm(h, w["rms2"], cfg.rms_eps)
    g = n2 @ w["wgate"].T
    return h + ((g * torch.sigmoid(g)) * (n2 @ w["wup"].T)) @ w["wdown"].T


def armt_cell(U, A, z, empty, w, cfg):
    eps, nu = cfg.assoc_eps, cfg.dpfp_nu
    if not empty:                                             # Eq. 6, added to its input
        f = dpfp(U @ w["wm_q"].T, nu)
        U = U + (f @ A.T) / (f @ z + eps)[:, None]
    Y = llama_block(U, w, cfg)
    Ym = Y[cfg.seg_len:]                                      # Eq. 3-5 on the memory rows of the output
    k = Ym @ w["wm_k"].T
    v = Ym @ w["wm_v"].T
    beta = torch.sigmoid((Ym @ w["wm_b"].T)[:, 0])
    f = dpfp(k, nu)
    zf = f @ z
    vbar = torch.zeros_like(v) if empty else (f @ A.T) / (zf + eps)[:, None]
    gamma = 1.0 - zf / ((f * f).sum(-1) + eps)
    return Y, A + (beta[:, None] * (v - vbar)).T @ f, z + gamma @ f


def _leaf(a):
    return torch.tensor(np.asarray(a, dtype=np.float64), dtype=F64, requires_grad=True)


def armt_forward_torch(cfg, W, mem_emb, x, A_in=None, z_in=None):
    """Sequential forward on torch tensors (leaves may require grad). Returns (hidden, A [L,...], z)."""
    L, d, P = cfg.n_layers, cfg.d_model, 2 * cfg.dpfp_nu * cfg.d_mem
    S = cfg.seg_len
    N = x.shape[0] // S
    assert x.shape[0] == N * S and N > 0
    if A_in is None:
        A = [torch.zeros(d, P, dtype=F64) for _ in range(L)]
        z = [torch.zeros(P, dtype=F64) for _ in range(L)]
        empty = [True] * L
    else:
        A, z, empty = [A_in[l] for l in range(L)], [z_in[l] for l in range(L)], [False] * L
    hidden = []
    for s in range(N):
        U = torch.cat([x[s * S:(s + 1) * S], mem_emb], dim=0)
        for l in range(L):
            U, A[l], z[l] = armt_cell(U, A[l], z[l], empty[l], W[l], cfg)
            empty[l] = False
        hidden.append(U[:S])
    return torch.cat(hidden, dim=0), torch.stack(A), torch.stack(z)


def armt_grad(cfg, layers, mem_emb, x, G_h, G_A=None, G_z=None, A_in=None, z_in=None):
    """Gradient of J = <hidden, G_h> + <A_out, G_A> + <z_out, G_z> (missing G = 0).
    Returns a dict: "layers" (list of dicts, one array per weight), "mem_emb", "x", and
    "A_in", "z_in" (None without a carried-in state); plus "hidden", "A", "z" of the forward."""
    W = [{k: _leaf(lw[k]) for k in WEIGHT_KEYS} for lw in layers]
    me, xx = _leaf(mem_emb), _leaf(x)
    Ai = None if A_in is None else _leaf(A_in)
    zi = None if z_in is None else _leaf(z_in)
    hidden, A, z = armt_forward_torch(cfg, W, me, xx, Ai, zi)
    J = (hidden * torch.as_tensor(np.asarray(G_h, dtype=np.float64))).sum()
    if G_A is not None:
        J = J + (A * torch.as_tensor(np.asarray(G_A, dtype=np.float64))).sum()
    if G_z is not None:
        J = J + (z * torch.as_tensor(np.asarray(G_z, dtype=np.float64))).sum()
    J.backward()

    def g(t):
        return np.zeros(tuple(t.shape)) if t.grad is None else t.grad.numpy().copy()

    return {"layers": [{k: g(w[k]) for k in WEIGHT_KEYS} for w in W], "mem_emb": g(me), "x": g(xx),
            "A_in": None if Ai is None else g(Ai), "z_in": None if zi is None else g(zi),
            "hidden": hidden.detach().numpy(), "A": A.detach().numpy(), "z": z.detach().numpy(), "J": float(J.detach())}


# --------------------------------------------------------------------------- token-level ends (Algorithm 1)
def lm_head_grad(hidden, final_gain, w_lm, eps, G_logits):
    """Gradient of <logits, G_logits>, logits = rmsnorm(hidden, final_gain) W_lm^T, with respect to hidden, final_gain
    and W_lm (autograd of the definition).  Returns (d_hidden, d_final_gain, d_w_lm)."""
    h, g, w = _leaf(hidden), _leaf(final_gain), _leaf(w_lm)
    logits = rmsnorm(h, g, eps) @ w.T
    (logits * torch.as_tensor(np.asarray(G_logits, dtype=np.float64))).sum().backward()
    return h.grad.numpy().copy(), g.grad.numpy().copy(), w.grad.numpy().copy()


def embed_tokens_grad(ids, dx, vocab):
    """Backward of the gather x[i] = table[ids[i]]: every row of dx is added to the table row it was read from."""
    out = np.zeros((vocab, np.asarray(dx).shape[1]))
    np.add.at(out, np.asarray(ids), np.asarray(dx, dtype=np.float64))
    return out

