"""Pins of the CPU oracle to things other than itself (all run without a GPU).

Each test names what fixes the expected value: a hand-worked fixture, a closed form
derived from Eq. 3-6 of the paper, a library routine, an invariant the paper states
(exact recurrence, dependency rule of Section 3.1, Lemma 3.1), or a brute-force
recomputation written separately in pure Python.
"""
import cmath
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import armt_synth as S
from oracle import armt_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def tiny_cfg(**kw):
    base = dict(name="t", n_layers=2, d_model=8, n_heads=2, n_kv_heads=1, head_dim=4, d_ff=12,
                seg_len=3, n_mem=2, d_mem=2, n_tokens=9, dtype="f32")
    base.update(kw)
    return S.ArmtShape(**base)


def rand_problem(cfg, seed=0, std=0.5, gain_std=0.2, mem_std=1.0):
    """Small problems use large weights so that every term (read, update, gains) matters."""
    layers, _ = S.make_weights(cfg, seed=seed, std=std, gain_std=gain_std)
    rng = np.random.default_rng(seed + 100)
    mem_emb = rng.standard_normal((cfg.n_mem, cfg.d_model)) * mem_std
    x = S.make_embeddings(cfg, seed=seed)
    return layers, mem_emb, x


# ------------------------------------------------------------------ DPFP (Section 2.1, phi)
def test_dpfp_handworked_fixture():
    n = 0
    for line in open(os.path.join(GOLDEN, "dpfp_handworked.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        nu, xs, ys = [p.strip() for p in line.split(";")]
        x = np.array([float(v) for v in xs.split()])
        want = np.array([float(v) for v in ys.split()])
        got = O.dpfp(x, int(nu))
        assert got.shape == want.shape
        assert np.array_equal(got, want), (line, got)
        n += 1
    assert n >= 4


def test_dpfp_properties():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((7, 16))
    f = O.dpfp(x, 3)
    assert f.shape == (7, 6 * 16)                    # A in R^{d_model x 6 d_mem}
    assert (f >= 0).all()
    # exactly one of relu(x_i), relu(-x_i) is non-zero, so each product is non-zero
    # only where both partners are; scaling x by c > 0 scales phi by c^2
    assert np.allclose(O.dpfp(2.5 * x, 3), 6.25 * f)
    # explicit index form of the definition
    r = np.concatenate([np.maximum(x, 0), np.maximum(-x, 0)], -1)
    for j in (1, 2, 3):
        for i in range(32):
            assert np.array_equal(f[:, (j - 1) * 32 + i], r[:, i] * r[:, (i - j) % 32])
    # phi(x) and phi(-x) hold the same products, moved by half a period
    g = O.dpfp(-x, 3)
    for j in range(3):
        blk_f, blk_g = f[:, j * 32:(j + 1) * 32], g[:, j * 32:(j + 1) * 32]
        assert np.allclose(np.roll(blk_f, 16, axis=-1), blk_g)


# ------------------------------------------------------------------ LLaMA block pieces
def test_rmsnorm_invariants():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((5, 32)) * 3
    y = O.rmsnorm(x, np.ones(32), 0.0)
    assert np.allclose(np.sqrt((y * y).mean(-1)), 1.0)
    assert np.allclose(O.rmsnorm(7.0 * x, np.ones(32), 0.0), y)
    g = rng.standard_normal(32)
    assert np.allclose(O.rmsnorm(x, g, 0.0), y * g)
    t = F.rms_norm(torch.from_numpy(x), (32,), torch.from_numpy(g), eps=1e-5).numpy()
    assert np.allclose(O.rmsnorm(x, g, 1e-5), t, rtol=1e-12, atol=1e-12)


def test_rope_invariants():
    rng = np.random.default_rng(3)
    T, H, dh, theta = 9, 3, 8, 500000.0
    x = rng.standard_normal((T, H, dh))
    y = O.rope(x, theta)
    assert np.allclose(y[0], x[0])                                   # position 0 is the identity
    assert np.allclose((y * y).sum(-1), (x * x).sum(-1))             # rotations preserve norms
    # complex form: (x_j + i x_{j+dh/2}) * exp(i p theta^(-2j/dh))
    for p in range(T):
        for j in range(dh // 2):
            w = cmath.exp(1j * p * theta ** (-2.0 * j / dh))
            for h in range(H):
                c = complex(x[p, h, j], x[p, h, j + dh // 2]) * w
                assert abs(c.real - y[p, h, j]) < 1e-12 and abs(c.imag - y[p, h, j + dh // 2]) < 1e-12
    # relative-position property: <rope(q)_p, rope(k)_r> depends on p - r only
    q = np.broadcast_to(rng.standard_normal((1, 1, dh)), (T, 1, dh)).copy()
    k = np.broadcast_to(rng.standard_normal((1, 1, dh)), (T, 1, dh)).copy()
    rq, rk = O.rope(q, theta)[:, 0], O.rope(k, theta)[:, 0]
    dots = rq @ rk.T
    for delta in range(-3, 4):
        diag = np.diagonal(dots, offset=-delta)
        assert np.allclose(diag, diag[0])
    # a small theta makes the angles large enough that a sign error shows
    y2 = O.rope(x, 10.0)
    assert not np.allclose(y2[1:], x[1:], atol=1e-2)


def test_attention_matches_library_sdpa():
    rng = np.random.default_rng(4)
    T, H, Hkv, dh = 13, 6, 2, 8
    q, k, v = (rng.standard_normal((T, n, dh)) for n in (H, Hkv, Hkv))
    got = O.causal_gqa_attention(q, k, v)
    tq, tk, tv = (torch.from_numpy(a).permute(1, 0, 2)[None] for a in (q, k, v))
    want = F.scaled_dot_product_attention(tq, tk, tv, is_causal=True, enable_gqa=True)[0].permute(1, 0, 2).numpy()
    assert np.allclose(got, want, rtol=1e-12, atol=1e-12)
    assert np.allclose(got[0], np.repeat(v[0], H // Hkv, axis=0))     # first row sees one key only
    # constant values: any convex combination returns the constant
    vc = np.ones((T, Hkv, dh)) * 3.0
    assert np.allclose(O.causal_gqa_attention(q, k, vc), 3.0)


def _library_block(U, w, cfg):
    """A LLaMA decoder block from library routines only, written apart from the oracle."""
    T = U.shape[0]
    H, Hkv, dh = cfg.n_heads, cfg.n_kv_heads, cfg.head_dim
    t = {k_: torch.from_numpy(np.asarray(v_, dtype=np.float64)) for k_, v_ in w.items()}
    x = torch.from_numpy(np.asarray(U, dtype=np.float64))

    def rot(a):     # [T, n, dh] -> rotary via complex multiplication on pairs (j, j + dh/2)
        half = dh // 2
        inv = cfg.rope_theta ** (-torch.arange(half, dtype=torch.float64) * 2.0 / dh)
        ang = torch.arange(T, dtype=torch.float64)[:, None] * inv[None]
        ph = torch.polar(torch.ones_like(ang), ang)[:, None, :]
        c = torch.complex(a[..., :half], a[..., half:]) * ph
        return torch.cat([c.real, c.imag], -1)

    n = F.rms_norm(x, (cfg.d_model,), t["rms1"], eps=cfg.rms_eps)
    q = rot(F.linear(n, t["wq"]).view(T, H, dh)).permute(1, 0, 2)[None]
    k = rot(F.linear(n, t["wk"]).view(T, Hkv, dh)).permute(1, 0, 2)[None]
    v = F.linear(n, t["wv"]).view(T, Hkv, dh).permute(1, 0, 2)[None]
    a = F.scaled_dot_product_attention(q, k, v, is_causal=True, enable_gqa=True)[0].permute(1, 0, 2).reshape(T, H * dh)
    h = x + F.linear(a, t["wo"])
    n2 = F.rms_norm(h, (cfg.d_model,), t["rms2"], eps=cfg.rms_eps)
    return (h + F.linear(F.silu(F.linear(n2, t["wgate"])) * F.linear(n2, t["wup"]), t["wdown"])).numpy()


def test_block_matches_library_transformer():
    cfg = S.get_shape("tiny")
    layers, mem_emb = S.make_weights(cfg, seed=5, std=0.2, gain_std=0.3)
    U = np.random.default_rng(5).standard_normal((cfg.T, cfg.d_model))
    got = O.llama_block(U, {k: v.astype(np.float64) for k, v in layers[0].items()}, cfg)
    want = _library_block(U, layers[0], cfg)
    assert np.allclose(got, want, rtol=1e-10, atol=1e-10)


def test_degenerate_armt_without_memory_is_a_plain_transformer():
    """With W_V^mem = 0 nothing is ever written to A, every read returns 0 and each segment is an
    independent decoder stack on [H_s, M] ("parallel RMT ... without memory association and
    update", Section 3.2)."""
    cfg = S.get_shape("tiny").replace(n_tokens=3 * 64)
    layers, mem_emb = S.make_weights(cfg, seed=6, std=0.2, gain_std=0.3)
    for lw in layers:
        lw["wm_v"][:] = 0.0
    x = S.make_embeddings(cfg, seed=6)
    hid, A, z = O.armt_forward_sequential(cfg, layers, mem_emb, x)
    assert np.all(A == 0.0) and np.abs(z).max() > 0.0
    for s in range(cfg.n_segments):
        U = np.concatenate([x[s * 64:(s + 1) * 64].astype(np.float64), mem_emb.astype(np.float64)], 0)
        for l in range(cfg.n_layers):
            U = _library_block(U, layers[l], cfg)
        assert np.allclose(hid[s * 64:(s + 1) * 64], U[:64], rtol=1e-9, atol=1e-9)


# ------------------------------------------------------------------ associative memory closed forms
def _one_token_weights(d, dm, k, v, b):
    """Weights such that the memory token e_0 produces exactly key k, value v, gate logit b."""
    w = dict(wm_k=np.zeros((dm, d)), wm_v=np.zeros((d, d)), wm_b=np.zeros((1, d)), wm_q=np.zeros((dm, d)))
    w["wm_k"][:, 0] = k
    w["wm_v"][:, 0] = v
    w["wm_b"][0, 0] = b
    w["wm_q"][:, 1] = k            # the query e_1 looks the same key up
    return w


def test_first_write_and_read_back_closed_form():
    rng = np.random.default_rng(7)
    d, dm, nu = 6, 4, 3
    k, v, b = rng.standard_normal(dm), rng.standard_normal(d), 0.3
    beta = 1 / (1 + math.exp(-b))
    w = _one_token_weights(d, dm, k, v, b)
    e0, e1 = np.eye(d)[0:1], np.eye(d)[1:2]
    A, z = O.assoc_update(e0, np.zeros((d, 6 * dm)), np.zeros(6 * dm), True, w, 0.0, nu)
    f = O.dpfp(k, nu)
    assert np.allclose(z, f)                                   # gamma = 1 - 0
    assert np.allclose(A, beta * np.outer(v, f))               # A = beta v (x) phi(k)
    back = O.assoc_read(e1, A, z, w["wm_q"], 0.0, nu)          # A f / z^T f = beta v |f|^2 / |f|^2
    assert np.allclose(back - e1, beta * v[None, :], rtol=1e-12, atol=1e-12)
    # querying c*k (c > 0) returns the same value: phi is homogeneous, numerator and denominator scale alike
    w2 = dict(w)
    w2["wm_q"] = 3.0 * w["wm_q"]
    assert np.allclose(O.assoc_read(e1, A, z, w2["wm_q"], 0.0, nu) - e1, beta * v[None, :])


def test_overwrite_is_delta_rule_interpolation():
    rng = np.random.default_rng(8)
    d, dm, nu = 5, 3, 3
    k, v1, v2 = rng.standard_normal(dm), rng.standard_normal(d), rng.standard_normal(d)
    b1, b2 = -0.4, 1.1
    be1, be2 = 1 / (1 + math.exp(-b1)), 1 / (1 + math.exp(-b2))
    e0, e1 = np.eye(d)[0:1], np.eye(d)[1:2]
    A, z = O.assoc_update(e0, np.zeros((d, 6 * dm)), np.zeros(6 * dm), True, _one_token_weights(d, dm, k, v1, b1), 0.0, nu)
    w = _one_token_weights(d, dm, k, v2, b2)
    A2, z2 = O.assoc_update(e0, A, z, False, w, 0.0, nu)
    assert np.allclose(z2, z)                                  # gamma = 1 - |f|^2/|f|^2 = 0
    want = be1 * v1 + be2 * (v2 - be1 * v1)                    # v_bar = beta1 v1
    assert np.allclose(O.assoc_read(e1, A2, z2, w["wm_q"], 0.0, nu) - e1, want[None, :], rtol=1e-12, atol=1e-12)


def test_orthogonal_keys_do_not_interfere_and_share_the_old_state():
    d, dm, nu = 4, 4, 3
    k1, k2 = np.array([1.0, 2.0, 0, 0]), np.array([0, 0, 3.0, 1.0])
    f1, f2 = O.dpfp(k1, nu), O.dpfp(k2, nu)
    assert f1 @ f2 == 0.0 and f1 @ f1 > 0 and f2 @ f2 > 0
    rng = np.random.default_rng(9)
    v = rng.standard_normal((2, d))
    w = dict(wm_k=np.zeros((dm, d)), wm_v=np.zeros((d, d)), wm_b=np.zeros((1, d)))
    w["wm_k"][:, 0], w["wm_k"][:, 1] = k1, k2
    w["wm_v"][:, 0], w["wm_v"][:, 1] = v[0], v[1]
    w["wm_b"][0, :2] = [0.7, -0.2]
    be = 1 / (1 + np.exp(-np.array([0.7, -0.2])))
    Ym = np.eye(d)[:2]
    A, z = O.assoc_update(Ym, np.zeros((d, 6 * dm)), np.zeros(6 * dm), True, w, 0.0, nu)
    wq = np.zeros((dm, d))
    wq[:, 2], wq[:, 3] = k1, k2
    U = np.eye(d)[2:4]
    rd = O.assoc_read(U, A, z, wq, 0.0, nu) - U
    assert np.allclose(rd[0], be[0] * v[0]) and np.allclose(rd[1], be[1] * v[1])
    # two tokens with the SAME key written together both see the old (empty) state:
    # A = (beta_a v_a + beta_b v_b) (x) f, z = 2 f  ->  read = (beta_a v_a + beta_b v_b) / 2
    w["wm_k"][:, 1] = k1
    A, z = O.assoc_update(Ym, np.zeros((d, 6 * dm)), np.zeros(6 * dm), True, w, 0.0, nu)
    assert np.allclose(z, 2 * f1)
    rd = O.assoc_read(U[:1], A, z, wq, 0.0, nu) - U[:1]
    assert np.allclose(rd[0], (be[0] * v[0] + be[1] * v[1]) / 2)


# ------------------------------------------------------------------ brute force, written separately
def _brute_force(cfg, layers, mem_emb, x):
    """Pure-python float64 recomputation straight from Eq. 2-6: naive loops, explicit T x T masked
    softmax, rotary by complex multiplication, and the memory A_s of each layer REBUILT at every use
    as the sum of all outer products stored by earlier segments."""
    L, d, H, Hkv, dh, Fd = cfg.n_layers, cfg.d_model, cfg.n_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_ff
    S_, m, dm, nu, T = cfg.seg_len, cfg.n_mem, cfg.d_mem, cfg.dpfp_nu, cfg.T
    P = 2 * nu * dm
    eps = cfg.assoc_eps
    W = [{k: np.asarray(v, dtype=np.float64).tolist() for k, v in lw.items()} for lw in layers]
    x = np.asarray(x, dtype=np.float64).tolist()
    mem_emb = np.asarray(mem_emb, dtype=np.float64).tolist()

    def matvec(Wm, vec):
        return [sum(Wm[o][i] * vec[i] for i in range(len(vec))) for o in range(len(Wm))]

    def phi(k):
        r = [max(a, 0.0) for a in k] + [max(-a, 0.0) for a in k]
        n = len(r)
        return [r[i] * r[(i - j) % n] for j in range(1, nu + 1) for i in range(n)]

    def rms(vec, g):
        ms = sum(a * a for a in vec) / len(vec)
        return [a / math.sqrt(ms + cfg.rms_eps) * gg for a, gg in zip(vec, g)]

    def rot(vec, p):    # one head
        out = [0.0] * dh
        for j in range(dh // 2):
            c = complex(vec[j], vec[j + dh // 2]) * cmath.exp(1j * p * cfg.rope_theta ** (-2.0 * j / dh))
            out[j], out[j + dh // 2] = c.real, c.imag
        return out

    writes = [[] for _ in range(L)]      # per layer: list of (coef[d], f[P]) and (gamma, f)

    def mem_A_times(l, f):               # A f with A rebuilt from the stored writes
        out = [0.0] * d
        for coef, fw, _ in writes[l]:
            dot = sum(a * b for a, b in zip(fw, f))
            for r_ in range(d):
                out[r_] += coef[r_] * dot
        return out

    def mem_z_dot(l, f):
        return sum(g * sum(a * b for a, b in zip(fw, f)) for _, fw, g in writes[l])

    hidden = []
    for s in range(len(x) // S_):
        U = [row[:] for row in x[s * S_:(s + 1) * S_]] + [row[:] for row in mem_emb]
        for l in range(L):
            w = W[l]
            if writes[l]:
                for i in range(T):
                    f = phi(matvec(w["wm_q"], U[i]))
                    num, den = mem_A_times(l, f), mem_z_dot(l, f) + eps
                    U[i] = [U[i][r_] + num[r_] / den for r_ in range(d)]
            q, k, v = [], [], []
            for i in range(T):
                n = rms(U[i], w["rms1"])
                qi, ki, vi = matvec(w["wq"], n), matvec(w["wk"], n), matvec(w["wv"], n)
                q.append([rot(qi[h * dh:(h + 1) * dh], i) for h in range(H)])
                k.append([rot(ki[g * dh:(g + 1) * dh], i) for g in range(Hkv)])
                v.append([vi[g * dh:(g + 1) * dh] for g in range(Hkv)])
            Y = []
            for i in range(T):
                att = []
                for h in range(H):
                    g = h // (H // Hkv)
                    sc = [sum(q[i][h][c] * k[j][g][c] for c in range(dh)) / math.sqrt(dh) for j in range(i + 1)]
                    mx = max(sc)
                    e = [math.exp(a - mx) for a in sc]
                    tot = sum(e)
                    att += [sum(e[j] / tot * v[j][g][c] for j in range(i + 1)) for c in range(dh)]
                o = matvec(w["wo"], att)
                hres = [U[i][r_] + o[r_] for r_ in range(d)]
                n2 = rms(hres, w["rms2"])
                gt, up = matvec(w["wgate"], n2), matvec(w["wup"], n2)
                act = [a / (1 + math.exp(-a)) * b for a, b in zip(gt, up)]
                dn = matvec(w["wdown"], act)
                Y.append([hres[r_] + dn[r_] for r_ in range(d)])
            new = []
            for i in range(S_, T):
                f = phi(matvec(w["wm_k"], Y[i]))
                vv = matvec(w["wm_v"], Y[i])
                beta = 1 / (1 + math.exp(-matvec(w["wm_b"], Y[i])[0]))
                zf = mem_z_dot(l, f)
                if writes[l]:
                    af = mem_A_times(l, f)
                    vbar = [a / (zf + eps) for a in af]
                else:
                    vbar = [0.0] * d
                gamma = 1 - zf / (sum(a * a for a in f) + eps)
                new.append(([beta * (vv[r_] - vbar[r_]) for r_ in range(d)], f, gamma))
            writes[l] += new          # all memory tokens of the segment saw the old state
            U = Y
        hidden += U[:S_]
    A = np.zeros((L, d, P))
    z = np.zeros((L, P))
    for l in range(L):
        for coef, f, g in writes[l]:
            A[l] += np.outer(coef, f)
            z[l] += g * np.asarray(f)
    return np.asarray(hidden), A, z


@pytest.mark.parametrize("seed,kw", [
    (0, {}),
    (1, dict(n_layers=3, n_heads=4, n_kv_heads=2, head_dim=2, n_tokens=12)),
    (2, dict(n_layers=1, n_heads=2, n_kv_heads=2, n_mem=1, seg_len=2, n_tokens=8, dpfp_nu=2)),
])
def test_forward_matches_brute_force(seed, kw):
    cfg = tiny_cfg(rope_theta=10.0, **kw)
    layers, mem_emb, x = rand_problem(cfg, seed)
    hid, A, z = O.armt_forward_sequential(cfg, layers, mem_emb, x)
    bh, bA, bz = _brute_force(cfg, layers, mem_emb, x)
    assert np.allclose(hid, bh, rtol=1e-9, atol=1e-10)
    assert np.allclose(A, bA, rtol=1e-8, atol=1e-10)
    assert np.allclose(z, bz, rtol=1e-8, atol=1e-10)
    # the memory path is not a rounding-level effect in this problem
    layers0 = [dict(lw) for lw in layers]
    for lw in layers0:
        lw["wm_v"] = np.zeros_like(lw["wm_v"])
    hid0, _, _ = O.armt_forward_sequential(cfg, layers0, mem_emb, x)
    assert np.abs(hid - hid0)[cfg.seg_len:].max() > 1e-3


# ------------------------------------------------------------------ recurrence invariants
def _problem(seed=0, n_seg=5, **kw):
    cfg = S.get_shape("tiny").replace(n_layers=3, d_model=32, n_heads=4, n_kv_heads=2, head_dim=8,
                                      d_ff=48, seg_len=6, n_mem=3, d_mem=4, n_tokens=6 * n_seg, **kw)
    layers, mem_emb, x = rand_problem(cfg, seed, std=0.2)
    return cfg, layers, mem_emb, x


def test_diagonal_order_is_bit_identical_to_sequential():
    """Exact recurrence: the anti-diagonal order only reorders independent cells (Lemma 3.1)."""
    for n_seg in (1, 2, 3, 7):
        cfg, layers, mem_emb, x = _problem(10 + n_seg, n_seg)
        a = O.armt_forward_sequential(cfg, layers, mem_emb, x)
        b = O.armt_forward_diagonal_order(cfg, layers, mem_emb, x)
        for u, v in zip(a, b):
            assert u.tobytes() == v.tobytes()
    cfg = S.get_shape("tiny")
    layers, mem_emb = S.make_weights(cfg, seed=0)
    x = S.make_embeddings(cfg, seed=0)
    a = O.armt_forward_sequential(cfg, layers, mem_emb, x)
    b = O.armt_forward_diagonal_order(cfg, layers, mem_emb, x)
    for u, v in zip(a, b):
        assert u.tobytes() == v.tobytes()


def test_lemma31_group_fixture():
    for line in open(os.path.join(GOLDEN, "lemma31_groups.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        lhs, rhs = line.split(":")
        L, N = (int(v) for v in lhs.split())
        sizes = [int(v) for v in rhs.split()]
        groups = O.diagonal_groups(L, N)
        assert len(groups) == L + N - 1 == len(sizes)
        assert [len(g) for g in groups] == sizes
        seen = set()
        for t, g in enumerate(groups):
            for (l, s) in g:
                assert l + s == t and 0 <= l < L and 0 <= s < N
                seen.add((l, s))
        assert len(seen) == L * N


def test_prefix_and_perturbation():
    """Cell (s, l) depends only on (s, l-1) and (s-1, l) (Section 3.1): outputs of segments < s'
    and the memory after segment s'-1 do not change when segment s' changes, and a run on the
    first k segments equals the first k segments of a longer run."""
    cfg, layers, mem_emb, x = _problem(20, 5)
    Sg = cfg.seg_len
    hid, A, z = O.armt_forward_sequential(cfg, layers, mem_emb, x)
    x2 = x.copy()
    x2[3 * Sg:4 * Sg] += 1.0
    hid2, _, _ = O.armt_forward_sequential(cfg, layers, mem_emb, x2)
    assert hid[:3 * Sg].tobytes() == hid2[:3 * Sg].tobytes()
    assert np.abs(hid[3 * Sg:4 * Sg] - hid2[3 * Sg:4 * Sg]).max() > 1e-3
    assert np.abs(hid[4 * Sg:] - hid2[4 * Sg:]).max() > 1e-6      # later segments see it through memory
    hk, Ak, zk = O.armt_forward_sequential(cfg, layers, mem_emb, x[:3 * Sg])
    assert hk.tobytes() == hid[:3 * Sg].tobytes()
    # carry-in: [0, k) then [k, N) from the exported state == one full run
    ht, At, zt = O.armt_forward_sequential(cfg, layers, mem_emb, x[3 * Sg:], A_in=Ak, z_in=zk)
    assert ht.tobytes() == hid[3 * Sg:].tobytes()
    assert At.tobytes() == A.tobytes() and zt.tobytes() == z.tobytes()
    # within a segment the block is causal: changing the last token of a segment leaves earlier rows alone
    x3 = x.copy()
    x3[Sg - 1] += 1.0
    hid3, _, _ = O.armt_forward_sequential(cfg, layers, mem_emb, x3)
    assert hid3[:Sg - 1].tobytes() == hid[:Sg - 1].tobytes()


def test_single_segment_has_no_memory_effect():
    """With one segment diagonal and sequential coincide trivially (the paper's error table prints
    0.00 % at one segment) and the result is the plain decoder stack on [H, M]."""
    cfg, layers, mem_emb, x = _problem(30, 1)
    hid, A, z = O.armt_forward_sequential(cfg, layers, mem_emb, x)
    U = np.concatenate([x.astype(np.float64), mem_emb], 0)
    for l in range(cfg.n_layers):
        U = _library_block(U, layers[l], cfg)
    assert np.allclose(hid, U[:cfg.seg_len], rtol=1e-10, atol=1e-10)
    assert np.abs(A).max() > 0


def test_read_is_well_conditioned_on_the_synthetic_workload():
    """Denominators z^T phi(.) stay positive on the N(0, 0.02) workload (z and phi are sums of
    non-negative terms as long as gamma stays positive), so parity on it is meaningful."""
    cfg = S.get_shape("tiny")
    layers, mem_emb = S.make_weights(cfg, seed=0)
    x = S.make_embeddings(cfg, seed=0)
    st = []
    hid, A, z = O.armt_forward_sequential(cfg, layers, mem_emb, x, stats=st)
    assert len(st) == cfg.n_layers * (cfg.n_segments - 1)
    assert all(e["min_den"] > 0 for e in st)
    assert np.isfinite(hid).all() and np.isfinite(A).all()
