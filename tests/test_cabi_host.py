"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the header
declares, implements the anti-diagonal schedule of Lemma 3.1, sizes its workspace, and turns bad
arguments into error codes before anything is launched."""
import ctypes as C
import os
import re

import pytest

import armt_synth as S

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module")
def lib():
    import paper_2506_05229_amd as P
    if not os.path.exists(P.library_path()):
        from paper_2506_05229_amd.build import build
        build()
    return P.load_library()


def _cfg(shape):
    import paper_2506_05229_amd as P
    return P.ArmtConfig.from_shape(shape)


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "armt.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = sorted(set(re.findall(r"\b(armt_[a-z0-9_]+)\s*\(", header)))
    assert {"armt_forward_sequential", "armt_forward_diagonal", "armt_workspace_bytes", "armt_grouped_gemm",
            "armt_segment_attention", "armt_assoc_read", "armt_assoc_update", "armt_diagonal_group"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_diagonal_schedule_matches_lemma_fixture(lib):
    for line in open(os.path.join(GOLDEN, "lemma31_groups.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        lhs, rhs = line.split(":")
        L, N = (int(v) for v in lhs.split())
        sizes = [int(v) for v in rhs.split()]
        seen = set()
        for t, want in enumerate(sizes):
            lo, hi = C.c_int32(-7), C.c_int32(-7)
            g = lib.armt_diagonal_group(L, N, t, C.byref(lo), C.byref(hi))
            assert g == want == hi.value - lo.value + 1
            for l in range(lo.value, hi.value + 1):
                s = t - l
                assert 0 <= l < L and 0 <= s < N          # node (segment s, layer l) sits in group s + l
                seen.add((l, s))
        assert len(seen) == L * N                          # every cell exactly once, in L + N - 1 groups
        lo, hi = C.c_int32(-7), C.c_int32(-7)
        for t in (-1, L + N - 1, L + N + 5):
            assert lib.armt_diagonal_group(L, N, t, C.byref(lo), C.byref(hi)) == 0
            assert lo.value == -7 and hi.value == -7
    assert lib.armt_diagonal_group(0, 3, 0, None, None) == 0
    assert lib.armt_diagonal_group(3, 0, 0, None, None) == 0
    assert lib.armt_diagonal_group(16, 128, 20, None, None) == 16


def test_auto_order_rule(lib):
    """One segment or one layer: sequential (the two orders coincide); otherwise diagonal; invalid input: -1."""
    tiny = S.get_shape("tiny")
    cfg = _cfg(tiny)
    assert lib.armt_auto_order(C.byref(cfg), tiny.seg_len) == 0
    assert lib.armt_auto_order(C.byref(cfg), 2 * tiny.seg_len) == 1
    assert lib.armt_auto_order(C.byref(cfg), 128 * tiny.seg_len) == 1
    assert lib.armt_auto_order(C.byref(cfg), tiny.seg_len + 1) == -1
    assert lib.armt_auto_order(C.byref(cfg), 0) == -1
    one_layer = _cfg(tiny.replace(n_layers=1))
    assert lib.armt_auto_order(C.byref(one_layer), 5 * tiny.seg_len) == 0
    assert lib.armt_auto_order(None, tiny.seg_len) == -1
    used = C.c_int32(-5)
    # argument errors of the call itself come back as status codes before anything is launched
    rc = lib.armt_forward_auto(C.byref(cfg), None, None, None, tiny.seg_len, None, None, None, None, None, None, 0, None,
                               C.byref(used))
    assert rc == 1
    rc = lib.armt_forward_diagonal_split(C.byref(cfg), None, None, None, tiny.seg_len, None, None, None, None, None, None,
                                         0, None, -1)
    assert rc == 2


def test_earliest_group_property(lib):
    """Each cell's group index s + l is one more than the latest of its two predecessors (s, l-1),
    (s-1, l): no cell could run earlier (Lemma 3.1)."""
    L, N = 5, 7
    group_of = {}
    for t in range(L + N - 1):
        lo, hi = C.c_int32(), C.c_int32()
        lib.armt_diagonal_group(L, N, t, C.byref(lo), C.byref(hi))
        for l in range(lo.value, hi.value + 1):
            group_of[(l, t - l)] = t
    for (l, s), t in group_of.items():
        preds = [group_of[p] for p in ((l - 1, s), (l, s - 1)) if p in group_of]
        assert t == (max(preds) + 1 if preds else 0)


def test_workspace_bytes(lib):
    for name in S.CONFIGS:
        assert lib.armt_workspace_bytes(C.byref(_cfg(S.get_shape(name)))) > 0
    big = lib.armt_workspace_bytes(C.byref(_cfg(S.get_shape("1b_128k"))))
    assert big == lib.armt_workspace_bytes(C.byref(_cfg(S.get_shape("1b_8k"))))     # independent of n_tokens
    assert big < 2 * 2 ** 30
    assert lib.armt_workspace_bytes(None) == 0
    tiny = S.get_shape("tiny")
    for bad in (dict(n_heads=3), dict(head_dim=31, d_model=124), dict(n_layers=0), dict(n_kv_heads=3), dict(d_mem=0),
                dict(dpfp_nu=64)):
        assert lib.armt_workspace_bytes(C.byref(_cfg(tiny.replace(**bad)))) == 0, bad
    c = _cfg(tiny)
    c.dtype = 7
    assert lib.armt_workspace_bytes(C.byref(c)) == 0


def test_forward_argument_errors_come_before_any_launch(lib):
    """All of these return before touching the GPU, so they run without one; the fake pointers are never
    dereferenced."""
    import paper_2506_05229_amd as P
    shape = S.get_shape("tiny")
    cfg = _cfg(shape)
    L = shape.n_layers
    layers = (P.ArmtLayerWeights * L)()
    fake = 0x1000
    for l in range(L):
        for f, _ in P.ArmtLayerWeights._fields_:
            setattr(layers[l], f, fake)
    ws_bytes = lib.armt_workspace_bytes(C.byref(cfg))
    ok_args = dict(cfg=C.byref(cfg), layers=layers, mem=fake, x=fake, n=shape.n_tokens, A_in=None, z_in=None,
                   hid=fake, A=fake, z=fake, ws=0x10000, wsb=ws_bytes, st=None)

    def call(fn, **kw):
        a = dict(ok_args, **kw)
        return fn(a["cfg"], a["layers"], a["mem"], a["x"], a["n"], a["A_in"], a["z_in"], a["hid"], a["A"], a["z"],
                  a["ws"], a["wsb"], a["st"])

    for fn in (lib.armt_forward_sequential, lib.armt_forward_diagonal):
        assert call(fn, cfg=None) == 1
        assert call(fn, mem=None) == 1 and call(fn, x=None) == 1 and call(fn, hid=None) == 1
        assert call(fn, A=None) == 1 and call(fn, z=None) == 1 and call(fn, layers=None) == 1
        assert call(fn, A_in=fake) == 1                     # A_in without z_in
        assert call(fn, n=0) == 2 and call(fn, n=-64) == 2 and call(fn, n=shape.n_tokens + 1) == 2
        assert call(fn, ws=None) == 4 and call(fn, wsb=ws_bytes - 1) == 4 and call(fn, ws=0x10001) == 4
        bad = _cfg(shape)
        bad.dtype = 9
        assert call(fn, cfg=C.byref(bad)) == 3
        assert call(fn, cfg=C.byref(_cfg(shape.replace(n_heads=3)))) == 2
        # bf16 shapes the matrix-core kernels do not cover are refused, not run slowly
        assert call(fn, cfg=C.byref(_cfg(shape.replace(dtype="bf16")))) == 6
        missing = (P.ArmtLayerWeights * L)()
        for l in range(L):
            for f, _ in P.ArmtLayerWeights._fields_:
                setattr(missing[l], f, fake)
        missing[L - 1].wm_b = None
        assert call(fn, layers=missing) == 1
    for code in range(0, 8):
        assert lib.armt_status_str(code)
    assert lib.armt_last_hip_error() is not None


def test_step_entry_argument_errors(lib):
    shape = S.get_shape("tiny")
    cfg = _cfg(shape)
    n = lib.armt_workspace_bytes(C.byref(cfg))
    fake = 0x1000
    assert lib.armt_segment_attention(C.byref(cfg), 0, fake, fake, 0x10000, n, None) == 2
    assert lib.armt_segment_attention(C.byref(cfg), shape.n_layers + 1, fake, fake, 0x10000, n, None) == 2
    assert lib.armt_segment_attention(C.byref(cfg), 1, fake, fake, 0x10000, n - 1, None) == 4
    assert lib.armt_segment_attention(C.byref(cfg), 1, None, fake, 0x10000, n, None) == 1
    arr = (C.c_void_p * 1)(fake)
    assert lib.armt_grouped_gemm(0, 1, 8, 8, 8, arr, arr, arr, None, 0, None) == 4
    assert lib.armt_grouped_gemm(1, 1, 8, 8, 40, arr, arr, arr, 0x10000, 4096, None) == 6      # bf16 needs K % 64 == 0
    assert lib.armt_grouped_gemm(5, 1, 8, 8, 8, arr, arr, arr, 0x10000, 4096, None) == 3
    assert lib.armt_grouped_gemm(0, 0, 8, 8, 8, arr, arr, arr, 0x10000, 4096, None) == 2
    assert lib.armt_assoc_update(C.byref(cfg), 1, fake, arr, arr, arr, 3, fake, fake, 0x10000, n, None) == 2
    assert lib.armt_profile_begin(99, 4) == 2
    assert lib.armt_set_gemm_tile_config(-1) == -1


def test_token_end_entry_argument_errors(lib):
    shape = S.get_shape("tiny")
    cfg = _cfg(shape)
    fake = 0x1000
    # embedding gather: null pointers, empty vocabulary, no tokens
    assert lib.armt_embed_tokens(C.byref(cfg), None, 10, fake, 4, fake, None) == 1
    assert lib.armt_embed_tokens(C.byref(cfg), fake, 0, fake, 4, fake, None) == 2
    assert lib.armt_embed_tokens(C.byref(cfg), fake, 10, fake, 0, fake, None) == 2
    # head: workspace grows with the rows (operand copy + row scales + pointer table), 0 for bad arguments
    n1, n2 = lib.armt_lm_head_workspace_bytes(C.byref(cfg), 1), lib.armt_lm_head_workspace_bytes(C.byref(cfg), 5000)
    assert n1 >= shape.d_model * 4 + 4 + 128 and n2 >= 5000 * (shape.d_model * 4 + 4) + 5 * 128 and n2 % 256 == 0
    assert lib.armt_lm_head_workspace_bytes(C.byref(cfg), 0) == 0
    assert lib.armt_lm_head(C.byref(cfg), None, 4, fake, fake, 10, fake, 0x10000, n1, None) == 1
    assert lib.armt_lm_head(C.byref(cfg), fake, 0, fake, fake, 10, fake, 0x10000, n1, None) == 2
    assert lib.armt_lm_head(C.byref(cfg), fake, 4, fake, fake, 0, fake, 0x10000, n1, None) == 2
    assert lib.armt_lm_head(C.byref(cfg), fake, 5000, fake, fake, 10, fake, 0x10000, n2 - 1, None) == 4
    assert lib.armt_lm_head(C.byref(cfg), fake, 4, fake, fake, 10, fake, 0x10010, n1, None) == 4     # misaligned
    bad = _cfg(shape)
    bad.head_dim = 31
    assert lib.armt_lm_head_workspace_bytes(C.byref(bad), 4) == 0
    assert lib.armt_embed_tokens(C.byref(bad), fake, 10, fake, 4, fake, None) != 0


def test_batched_workspace_and_argument_errors(lib):
    shape = S.get_shape("tiny")
    cfg = _cfg(shape)
    n1 = lib.armt_workspace_bytes(C.byref(cfg))
    lib.armt_workspace_bytes_batched.restype = C.c_size_t
    assert lib.armt_workspace_bytes_batched(C.byref(cfg), 1) == n1
    n3 = lib.armt_workspace_bytes_batched(C.byref(cfg), 3)
    assert 2 * n1 < n3 <= 3 * n1 + 4096                       # per-cell scratch grows with the batch, tables do not shrink
    assert lib.armt_workspace_bytes_batched(C.byref(cfg), 0) == 0
    assert lib.armt_workspace_bytes_batched(C.byref(cfg), 32768) == 0        # batch * n_layers beyond a launch grid
    layers = (__import__("paper_2506_05229_amd").ArmtLayerWeights * shape.n_layers)()
    fake = 0x1000
    args = lambda batch, ws_bytes: (C.byref(cfg), layers, fake, fake, batch, shape.seg_len, None, None, fake, fake, fake,
                                    0x10000, ws_bytes, None)
    assert lib.armt_forward_diagonal_batched(*args(0, n3)) == 2
    assert lib.armt_forward_diagonal_batched(*args(3, n3)) == 1          # null weight pointers
    for f in ("rms1", "wq", "wk", "wv", "wo", "rms2", "wgate", "wup", "wdown", "wm_q", "wm_k", "wm_v", "wm_b"):
        for l in range(shape.n_layers):
            setattr(layers[l], f, fake)
    assert lib.armt_forward_diagonal_batched(*args(3, n3 - 1)) == 4
    assert lib.armt_forward_sequential_batched(*args(3, n1)) == 4


def test_training_entry_argument_errors(lib):
    """Tape / workspace sizes and the argument checks of armt_forward_train and armt_backward; nothing is launched."""
    import paper_2506_05229_amd as P
    shape = S.get_shape("tiny")
    cfg = _cfg(shape)
    L, fake = shape.n_layers, 0x1000
    T, d, phi = shape.seg_len + shape.n_mem, shape.d_model, shape.phi
    rec = (T * d + d * phi + phi + 63) // 64 * 64
    tape_bytes = lib.armt_tape_bytes(C.byref(cfg), shape.n_tokens)
    assert tape_bytes == shape.n_segments * L * rec * 4
    assert lib.armt_tape_bytes(C.byref(cfg), shape.n_tokens + 1) == 0 and lib.armt_tape_bytes(C.byref(cfg), 0) == 0
    ws_bytes = lib.armt_backward_workspace_bytes(C.byref(cfg))
    assert ws_bytes > 0 and ws_bytes % 256 == 0
    big_m = _cfg(shape.replace(d_model=256, n_heads=1, n_kv_heads=1, head_dim=256))   # heads wider than the attention backward holds
    assert lib.armt_tape_bytes(C.byref(big_m), shape.n_tokens) == 0 and lib.armt_backward_workspace_bytes(C.byref(big_m)) == 0
    layers = (P.ArmtLayerWeights * L)()
    grads = (P.ArmtLayerGrads * L)()
    for l in range(L):
        for f, _ in P.ArmtLayerWeights._fields_:
            setattr(layers[l], f, fake)
            setattr(grads[l], f, fake)
    fwd_ws = lib.armt_workspace_bytes(C.byref(cfg))

    def train(**kw):
        a = dict(cfg=C.byref(cfg), tape=0x10000, tb=tape_bytes, n=shape.n_tokens, ws=0x20000, wsb=fwd_ws)
        a.update(kw)
        return lib.armt_forward_train(a["cfg"], layers, fake, fake, a["n"], None, None, fake, fake, fake, a["tape"], a["tb"],
                                      a["ws"], a["wsb"], None, 1)

    assert train(tape=None) == 1 and train(tb=tape_bytes - 1) == 4 and train(tape=0x10001) == 4
    assert train(n=shape.n_tokens + 3) == 2 and train(ws=None) == 4 and train(cfg=C.byref(big_m)) == 6

    def back(**kw):
        a = dict(cfg=C.byref(cfg), layers=layers, n=shape.n_tokens, tape=0x10000, tb=tape_bytes, dh=fake, dA=None, dz=None,
                 grads=grads, dmem=fake, dx=None, dAi=None, dzi=None, ws=0x20000, wsb=ws_bytes)
        a.update(kw)
        return lib.armt_backward(a["cfg"], a["layers"], a["n"], a["tape"], a["tb"], 0, a["dh"], a["dA"], a["dz"], a["grads"],
                                 a["dmem"], a["dx"], a["dAi"], a["dzi"], a["ws"], a["wsb"], None, 1)

    assert back(cfg=None) == 1 and back(layers=None) == 1 and back(tape=None) == 1 and back(dh=None) == 1
    assert back(grads=None) == 1 and back(dmem=None) == 1
    assert back(dA=fake) == 1 and back(dAi=fake) == 1            # one of a pair without the other
    assert back(n=0) == 2 and back(n=shape.n_tokens - 1) == 2
    assert back(tb=tape_bytes - 1) == 4 and back(ws=None) == 4 and back(wsb=ws_bytes - 1) == 4 and back(ws=0x20001) == 4
    assert back(cfg=C.byref(big_m)) == 6
    missing = (P.ArmtLayerGrads * L)()
    for l in range(L):
        for f, _ in P.ArmtLayerGrads._fields_:
            setattr(missing[l], f, fake)
    missing[0].wm_q = None
    assert back(grads=missing) == 1
    # batched variants: sizes scale with the batch, the batch is checked
    assert lib.armt_tape_bytes_batched(C.byref(cfg), 3, shape.n_tokens) == 3 * tape_bytes
    assert lib.armt_tape_bytes_batched(C.byref(cfg), 0, shape.n_tokens) == 0
    wsb3 = lib.armt_backward_workspace_bytes_batched(C.byref(cfg), 3)
    assert wsb3 > ws_bytes and lib.armt_backward_workspace_bytes_batched(C.byref(cfg), 0) == 0
    assert lib.armt_backward_workspace_bytes_batched(C.byref(cfg), 40000) == 0
    bb = lambda batch, tb, wsb: lib.armt_backward_batched(C.byref(cfg), layers, batch, shape.n_tokens, 0x10000, tb, 0, fake, None, None,
                                                          grads, fake, None, None, None, 0x20000, wsb, None, 1)
    assert bb(0, 3 * tape_bytes, wsb3) == 2 and bb(3, 3 * tape_bytes - 1, wsb3) == 4 and bb(3, 3 * tape_bytes, wsb3 - 1) == 4
    ft = lambda batch, tb: lib.armt_forward_train_batched(C.byref(cfg), layers, fake, fake, batch, shape.n_tokens, None, None, fake, fake,
                                                          fake, 0x10000, tb, 0x20000, lib.armt_workspace_bytes_batched(C.byref(cfg), 3),
                                                          None, 1)
    assert ft(0, 3 * tape_bytes) == 2 and ft(3, 3 * tape_bytes - 1) == 4


def test_token_end_backward_argument_errors(lib):
    shape = S.get_shape("tiny")
    cfg = _cfg(shape)
    fake, V, n = 0x1000, 301, 72
    need = lib.armt_lm_head_backward_workspace_bytes(C.byref(cfg), n, V)
    assert need > 0 and need % 256 == 0
    assert lib.armt_lm_head_backward_workspace_bytes(C.byref(cfg), 0, V) == 0
    assert lib.armt_lm_head_backward_workspace_bytes(C.byref(cfg), n, 0) == 0

    def head(**kw):
        a = dict(cfg=C.byref(cfg), h=fake, n=n, g=fake, w=fake, V=V, dl=fake, dh=fake, dg=fake, dw=fake, ws=0x10000, wsb=need)
        a.update(kw)
        return lib.armt_lm_head_backward(a["cfg"], a["h"], a["n"], a["g"], a["w"], a["V"], a["dl"], a["dh"], a["dg"], a["dw"],
                                         a["ws"], a["wsb"], None)

    assert head(cfg=None) == 1 and head(h=None) == 1 and head(dl=None) == 1 and head(dh=None) == 1 and head(dw=None) == 1
    assert head(n=0) == 2 and head(V=0) == 2
    assert head(ws=None) == 4 and head(wsb=need - 1) == 4 and head(ws=0x10001) == 4
    emb = lambda **kw: lib.armt_embed_tokens_backward(C.byref(cfg), kw.get("dx", fake), kw.get("ids", fake), kw.get("n", 8),
                                                      kw.get("V", V), kw.get("dt", fake), None)
    assert emb(dx=None) == 1 and emb(ids=None) == 1 and emb(dt=None) == 1 and emb(n=0) == 2 and emb(V=0) == 2


def test_microbench_needs_a_gpu_and_says_so(capsys):
    import torch
    if torch.cuda.is_available():
        pytest.skip("this checks the behaviour without a GPU")
    from paper_2506_05229_amd import microbench
    assert microbench.main(["gemm", "--iters", "1"]) == 2
    assert "GPU" in capsys.readouterr().err
