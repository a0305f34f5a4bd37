"""armt_lm_head_static, the entry point for callers that cannot allocate: its scratch memory is a fixed array inside the
library.  It must return the bits of armt_lm_head (same kernels), on two calls in a row of which the second is smaller
(the array keeps the first call's contents), and refuse inputs that do not fit before launching anything."""
import ctypes as C

import numpy as np
import pytest
import torch

import armt_synth as S

pytestmark = pytest.mark.gpu

STATIC_BYTES = 8454144


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_static_head_equals_workspace_head_on_two_calls(dtype):
    import paper_2506_05229_amd as P
    if dtype == "bf16":
        shape, vocab, rows = S.get_shape("1b_8k"), 4096, (1024 + 300, 272)     # whole 1024-row groups + a ragged rest
    else:
        shape, vocab, rows = S.get_shape("tiny"), 301, (200, 37)
    ids, E, gain, W = S.make_token_ends(shape, vocab=vocab, seed=3, gain_std=0.1)
    te = P.TokenEnds(shape, E, gain, W)
    lib = te.lib
    rng = np.random.default_rng(11)
    for call, n in enumerate(rows):
        assert lib.armt_lm_head_workspace_bytes(C.byref(te.cfg), n) <= STATIC_BYTES
        h = rng.standard_normal((n, shape.d_model)).astype(np.float32)
        hd = torch.from_numpy(S.round_to_bf16(h) if dtype == "bf16" else h).to(device="cuda", dtype=te.dt)
        print(f"lm_head_static {dtype} call {call}: {n} rows x vocab {vocab}", flush=True)
        want = te.logits(hd)
        got = torch.full((n, vocab), float("nan"), dtype=torch.float32, device="cuda")
        te.logits_static(hd, got)
        torch.cuda.synchronize()
        assert torch.isfinite(got).all()
        assert torch.equal(got, want), (dtype, call, n)


def test_static_head_refuses_what_does_not_fit():
    import paper_2506_05229_amd as P
    shape = S.get_shape("1b_8k")
    lib = P.load_library()
    cfg = P.ArmtConfig.from_shape(shape)
    n = 4096                                     # 16 MB of normalised bf16 rows: more than the array holds
    assert lib.armt_lm_head_workspace_bytes(C.byref(cfg), n) > STATIC_BYTES
    fake = C.c_void_p(256)
    rc = lib.armt_lm_head_static(C.byref(cfg), fake, n, fake, fake, 1000, fake, None)
    assert rc == 7 and b"scratch" in lib.armt_status_str(rc)
    assert lib.armt_lm_head_static(C.byref(cfg), None, 16, fake, fake, 1000, fake, None) == 1
    assert lib.armt_lm_head_static(C.byref(cfg), fake, 0, fake, fake, 1000, fake, None) == 2
