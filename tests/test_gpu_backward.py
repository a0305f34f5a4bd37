"""Parity of the HIP backward pass (through the C ABI) against the backward oracle (float64 autograd of the
restated forward).  Every gradient tensor is compared by relative Frobenius error.
fp32 configurations: <= 2e-4.
bf16 configurations: <= 5e-2 for the decoder block's weights, the embeddings and W_V, W_beta of the memory (every
gradient GEMM takes bf16 operands and accumulates in fp32, the attention backward rounds P and dS to bf16 like the
forward rounds P; measured 0.5 - 3.5 %, growing by about 0.5 % per layer the gradient crosses; the same cases through
fp32 arithmetic on the same bf16-stored tensors give 0.7 - 2.7 %); <= 1.5e-1 (measured 2 - 11 %) for W_Q and W_K of the
memory.  Where that looser bound comes from is measured by test_bf16_backward_kernels_on_an_oracle_tape, which hands
armt_backward a tape from the float64 forward oracle, so that the deviation of the bf16 forward pass between cells is
out of the comparison: then the gradients of the carried-in state are good to 1.4e-2 / 5e-3 and are held to 5e-2 like
everything else, W_Q comes out at 4e-2 and W_K at 7e-2.  So about two thirds of the W_K error are the backward pass's own:
its gradient runs through gamma = 1 - z.phi / (|phi|^2 + eps) and v - v_bar (Eq. 4), differences whose relative error is
that of phi(k) -- twice the bf16 error of the memory rows the step recomputes -- divided by gamma, and the test inputs sit
on purpose at the edge of the well-conditioned range, where gamma comes close to zero; the rest is the forward's bf16
deviation in A and z between cells, which these gradients are linear in.  Bound: 1e-1 on an oracle tape, 1.5e-1 end to
end (margin over the measured 7e-2 and 1.1e-1)."""
import numpy as np
import pytest

import armt_synth as S
from gpu_util import make_problem, rel_fro
from oracle import armt_oracle_grad as G

pytestmark = pytest.mark.gpu

F32_REL = 2e-4
BF16_REL = 5e-2
BF16_REL_MEM = 1.5e-1
BF16_REL_TAPE = 1e-1


def upstream(shape, seed, with_state):
    rng = np.random.default_rng(seed + 1000)
    Gh = rng.standard_normal((shape.n_tokens, shape.d_model)).astype(np.float32)
    if shape.dtype == "bf16":
        Gh = S.round_to_bf16(Gh)
    if not with_state:
        return Gh, None, None
    GA = (rng.standard_normal((shape.n_layers, shape.d_model, shape.phi)) * 0.1).astype(np.float32)
    Gz = (rng.standard_normal((shape.n_layers, shape.phi)) * 0.1).astype(np.float32)
    return Gh, GA, Gz


def carried(shape, seed):
    rng = np.random.default_rng(seed + 2000)
    A = (rng.standard_normal((shape.n_layers, shape.d_model, shape.phi)) * 0.05).astype(np.float32)
    z = rng.uniform(0.5, 1.5, (shape.n_layers, shape.phi)).astype(np.float32)
    return A, z


def well_conditioned(shape, seed):
    """Inputs on which parity means something: the recurrence of Eq. 4-5 can drive z.phi through zero (a property of
    the equations, the forward oracle shows it), and gradients there are unbounded.  Take the largest key scale 2^-p
    for which the forward oracle keeps every denominator positive and the values read back of order one."""
    from oracle import armt_oracle as O
    x = S.make_embeddings(shape, seed=seed)
    for p in (0, 2, 4, 6, 8, 10, 12):
        shape = shape.replace(mem_k_scale=2.0 ** -p, mem_v_scale=16.0)
        layers, mem_emb = S.make_weights(shape, seed=seed, gain_std=0.1)
        stats = []
        O.armt_forward_sequential(shape, layers, mem_emb, x, stats=stats)
        if all(r["min_den"] > 0.0 for r in stats) and max(r["max_abs_read"] for r in stats) < 2.0:
            print(f"key scale 2^-{p}: max read {max(r['max_abs_read'] for r in stats):.2f}", flush=True)
            return shape, layers, mem_emb, x
    pytest.skip("no well-conditioned key scale found")


def run_hip_grad(shape, layers, mem_emb, x, Gs, state, diagonal):
    import torch
    import paper_2506_05229_amd as P
    model = P.Armt(shape, layers, mem_emb)
    xd = model.embed(x)
    dev = lambda a: None if a is None else torch.as_tensor(a, dtype=torch.float32).cuda().contiguous()
    A_in, z_in = (dev(state[0]), dev(state[1])) if state else (None, None)
    hidden, A, z, tape = model.forward_train(xd, diagonal=diagonal, A_in=A_in, z_in=z_in)
    ref = model.forward(xd, diagonal=diagonal, A_in=A_in, z_in=z_in)
    for a, b in zip((hidden, A, z), ref):
        assert torch.equal(a, b)                     # the tape does not change the forward result
    g = model.backward(tape, x.shape[0], model.embed(Gs[0]), dev(Gs[1]), dev(Gs[2]), carry_in=state is not None,
                       diagonal=diagonal)
    torch.cuda.synchronize()
    np_ = lambda t: None if t is None else t.float().cpu().numpy()
    return {"layers": [{k: np_(v) for k, v in lw.items()} for lw in g["layers"]], "mem_emb": np_(g["mem_emb"]),
            "x": np_(g["x"]), "A_in": np_(g["A_in"]), "z_in": np_(g["z_in"]), "hidden": np_(hidden), "A": np_(A), "z": np_(z)}


def compare(got, want, tol, what, tol_mem=None):
    """tol_mem: tolerance of the tensors whose gradient passes through the associative read or update."""
    errs = {}
    def one(name, a, b, t):
        assert np.isfinite(a).all(), (what, name)
        e = rel_fro(a, b)
        key = name.split()[-1]
        errs[key] = max(errs.get(key, 0.0), e)
        return [] if e <= t else [(name, e, t)]
    bad = []
    tm = tol if tol_mem is None else tol_mem
    for l, (gl, wl) in enumerate(zip(got["layers"], want["layers"])):
        for k in G.WEIGHT_KEYS:
            bad += one(f"layer {l} {k}", gl[k].reshape(wl[k].shape), wl[k], tm if k in ("wm_q", "wm_k") else tol)
    bad += one("mem_emb", got["mem_emb"], want["mem_emb"], tol)
    bad += one("x", got["x"], want["x"], tol)
    if want["A_in"] is not None:
        bad += one("A_in", got["A_in"], want["A_in"], tm)
        bad += one("z_in", got["z_in"], want["z_in"], tm)
    fwd = " ".join(f"{k}={rel_fro(got[k], want[k]):.2e}" for k in ("hidden", "A", "z"))
    print(f"{what}: forward {fwd}; gradients " + " ".join(f"{k}={v:.2e}" for k, v in errs.items()), flush=True)
    assert not bad, (what, bad)


@pytest.mark.parametrize("diagonal", [False, True])
@pytest.mark.parametrize("case", ["plain", "carry_and_state_grads", "ragged"])
def test_f32_backward_matches_oracle(case, diagonal):
    base = S.get_shape("tiny")
    if case == "ragged":
        shape = base.replace(n_layers=3, d_model=120, n_heads=6, n_kv_heads=3, head_dim=20, d_ff=200,
                             seg_len=37, n_mem=5, d_mem=12, n_tokens=37 * 4, dpfp_nu=2)
    else:
        shape = base.replace(n_tokens=5 * 64)
    layers, mem_emb, x = make_problem(shape, seed=3, std=0.02, gain_std=0.1, v_scale=64.0)
    state = carried(shape, 3) if case == "carry_and_state_grads" else None
    Gs = upstream(shape, 3, with_state=(case != "plain"))
    want = G.armt_grad(shape, layers, mem_emb, x, *Gs, A_in=state[0] if state else None, z_in=state[1] if state else None)
    got = run_hip_grad(shape, layers, mem_emb, x, Gs, state, diagonal)
    compare(got, want, F32_REL, f"f32 {case} diag={diagonal}")


SMALL_BF16 = dict(n_layers=3, d_model=256, n_heads=4, n_kv_heads=2, head_dim=64, d_ff=512, seg_len=144,
                  n_mem=16, d_mem=32, n_tokens=144 * 4, dtype="bf16")


@pytest.mark.parametrize("diagonal", [False, True])
@pytest.mark.parametrize("heads", ["4x64_kv2", "4x128_kv1", "8x64_kv1", "4x64_kv4"])
def test_small_bf16_backward_matches_oracle(heads, diagonal):
    """Head layouts of the attention-backward configurations: head_dim 64 and 128; 1, 2, 4 and 8 query heads per KV head
    (with 1 and 2 a workgroup of the dQ and of the forward kernel takes 4 and 2 row tiles)."""
    kw = {"4x64_kv2": dict(), "4x128_kv1": dict(d_model=512, n_heads=4, n_kv_heads=1, head_dim=128),
          "8x64_kv1": dict(d_model=512, n_heads=8, n_kv_heads=1, head_dim=64),
          "4x64_kv4": dict(n_heads=4, n_kv_heads=4, seg_len=200, n_tokens=200 * 4)}[heads]
    shape, layers, mem_emb, x = well_conditioned(S.get_shape("tiny").replace(**dict(SMALL_BF16, **kw)), seed=11)
    Gs = upstream(shape, 11, with_state=True)
    want = G.armt_grad(shape, layers, mem_emb, x, *Gs)
    got = run_hip_grad(shape, layers, mem_emb, x, Gs, None, diagonal)
    compare(got, want, BF16_REL, f"bf16 {heads} diag={diagonal}", tol_mem=BF16_REL_MEM)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_many_memory_tokens_backward_matches_oracle(dtype):
    """n_mem above the 16 tokens the delta-rule backward holds at once: several chunks, the last one ragged (fp32)."""
    if dtype == "f32":
        shape = S.get_shape("tiny").replace(n_mem=40, n_tokens=4 * 64)
    else:
        shape = S.get_shape("tiny").replace(**dict(SMALL_BF16, n_mem=48, n_tokens=144 * 3))
    shape, layers, mem_emb, x = well_conditioned(shape, seed=4)
    Gs = upstream(shape, 4, with_state=True)
    want = G.armt_grad(shape, layers, mem_emb, x, *Gs)
    got = run_hip_grad(shape, layers, mem_emb, x, Gs, None, True)
    if dtype == "f32":
        compare(got, want, F32_REL, "f32 n_mem 40")
    else:
        compare(got, want, BF16_REL, "bf16 n_mem 48", tol_mem=BF16_REL_MEM)


def _oracle_tape(shape, layers, mem_emb, x, A_in=None, z_in=None):
    """The tape of include/armt.h filled from the float64 forward oracle (rounded to fp32 once)."""
    from oracle import armt_oracle as O
    trace = []
    O.armt_forward_sequential(shape, layers, mem_emb, x, A_in=A_in, z_in=z_in, trace=trace)
    T, d, P = shape.T, shape.d_model, shape.phi
    R = (T * d + d * P + P + 63) // 64 * 64
    tape = np.zeros((shape.n_segments * shape.n_layers, R), dtype=np.float32)
    for (s, l, U, A, z) in trace:
        rec = tape[s * shape.n_layers + l]
        rec[:T * d] = U.reshape(-1)
        rec[T * d:T * d + d * P] = A.reshape(-1)
        rec[T * d + d * P:T * d + d * P + P] = z
    return tape


@pytest.mark.parametrize("diagonal", [False, True])
def test_bf16_backward_kernels_on_an_oracle_tape(diagonal):
    """The backward kernels alone: armt_backward is given a tape built from the float64 forward oracle (cell inputs and
    memory states rounded to fp32 once), so that the deviation of the bf16 FORWARD pass is out of the comparison.  Then
    every gradient, those of the carried-in state included, is held to the 5e-2 of the other tensors, W_Q and W_K of the
    memory to 1e-1 (see the header of this file).  The state is carried in from an oracle run over two earlier segments (a well-conditioned state)."""
    import torch
    import paper_2506_05229_amd as P
    from oracle import armt_oracle as O
    shape, layers, mem_emb, x = well_conditioned(S.get_shape("tiny").replace(**dict(SMALL_BF16, n_tokens=144 * 6)), seed=11)
    Sg = shape.seg_len
    _, A0, z0 = O.armt_forward_sequential(shape, layers, mem_emb, x[:2 * Sg])
    A0, z0 = A0.astype(np.float32), z0.astype(np.float32)
    rest = shape.replace(n_tokens=4 * Sg)
    xr = x[2 * Sg:]
    Gs = upstream(rest, 11, with_state=True)
    want = G.armt_grad(rest, layers, mem_emb, xr, *Gs, A_in=A0, z_in=z0)
    tape = torch.from_numpy(_oracle_tape(rest, layers, mem_emb, xr, A_in=A0.astype(np.float64), z_in=z0.astype(np.float64))).cuda()
    model = P.Armt(rest, layers, mem_emb)
    dev = lambda a: torch.as_tensor(a, dtype=torch.float32).cuda().contiguous()
    g = model.backward(tape.view(torch.uint8).reshape(-1), rest.n_tokens, model.embed(Gs[0]), dev(Gs[1]), dev(Gs[2]), carry_in=True,
                       diagonal=diagonal)
    torch.cuda.synchronize()
    np_ = lambda t: t.float().cpu().numpy()
    got = {"layers": [{k: np_(v) for k, v in lw.items()} for lw in g["layers"]], "mem_emb": np_(g["mem_emb"]),
           "x": np_(g["x"]), "A_in": np_(g["A_in"]), "z_in": np_(g["z_in"]),
           "hidden": want["hidden"], "A": want["A"], "z": want["z"]}      # the forward is the oracle's own here
    # the carried-in state's gradients are held to the bound of every other tensor here; W_Q, W_K of the memory to 1e-1
    compare(got, want, BF16_REL, f"bf16 backward on an oracle tape, diag={diagonal}", tol_mem=BF16_REL_TAPE)
    assert rel_fro(got["A_in"], want["A_in"]) <= BF16_REL and rel_fro(got["z_in"], want["z_in"]) <= BF16_REL


def test_backward_orders_agree():
    """Reverse diagonal and reverse sequential order: the same cells and the same per-cell arithmetic, so everything that
    flows from cell to cell (dx, d_mem_emb, the gradient of the state) is bit-identical; a layer's weight gradient is a
    sum over its segments that the diagonal order adds eight segments at a time, so it agrees to fp32 rounding."""
    shape = S.get_shape("tiny").replace(n_tokens=6 * 64)
    layers, mem_emb, x = make_problem(shape, seed=5, std=0.02, gain_std=0.1, v_scale=64.0)
    Gs = upstream(shape, 5, with_state=True)
    state = carried(shape, 5)
    a = run_hip_grad(shape, layers, mem_emb, x, Gs, state, False)
    b = run_hip_grad(shape, layers, mem_emb, x, Gs, state, True)
    for la, lb in zip(a["layers"], b["layers"]):
        for k in G.WEIGHT_KEYS:
            assert rel_fro(la[k], lb[k]) <= 2e-6, k
    for k in ("x", "mem_emb", "A_in", "z_in"):
        assert np.array_equal(a[k], b[k]), k


def test_1b_width_bf16_backward_matches_oracle():
    """Two layers of the 1B shape (d_model 2048, 32/8 heads of 64, d_ff 8192, segment 1024 + 16 memory tokens,
    d_mem 64) over three segments, diagonal order: the tile configurations and launch shapes of the full model."""
    shape = S.get_shape("1b_8k").replace(n_layers=2, n_tokens=3 * 1024)
    layers, mem_emb, x = make_problem(shape, seed=2, std=0.02)
    Gs = upstream(shape, 2, with_state=True)
    want = G.armt_grad(shape, layers, mem_emb, x, *Gs)
    got = run_hip_grad(shape, layers, mem_emb, x, Gs, None, True)
    compare(got, want, BF16_REL, "1B width, 2 layers, 3 segments", tol_mem=BF16_REL_MEM)


def test_full_1b_model_backward_properties():
    """The whole 1B model (16 layers) over 8 segments, in the launch configuration bench.py times; the oracle cannot
    differentiate this size in minutes, so properties that hold at any size: (i) an upstream gradient on segment 2 only
    leaves the embeddings of segments 3.. without gradient, exactly (dependency rule of Section 3.1); (ii) reverse
    diagonal and reverse sequential order agree (bit for bit on what flows between cells, to fp32 rounding on the
    weight gradients, which the diagonal order adds eight segments at a time); (iii) everything is finite and non-zero."""
    import torch
    import paper_2506_05229_amd as P
    shape = S.get_shape("1b_8k")
    layers, mem_emb = S.make_weights(shape, seed=0)
    x = S.make_embeddings(shape, seed=0)
    model = P.Armt(shape, layers, mem_emb)
    xd = model.embed(x)
    Sg = shape.seg_len
    Gh = torch.zeros(shape.n_tokens, shape.d_model, device="cuda", dtype=model.act_dtype)
    Gh[2 * Sg:3 * Sg] = torch.randn(Sg, shape.d_model, device="cuda", generator=torch.Generator(device="cuda").manual_seed(3)).to(
        model.act_dtype)
    _, _, _, tape = model.forward_train(xd, diagonal=True)
    gd = model.backward(tape, shape.n_tokens, Gh, diagonal=True)
    gs = model.backward(tape, shape.n_tokens, Gh, diagonal=False)
    torch.cuda.synchronize()
    assert not gd["x"][3 * Sg:].any().item()                       # (i)
    assert gd["x"][:3 * Sg].abs().max().item() > 0
    assert torch.equal(gd["x"], gs["x"]) and torch.equal(gd["mem_emb"], gs["mem_emb"])      # (ii)
    worst = 0.0
    for ld, ls in zip(gd["layers"], gs["layers"]):
        for k in G.WEIGHT_KEYS:
            a, b = ld[k].double(), ls[k].double()
            assert torch.isfinite(a).all().item() and a.abs().max().item() > 0, k                 # (iii)
            worst = max(worst, ((a - b).norm() / b.norm()).item())
    print(f"full 1B model: worst relative difference between the two orders {worst:.2e}", flush=True)
    assert worst <= 1e-5


@pytest.mark.parametrize("dtype,diagonal", [("f32", True), ("f32", False), ("bf16", True)])
def test_batched_backward_matches_oracle(dtype, diagonal):
    """Three sequences in one call, with gradients into the final state (fp32: also a carried-in state): the gradients of the shared
    weights and of mem_emb are the sums of the oracle's per-sequence gradients; dx, dA_in, dz_in are per sequence."""
    import torch
    import paper_2506_05229_amd as P
    B = 3
    if dtype == "f32":
        shape, tol, tol_mem = S.get_shape("tiny").replace(n_tokens=5 * 64), F32_REL, None
        layers, mem_emb, _ = make_problem(shape, seed=3, std=0.02, gain_std=0.1, v_scale=64.0)
    else:
        shape, layers, mem_emb, _ = well_conditioned(S.get_shape("tiny").replace(**SMALL_BF16), seed=11)
        tol, tol_mem = BF16_REL, BF16_REL_MEM
    xs = [S.make_embeddings(shape, seed=20 + b) for b in range(B)]
    carry = dtype == "f32"       # a random carried-in state drives z.phi through zero on the bf16 shape (the oracle shows it)
    states = [carried(shape, 30 + b) if carry else (None, None) for b in range(B)]
    Gss = [upstream(shape, 40 + b, with_state=True) for b in range(B)]
    wants = [G.armt_grad(shape, layers, mem_emb, xs[b], *Gss[b], A_in=states[b][0], z_in=states[b][1]) for b in range(B)]
    model = P.Armt(shape, layers, mem_emb)
    dev = lambda a: torch.as_tensor(np.stack(a), dtype=torch.float32).cuda().contiguous()
    xd = model.embed(np.stack(xs))
    A_in, z_in = (dev([s[0] for s in states]), dev([s[1] for s in states])) if carry else (None, None)
    hidden, A, z, tape = model.forward_train(xd, diagonal=diagonal, A_in=A_in, z_in=z_in)
    ref = model.forward_batched(xd, diagonal=diagonal, A_in=A_in, z_in=z_in)
    for a, b in zip((hidden, A, z), ref):
        assert torch.equal(a, b)
    g = model.backward(tape, shape.n_tokens, model.embed(np.stack([q[0] for q in Gss])), dev([q[1] for q in Gss]),
                       dev([q[2] for q in Gss]), carry_in=carry, diagonal=diagonal)
    torch.cuda.synchronize()
    np_ = lambda t: None if t is None else t.float().cpu().numpy()
    got = {"layers": [{k: np_(v) for k, v in lw.items()} for lw in g["layers"]], "mem_emb": np_(g["mem_emb"]),
           "x": np_(g["x"]), "A_in": np_(g["A_in"]), "z_in": np_(g["z_in"]), "hidden": np_(hidden), "A": np_(A), "z": np_(z)}
    want = {"layers": [{k: sum(w["layers"][l][k] for w in wants) for k in G.WEIGHT_KEYS} for l in range(shape.n_layers)],
            "mem_emb": sum(w["mem_emb"] for w in wants)}
    for k in ("x", "A_in", "z_in", "hidden", "A", "z"):
        want[k] = None if wants[0][k] is None else np.stack([w[k] for w in wants])
    compare(got, want, tol, f"batch of {B}, {dtype}, diag={diagonal}", tol_mem=tol_mem)

