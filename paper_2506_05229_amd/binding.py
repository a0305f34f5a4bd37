"""ctypes binding of include/armt.h: argument marshalling only.

Every step of the path runs inside the shared library; torch is used for device memory and
the current stream.  There is no fallback: if the library is missing, loading raises."""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))

ARMT_F32, ARMT_BF16 = 0, 1
LAYER_FIELDS = ("rms1", "wq", "wk", "wv", "wo", "rms2", "wgate", "wup", "wdown",
                "wm_q", "wm_k", "wm_v", "wm_b")


class ArmtError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"armt status {code}: {text}")
        self.code = code


class ArmtConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "n_kv_heads", "head_dim", "d_ff",
                                         "seg_len", "n_mem", "d_mem", "dpfp_nu", "dtype")] + \
               [(n, C.c_float) for n in ("rms_eps", "rope_theta", "assoc_eps")]

    @classmethod
    def from_shape(cls, s) -> "ArmtConfig":
        return cls(n_layers=s.n_layers, d_model=s.d_model, n_heads=s.n_heads, n_kv_heads=s.n_kv_heads,
                   head_dim=s.head_dim, d_ff=s.d_ff, seg_len=s.seg_len, n_mem=s.n_mem, d_mem=s.d_mem,
                   dpfp_nu=s.dpfp_nu, dtype=ARMT_BF16 if s.dtype == "bf16" else ARMT_F32,
                   rms_eps=s.rms_eps, rope_theta=s.rope_theta, assoc_eps=s.assoc_eps)


class ArmtLayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in LAYER_FIELDS]


class ArmtLayerGrads(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in LAYER_FIELDS]


def library_path() -> str:
    return os.environ.get("ARMT_HIP_LIBRARY", os.path.join(HERE, "libarmt_hip.so"))


_LIB = None


def load_library():
    """Load libarmt_hip.so (built in-tree by paper_2506_05229_amd.build) and declare its C ABI."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} not found: build it with `python -m paper_2506_05229_amd.build`")
    lib = C.CDLL(path)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    fwd = [C.POINTER(ArmtConfig), C.POINTER(ArmtLayerWeights), vp, vp, i64, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.armt_workspace_bytes.argtypes = [C.POINTER(ArmtConfig)]
    lib.armt_workspace_bytes.restype = sz
    for name in ("armt_forward_sequential", "armt_forward_diagonal"):
        getattr(lib, name).argtypes = fwd
        getattr(lib, name).restype = C.c_int
    lib.armt_forward_auto.argtypes = fwd + [C.POINTER(i32)]
    lib.armt_forward_auto.restype = C.c_int
    lib.armt_forward_diagonal_split.argtypes = fwd + [i32]
    lib.armt_forward_diagonal_split.restype = C.c_int
    lib.armt_auto_order.argtypes = [C.POINTER(ArmtConfig), i64]
    lib.armt_auto_order.restype = i32
    fwdb = fwd[:4] + [i32] + fwd[4:]
    for name in ("armt_forward_sequential_batched", "armt_forward_diagonal_batched"):
        getattr(lib, name).argtypes = fwdb
        getattr(lib, name).restype = C.c_int
    lib.armt_workspace_bytes_batched.argtypes = [C.POINTER(ArmtConfig), i32]
    lib.armt_workspace_bytes_batched.restype = sz
    lib.armt_tape_bytes.argtypes = [C.POINTER(ArmtConfig), i64]
    lib.armt_tape_bytes.restype = sz
    lib.armt_backward_workspace_bytes.argtypes = [C.POINTER(ArmtConfig)]
    lib.armt_backward_workspace_bytes.restype = sz
    lib.armt_forward_train.argtypes = [C.POINTER(ArmtConfig), C.POINTER(ArmtLayerWeights), vp, vp, i64, vp, vp, vp, vp, vp,
                                       vp, sz, vp, sz, vp, i32]
    lib.armt_forward_train.restype = C.c_int
    lib.armt_backward.argtypes = [C.POINTER(ArmtConfig), C.POINTER(ArmtLayerWeights), i64, vp, sz, i32, vp, vp, vp,
                                  C.POINTER(ArmtLayerGrads), vp, vp, vp, vp, vp, sz, vp, i32]
    lib.armt_backward.restype = C.c_int
    lib.armt_tape_bytes_batched.argtypes = [C.POINTER(ArmtConfig), i32, i64]
    lib.armt_tape_bytes_batched.restype = sz
    lib.armt_backward_workspace_bytes_batched.argtypes = [C.POINTER(ArmtConfig), i32]
    lib.armt_backward_workspace_bytes_batched.restype = sz
    lib.armt_forward_train_batched.argtypes = [C.POINTER(ArmtConfig), C.POINTER(ArmtLayerWeights), vp, vp, i32, i64, vp, vp, vp, vp,
                                               vp, vp, sz, vp, sz, vp, i32]
    lib.armt_forward_train_batched.restype = C.c_int
    lib.armt_backward_batched.argtypes = [C.POINTER(ArmtConfig), C.POINTER(ArmtLayerWeights), i32, i64, vp, sz, i32, vp, vp, vp,
                                          C.POINTER(ArmtLayerGrads), vp, vp, vp, vp, vp, sz, vp, i32]
    lib.armt_backward_batched.restype = C.c_int
    lib.armt_diagonal_group.argtypes = [i32, i32, i32, C.POINTER(i32), C.POINTER(i32)]
    lib.armt_diagonal_group.restype = i32
    pp = C.POINTER(C.c_void_p)
    lib.armt_grouped_gemm.argtypes = [i32, i32, i32, i32, i32, pp, pp, pp, vp, sz, vp]
    lib.armt_grouped_gemm.restype = C.c_int
    lib.armt_segment_attention.argtypes = [C.POINTER(ArmtConfig), i32, vp, vp, vp, sz, vp]
    lib.armt_segment_attention.restype = C.c_int
    lib.armt_assoc_read.argtypes = [C.POINTER(ArmtConfig), i32, vp, pp, vp, vp, vp, sz, vp]
    lib.armt_assoc_read.restype = C.c_int
    lib.armt_assoc_update.argtypes = [C.POINTER(ArmtConfig), i32, vp, pp, pp, pp, i32, vp, vp, vp, sz, vp]
    lib.armt_assoc_update.restype = C.c_int
    lib.armt_embed_tokens.argtypes = [C.POINTER(ArmtConfig), vp, i32, vp, i64, vp, vp]
    lib.armt_embed_tokens.restype = C.c_int
    lib.armt_lm_head_workspace_bytes.argtypes = [C.POINTER(ArmtConfig), i64]
    lib.armt_lm_head_workspace_bytes.restype = sz
    lib.armt_lm_head.argtypes = [C.POINTER(ArmtConfig), vp, i64, vp, vp, i32, vp, vp, sz, vp]
    lib.armt_lm_head.restype = C.c_int
    lib.armt_lm_head_static.argtypes = [C.POINTER(ArmtConfig), vp, i64, vp, vp, i32, vp, vp]
    lib.armt_lm_head_static.restype = C.c_int
    lib.armt_lm_head_backward_workspace_bytes.argtypes = [C.POINTER(ArmtConfig), i64, i32]
    lib.armt_lm_head_backward_workspace_bytes.restype = sz
    lib.armt_lm_head_backward.argtypes = [C.POINTER(ArmtConfig), vp, i64, vp, vp, i32, vp, vp, vp, vp, vp, sz, vp]
    lib.armt_lm_head_backward.restype = C.c_int
    lib.armt_embed_tokens_backward.argtypes = [C.POINTER(ArmtConfig), vp, vp, i64, i32, vp, vp]
    lib.armt_embed_tokens_backward.restype = C.c_int
    lib.armt_set_gemm_tile_config.argtypes = [i32]
    lib.armt_set_gemm_tile_config.restype = i32
    lib.armt_profile_begin.argtypes = [i32, i32]
    lib.armt_profile_begin.restype = C.c_int
    lib.armt_profile_end.argtypes = [C.POINTER(C.c_double), C.POINTER(i64), C.POINTER(i64)]
    lib.armt_profile_end.restype = C.c_int
    lib.armt_status_str.argtypes = [C.c_int]
    lib.armt_status_str.restype = C.c_char_p
    lib.armt_last_hip_error.argtypes = []
    lib.armt_last_hip_error.restype = C.c_char_p
    _LIB = lib
    return lib


def _check(lib, code: int):
    if code != 0:
        text = lib.armt_status_str(code).decode()
        if code == 5:
            text += " (" + lib.armt_last_hip_error().decode() + ")"
        raise ArmtError(code, text)


def diagonal_group(n_layers: int, n_segments: int, t: int):
    """(l_lo, l_hi) of step t of the anti-diagonal schedule, or None outside 0 .. L+N-2."""
    lib = load_library()
    lo, hi = C.c_int32(-1), C.c_int32(-1)
    g = lib.armt_diagonal_group(n_layers, n_segments, t, C.byref(lo), C.byref(hi))
    return None if g == 0 else (lo.value, hi.value)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


class Armt:
    """An ARMT model resident in HBM: config + per-layer weight pointers + workspace."""

    def __init__(self, shape, layers, mem_emb, device="cuda:0"):
        import torch
        self.torch = torch
        self.lib = load_library()
        self.shape = shape
        self.cfg = ArmtConfig.from_shape(shape)
        self.device = torch.device(device)
        self.act_dtype = torch.bfloat16 if shape.dtype == "bf16" else torch.float32
        to = lambda a: torch.as_tensor(a).to(device=self.device, dtype=self.act_dtype).contiguous()
        self.layers = [{f: to(lw[f]) for f in LAYER_FIELDS} for lw in layers]
        self.mem_emb = to(mem_emb)
        self.c_layers = (ArmtLayerWeights * shape.n_layers)()
        for l, lw in enumerate(self.layers):
            for f in LAYER_FIELDS:
                setattr(self.c_layers[l], f, lw[f].data_ptr())
        nbytes = self.lib.armt_workspace_bytes(C.byref(self.cfg))
        if nbytes == 0:
            raise ArmtError(2, "configuration rejected by armt_workspace_bytes")
        self.workspace_bytes = nbytes
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)

    def embed(self, x):
        return self.torch.as_tensor(x).to(device=self.device, dtype=self.act_dtype).contiguous()

    def forward(self, x, diagonal=True, A_in=None, z_in=None, out=None, split_upto=None):
        """x: [n_tokens, d] device tensor of the activation type.  Returns (hidden, A, z).
        diagonal: True / False, or "auto" (armt_forward_auto; the order it took is left in self.order_used).
        split_upto: if given, armt_forward_diagonal_split with that threshold."""
        torch, s = self.torch, self.shape
        assert x.is_cuda and x.dtype == self.act_dtype and x.is_contiguous()
        n_tokens = x.shape[0]
        if out is None:
            hidden = torch.empty((n_tokens, s.d_model), dtype=self.act_dtype, device=self.device)
            A = torch.empty((s.n_layers, s.d_model, s.phi), dtype=torch.float32, device=self.device)
            z = torch.empty((s.n_layers, s.phi), dtype=torch.float32, device=self.device)
        else:
            hidden, A, z = out
        stream = torch.cuda.current_stream(self.device).cuda_stream
        args = (C.byref(self.cfg), self.c_layers, _ptr(self.mem_emb), _ptr(x), n_tokens, _ptr(A_in), _ptr(z_in),
                _ptr(hidden), _ptr(A), _ptr(z), _ptr(self.workspace), self.workspace_bytes, C.c_void_p(stream))
        if split_upto is not None:
            code = self.lib.armt_forward_diagonal_split(*args, int(split_upto))
        elif diagonal == "auto":
            used = C.c_int32(-1)
            code = self.lib.armt_forward_auto(*args, C.byref(used))
            self.order_used = used.value
        else:
            fn = self.lib.armt_forward_diagonal if diagonal else self.lib.armt_forward_sequential
            code = fn(*args)
        _check(self.lib, code)
        return hidden, A, z

    def forward_batched(self, x, diagonal=True, A_in=None, z_in=None, out=None):
        """x: [B, n_tokens, d] device tensor: B independent sequences.  Returns (hidden [B, n_tokens, d],
        A [B, L, d, Phi], z [B, L, Phi])."""
        torch, s = self.torch, self.shape
        assert x.is_cuda and x.dtype == self.act_dtype and x.is_contiguous() and x.dim() == 3
        B, n_tokens = x.shape[0], x.shape[1]
        need = self.lib.armt_workspace_bytes_batched(C.byref(self.cfg), B)
        if need == 0:
            raise ArmtError(2, "configuration or batch rejected by armt_workspace_bytes_batched")
        if self.workspace.numel() < need:
            self.workspace = torch.empty(need, dtype=torch.uint8, device=self.device)
        if out is None:
            hidden = torch.empty((B, n_tokens, s.d_model), dtype=self.act_dtype, device=self.device)
            A = torch.empty((B, s.n_layers, s.d_model, s.phi), dtype=torch.float32, device=self.device)
            z = torch.empty((B, s.n_layers, s.phi), dtype=torch.float32, device=self.device)
        else:
            hidden, A, z = out
        fn = self.lib.armt_forward_diagonal_batched if diagonal else self.lib.armt_forward_sequential_batched
        stream = torch.cuda.current_stream(self.device).cuda_stream
        code = fn(C.byref(self.cfg), self.c_layers, _ptr(self.mem_emb), _ptr(x), B, n_tokens, _ptr(A_in), _ptr(z_in),
                  _ptr(hidden), _ptr(A), _ptr(z), _ptr(self.workspace), self.workspace.numel(), C.c_void_p(stream))
        _check(self.lib, code)
        return hidden, A, z

    # ------------------------------------------------------------ training
    def forward_train(self, x, diagonal=True, A_in=None, z_in=None):
        """Forward pass that also records the tape the backward pass needs.  x: [n_tokens, d] or, for a batch of
        sequences, [B, n_tokens, d] (then hidden is [B, n_tokens, d], A [B, L, d, Phi], z [B, L, Phi]).
        Returns (hidden, A, z, tape)."""
        torch, s = self.torch, self.shape
        assert x.is_cuda and x.dtype == self.act_dtype and x.is_contiguous() and x.dim() in (2, 3)
        B = x.shape[0] if x.dim() == 3 else 1
        lead = (B,) if x.dim() == 3 else ()
        n_tokens = x.shape[-2]
        nbytes = self.lib.armt_tape_bytes_batched(C.byref(self.cfg), B, n_tokens)
        if nbytes == 0:
            raise ArmtError(6, "configuration, batch or length rejected by armt_tape_bytes_batched")
        need = self.lib.armt_workspace_bytes_batched(C.byref(self.cfg), B)
        if self.workspace.numel() < need:
            self.workspace = torch.empty(need, dtype=torch.uint8, device=self.device)
        tape = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        hidden = torch.empty(lead + (n_tokens, s.d_model), dtype=self.act_dtype, device=self.device)
        A = torch.empty(lead + (s.n_layers, s.d_model, s.phi), dtype=torch.float32, device=self.device)
        z = torch.empty(lead + (s.n_layers, s.phi), dtype=torch.float32, device=self.device)
        stream = torch.cuda.current_stream(self.device).cuda_stream
        code = self.lib.armt_forward_train_batched(C.byref(self.cfg), self.c_layers, _ptr(self.mem_emb), _ptr(x), B, n_tokens,
                                                   _ptr(A_in), _ptr(z_in), _ptr(hidden), _ptr(A), _ptr(z), _ptr(tape), nbytes,
                                                   _ptr(self.workspace), self.workspace.numel(), C.c_void_p(stream),
                                                   1 if diagonal else 0)
        _check(self.lib, code)
        return hidden, A, z, tape

    def backward(self, tape, n_tokens, d_hidden, dA_out=None, dz_out=None, carry_in=False, diagonal=True,
                 want_dx=True, grads=None):
        """Gradients of <hidden, d_hidden> + <A_out, dA_out> + <z_out, dz_out>; d_hidden [n_tokens, d] or [B, n_tokens, d]
        as in forward_train.  Returns a dict: "layers" (list of dicts of fp32 tensors, accumulated into `grads["layers"]`
        if given; summed over the sequences of a batch), "mem_emb", "x", "A_in", "z_in" (per sequence)."""
        torch, s = self.torch, self.shape
        f32 = dict(dtype=torch.float32, device=self.device)
        assert d_hidden.is_cuda and d_hidden.dtype == self.act_dtype and d_hidden.is_contiguous() and d_hidden.dim() in (2, 3)
        B = d_hidden.shape[0] if d_hidden.dim() == 3 else 1
        lead = (B,) if d_hidden.dim() == 3 else ()
        if grads is None:
            grads = {"layers": [{f: torch.zeros(tuple(lw[f].shape), **f32) for f in LAYER_FIELDS} for lw in self.layers],
                     "mem_emb": torch.zeros(tuple(self.mem_emb.shape), **f32)}
        c_grads = (ArmtLayerGrads * s.n_layers)()
        for l, g in enumerate(grads["layers"]):
            for f in LAYER_FIELDS:
                setattr(c_grads[l], f, g[f].data_ptr())
        dx = torch.empty(lead + (n_tokens, s.d_model), **f32) if want_dx else None
        dA_in = torch.empty(lead + (s.n_layers, s.d_model, s.phi), **f32) if carry_in else None
        dz_in = torch.empty(lead + (s.n_layers, s.phi), **f32) if carry_in else None
        need = self.lib.armt_backward_workspace_bytes_batched(C.byref(self.cfg), B)
        if need == 0:
            raise ArmtError(6, "configuration or batch rejected by armt_backward_workspace_bytes_batched")
        if getattr(self, "bwd_workspace", None) is None or self.bwd_workspace.numel() < need:
            self.bwd_workspace = torch.empty(need, dtype=torch.uint8, device=self.device)
        stream = torch.cuda.current_stream(self.device).cuda_stream
        code = self.lib.armt_backward_batched(C.byref(self.cfg), self.c_layers, B, n_tokens, _ptr(tape), tape.numel(),
                                              1 if carry_in else 0, _ptr(d_hidden), _ptr(dA_out), _ptr(dz_out), c_grads,
                                              _ptr(grads["mem_emb"]), _ptr(dx), _ptr(dA_in), _ptr(dz_in),
                                              _ptr(self.bwd_workspace), self.bwd_workspace.numel(), C.c_void_p(stream),
                                              1 if diagonal else 0)
        _check(self.lib, code)
        grads.update({"x": dx, "A_in": dA_in, "z_in": dz_in})
        return grads


# ---------------------------------------------------------------- single steps (tests, micro-benchmarks)
def _ptr_array(tensors):
    arr = (C.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i] = t.data_ptr()
    return arr


def _stream(torch):
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def set_gemm_tile_config(config: int) -> int:
    return load_library().armt_set_gemm_tile_config(config)


GEMM_KINDS = {"mem_q": 0, "mem_read": 1, "qkv": 2, "attn_out": 3, "gate_up": 4, "down": 5, "mem_kv": 6,
              "dpfp_read": 7, "update_prep": 8, "delta_rule": 9, "attention": 10}


def profile_begin(kind: str, max_launches: int):
    lib = load_library()
    _check(lib, lib.armt_profile_begin(GEMM_KINDS[kind], max_launches))


def profile_end():
    """(total kernel ms, launches, groups) of the GEMM kind selected by profile_begin."""
    lib = load_library()
    ms, n, g = C.c_double(0.0), C.c_int64(0), C.c_int64(0)
    _check(lib, lib.armt_profile_end(C.byref(ms), C.byref(n), C.byref(g)))
    return ms.value, n.value, g.value


def grouped_gemm(a_list, b_list, out_list=None, workspace=None):
    """C_i = A_i B_i^T; lists of device tensors A_i [M, K], B_i [N, K] (fp32 or bf16)."""
    import torch
    lib = load_library()
    g = len(a_list)
    M, K = a_list[0].shape
    N = b_list[0].shape[0]
    dt = a_list[0].dtype
    if out_list is None:
        out_list = [torch.empty((M, N), dtype=dt, device=a_list[0].device) for _ in range(g)]
    if workspace is None:
        workspace = torch.empty(max(256, g * 128), dtype=torch.uint8, device=a_list[0].device)
    code = lib.armt_grouped_gemm(ARMT_BF16 if dt == torch.bfloat16 else ARMT_F32, g, M, N, K, _ptr_array(a_list),
                                 _ptr_array(b_list), _ptr_array(out_list), _ptr(workspace), workspace.numel(),
                                 _stream(torch))
    _check(lib, code)
    return out_list


class ArmtSteps:
    """Single steps of the path on caller buffers, with the sizes of one configuration."""

    def __init__(self, shape, device="cuda:0"):
        import torch
        self.torch, self.shape = torch, shape
        self.lib = load_library()
        self.cfg = ArmtConfig.from_shape(shape)
        self.act_dtype = torch.bfloat16 if shape.dtype == "bf16" else torch.float32
        n = self.lib.armt_workspace_bytes(C.byref(self.cfg))
        if n == 0:
            raise ArmtError(2, "configuration rejected by armt_workspace_bytes")
        self.ws = torch.empty(n, dtype=torch.uint8, device=device)

    def segment_attention(self, qkv):
        """qkv [g, T, (H + 2 Hkv) dh] (rotated in place) -> out [g, T, H dh]."""
        torch, s = self.torch, self.shape
        g = qkv.shape[0]
        out = torch.empty((g, s.T, s.n_heads * s.head_dim), dtype=self.act_dtype, device=qkv.device)
        _check(self.lib, self.lib.armt_segment_attention(C.byref(self.cfg), g, _ptr(qkv), _ptr(out), _ptr(self.ws),
                                                         self.ws.numel(), _stream(torch)))
        return out

    def assoc_read(self, x, wm_q_list, A, z):
        """x [g, T, d] fp32, updated in place."""
        _check(self.lib, self.lib.armt_assoc_read(C.byref(self.cfg), x.shape[0], _ptr(x), _ptr_array(wm_q_list), _ptr(A),
                                                  _ptr(z), _ptr(self.ws), self.ws.numel(), _stream(self.torch)))
        return x

    def assoc_update(self, ym, wm_k_list, wm_v_list, wm_b_list, A, z, empty_group=-1):
        """ym [g, m, d] fp32; A [g, d, Phi], z [g, Phi] fp32 updated in place."""
        _check(self.lib, self.lib.armt_assoc_update(C.byref(self.cfg), ym.shape[0], _ptr(ym), _ptr_array(wm_k_list),
                                                    _ptr_array(wm_v_list), _ptr_array(wm_b_list), empty_group, _ptr(A),
                                                    _ptr(z), _ptr(self.ws), self.ws.numel(), _stream(self.torch)))
        return A, z


class TokenEnds:
    """Token-level ends of Algorithm 1 around a forward call: ids -> embeddings, hidden states -> logits."""

    def __init__(self, shape, emb_table, final_gain, w_lm, device="cuda:0"):
        import torch
        self.torch, self.shape = torch, shape
        self.lib = load_library()
        self.cfg = ArmtConfig.from_shape(shape)
        self.dt = torch.bfloat16 if shape.dtype == "bf16" else torch.float32
        dev = lambda a: a if isinstance(a, torch.Tensor) else torch.from_numpy(a).to(device=device, dtype=self.dt)
        self.emb_table, self.final_gain, self.w_lm = dev(emb_table), dev(final_gain), dev(w_lm)
        self.vocab = int(self.emb_table.shape[0])
        self.ws = None

    def embed(self, ids):
        """ids [n] int32 device tensor -> x [n, d_model]."""
        torch = self.torch
        x = torch.empty((ids.numel(), self.shape.d_model), dtype=self.dt, device=ids.device)
        _check(self.lib, self.lib.armt_embed_tokens(C.byref(self.cfg), _ptr(self.emb_table), self.vocab, _ptr(ids),
                                                    ids.numel(), _ptr(x), _stream(torch)))
        return x

    def logits(self, hidden, out=None):
        """hidden [n, d_model] -> logits [n, vocab] fp32."""
        torch = self.torch
        n = hidden.shape[0]
        need = self.lib.armt_lm_head_workspace_bytes(C.byref(self.cfg), n)
        if need == 0:
            raise ArmtError(2, "configuration or row count rejected by armt_lm_head_workspace_bytes")
        if self.ws is None or self.ws.numel() < need:
            self.ws = torch.empty(need, dtype=torch.uint8, device=hidden.device)
        V = int(self.w_lm.shape[0])
        if out is None:
            out = torch.empty((n, V), dtype=torch.float32, device=hidden.device)
        _check(self.lib, self.lib.armt_lm_head(C.byref(self.cfg), _ptr(hidden), n, _ptr(self.final_gain),
                                               _ptr(self.w_lm), V, _ptr(out), _ptr(self.ws), self.ws.numel(),
                                               _stream(torch)))
        return out

    def logits_static(self, hidden, out):
        """armt_lm_head_static: as logits(), with the library's own fixed scratch array; `out` must be given (this call
        and everything under it allocate nothing)."""
        n, V = hidden.shape[0], int(self.w_lm.shape[0])
        _check(self.lib, self.lib.armt_lm_head_static(C.byref(self.cfg), _ptr(hidden), n, _ptr(self.final_gain),
                                                      _ptr(self.w_lm), V, _ptr(out), _stream(self.torch)))
        return out

    def logits_backward(self, hidden, d_logits, grads=None):
        """Gradients of <logits, d_logits>: returns (d_hidden [n, d_model] fp32, d_final_gain [d_model], d_w_lm [vocab, d_model]);
        the last two are accumulated into `grads = (d_final_gain, d_w_lm)` if given."""
        torch = self.torch
        n, V = hidden.shape[0], int(self.w_lm.shape[0])
        assert d_logits.dtype == torch.float32 and d_logits.is_contiguous() and tuple(d_logits.shape) == (n, V)
        need = self.lib.armt_lm_head_backward_workspace_bytes(C.byref(self.cfg), n, V)
        if need == 0:
            raise ArmtError(2, "configuration or sizes rejected by armt_lm_head_backward_workspace_bytes")
        if getattr(self, "bws", None) is None or self.bws.numel() < need:
            self.bws = torch.empty(need, dtype=torch.uint8, device=hidden.device)
        f32 = dict(dtype=torch.float32, device=hidden.device)
        d_hidden = torch.empty((n, self.shape.d_model), **f32)
        d_gain, d_w = grads if grads is not None else (torch.zeros(self.shape.d_model, **f32), torch.zeros((V, self.shape.d_model), **f32))
        _check(self.lib, self.lib.armt_lm_head_backward(C.byref(self.cfg), _ptr(hidden), n, _ptr(self.final_gain), _ptr(self.w_lm), V,
                                                        _ptr(d_logits), _ptr(d_hidden), _ptr(d_gain), _ptr(d_w), _ptr(self.bws),
                                                        self.bws.numel(), _stream(torch)))
        return d_hidden, d_gain, d_w

    def embed_backward(self, ids, dx, d_table=None):
        """d_table[ids[i]] += dx[i] (fp32 [vocab, d_model]; allocated as zeros if not given)."""
        torch = self.torch
        assert dx.dtype == torch.float32 and dx.is_contiguous()
        if d_table is None:
            d_table = torch.zeros((self.vocab, self.shape.d_model), dtype=torch.float32, device=dx.device)
        _check(self.lib, self.lib.armt_embed_tokens_backward(C.byref(self.cfg), _ptr(dx), _ptr(ids), ids.numel(), self.vocab,
                                                             _ptr(d_table), _stream(torch)))
        return d_table

