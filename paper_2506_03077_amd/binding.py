"""Thin ctypes binding over libstreambp.so: argument marshalling only.

Function names mirror the C ABI in include/streambp.h.  torch is used for
device memory and the current HIP stream, nothing else: every step of the
path runs in the library's kernels.  If the library is missing the import of
any entry point raises - there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("STREAMBP_LIB") or os.path.join(_PKG, "libstreambp.so")   # (the override serves A/B runs of two builds)

SBP_F32, SBP_BF16 = 0, 1
SBP_OBJ_SFT, SBP_OBJ_GRPO, SBP_OBJ_DPO = 0, 1, 2
WEIGHT_NAMES = ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown", "g1", "g2")


class StreamBPError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"libstreambp error {code}: {msg}")
        self.code = code


class LayerCfg(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("batch", C.c_int32), ("seq_len", C.c_int32), ("chunk", C.c_int32),
                ("hidden", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("mlp_width", C.c_int32), ("rms_eps", C.c_float), ("rope_theta", C.c_float), ("pos_offset", C.c_int32),
                ("grad_dtype", C.c_int32), ("dw_group_rows", C.c_int32), ("window", C.c_int32),
                ("seq_first", C.POINTER(C.c_int32))]


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in WEIGHT_NAMES]


class LayerGrads(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in WEIGHT_NAMES]


MATRIX_NAMES = WEIGHT_NAMES[:7]


class LoraAdapters(C.Structure):
    _fields_ = [("rank", C.c_int32), ("scale", C.c_float), ("a", C.c_void_p * 7), ("b", C.c_void_p * 7)]


class LoraGrads(C.Structure):
    _fields_ = [("da", C.c_void_p * 7), ("db", C.c_void_p * 7)]


class HeadCfg(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("batch", C.c_int32), ("seq_len", C.c_int32), ("chunk", C.c_int32),
                ("hidden", C.c_int32), ("vocab", C.c_int32), ("objective", C.c_int32), ("loss_scale", C.c_float),
                ("clip_eps", C.c_float), ("kl_beta", C.c_float), ("kl_mode", C.c_int32), ("grad_dtype", C.c_int32), ("dw_group_rows", C.c_int32)]


class AttnCfg(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("q_start", C.c_int32), ("q_len", C.c_int32), ("scale", C.c_float), ("window", C.c_int32),
                ("kv_first", C.c_int32)]


class StackCfg(C.Structure):
    _fields_ = [("layer", LayerCfg), ("n_layers", C.c_int32), ("vocab", C.c_int32), ("head_chunk", C.c_int32),
                ("objective", C.c_int32), ("loss_scale", C.c_float), ("clip_eps", C.c_float), ("kl_beta", C.c_float),
                ("kl_mode", C.c_int32), ("final_eps", C.c_float)]


_lib = None


def lib():
    """Load the C-ABI library (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2506_03077_amd.build` "
                "(there is no CPU or PyTorch fallback)")
        L = C.CDLL(LIB_PATH)
        vp, sz, i32, i64, f32 = C.c_void_p, C.c_size_t, C.c_int32, C.c_int64, C.c_float
        L.streambp_version.restype = C.c_char_p
        L.streambp_last_error.restype = C.c_char_p
        L.streambp_layer_workspace_bytes.restype = sz
        L.streambp_layer_workspace_bytes.argtypes = [C.POINTER(LayerCfg)]
        L.streambp_layer_backward.restype = i32
        L.streambp_layer_backward.argtypes = [C.POINTER(LayerCfg), C.POINTER(LayerWeights), vp, vp, vp,
                                              C.POINTER(LayerGrads), vp, sz, vp]
        L.streambp_layer_lora_workspace_bytes.restype = sz
        L.streambp_layer_lora_workspace_bytes.argtypes = [C.POINTER(LayerCfg), C.POINTER(LoraAdapters)]
        L.streambp_layer_lora_backward.restype = i32
        L.streambp_layer_lora_backward.argtypes = [C.POINTER(LayerCfg), C.POINTER(LayerWeights), C.POINTER(LoraAdapters), vp, vp, vp,
                                                   C.POINTER(LoraGrads), vp, sz, vp]
        L.streambp_layer_forward.restype = i32
        L.streambp_layer_forward.argtypes = [C.POINTER(LayerCfg), C.POINTER(LayerWeights), vp, vp, vp, sz, vp]
        L.streambp_lmhead_workspace_bytes.restype = sz
        L.streambp_lmhead_workspace_bytes.argtypes = [C.POINTER(HeadCfg)]
        L.streambp_lmhead_ce_backward.restype = i32
        L.streambp_lmhead_ce_backward.argtypes = [C.POINTER(HeadCfg), vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.streambp_attn_workspace_bytes.restype = sz
        L.streambp_attn_workspace_bytes.argtypes = [C.POINTER(AttnCfg)]
        L.streambp_attn_chunk_forward.restype = i32
        L.streambp_attn_chunk_forward.argtypes = [C.POINTER(AttnCfg), vp, vp, vp, vp, vp, vp]
        L.streambp_attn_chunk_backward.restype = i32
        L.streambp_attn_chunk_backward.argtypes = [C.POINTER(AttnCfg), vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.streambp_attn_chunk_backward_noalloc.restype = i32
        L.streambp_attn_chunk_backward_noalloc.argtypes = [C.POINTER(AttnCfg), vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.streambp_rmsnorm_workspace_bytes.restype = sz
        L.streambp_rmsnorm_workspace_bytes.argtypes = [i64, i32]
        L.streambp_rmsnorm_forward.restype = i32
        L.streambp_rmsnorm_forward.argtypes = [i32, i64, i32, f32, vp, vp, vp, vp]
        L.streambp_rmsnorm_backward.restype = i32
        L.streambp_rmsnorm_backward.argtypes = [i32, i64, i32, f32, vp, vp, vp, vp, vp, vp, sz, vp]
        L.streambp_embedding_forward.restype = i32
        L.streambp_embedding_forward.argtypes = [i32, i64, i32, i32, vp, vp, vp, vp]
        L.streambp_embedding_backward.restype = i32
        L.streambp_embedding_backward.argtypes = [i32, i64, i32, i32, vp, vp, vp, vp]
        L.streambp_attn_tile_pairs.restype = i64
        L.streambp_attn_tile_pairs.argtypes = [i32, i32, C.POINTER(i32), C.POINTER(i32)]
        L.streambp_layer_fast_path.restype = i32
        L.streambp_layer_fast_path.argtypes = [C.POINTER(LayerCfg)]
        L.streambp_lmhead_fast_path.restype = i32
        L.streambp_lmhead_fast_path.argtypes = [C.POINTER(HeadCfg)]
        L.streambp_generic_launches.restype = i64
        L.streambp_generic_launches.argtypes = []
        L.streambp_debug_set_fusions.restype = None
        L.streambp_debug_set_fusions.argtypes = [C.c_int]
        L.streambp_debug_get_fusions.restype = C.c_int
        L.streambp_debug_force_generic.restype = None
        L.streambp_debug_force_generic.argtypes = [C.c_int, C.c_int]
        L.streambp_debug_gemm.restype = C.c_int
        L.streambp_debug_gemm.argtypes = [C.c_int] * 8 + [vp, vp, vp, C.c_longlong, C.c_longlong, C.c_longlong, vp, sz, vp, vp, vp, vp]
        L.streambp_stack_workspace_bytes.restype = sz
        L.streambp_stack_workspace_bytes.argtypes = [C.POINTER(StackCfg)]
        L.streambp_stack_forward.restype = i32
        L.streambp_stack_forward.argtypes = [C.POINTER(StackCfg), C.POINTER(LayerWeights), vp, vp, C.POINTER(vp), vp, sz, vp]
        L.streambp_stack_backward.restype = i32
        L.streambp_stack_backward.argtypes = [C.POINTER(StackCfg), C.POINTER(LayerWeights), vp, vp, C.POINTER(vp), vp, vp, vp, vp,
                                              vp, C.POINTER(LayerGrads), vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.streambp_debug_gemm_dw_segments.restype = C.c_int
        L.streambp_debug_gemm_dw_segments.argtypes = [C.c_int, C.c_int, C.c_int, C.POINTER(C.c_int), C.POINTER(vp), C.POINTER(vp),
                                                      C.POINTER(vp), vp, C.c_longlong, C.c_longlong, C.c_longlong, C.c_int, C.c_int, vp]
        L.streambp_debug_profile_begin.restype = C.c_int
        L.streambp_debug_profile_begin.argtypes = [C.c_int]
        L.streambp_debug_profile_end.restype = C.c_int
        L.streambp_debug_profile_end.argtypes = [C.POINTER(C.c_longlong), C.POINTER(C.c_double), C.POINTER(C.c_double),
                                                 C.POINTER(C.c_double)]
        L.streambp_debug_profile_kinds.restype = C.c_int
        L.streambp_debug_gemm_numerators.restype = C.c_int
        L.streambp_debug_gemm_numerators.argtypes = [C.c_int, C.c_int, C.c_int, vp, vp, vp, C.c_longlong, C.c_longlong, C.c_longlong,
                                                     vp, vp, vp, vp, vp]
        L.streambp_debug_mfma_rate.restype = C.c_int
        L.streambp_debug_mfma_rate.argtypes = [vp, vp, C.c_int, C.c_int, C.c_int, vp]
        _lib = L
    return _lib


def _check(rc):
    if rc != 0:
        raise StreamBPError(rc, lib().streambp_last_error().decode())


def _torch():
    import torch
    return torch


def _dt_code(t):
    torch = _torch()
    if t.dtype == torch.float32:
        return SBP_F32
    if t.dtype == torch.bfloat16:
        return SBP_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ptr(t):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "tensors must be contiguous device tensors"
    return t.data_ptr()


def _stream(stream):
    torch = _torch()
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream


def _workspace(nbytes, device):
    torch = _torch()
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def streambp_version():
    return lib().streambp_version().decode()


def layer_cfg(dtype, batch, seq_len, chunk, hidden, n_q_heads, n_kv_heads, head_dim, mlp_width,
              rms_eps=1e-6, rope_theta=1e4, pos_offset=0, grad_dtype=SBP_F32, dw_group_rows=0, window=0, seq_first=None):
    """seq_first: optional list of `batch` ints (rows of padding in front of every sequence); held by the returned struct."""
    cfg = LayerCfg(int(dtype), batch, seq_len, chunk, hidden, n_q_heads, n_kv_heads, head_dim, mlp_width,
                   rms_eps, rope_theta, pos_offset, int(grad_dtype), int(dw_group_rows), int(window), None)
    if seq_first is not None:
        assert len(seq_first) == batch
        cfg._seq_first = (C.c_int32 * batch)(*[int(v) for v in seq_first])     # kept alive with the struct
        cfg.seq_first = C.cast(cfg._seq_first, C.POINTER(C.c_int32))
    return cfg


def streambp_layer_workspace_bytes(cfg: LayerCfg) -> int:
    return int(lib().streambp_layer_workspace_bytes(C.byref(cfg)))


def _weights_struct(w):
    return LayerWeights(*[_ptr(w[n]) for n in WEIGHT_NAMES])


def _grad_torch_dtype(grad_dtype):
    torch = _torch()
    return torch.bfloat16 if int(grad_dtype) == SBP_BF16 else torch.float32


def new_layer_grads(w, grad_dtype=SBP_F32):
    """Zero accumulators shaped like the weights: matrices in grad_dtype, the two norm gains always fp32."""
    torch = _torch()
    mat = _grad_torch_dtype(grad_dtype)
    return {n: torch.zeros(w[n].shape, dtype=(torch.float32 if n in ("g1", "g2") else mat), device=w[n].device)
            for n in WEIGHT_NAMES}


def streambp_layer_backward(cfg: LayerCfg, w, x, dy, dx=None, dw=None, workspace=None, stream=None):
    """x, dy [B,T,d]; returns (dx, dw).  dw (dict of fp32 tensors) is accumulated into."""
    torch = _torch()
    if dx is None:
        dx = torch.empty_like(x)
    if dw is None:
        dw = new_layer_grads(w, cfg.grad_dtype)
    for n in WEIGHT_NAMES:
        want = torch.float32 if n in ("g1", "g2") else _grad_torch_dtype(cfg.grad_dtype)
        assert dw[n].dtype == want, f"dw[{n}] must be {want} for this cfg"
    if workspace is None:
        workspace = _workspace(streambp_layer_workspace_bytes(cfg), x.device)
    ws, gs = _weights_struct(w), LayerGrads(*[_ptr(dw[n]) for n in WEIGHT_NAMES])
    _check(lib().streambp_layer_backward(C.byref(cfg), C.byref(ws), _ptr(x), _ptr(dy), _ptr(dx), C.byref(gs),
                                         _ptr(workspace), workspace.numel(), _stream(stream)))
    return dx, dw


def _lora_struct(adapters, rank, scale):
    a = (C.c_void_p * 7)(*[(_ptr(adapters[n][0]) if n in adapters else None) for n in MATRIX_NAMES])
    b = (C.c_void_p * 7)(*[(_ptr(adapters[n][1]) if n in adapters else None) for n in MATRIX_NAMES])
    return LoraAdapters(int(rank), float(scale), a, b)


def streambp_layer_lora_workspace_bytes(cfg: LayerCfg, adapters, rank, scale=1.0) -> int:
    ad = _lora_struct(adapters, rank, scale)
    return int(lib().streambp_layer_lora_workspace_bytes(C.byref(cfg), C.byref(ad)))


def streambp_layer_lora_backward(cfg: LayerCfg, w, adapters, rank, scale, x, dy, dx=None, da=None, db=None, workspace=None,
                                 stream=None):
    """adapters: dict matrix name -> (A [r, in], B [out, r]) device tensors; returns (dx, da, db) with da / db dicts of fp32
    tensors (accumulated into when given)."""
    torch = _torch()
    if dx is None:
        dx = torch.empty_like(x)
    if da is None:
        da = {n: torch.zeros(ab[0].shape, dtype=torch.float32, device=x.device) for n, ab in adapters.items()}
    if db is None:
        db = {n: torch.zeros(ab[1].shape, dtype=torch.float32, device=x.device) for n, ab in adapters.items()}
    ad = _lora_struct(adapters, rank, scale)
    if workspace is None:
        workspace = _workspace(lib().streambp_layer_lora_workspace_bytes(C.byref(cfg), C.byref(ad)), x.device)
    gs = LoraGrads((C.c_void_p * 7)(*[(_ptr(da[n]) if n in adapters else None) for n in MATRIX_NAMES]),
                   (C.c_void_p * 7)(*[(_ptr(db[n]) if n in adapters else None) for n in MATRIX_NAMES]))
    ws = _weights_struct(w)
    _check(lib().streambp_layer_lora_backward(C.byref(cfg), C.byref(ws), C.byref(ad), _ptr(x), _ptr(dy), _ptr(dx), C.byref(gs),
                                              _ptr(workspace), workspace.numel(), _stream(stream)))
    return dx, da, db


def streambp_layer_forward(cfg: LayerCfg, w, x, y=None, workspace=None, stream=None):
    torch = _torch()
    if y is None:
        y = torch.empty_like(x)
    if workspace is None:
        workspace = _workspace(streambp_layer_workspace_bytes(cfg), x.device)
    ws = _weights_struct(w)
    _check(lib().streambp_layer_forward(C.byref(cfg), C.byref(ws), _ptr(x), _ptr(y), _ptr(workspace),
                                        workspace.numel(), _stream(stream)))
    return y


def head_cfg(dtype, batch, seq_len, chunk, hidden, vocab, objective=SBP_OBJ_SFT, loss_scale=1.0,
             clip_eps=0.2, kl_beta=0.04, kl_mode=0, grad_dtype=SBP_F32, dw_group_rows=0):
    return HeadCfg(int(dtype), batch, seq_len, chunk, hidden, vocab, objective, loss_scale, clip_eps, kl_beta, kl_mode,
                   int(grad_dtype), int(dw_group_rows))


def streambp_lmhead_workspace_bytes(cfg: HeadCfg) -> int:
    return int(lib().streambp_lmhead_workspace_bytes(C.byref(cfg)))


def streambp_lmhead_ce_backward(cfg: HeadCfg, w, h, targets, old_logp=None, ref_logp=None, advantages=None,
                                dh=None, dw=None, loss=None, n_active=None, workspace=None, stream=None):
    """Returns (dh, dw, loss, n_active) - loss and n_active are 1-element device tensors."""
    torch = _torch()
    dev = h.device
    if dh is None:
        dh = torch.empty_like(h)
    if dw is None:
        dw = torch.zeros(w.shape, dtype=_grad_torch_dtype(cfg.grad_dtype), device=dev)
    assert dw.dtype == _grad_torch_dtype(cfg.grad_dtype), "dw must have the element type cfg.grad_dtype names"
    if loss is None:
        loss = torch.zeros(1, dtype=torch.float32, device=dev)
    if n_active is None:
        n_active = torch.zeros(1, dtype=torch.int64, device=dev)
    if workspace is None:
        workspace = _workspace(streambp_lmhead_workspace_bytes(cfg), dev)
    assert targets.dtype == torch.int32
    _check(lib().streambp_lmhead_ce_backward(C.byref(cfg), _ptr(w), _ptr(h), _ptr(targets), _ptr(old_logp),
                                             _ptr(ref_logp), _ptr(advantages), _ptr(dh), _ptr(dw), _ptr(loss),
                                             _ptr(n_active), _ptr(workspace), workspace.numel(), _stream(stream)))
    return dh, dw, loss, n_active


def attn_cfg(dtype, n_q_heads, n_kv_heads, head_dim, q_start, q_len, scale, window=0, kv_first=0):
    return AttnCfg(int(dtype), n_q_heads, n_kv_heads, head_dim, q_start, q_len, scale, int(window), int(kv_first))


def streambp_attn_workspace_bytes(cfg: AttnCfg) -> int:
    return int(lib().streambp_attn_workspace_bytes(C.byref(cfg)))


def streambp_attn_chunk_forward(cfg: AttnCfg, q, k, v, o=None, lse=None, stream=None):
    torch = _torch()
    if o is None:
        o = torch.empty_like(q)
    if lse is None:
        lse = torch.empty((cfg.n_q_heads, cfg.q_len), dtype=torch.float32, device=q.device)
    _check(lib().streambp_attn_chunk_forward(C.byref(cfg), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _stream(stream)))
    return o, lse


def streambp_attn_chunk_backward(cfg: AttnCfg, q, k, v, o, lse, d_o, dq=None, dk=None, dv=None, workspace=None,
                                 stream=None):
    """dk, dv [>= s+c, Hkv, dh] fp32 are accumulated into (zero tensors are made if not given)."""
    torch = _torch()
    if dq is None:
        dq = torch.empty_like(q)
    if dk is None:
        dk = torch.zeros(k.shape, dtype=torch.float32, device=q.device)
    if dv is None:
        dv = torch.zeros(v.shape, dtype=torch.float32, device=q.device)
    if workspace is None:
        workspace = _workspace(streambp_attn_workspace_bytes(cfg), q.device)
    _check(lib().streambp_attn_chunk_backward(C.byref(cfg), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(d_o),
                                              _ptr(dq), _ptr(dk), _ptr(dv), _ptr(workspace), workspace.numel(),
                                              _stream(stream)))
    return dq, dk, dv


def streambp_attn_chunk_backward_noalloc(cfg: AttnCfg, q, k, v, o, lse, d_o, dq, dk, dv, stream=None):
    """The backward without a workspace (the library's built-in scratch); every output tensor is the caller's."""
    _check(lib().streambp_attn_chunk_backward_noalloc(C.byref(cfg), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(d_o),
                                                      _ptr(dq), _ptr(dk), _ptr(dv), _stream(stream)))
    return dq, dk, dv


def streambp_rmsnorm_forward(x, g, eps=1e-6, y=None, stream=None):
    torch = _torch()
    if y is None:
        y = torch.empty_like(x)
    d = x.shape[-1]
    _check(lib().streambp_rmsnorm_forward(_dt_code(x), x.numel() // d, d, eps, _ptr(x), _ptr(g), _ptr(y), _stream(stream)))
    return y


def streambp_rmsnorm_backward(x, g, dy, eps=1e-6, dx=None, dg=None, workspace=None, stream=None):
    torch = _torch()
    d = x.shape[-1]
    n = x.numel() // d
    if dx is None:
        dx = torch.empty_like(x)
    if dg is None:
        dg = torch.zeros(d, dtype=torch.float32, device=x.device)
    if workspace is None:
        workspace = _workspace(lib().streambp_rmsnorm_workspace_bytes(n, d), x.device)
    _check(lib().streambp_rmsnorm_backward(_dt_code(x), n, d, eps, _ptr(x), _ptr(g), _ptr(dy), _ptr(dx), _ptr(dg),
                                           _ptr(workspace), workspace.numel(), _stream(stream)))
    return dx, dg


def streambp_embedding_forward(ids, emb, x=None, stream=None):
    torch = _torch()
    V, d = emb.shape
    if x is None:
        x = torch.empty((ids.numel(), d), dtype=emb.dtype, device=emb.device)
    _check(lib().streambp_embedding_forward(_dt_code(emb), ids.numel(), d, V, _ptr(ids), _ptr(emb), _ptr(x), _stream(stream)))
    return x


def streambp_embedding_backward(ids, dx, vocab, demb=None, stream=None):
    torch = _torch()
    d = dx.shape[-1]
    if demb is None:
        demb = torch.zeros((vocab, d), dtype=torch.float32, device=dx.device)
    _check(lib().streambp_embedding_backward(_dt_code(dx), ids.numel(), d, vocab, _ptr(ids), _ptr(dx), _ptr(demb), _stream(stream)))
    return demb


def streambp_layer_fast_path(cfg: LayerCfg) -> int:
    """1: the whole configuration runs on the bf16 MFMA kernels; 0: part of it on the shape-agnostic kernels."""
    return int(lib().streambp_layer_fast_path(C.byref(cfg)))


def streambp_lmhead_fast_path(cfg: HeadCfg) -> int:
    return int(lib().streambp_lmhead_fast_path(C.byref(cfg)))


def streambp_generic_launches() -> int:
    """bf16 launches that ran on the shape-agnostic kernels since the library was loaded."""
    return int(lib().streambp_generic_launches())


def streambp_attn_tile_pairs(q_start, q_len):
    tq, tk = C.c_int32(0), C.c_int32(0)
    n = lib().streambp_attn_tile_pairs(q_start, q_len, C.byref(tq), C.byref(tk))
    return int(n), tq.value, tk.value


def debug_set_fusions(mask):
    """Optional fusions (bit 0: SwiGLU adjoint in the dact GEMM's epilogue; bit 1: RoPE of q / dq inside the attention
    kernels; bit 2: the LM head's logits GEMM stores bf16 softmax numerators instead of fp32 logits); returns the previous mask."""
    old = lib().streambp_debug_get_fusions()
    lib().streambp_debug_set_fusions(int(mask))
    return old


def debug_force_generic(gemm=False, attn=False):
    """Route GEMMs / attention through the shape-agnostic kernels (A/B testing of the MFMA kernels)."""
    lib().streambp_debug_force_generic(int(gemm), int(attn))


def debug_gemm(A, B, C_out, M, N, K, ta, tb, acc=False, scratch=None, stream=None, A2=None, B2=None, row_stats=None):
    """C[M,N] (=|+=) op(A) op(B) [+ op(A2) op(B2)] through the library's GEMM dispatcher; returns 1 if the MFMA kernel
    ran, 0 if the shape-agnostic one did.  A(m,k) = A[k,m] if ta else A[m,k]; B(k,n) = B[n,k] if tb else B[k,n].
    row_stats: optional fp32 [M, N/256, 2] output, (max, sum of exp(c - max)) of every row over every block of 256 columns
    (MFMA store form C = A B^T with fp32 C only; the launch fails where that kernel cannot take the problem)."""
    assert C_out.is_cuda and C_out.stride(-1) == 1      # C may be a column slice of a wider buffer (ldc = its row stride)
    rc = lib().streambp_debug_gemm(M, N, K, int(ta), int(tb), _dt_code(A), _dt_code(C_out), int(acc), _ptr(A), _ptr(B),
                                   C_out.data_ptr(), A.stride(0), B.stride(0), C_out.stride(0), _ptr(scratch),
                                   0 if scratch is None else scratch.numel() * scratch.element_size(), _stream(stream),
                                   _ptr(A2), _ptr(B2), _ptr(row_stats))
    if rc < 0:
        raise StreamBPError(rc, "debug_gemm launch failed")
    return rc


def debug_gemm_dw_segments(As, Bs, C_out, M, N, Ks, rows_dev=None, stream=None):
    """C[M,N] += sum_s As[s]^T Bs[s] (As[s] [K_s, M], Bs[s] [K_s, N]) through the library's batched dispatcher; rows_dev: optional
    list of int32 device scalars (or None) limiting each segment's row count.  Returns 1 if one segmented MFMA launch did it."""
    n = len(As)
    Ka = (C.c_int * n)(*Ks)
    Aa = (C.c_void_p * n)(*[_ptr(a) for a in As])
    Ba = (C.c_void_p * n)(*[_ptr(b) for b in Bs])
    Ra = (C.c_void_p * n)(*[(_ptr(r) if r is not None else None) for r in (rows_dev or [None] * n)])
    rc = lib().streambp_debug_gemm_dw_segments(n, M, N, Ka, Aa, Ba, Ra, _ptr(C_out), As[0].stride(0), Bs[0].stride(0),
                                               C_out.stride(0), _dt_code(As[0]), _dt_code(C_out), _stream(stream))
    if rc < 0:
        raise StreamBPError(rc, "debug_gemm_dw_segments launch failed")
    return rc


def debug_gemm_numerators(A, B, E, stats, targets, target_value, row_index=None, stream=None):
    """E (bf16 [M,N]) = exp(A B^T - block max), stats [M, ceil(N/256), 2], target_value [M] (see streambp_debug.h).  Returns 1
    if the MFMA kernel ran."""
    M, K = A.shape
    N = B.shape[0]
    rc = lib().streambp_debug_gemm_numerators(M, N, K, _ptr(A), _ptr(B), _ptr(E), A.stride(0), B.stride(0), E.stride(0), _ptr(stats),
                                              _ptr(targets), _ptr(row_index) if row_index is not None else None, _ptr(target_value),
                                              _stream(stream))
    if rc < 0:
        raise StreamBPError(rc, "debug_gemm_numerators launch failed")
    return rc


def debug_mfma_rate(operands, workgroups=512, iters=10000, repeats=12, lds_reads=0, stream=None):
    """TFLOP/s the matrix pipe sustains on fragments taken from `operands` (a bf16 device tensor of 32768 values: the rate
    depends on the values) with no global memory traffic, `lds_reads` (0, 6, 8) of every eight A fragments re-read from LDS:
    streambp_debug_mfma_rate timed with events on the launch stream.  The
    default launches keep the chip busy for 0.1-0.15 s: the power management settles within the first tens of milliseconds."""
    import torch
    assert operands.dtype == torch.bfloat16 and operands.numel() == 32768 and operands.is_contiguous()
    sink = torch.empty(workgroups * 512, dtype=torch.float32, device=operands.device)
    launch = lambda n: lib().streambp_debug_mfma_rate(_ptr(operands), _ptr(sink), workgroups, n, lds_reads, _stream(stream))
    if launch(max(1, iters // 10)) != 0:
        raise StreamBPError(-5, "debug_mfma_rate launch failed")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(repeats):
        if launch(iters) != 0:
            raise StreamBPError(-5, "debug_mfma_rate launch failed")
    e1.record()
    e1.synchronize()
    flops = 2.0 * 32 * 32 * 16 * 8 * iters * 8 * workgroups * repeats
    return flops / (e0.elapsed_time(e1) * 1e-3) / 1e12


def _profile_kind_names():
    lay = (("false, true", "NT"), ("false, false", "NN"), ("true, false", "TN"))
    names = [f"gemm_mfma_k<{t}, {m}>" for t, _ in lay for m in range(4)]
    names += [f"gemm_mfma_group_k<{t}, {m}>" for t, _ in lay for m in range(4)]
    names += ["gemm_generic_k", "attn_fwd (launch sequence)", "attn_bwd (delta + dq + dkv launch sequence)", "gemm_mfma_seg_k",
              "gemm_mfma_k<false, true, 5>", "gemm_mfma_k<false, false, 6>", "gemm_mfma_k<false, true, 7>"]
    return tuple(names)


PROFILE_KINDS = _profile_kind_names()   # GEMM entries are the kernel symbols rocprofv3 reports (sbp:: prefix dropped)


def debug_profile_begin(max_records=100000):
    """Start per-launch HIP-event timing of the GEMM kernels / attention launch sequences (events are created here)."""
    rc = lib().streambp_debug_profile_begin(max_records)
    if rc != 0:
        raise StreamBPError(rc, "profile_begin failed")


def debug_profile_end():
    """Stop timing; returns {kind: dict(count, ms, flops, flops_bounded)} summed over the launches since begin.
    flops_bounded is the work of launches whose row count was only known on the device, computed from the host-side
    upper bound (scale it by the fraction of rows that were really there)."""
    n = len(PROFILE_KINDS)
    assert n == lib().streambp_debug_profile_kinds()
    cnt, ms, work, wb = (C.c_longlong * n)(), (C.c_double * n)(), (C.c_double * n)(), (C.c_double * n)()
    rc = lib().streambp_debug_profile_end(cnt, ms, work, wb)
    if rc != 0:
        raise StreamBPError(rc, "profile_end failed")
    return {k: dict(count=int(cnt[i]), ms=float(ms[i]), flops=float(work[i]), flops_bounded=float(wb[i]))
            for i, k in enumerate(PROFILE_KINDS)}


def stack_cfg(layer: LayerCfg, n_layers, vocab, head_chunk, objective=SBP_OBJ_SFT, loss_scale=1.0, clip_eps=0.2,
              kl_beta=0.04, kl_mode=0, final_eps=1e-6):
    sc = StackCfg(layer, n_layers, vocab, head_chunk, objective, loss_scale, clip_eps, kl_beta, kl_mode, final_eps)
    sc._layer = layer            # the copy shares layer.seq_first: keep the array's owner alive
    return sc


def streambp_stack_workspace_bytes(cfg: StackCfg) -> int:
    return int(lib().streambp_stack_workspace_bytes(C.byref(cfg)))


def _ptr_array(tensors):
    return (C.c_void_p * len(tensors))(*[_ptr(t) for t in tensors])


def streambp_stack_forward(cfg: StackCfg, layers, ckpt, emb=None, ids=None, workspace=None, stream=None):
    """layers: list of weight dicts; ckpt: list of L+1 [B,T,d] tensors (filled: ckpt[l] = input of layer l)."""
    if workspace is None:
        workspace = _workspace(streambp_stack_workspace_bytes(cfg), ckpt[0].device)
    ws = (LayerWeights * len(layers))(*[_weights_struct(w) for w in layers])
    _check(lib().streambp_stack_forward(C.byref(cfg), ws, _ptr(emb), _ptr(ids), _ptr_array(ckpt), _ptr(workspace),
                                        workspace.numel(), _stream(stream)))
    return ckpt


def streambp_stack_backward(cfg: StackCfg, layers, g_final, w_head, ckpt, targets, ids=None, old_logp=None, ref_logp=None,
                            advantages=None, dlayers=None, dg_final=None, dw_head=None, demb=None, dx0=None, loss=None,
                            n_active=None, workspace=None, stream=None):
    """Returns dict(dlayers, dg_final, dw_head, demb, dx0, loss, n_active); gradient tensors are accumulated into."""
    torch = _torch()
    dev = ckpt[0].device
    if dlayers is None:
        dlayers = [new_layer_grads(w, cfg.layer.grad_dtype) for w in layers]
    if dg_final is None:
        dg_final = torch.zeros(g_final.shape, dtype=torch.float32, device=dev)
    if dw_head is None:
        dw_head = torch.zeros(w_head.shape, dtype=_grad_torch_dtype(cfg.layer.grad_dtype), device=dev)
    if ids is not None and demb is None:
        demb = torch.zeros(w_head.shape, dtype=torch.float32, device=dev)
    if dx0 is None:
        dx0 = torch.empty_like(ckpt[0])
    if loss is None:
        loss = torch.zeros(1, dtype=torch.float32, device=dev)
    if n_active is None:
        n_active = torch.zeros(1, dtype=torch.int64, device=dev)
    if workspace is None:
        workspace = _workspace(streambp_stack_workspace_bytes(cfg), dev)
    ws = (LayerWeights * len(layers))(*[_weights_struct(w) for w in layers])
    gs = (LayerGrads * len(layers))(*[LayerGrads(*[_ptr(g[n]) for n in WEIGHT_NAMES]) for g in dlayers])
    _check(lib().streambp_stack_backward(C.byref(cfg), ws, _ptr(g_final), _ptr(w_head), _ptr_array(ckpt), _ptr(ids),
                                         _ptr(targets), _ptr(old_logp), _ptr(ref_logp), _ptr(advantages), gs,
                                         _ptr(dg_final), _ptr(dw_head), _ptr(demb), _ptr(dx0), _ptr(loss), _ptr(n_active),
                                         _ptr(workspace), workspace.numel(), _stream(stream)))
    return dict(dlayers=dlayers, dg_final=dg_final, dw_head=dw_head, demb=demb, dx0=dx0, loss=loss, n_active=n_active)


def streambp_rmsnorm_workspace_bytes(n_rows, hidden) -> int:
    return int(lib().streambp_rmsnorm_workspace_bytes(n_rows, hidden))


def streambp_last_error():
    return lib().streambp_last_error().decode()
