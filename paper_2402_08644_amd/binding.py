"""ctypes binding of libtandem.so: argument marshalling only.

Each function has the name of the C entry point it calls (include/tandem.h).  Tensors are
torch tensors used purely as handles to device memory (``data_ptr()``) and to the current
HIP stream; no torch operator takes part in the computation.  There is no fallback: if the
library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import math
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtandem.so")

OK, ERR_NULL, ERR_SHAPE, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP = range(6)
F32, BF16 = 0, 1
ACT_NONE, ACT_GELU, ACT_RELU = 0, 1, 2
MAX_QLEN = 32
MAX_PREFILL = 128
_ACT = {None: ACT_NONE, "none": ACT_NONE, "gelu": ACT_GELU, "relu": ACT_RELU}


class TandemError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


class AttnDesc(C.Structure):
    _fields_ = [
        ("B", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("dh", C.c_int32),
        ("T_max", C.c_int64), ("gamma_max", C.c_int32), ("scale", C.c_float), ("dtype", C.c_int32),
    ]


class FFDesc(C.Structure):
    _fields_ = [
        ("d_L", C.c_int32), ("d_hidden", C.c_int32), ("d_S", C.c_int32), ("act", C.c_int32), ("dtype", C.c_int32),
        ("W1", C.c_void_p), ("b1", C.c_void_p), ("W2", C.c_void_p), ("b2", C.c_void_p),
        ("W1p", C.c_void_p), ("W2p", C.c_void_p),
    ]


class LayerWeights(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in ("g_attn", "Wqkv", "Wo", "g_mlp", "W1", "b1", "W2", "b2")]


class DecoderDesc(C.Structure):
    _fields_ = [
        ("n_layers", C.c_int32), ("d", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("dh", C.c_int32),
        ("d_ff", C.c_int32), ("vocab", C.c_int32),
        ("emb", C.c_void_p), ("g_final", C.c_void_p), ("W_out", C.c_void_p), ("layers", C.POINTER(LayerWeights)),
    ]


class ModelDesc(C.Structure):
    _fields_ = [
        ("L", DecoderDesc), ("S", DecoderDesc), ("ell", C.POINTER(C.c_int32)), ("ff", C.POINTER(FFDesc)),
        ("rms_eps", C.c_float), ("dtype", C.c_int32), ("flags", C.c_int32),
    ]


class StateDesc(C.Structure):
    _fields_ = [
        ("B", C.c_int32), ("T_max", C.c_int64), ("gamma_max", C.c_int32),
        ("KL", C.POINTER(C.c_void_p)), ("VL", C.POINTER(C.c_void_p)),
        ("Khat", C.POINTER(C.c_void_p)), ("Vhat", C.POINTER(C.c_void_p)),
        ("Kcur", C.POINTER(C.c_void_p)), ("Vcur", C.POINTER(C.c_void_p)),
        ("n", C.c_void_p), ("pending", C.c_void_p),
    ]


class StepAux(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in ("draft", "verify", "y_small", "x_large", "logits_S", "logits_L")]


class PromptDesc(C.Structure):
    _fields_ = [("samples", C.c_int32), ("T_prompt", C.c_int64),
                ("KLp", C.POINTER(C.c_void_p)), ("VLp", C.POINTER(C.c_void_p)),
                ("Khp", C.POINTER(C.c_void_p)), ("Vhp", C.POINTER(C.c_void_p)), ("n_prompt", C.c_void_p)]


class DeepStateDesc(C.Structure):
    _fields_ = [("B", C.c_int32), ("T_max", C.c_int64),
                ("KL", C.POINTER(C.c_void_p)), ("VL", C.POINTER(C.c_void_p)),
                ("KS", C.POINTER(C.c_void_p)), ("VS", C.POINTER(C.c_void_p))]


class RouterDesc(C.Structure):
    _fields_ = [("k", C.c_int32), ("d_hidden", C.c_int32), ("dtype", C.c_int32), ("tau", C.c_float),
                ("W1", C.c_void_p), ("b1", C.c_void_p), ("w2", C.c_void_p), ("b2", C.c_void_p)]


ROUTER_MAX_K = 8
STEP_FREE_TOKEN = 1
PREFILL_EMIT = 1

EXPORTS = (
    "tandem_status_string", "tandem_read_stream",
    "tandem_project_workspace", "tandem_block_attn_workspace", "tandem_draft_attn_workspace",
    "tandem_packed_weight_bytes", "tandem_pack_weight",
    "tandem_project", "tandem_block_attn", "tandem_draft_attn", "tandem_draft_attn_static",
    "tandem_block_attn_shared_workspace", "tandem_block_attn_shared",
    "tandem_draft_attn_shared_workspace", "tandem_draft_attn_shared",
    "tandem_mixed_attn_workspace", "tandem_mixed_attn",
    "tandem_block_prefix_attn_workspace", "tandem_block_prefix_attn",
    "tandem_model_create", "tandem_model_destroy", "tandem_model_packed_bytes", "tandem_model_pack",
    "tandem_decode_step_workspace", "tandem_decode_step",
    "tandem_prefill_workspace", "tandem_prefill",
    "tandem_router_eval", "tandem_decode_step_adaptive",
    "tandem_score_workspace", "tandem_score",
    "tandem_deep_score_workspace", "tandem_deep_begin", "tandem_deep_score", "tandem_deep_step",
    "tandem_decode_step_shared_workspace", "tandem_decode_step_shared",
)

_lib = None


def lib():
    """Loads libtandem.so (built in-tree by paper_2402_08644_amd.build).  No fallback."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'` first")
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    L.tandem_status_string.restype = C.c_char_p
    L.tandem_status_string.argtypes = [C.c_int]
    L.tandem_read_stream.restype = C.c_int
    L.tandem_read_stream.argtypes = [vp, sz, vp, vp]
    L.tandem_project_workspace.restype = sz
    L.tandem_project_workspace.argtypes = [C.POINTER(FFDesc), i64]
    L.tandem_decode_step_shared_workspace.restype = sz
    L.tandem_decode_step_shared_workspace.argtypes = [vp, i32, i32, i32]
    L.tandem_decode_step_shared.restype = C.c_int
    L.tandem_decode_step_shared.argtypes = [vp, C.POINTER(StateDesc), C.POINTER(PromptDesc), i32, i32, vp, vp,
                                            C.POINTER(StepAux), vp, sz, vp]
    L.tandem_score_workspace.restype = sz
    L.tandem_score_workspace.argtypes = [vp, i32, i32]
    L.tandem_score.restype = C.c_int
    L.tandem_score.argtypes = [vp, C.POINTER(StateDesc), C.POINTER(vp), C.POINTER(vp), vp, vp, i32, i32, vp, vp, vp, vp,
                               sz, vp]
    L.tandem_deep_score_workspace.restype = sz
    L.tandem_deep_score_workspace.argtypes = [vp, C.POINTER(FFDesc), i32, i32]
    L.tandem_deep_begin.restype = C.c_int
    L.tandem_deep_begin.argtypes = [vp, C.POINTER(FFDesc), C.POINTER(DeepStateDesc), vp, sz, vp]
    L.tandem_deep_step.restype = C.c_int
    L.tandem_deep_step.argtypes = [vp, C.POINTER(FFDesc), C.POINTER(DeepStateDesc), vp, i64, vp, i32, vp, vp, vp, vp, vp, sz,
                                   vp]
    L.tandem_deep_score.restype = C.c_int
    L.tandem_deep_score.argtypes = [vp, C.POINTER(FFDesc), C.POINTER(DeepStateDesc), vp, i64, vp, i32, i32, vp, vp, vp, vp,
                                    vp, sz, vp]
    L.tandem_router_eval.restype = C.c_int
    L.tandem_router_eval.argtypes = [C.POINTER(RouterDesc), vp, vp, i32, i32, i32, vp, vp]
    L.tandem_decode_step_adaptive.restype = C.c_int
    L.tandem_decode_step_adaptive.argtypes = [vp, C.POINTER(StateDesc), C.POINTER(RouterDesc), i32, i32, vp, vp, vp, vp,
                                              C.POINTER(StepAux), vp, sz, vp]
    L.tandem_block_prefix_attn_workspace.restype = sz
    L.tandem_block_prefix_attn_workspace.argtypes = [C.POINTER(AttnDesc), i32]
    L.tandem_block_prefix_attn.restype = C.c_int
    L.tandem_block_prefix_attn.argtypes = [C.POINTER(AttnDesc), vp, vp, vp, vp, i32, i32, vp, vp, sz, vp]
    L.tandem_mixed_attn_workspace.restype = sz
    L.tandem_mixed_attn_workspace.argtypes = [C.POINTER(AttnDesc), i32]
    L.tandem_mixed_attn.restype = C.c_int
    L.tandem_mixed_attn.argtypes = [C.POINTER(AttnDesc), vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, sz, vp]
    L.tandem_draft_attn_shared_workspace.restype = sz
    L.tandem_draft_attn_shared_workspace.argtypes = [C.POINTER(AttnDesc), i32, i64]
    L.tandem_draft_attn_shared.restype = C.c_int
    L.tandem_draft_attn_shared.argtypes = [C.POINTER(AttnDesc), i32, i64] + [vp] * 11 + [vp, sz, vp]
    L.tandem_block_attn_shared_workspace.restype = sz
    L.tandem_block_attn_shared_workspace.argtypes = [C.POINTER(AttnDesc), i32, i64, i32]
    L.tandem_block_attn_shared.restype = C.c_int
    L.tandem_block_attn_shared.argtypes = [C.POINTER(AttnDesc), i32, i64, vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, sz, vp]
    L.tandem_block_attn_workspace.restype = sz
    L.tandem_block_attn_workspace.argtypes = [C.POINTER(AttnDesc), i32]
    L.tandem_draft_attn_workspace.restype = sz
    L.tandem_draft_attn_workspace.argtypes = [C.POINTER(AttnDesc)]
    L.tandem_packed_weight_bytes.restype = sz
    L.tandem_packed_weight_bytes.argtypes = [i64, i64, i32]
    L.tandem_pack_weight.restype = C.c_int
    L.tandem_pack_weight.argtypes = [vp, i64, i64, i32, vp, vp]
    L.tandem_project.restype = C.c_int
    L.tandem_project.argtypes = [C.POINTER(FFDesc), vp, vp, i64, vp, sz, vp]
    L.tandem_block_attn.restype = C.c_int
    L.tandem_block_attn.argtypes = [C.POINTER(AttnDesc), vp, vp, vp, vp, i32, vp, vp, sz, vp]
    L.tandem_draft_attn.restype = C.c_int
    L.tandem_draft_attn.argtypes = [C.POINTER(AttnDesc), vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    L.tandem_draft_attn_static.restype = C.c_int
    L.tandem_draft_attn_static.argtypes = [C.POINTER(AttnDesc), vp, vp, vp, vp, vp, vp, vp, vp, vp]
    L.tandem_model_create.restype = C.c_int
    L.tandem_model_create.argtypes = [C.POINTER(ModelDesc), C.POINTER(vp)]
    L.tandem_model_destroy.restype = None
    L.tandem_model_destroy.argtypes = [vp]
    L.tandem_model_packed_bytes.restype = sz
    L.tandem_model_packed_bytes.argtypes = [vp]
    L.tandem_model_pack.restype = C.c_int
    L.tandem_model_pack.argtypes = [vp, vp, sz, vp]
    L.tandem_decode_step_workspace.restype = sz
    L.tandem_decode_step_workspace.argtypes = [vp, i32, i32]
    L.tandem_decode_step.restype = C.c_int
    L.tandem_decode_step.argtypes = [vp, C.POINTER(StateDesc), i32, i32, vp, vp, vp, C.POINTER(StepAux), vp, sz, vp]
    L.tandem_prefill_workspace.restype = sz
    L.tandem_prefill_workspace.argtypes = [vp, i32, i32]
    L.tandem_prefill.restype = C.c_int
    L.tandem_prefill.argtypes = [vp, C.POINTER(StateDesc), vp, i32, i32, vp, vp, sz, vp]
    _lib = L
    return L


def status_string(status: int) -> str:
    return lib().tandem_status_string(int(status)).decode()


def _check(rc, where):
    if rc != OK:
        raise TandemError(rc, where)


def _dtype_code(t):
    import torch

    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float32:
        return F32
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    import torch

    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _need(t, shape, what):
    if tuple(t.shape) != tuple(shape) or not t.is_contiguous() or not t.is_cuda:
        raise ValueError(f"{what}: expected contiguous device tensor of shape {tuple(shape)}, got {tuple(t.shape)}")


def _workspace(nbytes, like):
    import torch

    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=like.device)


def workspace(nbytes, device="cuda"):
    """Device scratch of at least nbytes for the *_workspace() sizes (at least 256 bytes)."""
    import torch

    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


READ_STREAM_BLOCKS = 2048


def tandem_read_stream(src, sink, stream=None):
    """Plain read-only stream over the bytes of `src` (measurement helper); sink: int32 device tensor of
    READ_STREAM_BLOCKS elements."""
    _check(lib().tandem_read_stream(_ptr(src), src.numel() * src.element_size(), _ptr(sink), _stream(stream)),
           "tandem_read_stream")


def attn_desc(B, Hq, Hkv, dh, T_max, gamma_max, scale, dtype_code):
    return AttnDesc(B, Hq, Hkv, dh, T_max, gamma_max, scale, dtype_code)


def tandem_draft_attn_workspace(desc: AttnDesc) -> int:
    return int(lib().tandem_draft_attn_workspace(C.byref(desc)))


def tandem_block_attn_workspace(desc: AttnDesc, q_len: int) -> int:
    return int(lib().tandem_block_attn_workspace(C.byref(desc), q_len))


STATIC_SCRATCH_BYTES = 1 << 20


def tandem_draft_attn_static(q, k_hat, v_hat, n_large, k_cur, v_cur, n_cur, out, scale=None, stream=None):
    """tandem_draft_attn without a workspace argument: the library's own static device scratch holds the split
    partials.  `out` is required (the call allocates nothing, this wrapper included)."""
    B, Hq, dh = q.shape
    _, Hkv, T_max, _ = k_hat.shape
    d = attn_desc(B, Hq, Hkv, dh, T_max, k_cur.shape[2], (1.0 / math.sqrt(dh)) if scale is None else scale, _dtype_code(q))
    rc = lib().tandem_draft_attn_static(C.byref(d), _ptr(q), _ptr(k_hat), _ptr(v_hat), _ptr(n_large), _ptr(k_cur),
                                        _ptr(v_cur), _ptr(n_cur), _ptr(out), _stream(stream))
    _check(rc, "tandem_draft_attn_static")
    return out


def tandem_draft_attn(q, k_hat, v_hat, n_large, k_cur, v_cur, n_cur, scale=None, out=None, ws=None, stream=None):
    """q [B,Hq,dh]; k_hat,v_hat [B,Hkv,T_max,dh]; k_cur,v_cur [B,Hkv,gamma_max,dh]; n_large,n_cur int32 [B]."""
    import torch

    B, Hq, dh = q.shape
    _, Hkv, T_max, _ = k_hat.shape
    gmax = k_cur.shape[2]
    _need(q, (B, Hq, dh), "q")
    for t, nm in ((k_hat, "k_hat"), (v_hat, "v_hat")):
        _need(t, (B, Hkv, T_max, dh), nm)
    for t, nm in ((k_cur, "k_cur"), (v_cur, "v_cur")):
        _need(t, (B, Hkv, gmax, dh), nm)
    for t, nm in ((n_large, "n_large"), (n_cur, "n_cur")):
        _need(t, (B,), nm)
        if t.dtype != torch.int32:
            raise TypeError(f"{nm} must be int32")
    for t in (k_hat, v_hat, k_cur, v_cur):
        if t.dtype != q.dtype:
            raise TypeError("q / K / V dtypes differ")
    d = attn_desc(B, Hq, Hkv, dh, T_max, gmax, (1.0 / math.sqrt(dh)) if scale is None else scale, _dtype_code(q))
    if out is None:
        out = torch.empty_like(q)
    need = tandem_draft_attn_workspace(d)
    if ws is None:
        ws = _workspace(need, q)
    rc = lib().tandem_draft_attn(C.byref(d), _ptr(q), _ptr(k_hat), _ptr(v_hat), _ptr(n_large), _ptr(k_cur), _ptr(v_cur),
                                 _ptr(n_cur), _ptr(out), _ptr(ws), ws.numel(), _stream(stream))
    _check(rc, "tandem_draft_attn")
    return out


def tandem_block_attn(q, k_cache, v_cache, n_prefix, scale=None, out=None, ws=None, stream=None):
    """q [B,q_len,Hq,dh]; k_cache,v_cache [B,Hkv,T_max,dh]; n_prefix int32 [B]."""
    import torch

    B, q_len, Hq, dh = q.shape
    _, Hkv, T_max, _ = k_cache.shape
    _need(q, (B, q_len, Hq, dh), "q")
    _need(k_cache, (B, Hkv, T_max, dh), "k_cache")
    _need(v_cache, (B, Hkv, T_max, dh), "v_cache")
    _need(n_prefix, (B,), "n_prefix")
    if n_prefix.dtype != torch.int32:
        raise TypeError("n_prefix must be int32")
    if k_cache.dtype != q.dtype or v_cache.dtype != q.dtype:
        raise TypeError("q / K / V dtypes differ")
    d = attn_desc(B, Hq, Hkv, dh, T_max, 0, (1.0 / math.sqrt(dh)) if scale is None else scale, _dtype_code(q))
    if out is None:
        out = torch.empty_like(q)
    need = tandem_block_attn_workspace(d, q_len)
    if ws is None:
        ws = _workspace(need, q)
    rc = lib().tandem_block_attn(C.byref(d), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(n_prefix), q_len, _ptr(out),
                                 _ptr(ws), ws.numel(), _stream(stream))
    _check(rc, "tandem_block_attn")
    return out


def tandem_draft_attn_shared(q, k_hat_shared, v_hat_shared, n_shared, k_hat_own, v_hat_own, n_own, k_cur, v_cur, n_cur,
                             scale=None, out=None, ws=None, stream=None):
    """q [B,samples,Hq,dh]; k_hat_shared,v_hat_shared [B,Hkv,T_max,dh], n_shared int32 [B]; k_hat_own,v_hat_own
    [B*samples,Hkv,T_own,dh], n_own int32 [B*samples]; k_cur,v_cur [B*samples,Hkv,gamma_max,dh], n_cur int32 [B*samples]."""
    import torch

    B, ns, Hq, dh = q.shape
    _, Hkv, T_max, _ = k_hat_shared.shape
    T_own, gmax = k_hat_own.shape[2], k_cur.shape[2]
    _need(q, (B, ns, Hq, dh), "q")
    for t, nm in ((k_hat_shared, "k_hat_shared"), (v_hat_shared, "v_hat_shared")):
        _need(t, (B, Hkv, T_max, dh), nm)
    for t, nm in ((k_hat_own, "k_hat_own"), (v_hat_own, "v_hat_own")):
        _need(t, (B * ns, Hkv, T_own, dh), nm)
    for t, nm in ((k_cur, "k_cur"), (v_cur, "v_cur")):
        _need(t, (B * ns, Hkv, gmax, dh), nm)
    _need(n_shared, (B,), "n_shared")
    for t, nm in ((n_own, "n_own"), (n_cur, "n_cur")):
        _need(t, (B * ns,), nm)
    for t, nm in ((n_shared, "n_shared"), (n_own, "n_own"), (n_cur, "n_cur")):
        if t.dtype != torch.int32:
            raise TypeError(f"{nm} must be int32")
    for t in (k_hat_shared, v_hat_shared, k_hat_own, v_hat_own, k_cur, v_cur):
        if t.dtype != q.dtype:
            raise TypeError("q / K / V dtypes differ")
    d = attn_desc(B, Hq, Hkv, dh, T_max, gmax, (1.0 / math.sqrt(dh)) if scale is None else scale, _dtype_code(q))
    if out is None:
        out = torch.empty_like(q)
    if ws is None:
        ws = _workspace(int(lib().tandem_draft_attn_shared_workspace(C.byref(d), ns, T_own)), q)
    rc = lib().tandem_draft_attn_shared(C.byref(d), ns, T_own, _ptr(q), _ptr(k_hat_shared), _ptr(v_hat_shared),
                                        _ptr(n_shared), _ptr(k_hat_own), _ptr(v_hat_own), _ptr(n_own), _ptr(k_cur),
                                        _ptr(v_cur), _ptr(n_cur), _ptr(out), _ptr(ws), ws.numel(), _stream(stream))
    _check(rc, "tandem_draft_attn_shared")
    return out


def tandem_block_attn_shared_workspace(desc: AttnDesc, samples: int, T_own: int, q_len: int) -> int:
    return int(lib().tandem_block_attn_shared_workspace(C.byref(desc), samples, T_own, q_len))


def tandem_block_attn_shared(q, k_shared, v_shared, n_shared, k_own, v_own, n_own, scale=None, out=None, ws=None,
                             stream=None):
    """q [B,samples,q_len,Hq,dh]; k_shared,v_shared [B,Hkv,T_max,dh], n_shared int32 [B]; k_own,v_own
    [B*samples,Hkv,T_own,dh], n_own int32 [B*samples]."""
    import torch

    B, ns, q_len, Hq, dh = q.shape
    _, Hkv, T_max, _ = k_shared.shape
    T_own = k_own.shape[2]
    _need(q, (B, ns, q_len, Hq, dh), "q")
    for t, nm in ((k_shared, "k_shared"), (v_shared, "v_shared")):
        _need(t, (B, Hkv, T_max, dh), nm)
    for t, nm in ((k_own, "k_own"), (v_own, "v_own")):
        _need(t, (B * ns, Hkv, T_own, dh), nm)
    _need(n_shared, (B,), "n_shared")
    _need(n_own, (B * ns,), "n_own")
    for t, nm in ((n_shared, "n_shared"), (n_own, "n_own")):
        if t.dtype != torch.int32:
            raise TypeError(f"{nm} must be int32")
    for t in (k_shared, v_shared, k_own, v_own):
        if t.dtype != q.dtype:
            raise TypeError("q / K / V dtypes differ")
    d = attn_desc(B, Hq, Hkv, dh, T_max, 0, (1.0 / math.sqrt(dh)) if scale is None else scale, _dtype_code(q))
    if out is None:
        out = torch.empty_like(q)
    need = tandem_block_attn_shared_workspace(d, ns, T_own, q_len)
    if ws is None:
        ws = _workspace(max(need, 256), q)
    rc = lib().tandem_block_attn_shared(C.byref(d), ns, T_own, _ptr(q), _ptr(k_shared), _ptr(v_shared), _ptr(n_shared),
                                        _ptr(k_own), _ptr(v_own), _ptr(n_own), q_len, _ptr(out), _ptr(ws), ws.numel(),
                                        _stream(stream))
    _check(rc, "tandem_block_attn_shared")
    return out


def tandem_block_prefix_attn(q, k_cache, v_cache, n_prefix, gamma, scale=None, out=None, ws=None, stream=None):
    """Deep Tandem's large-model attention: q [B,q_len,Hq,dh]; k_cache,v_cache [B,Hkv,T_max,dh]; n_prefix int32 [B]."""
    import torch

    B, q_len, Hq, dh = q.shape
    _, Hkv, T_max, _ = k_cache.shape
    _need(q, (B, q_len, Hq, dh), "q")
    _need(k_cache, (B, Hkv, T_max, dh), "k_cache")
    _need(v_cache, (B, Hkv, T_max, dh), "v_cache")
    _need(n_prefix, (B,), "n_prefix")
    if n_prefix.dtype != torch.int32:
        raise TypeError("n_prefix must be int32")
    if k_cache.dtype != q.dtype or v_cache.dtype != q.dtype:
        raise TypeError("q / K / V dtypes differ")
    d = attn_desc(B, Hq, Hkv, dh, T_max, 0, (1.0 / math.sqrt(dh)) if scale is None else scale, _dtype_code(q))
    if out is None:
        out = torch.empty_like(q)
    if ws is None:
        ws = _workspace(int(lib().tandem_block_prefix_attn_workspace(C.byref(d), q_len)), q)
    rc = lib().tandem_block_prefix_attn(C.byref(d), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(n_prefix), q_len,
                                        int(gamma), _ptr(out), _ptr(ws), ws.numel(), _stream(stream))
    _check(rc, "tandem_block_prefix_attn")
    return out


def tandem_mixed_attn_workspace(desc: AttnDesc, q_len: int) -> int:
    return int(lib().tandem_mixed_attn_workspace(C.byref(desc), q_len))


def tandem_mixed_attn(q, k_hat, v_hat, k_own, v_own, n_prefix, gamma, scale=None, out=None, ws=None, stream=None):
    """q [B,q_len,Hq,dh]; k_hat,v_hat,k_own,v_own [B,Hkv,T_max,dh] indexed by position; n_prefix int32 [B]."""
    import torch

    B, q_len, Hq, dh = q.shape
    _, Hkv, T_max, _ = k_hat.shape
    _need(q, (B, q_len, Hq, dh), "q")
    for t, nm in ((k_hat, "k_hat"), (v_hat, "v_hat"), (k_own, "k_own"), (v_own, "v_own")):
        _need(t, (B, Hkv, T_max, dh), nm)
        if t.dtype != q.dtype:
            raise TypeError("q / K / V dtypes differ")
    _need(n_prefix, (B,), "n_prefix")
    if n_prefix.dtype != torch.int32:
        raise TypeError("n_prefix must be int32")
    d = attn_desc(B, Hq, Hkv, dh, T_max, 0, (1.0 / math.sqrt(dh)) if scale is None else scale, _dtype_code(q))
    if out is None:
        out = torch.empty_like(q)
    need = tandem_mixed_attn_workspace(d, q_len)
    if ws is None:
        ws = _workspace(need, q)
    rc = lib().tandem_mixed_attn(C.byref(d), _ptr(q), _ptr(k_hat), _ptr(v_hat), _ptr(k_own), _ptr(v_own),
                                 _ptr(n_prefix), q_len, int(gamma), _ptr(out), _ptr(ws), ws.numel(), _stream(stream))
    _check(rc, "tandem_mixed_attn")
    return out


def ff_desc(ff: dict, dtype_code=None) -> FFDesc:
    """ff: {"W","b"} (linear) or {"W1","b1","W2","b2","act"} of device tensors, weights [out, in]; optional
    "Wp" / "W1p","W2p": the same weights packed by tandem_pack_weight."""
    opt = lambda k: ff[k].data_ptr() if ff.get(k) is not None else None
    if "W" in ff:
        W = ff["W"]
        return FFDesc(W.shape[1], 0, W.shape[0], ACT_NONE, _dtype_code(W), W.data_ptr(), opt("b"), None, None,
                      opt("Wp"), None)
    W1, W2 = ff["W1"], ff["W2"]
    return FFDesc(W1.shape[1], W1.shape[0], W2.shape[0], _ACT[ff.get("act", "gelu")], _dtype_code(W1), W1.data_ptr(),
                  opt("b1"), W2.data_ptr(), opt("b2"), opt("W1p"), opt("W2p"))


def tandem_packed_weight_bytes(N: int, K: int, dtype_code: int) -> int:
    return int(lib().tandem_packed_weight_bytes(N, K, dtype_code))


def tandem_pack_weight(W, stream=None):
    """W [N, K] device tensor -> its packed copy (a tensor of the same shape and dtype holding the tile layout),
    or None when the shape or dtype has no packed form."""
    import torch

    N, K = W.shape
    if not W.is_contiguous():
        raise ValueError("W must be contiguous")
    if tandem_packed_weight_bytes(N, K, _dtype_code(W)) == 0:
        return None
    Wp = torch.empty_like(W)
    _check(lib().tandem_pack_weight(_ptr(W), N, K, _dtype_code(W), _ptr(Wp), _stream(stream)), "tandem_pack_weight")
    return Wp


def tandem_project_workspace(desc: FFDesc, M: int) -> int:
    return int(lib().tandem_project_workspace(C.byref(desc), M))


def tandem_project(ff: dict, x, out=None, ws=None, stream=None):
    """x [M, d_L] -> y_hat [M, d_S]."""
    import torch

    d = ff_desc(ff)
    M = x.shape[0]
    _need(x, (M, d.d_L), "x")
    if _dtype_code(x) != d.dtype:
        raise TypeError("x dtype differs from the weights'")
    if out is None:
        out = torch.empty((M, d.d_S), dtype=x.dtype, device=x.device)
    need = tandem_project_workspace(d, M)
    if ws is None:
        ws = _workspace(need, x)
    rc = lib().tandem_project(C.byref(d), _ptr(x), _ptr(out), M, _ptr(ws), ws.numel(), _stream(stream))
    _check(rc, "tandem_project")
    return out


# ------------------------------------------------------------------ decode step
def _dev(t):
    """HostTensor (paper_2402_08644_amd.inputs) or torch tensor -> device torch tensor."""
    return t.to_torch() if hasattr(t, "to_torch") else t


class TandemModel:
    """Owns the device copies of a Tandem pair's weights and the opaque tandem_model handle.

    `weights` has the layout produced by inputs.tandem_weights: {"L": decoder, "S": decoder,
    "ell": [...], "ff": [...], "eps": float} with per-layer Wq / Wk / Wv stored separately; they are
    stacked here into the Wqkv operand the C ABI takes.  pack_weights: also hold a buffer with the packed copies of
    the weight matrices (tandem_model_pack: faster decode-time products, as much device memory again as those
    matrices; packed on the current stream)."""

    def __init__(self, weights, pack_weights=True):
        import torch

        self._keep = []
        self.eps = float(weights["eps"])
        self.ell = [int(v) for v in weights["ell"]]

        def hold(t):
            t = _dev(t).contiguous()
            self._keep.append(t)
            return t

        def decoder(M):
            layers = (LayerWeights * len(M["layers"]))()
            for i, lay in enumerate(M["layers"]):
                wqkv = hold(torch.cat([_dev(lay["Wq"]), _dev(lay["Wk"]), _dev(lay["Wv"])], dim=0))
                vals = dict(g_attn=hold(lay["g_attn"]), Wqkv=wqkv, Wo=hold(lay["Wo"]), g_mlp=hold(lay["g_mlp"]),
                            W1=hold(lay["W1"]), b1=hold(lay["b1"]) if lay.get("b1") is not None else None,
                            W2=hold(lay["W2"]), b2=hold(lay["b2"]) if lay.get("b2") is not None else None)
                for k, v in vals.items():
                    setattr(layers[i], k, None if v is None else v.data_ptr())
            self._keep.append(layers)
            emb, gf, wo = hold(M["emb"]), hold(M["g_final"]), hold(M["W_out"])
            d = DecoderDesc(len(M["layers"]), emb.shape[1], M["Hq"], M["Hkv"], M["dh"], M["layers"][0]["W1"].shape[0],
                            emb.shape[0], emb.data_ptr(), gf.data_ptr(), wo.data_ptr(), layers)
            return d, emb

        L, embL = decoder(weights["L"])
        S, embS = decoder(weights["S"])
        self.dtype = embL.dtype
        self.dtype_code = _dtype_code(embL)
        self.L, self.S = L, S
        ffs = (FFDesc * len(weights["ff"]))()
        for j, ff in enumerate(weights["ff"]):
            held = {k: (hold(v) if hasattr(v, "shape") else v) for k, v in ff.items()}
            ffs[j] = ff_desc(held)
        ell = (C.c_int32 * len(self.ell))(*self.ell)
        self._keep += [ffs, ell]
        desc = ModelDesc(L, S, ell, ffs, self.eps, self.dtype_code, 0)
        handle = C.c_void_p()
        _check(lib().tandem_model_create(C.byref(desc), C.byref(handle)), "tandem_model_create")
        self.handle = handle
        self.packed = None
        if pack_weights:
            need = int(lib().tandem_model_packed_bytes(handle))
            if need > 0:
                self.packed = torch.empty(need, dtype=torch.uint8, device=embL.device)
                _check(lib().tandem_model_pack(handle, _ptr(self.packed), need, _stream(None)), "tandem_model_pack")

    def __del__(self):
        h = getattr(self, "handle", None)
        if h:
            lib().tandem_model_destroy(h)
            self.handle = None


def kv_pair_out_of_phase(mk, shape, dtype, device):
    """K and V caches [B, Hkv, T_max, dh] of one layer for the block-mode attention, placed so that V's rows start
    1 MB out of phase with K's when a (sequence, head) region is a multiple of 2 MB.  A workgroup of the block
    attention streams the K and the V region of one (sequence, head) side by side; with both on the same 2 MB phase
    the launch measured 2.5 % slower (182.8 against 178.0 us at B=32, 8 KV heads, 8192 rows of 128) - the two streams
    press on the same part of the memory system at every instant.  Other shapes get two ordinary tensors."""
    import torch

    B, H, T, dh = shape
    es = torch.empty((), dtype=dtype).element_size()
    region, nbytes = T * dh * es, B * H * T * dh * es
    if region % (2 << 20) != 0 or not str(device).startswith("cuda"):
        return mk(*shape), mk(*shape)
    buf = torch.empty(2 * nbytes + (3 << 20), dtype=torch.uint8, device=device)
    pad = (-buf.data_ptr()) % (2 << 20)
    K = buf[pad: pad + nbytes].view(dtype).view(*shape)
    V = buf[pad + nbytes + (1 << 20): pad + 2 * nbytes + (1 << 20)].view(dtype).view(*shape)
    K.copy_(mk(*shape))
    V.copy_(mk(*shape))
    return K, V


class TandemState:
    """Caller-owned caches and per-sequence state of tandem_decode_step, as torch tensors."""

    def __init__(self, model: TandemModel, B, T_max, gamma_max, device="cuda", fill=None):
        import torch

        self.B, self.T_max, self.gamma_max = B, T_max, gamma_max
        L, S = model.L, model.S
        mk = (lambda *s: torch.zeros(s, dtype=model.dtype, device=device)) if fill is None else fill
        pairs = [kv_pair_out_of_phase(mk, (B, L.Hkv, T_max, L.dh), model.dtype, device) for _ in range(L.n_layers)]
        self.KL, self.VL = [p[0] for p in pairs], [p[1] for p in pairs]
        self.Khat = [mk(B, S.Hkv, T_max, S.dh) for _ in range(S.n_layers)]
        self.Vhat = [mk(B, S.Hkv, T_max, S.dh) for _ in range(S.n_layers)]
        self.Kcur = [torch.zeros((B, S.Hkv, gamma_max, S.dh), dtype=model.dtype, device=device) for _ in range(S.n_layers)]
        self.Vcur = [torch.zeros((B, S.Hkv, gamma_max, S.dh), dtype=model.dtype, device=device) for _ in range(S.n_layers)]
        self.n = torch.zeros(B, dtype=torch.int32, device=device)
        self.pending = torch.zeros(B, dtype=torch.int32, device=device)
        self._arrays = {}
        self.desc = self._make_desc()

    def _make_desc(self):
        def arr(name):
            ts = getattr(self, name)
            a = (C.c_void_p * len(ts))(*[t.data_ptr() for t in ts])
            self._arrays[name] = a
            return a

        return StateDesc(self.B, self.T_max, self.gamma_max, arr("KL"), arr("VL"), arr("Khat"), arr("Vhat"), arr("Kcur"),
                         arr("Vcur"), self.n.data_ptr(), self.pending.data_ptr())


class TandemPrompt:
    """The prompts of a step with several samples per prompt: the caches and lengths of a TandemState that
    tandem_prefill filled for `prompts` sequences, read by every sample of a prompt."""

    def __init__(self, prompt_state: TandemState, samples: int):
        self.state, self.samples = prompt_state, samples
        self._arrays = [(C.c_void_p * len(ts))(*[t.data_ptr() for t in ts])
                        for ts in (prompt_state.KL, prompt_state.VL, prompt_state.Khat, prompt_state.Vhat)]
        self.desc = PromptDesc(samples, prompt_state.T_max, *self._arrays, prompt_state.n.data_ptr())


def tandem_decode_step_shared_workspace(model: TandemModel, B: int, samples: int, gamma: int) -> int:
    return int(lib().tandem_decode_step_shared_workspace(model.handle, B, samples, gamma))


def tandem_decode_step_workspace(model: TandemModel, B: int, gamma: int) -> int:
    return int(lib().tandem_decode_step_workspace(model.handle, B, gamma))


def router_desc(router: dict, tau: float = 0.8) -> RouterDesc:
    """router: {"k", "W1" [H, 1+k+k*d], "w2" [H], optional "b1" [H], "b2" [1]} of device tensors of one dtype."""
    W1 = router["W1"]
    opt = lambda k: router[k].data_ptr() if router.get(k) is not None else None
    for k in ("W1", "b1", "w2", "b2"):
        t = router.get(k)
        if t is not None and (not t.is_cuda or not t.is_contiguous() or t.dtype != W1.dtype):
            raise ValueError(f"router {k}: expected a contiguous device tensor of the dtype of W1")
    if router["w2"].numel() != W1.shape[0] or (router.get("b1") is not None and router["b1"].numel() != W1.shape[0]):
        raise ValueError("router: b1 / w2 do not match the rows of W1")
    return RouterDesc(int(router["k"]), W1.shape[0], _dtype_code(W1), float(tau), W1.data_ptr(), opt("b1"),
                      router["w2"].data_ptr(), opt("b2"))


def tandem_router_eval(router: dict, logits, emb, out=None, stream=None):
    """The router's probability for every logits row: logits [rows, vocab], emb [vocab, d] -> fp32 [rows]."""
    import torch

    rows, vocab = logits.shape
    d = emb.shape[1]
    _need(logits, (rows, vocab), "logits")
    _need(emb, (vocab, d), "emb")
    rd = router_desc(router)
    if router["W1"].shape[1] != 1 + rd.k * (d + 1):
        raise ValueError("router W1: expected 1 + k + k*d columns")
    if logits.dtype != router["W1"].dtype or emb.dtype != router["W1"].dtype:
        raise TypeError("logits / emb / router dtypes differ")
    if out is None:
        out = torch.empty((rows,), dtype=torch.float32, device=logits.device)
    rc = lib().tandem_router_eval(C.byref(rd), _ptr(logits), _ptr(emb), rows, vocab, d, _ptr(out), _stream(stream))
    _check(rc, "tandem_router_eval")
    return out


def tandem_decode_step(model: TandemModel, state: TandemState, gamma: int, forced=None, aux=False, ws=None, out=None,
                       stream=None, free_token=False, router=None, tau=0.8, prompt=None):
    """Runs one step.  q = gamma, or gamma + 1 with free_token (M_L also verifies the last draft and always
    emits its own token after the accepted prefix).  Returns a dict with "tokens" [B,q] and "n_accepted" [B]
    (int32 device tensors) and, with aux=True, "draft" [B,gamma], "verify" [B,q], "y_small", "x_large",
    "logits_S", "logits_L".  With router (see router_desc) the block length adapts per sequence up to gamma:
    the dict then also holds "n_drafted" [B] (int32) and "router_p" [B,gamma] (fp32).  With prompt (a TandemPrompt)
    the state's sequences are samples of its prompts and the state's caches hold only their rows after the prompt."""
    import torch

    B = state.B
    dev = state.n.device
    q = gamma + 1 if free_token else gamma
    if out is None:
        out = {"tokens": torch.empty((B, q), dtype=torch.int32, device=dev),
               "n_accepted": torch.empty((B,), dtype=torch.int32, device=dev)}
        if aux:
            out.update(
                draft=torch.empty((B, gamma), dtype=torch.int32, device=dev),
                verify=torch.empty((B, q), dtype=torch.int32, device=dev),
                y_small=torch.empty((B, gamma, model.S.d), dtype=model.dtype, device=dev),
                x_large=torch.empty((B, q, model.L.d), dtype=model.dtype, device=dev),
                logits_S=torch.empty((B, gamma, model.S.vocab), dtype=model.dtype, device=dev),
                logits_L=torch.empty((B, q, model.L.vocab), dtype=model.dtype, device=dev),
            )
    _need(out["tokens"], (B, q), "out tokens")
    a = None
    if "draft" in out:
        a = StepAux(*[out[k].data_ptr() for k in ("draft", "verify", "y_small", "x_large", "logits_S", "logits_L")])
    if forced is not None:
        _need(forced, (B, gamma), "forced")
        if forced.dtype != torch.int32:
            raise TypeError("forced must be int32")
    if prompt is not None:
        if forced is not None or router is not None:
            raise ValueError("the shared-prompt step takes neither forced tokens nor a router")
        if ws is None:
            ws = _workspace(tandem_decode_step_shared_workspace(model, B, prompt.samples, gamma), state.n)
        rc = lib().tandem_decode_step_shared(model.handle, C.byref(state.desc), C.byref(prompt.desc), gamma,
                                             STEP_FREE_TOKEN if free_token else 0, _ptr(out["tokens"]),
                                             _ptr(out["n_accepted"]), C.byref(a) if a is not None else None, _ptr(ws),
                                             ws.numel(), _stream(stream))
        _check(rc, "tandem_decode_step_shared")
        return out
    if ws is None:
        ws = _workspace(tandem_decode_step_workspace(model, B, gamma), state.n)
    if router is not None:
        if forced is not None:
            raise ValueError("forced tokens and the adaptive block length exclude each other")
        rd = router_desc(router, tau)
        if router["W1"].shape[1] != 1 + rd.k * (model.S.d + 1):
            raise ValueError("router W1: expected 1 + k + k*d columns")
        out.setdefault("n_drafted", torch.empty((B,), dtype=torch.int32, device=dev))
        out.setdefault("router_p", torch.empty((B, gamma), dtype=torch.float32, device=dev))
        rc = lib().tandem_decode_step_adaptive(model.handle, C.byref(state.desc), C.byref(rd), gamma,
                                               STEP_FREE_TOKEN if free_token else 0, _ptr(out["tokens"]),
                                               _ptr(out["n_accepted"]), _ptr(out["n_drafted"]), _ptr(out["router_p"]),
                                               C.byref(a) if a is not None else None, _ptr(ws), ws.numel(),
                                               _stream(stream))
        _check(rc, "tandem_decode_step_adaptive")
        return out
    rc = lib().tandem_decode_step(model.handle, C.byref(state.desc), gamma, STEP_FREE_TOKEN if free_token else 0,
                                  _ptr(forced), _ptr(out["tokens"]),
                                  _ptr(out["n_accepted"]), C.byref(a) if a is not None else None, _ptr(ws), ws.numel(),
                                  _stream(stream))
    _check(rc, "tandem_decode_step")
    return out


def tandem_score_workspace(model: TandemModel, B: int, q_len: int) -> int:
    return int(lib().tandem_score_workspace(model.handle, B, q_len))


def own_caches(model: TandemModel, state: TandemState):
    """Zeroed position-indexed caches for the small model's own K/V rows (tandem_score): two lists over its layers."""
    import torch

    S = model.S
    mk = lambda: [torch.zeros((state.B, S.Hkv, state.T_max, S.dh), dtype=model.dtype, device=state.n.device)
                  for _ in range(S.n_layers)]
    return mk(), mk()


def tandem_score(model: TandemModel, state: TandemState, k_own, v_own, pos, tokens, gamma, logits=False, y_small=False,
                 ws=None, stream=None):
    """Teacher-forced small-model pass over tokens [B, q_len] (int32) at positions pos[b].. (int32 [B]); k_own, v_own
    from own_caches().  Returns {"greedy" [B,q_len] int32, optionally "logits" [B,q_len,vocab], "y_small" [B,q_len,d]}."""
    import torch

    B, q_len = tokens.shape
    _need(tokens, (state.B, q_len), "tokens")
    _need(pos, (state.B,), "pos")
    if tokens.dtype != torch.int32 or pos.dtype != torch.int32:
        raise TypeError("tokens and pos must be int32")
    S = model.S
    for ts, nm in ((k_own, "k_own"), (v_own, "v_own")):
        if len(ts) != S.n_layers:
            raise ValueError(f"{nm}: one tensor per small layer")
        for t in ts:
            _need(t, (B, S.Hkv, state.T_max, S.dh), nm)
            if t.dtype != model.dtype:
                raise TypeError(f"{nm}: model dtype expected")
    dev = state.n.device
    out = {"greedy": torch.empty((B, q_len), dtype=torch.int32, device=dev)}
    if logits:
        out["logits"] = torch.empty((B, q_len, S.vocab), dtype=model.dtype, device=dev)
    if y_small:
        out["y_small"] = torch.empty((B, q_len, S.d), dtype=model.dtype, device=dev)
    if ws is None:
        ws = _workspace(tandem_score_workspace(model, B, q_len), state.n)
    ka = (C.c_void_p * S.n_layers)(*[t.data_ptr() for t in k_own])
    va = (C.c_void_p * S.n_layers)(*[t.data_ptr() for t in v_own])
    rc = lib().tandem_score(model.handle, C.byref(state.desc), ka, va, _ptr(pos), _ptr(tokens), q_len, int(gamma),
                            _ptr(out["greedy"]), _ptr(out.get("logits")), _ptr(out.get("y_small")), _ptr(ws), ws.numel(),
                            _stream(stream))
    _check(rc, "tandem_score")
    return out


class DeepState:
    """Caller-owned caches of the Deep Tandem pass (Sec. 5): M_L's K/V rows and M_S's own K/V rows, by position."""

    def __init__(self, model: TandemModel, B, T_max, device="cuda"):
        import torch

        self.B, self.T_max = B, T_max
        L, S = model.L, model.S
        mk = lambda D: [torch.zeros((B, D.Hkv, T_max, D.dh), dtype=model.dtype, device=device) for _ in range(D.n_layers)]
        zeros = lambda *s: torch.zeros(s, dtype=model.dtype, device=device)
        pairs = [kv_pair_out_of_phase(zeros, (B, L.Hkv, T_max, L.dh), model.dtype, device) for _ in range(L.n_layers)]
        self.KL, self.VL, self.KS, self.VS = [p[0] for p in pairs], [p[1] for p in pairs], mk(S), mk(S)
        self._arrays = [(C.c_void_p * len(ts))(*[t.data_ptr() for t in ts]) for ts in (self.KL, self.VL, self.KS, self.VS)]
        self.desc = DeepStateDesc(B, T_max, *self._arrays)


def tandem_deep_begin(model: TandemModel, ff_deep: dict, state: DeepState, ws=None, stream=None):
    """M_L's row 0 of every sequence (before the first tandem_deep_score)."""
    d = ff_desc(ff_deep)
    if ws is None:
        ws = _workspace(int(lib().tandem_deep_score_workspace(model.handle, C.byref(d), state.B, 1)), state.KL[0])
    _check(lib().tandem_deep_begin(model.handle, C.byref(d), C.byref(state.desc), _ptr(ws), ws.numel(), _stream(stream)),
           "tandem_deep_begin")


def tandem_deep_score(model: TandemModel, ff_deep: dict, state: DeepState, tokens, pos, q_len, gamma, logits=False,
                      y_small=False, sketch=False, ws=None, stream=None):
    """One chunk of the teacher-forced Deep Tandem pass: tokens int32 [B, n_tokens] (all known tokens), pos int32 [B].
    Returns {"greedy" [B,q_len], optionally "logits", "y_small", "sketch"}."""
    import torch

    B, n_tokens = tokens.shape
    _need(tokens, (state.B, n_tokens), "tokens")
    _need(pos, (state.B,), "pos")
    if tokens.dtype != torch.int32 or pos.dtype != torch.int32:
        raise TypeError("tokens and pos must be int32")
    d = ff_desc(ff_deep)
    dev = tokens.device
    out = {"greedy": torch.empty((B, q_len), dtype=torch.int32, device=dev)}
    if logits:
        out["logits"] = torch.empty((B, q_len, model.S.vocab), dtype=model.dtype, device=dev)
    if y_small:
        out["y_small"] = torch.empty((B, q_len, model.S.d), dtype=model.dtype, device=dev)
    if sketch:
        out["sketch"] = torch.empty((B, q_len, model.L.d), dtype=model.dtype, device=dev)
    if ws is None:
        ws = _workspace(int(lib().tandem_deep_score_workspace(model.handle, C.byref(d), B, q_len)), tokens)
    rc = lib().tandem_deep_score(model.handle, C.byref(d), C.byref(state.desc), _ptr(tokens), n_tokens, _ptr(pos), q_len,
                                 int(gamma), _ptr(out["greedy"]), _ptr(out.get("logits")), _ptr(out.get("y_small")),
                                 _ptr(out.get("sketch")), _ptr(ws), ws.numel(), _stream(stream))
    _check(rc, "tandem_deep_score")
    return out


def tandem_deep_step(model: TandemModel, ff_deep: dict, state: DeepState, tokens, length, gamma, logits=False,
                     y_small=False, sketch=False, ws=None, stream=None):
    """One Deep Tandem decoding step: tokens int32 [B, n_tokens] (updated in place), length int32 [B] (advanced by gamma).
    Returns {"tokens" [B, gamma], optionally "logits", "y_small", "sketch"}."""
    import torch

    B, n_tokens = tokens.shape
    _need(tokens, (state.B, n_tokens), "tokens")
    _need(length, (state.B,), "length")
    if tokens.dtype != torch.int32 or length.dtype != torch.int32:
        raise TypeError("tokens and length must be int32")
    d = ff_desc(ff_deep)
    dev = tokens.device
    out = {"tokens": torch.empty((B, gamma), dtype=torch.int32, device=dev)}
    if logits:
        out["logits"] = torch.empty((B, gamma, model.S.vocab), dtype=model.dtype, device=dev)
    if y_small:
        out["y_small"] = torch.empty((B, gamma, model.S.d), dtype=model.dtype, device=dev)
    if sketch:
        out["sketch"] = torch.empty((B, gamma, model.L.d), dtype=model.dtype, device=dev)
    if ws is None:
        ws = _workspace(int(lib().tandem_deep_score_workspace(model.handle, C.byref(d), B, gamma)), tokens)
    rc = lib().tandem_deep_step(model.handle, C.byref(d), C.byref(state.desc), _ptr(tokens), n_tokens, _ptr(length),
                                int(gamma), _ptr(out["tokens"]), _ptr(out.get("logits")), _ptr(out.get("y_small")),
                                _ptr(out.get("sketch")), _ptr(ws), ws.numel(), _stream(stream))
    _check(rc, "tandem_deep_step")
    return out


def tandem_prefill_workspace(model: TandemModel, B: int, q_len: int) -> int:
    return int(lib().tandem_prefill_workspace(model.handle, B, q_len))


def tandem_prefill(model: TandemModel, state: TandemState, tokens, emit=False, x_large=None, ws=None, stream=None):
    """Ingests tokens [B, q_len] (int32 device tensor, q_len <= 128) for every sequence: M_L's block pass plus the
    Khat / Vhat rows; n += q_len; with emit, pending = M_L's greedy token after the last row."""
    import torch

    B, q_len = tokens.shape
    _need(tokens, (state.B, q_len), "tokens")
    if tokens.dtype != torch.int32:
        raise TypeError("tokens must be int32")
    if ws is None:
        ws = _workspace(tandem_prefill_workspace(model, B, q_len), state.n)
    rc = lib().tandem_prefill(model.handle, C.byref(state.desc), _ptr(tokens), q_len, PREFILL_EMIT if emit else 0,
                              _ptr(x_large), _ptr(ws), ws.numel(), _stream(stream))
    _check(rc, "tandem_prefill")
