"""ctypes binding of libqjl.so: argument marshalling only.

Each function has the name and meaning of the C entry point declared in
include/qjl.h; torch is used for device memory and the current stream.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

QJL_F32, QJL_F16, QJL_BF16 = 0, 1, 2
_DTYPE_TAG = {torch.float32: QJL_F32, torch.float16: QJL_F16, torch.bfloat16: QJL_BF16}

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libqjl.so")
_lib: Optional[ctypes.CDLL] = None


class QJLError(RuntimeError):
    def __init__(self, fn: str, status: int, text: str):
        super().__init__(f"{fn} failed with status {status} ({text})")
        self.status = status


class QJLShape(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("q_heads", ctypes.c_int32), ("kv_heads", ctypes.c_int32),
                ("n", ctypes.c_int32), ("d", ctypes.c_int32), ("m", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("scale", ctypes.c_float)]


def lib_path() -> str:
    return _LIB_PATH


def lib() -> ctypes.CDLL:
    """The loaded C library.  Raises if it has not been built: there is no fallback."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is missing: build it with "
                           "`python -m paper_2406_03482_amd.build` (needs hipcc)")
    L = ctypes.CDLL(_LIB_PATH)
    vp, sp = ctypes.c_void_p, ctypes.POINTER(QJLShape)
    L.qjl_version.restype = ctypes.c_int
    L.qjl_version.argtypes = []
    L.qjl_status_string.restype = ctypes.c_char_p
    L.qjl_status_string.argtypes = [ctypes.c_int]
    L.qjl_make_sketch.restype = ctypes.c_int
    L.qjl_make_sketch.argtypes = [ctypes.c_uint64, ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, vp]
    L.qjl_make_sketch_orthogonal.restype = ctypes.c_int
    L.qjl_make_sketch_orthogonal.argtypes = [ctypes.c_uint64, ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, vp]
    L.qjl_quantize_keys.restype = ctypes.c_int
    L.qjl_quantize_keys.argtypes = [sp, vp, vp, vp, vp, vp]
    L.qjl_project_query.restype = ctypes.c_int
    L.qjl_project_query.argtypes = [sp, vp, vp, vp, vp]
    L.qjl_scores.restype = ctypes.c_int
    L.qjl_scores.argtypes = [sp, vp, vp, vp, vp, vp]
    L.qjl_decode_workspace_bytes.restype = ctypes.c_size_t
    L.qjl_decode_workspace_bytes.argtypes = [sp]
    L.qjl_decode_attention.restype = ctypes.c_int
    L.qjl_decode_attention.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    L.qjl_decode_plan.restype = ctypes.c_size_t
    L.qjl_decode_plan.argtypes = [sp, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_int32)]
    L.qjl_decode_attention_splits.restype = ctypes.c_int
    L.qjl_decode_attention_splits.argtypes = [sp, ctypes.c_int, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    L.qjl_decode_noalloc_max_bytes.restype = ctypes.c_size_t
    L.qjl_decode_noalloc_max_bytes.argtypes = []
    L.qjl_decode_attention_noalloc.restype = ctypes.c_int
    L.qjl_decode_attention_noalloc.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp]
    L.qjl_decode_attention_timed.restype = ctypes.c_int
    L.qjl_decode_attention_timed.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp, vp, vp]
    ip = ctypes.c_int
    L.qjl_outlier_workspace_bytes.restype = ctypes.c_size_t
    L.qjl_outlier_workspace_bytes.argtypes = [sp]
    L.qjl_select_outliers.restype = ctypes.c_int
    L.qjl_select_outliers.argtypes = [sp, vp, ip, vp, vp, ctypes.c_size_t, vp]
    L.qjl_make_dual_sketch.restype = ctypes.c_int
    L.qjl_make_dual_sketch.argtypes = [sp, ip, vp, vp, vp, ip, vp, vp]
    L.qjl_quantize_keys_dual.restype = ctypes.c_int
    L.qjl_quantize_keys_dual.argtypes = [sp, ip, vp, vp, vp, ip, vp, vp, vp, vp]
    L.qjl_decode_dual_workspace_bytes.restype = ctypes.c_size_t
    L.qjl_decode_dual_workspace_bytes.argtypes = [sp, ip]
    L.qjl_decode_attention_dual.restype = ctypes.c_int
    L.qjl_decode_attention_dual.argtypes = [sp, ip, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp, vp, vp]
    L.qjl_quantize_values.restype = ctypes.c_int
    L.qjl_quantize_values.argtypes = [sp, ip, vp, vp, vp, vp, vp]
    L.qjl_decode_attention_vq.restype = ctypes.c_int
    L.qjl_decode_attention_vq.argtypes = [sp, ip, vp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp, vp, vp]
    L.qjl_decode_attention_dual_vq.restype = ctypes.c_int
    L.qjl_decode_attention_dual_vq.argtypes = [sp, ip, ip, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp, vp, vp]
    L.qjl_generation_step.restype = ctypes.c_int
    L.qjl_generation_step.argtypes = [sp, ip, ip, ip, vp, vp, vp, vp, vp, ip, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    L.qjl_generation_step_devpos.restype = ctypes.c_int
    L.qjl_generation_step_devpos.argtypes = [sp, ip, ip, vp, vp, vp, vp, vp, vp, ip, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    L.qjl_append_keys.restype = ctypes.c_int
    L.qjl_append_keys.argtypes = [sp, ip, ip, vp, vp, vp, vp, vp]
    L.qjl_decode_step.restype = ctypes.c_int
    L.qjl_decode_step.argtypes = [sp, ip, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    _lib = L
    return L


def _check(fn: str, status: int) -> None:
    if status != 0:
        raise QJLError(fn, status, lib().qjl_status_string(status).decode())


def _stream(t: torch.Tensor) -> int:
    return torch.cuda.current_stream(t.device).cuda_stream


def _dev(t: torch.Tensor, name: str) -> int:
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr()


def _tag(t: torch.Tensor) -> int:
    try:
        return _DTYPE_TAG[t.dtype]
    except KeyError:
        raise ValueError(f"unsupported dtype {t.dtype}") from None


def _shape(batch, q_heads, kv_heads, n, d, m, dtype_tag, scale=1.0) -> QJLShape:
    return QJLShape(batch, q_heads, kv_heads, n, d, m, dtype_tag, scale)


def qjl_make_sketch(seed: int, m: int, d: int, dtype: torch.dtype = torch.bfloat16,
                    device="cuda") -> torch.Tensor:
    """S[m,d] with i.i.d. N(0,1) entries that depend only on (seed, m, d, dtype)."""
    S = torch.empty((m, d), dtype=dtype, device=device)
    _check("qjl_make_sketch",
           lib().qjl_make_sketch(seed & (2 ** 64 - 1), m, d, _tag(S), _dev(S, "S"), _stream(S)))
    return S


def qjl_make_sketch_orthogonal(seed: int, m: int, d: int, dtype: torch.dtype = torch.bfloat16,
                               device="cuda") -> torch.Tensor:
    """The sketch of qjl_make_sketch(seed, ...) with the rows of every block of d rows orthogonalised."""
    S = torch.empty((m, d), dtype=dtype, device=device)
    _check("qjl_make_sketch_orthogonal",
           lib().qjl_make_sketch_orthogonal(seed & (2 ** 64 - 1), m, d, _tag(S), _dev(S, "S"), _stream(S)))
    return S


def qjl_quantize_keys(K: torch.Tensor, S: torch.Tensor, bits: Optional[torch.Tensor] = None,
                      norms: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """K[B,Hkv,n,d], S[m,d] -> (bits uint8 [B,Hkv,n,m/8], norms float16 [B,Hkv,n])."""
    B, Hkv, n, d = K.shape
    m = S.shape[0]
    if S.shape[1] != d or S.dtype != K.dtype:
        raise ValueError("S must be [m,d] with the dtype of K")
    if bits is None:
        bits = torch.empty((B, Hkv, n, m // 8), dtype=torch.uint8, device=K.device)
    if norms is None:
        norms = torch.empty((B, Hkv, n), dtype=torch.float16, device=K.device)
    if tuple(bits.shape) != (B, Hkv, n, m // 8) or bits.dtype != torch.uint8:
        raise ValueError("bits must be uint8 [B,Hkv,n,m/8]")
    if tuple(norms.shape) != (B, Hkv, n) or norms.dtype != torch.float16:
        raise ValueError("norms must be float16 [B,Hkv,n]")
    sh = _shape(B, Hkv, Hkv, n, d, m, _tag(K))
    _check("qjl_quantize_keys",
           lib().qjl_quantize_keys(ctypes.byref(sh), _dev(K, "K"), _dev(S, "S"), _dev(bits, "bits"),
                                   _dev(norms, "norms"), _stream(K)))
    return bits, norms


def qjl_project_query(Q: torch.Tensor, S: torch.Tensor, SQ: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Q[B,Hq,d], S[m,d] -> SQ float32 [B,Hq,m] = S q (unquantized)."""
    B, Hq, d = Q.shape
    m = S.shape[0]
    if S.shape[1] != d or S.dtype != Q.dtype:
        raise ValueError("S must be [m,d] with the dtype of Q")
    if SQ is None:
        SQ = torch.empty((B, Hq, m), dtype=torch.float32, device=Q.device)
    sh = _shape(B, Hq, 1, 1, d, m, _tag(Q))
    _check("qjl_project_query",
           lib().qjl_project_query(ctypes.byref(sh), _dev(Q, "Q"), _dev(S, "S"), _dev(SQ, "SQ"),
                                   _stream(Q)))
    return SQ


def qjl_scores(SQ: torch.Tensor, bits: torch.Tensor, norms: torch.Tensor, scale: float = 1.0,
               out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """SQ[B,Hq,m], bits[B,Hkv,n,m/8], norms[B,Hkv,n] -> float32 [B,Hq,n] (pre-softmax)."""
    B, Hq, m = SQ.shape
    _, Hkv, n, mb = bits.shape
    if mb * 8 != m or SQ.dtype != torch.float32:
        raise ValueError("SQ must be float32 [B,Hq,m] with m = 8 * bits.shape[-1]")
    if out is None:
        out = torch.empty((B, Hq, n), dtype=torch.float32, device=SQ.device)
    sh = _shape(B, Hq, Hkv, n, 128, m, QJL_F32, scale)
    _check("qjl_scores",
           lib().qjl_scores(ctypes.byref(sh), _dev(SQ, "SQ"), _dev(bits, "bits"),
                            _dev(norms, "norms"), _dev(out, "out"), _stream(SQ)))
    return out


def qjl_decode_workspace_bytes(batch: int, q_heads: int, kv_heads: int, n: int, d: int, m: int,
                               dtype: torch.dtype = torch.bfloat16) -> int:
    sh = _shape(batch, q_heads, kv_heads, n, d, m, _DTYPE_TAG[dtype])
    return int(lib().qjl_decode_workspace_bytes(ctypes.byref(sh)))


def qjl_decode_plan(batch: int, q_heads: int, kv_heads: int, n: int, d: int, m: int, m_out: int = 0,
                    splits: int = 0, dtype: torch.dtype = torch.bfloat16):
    """(workspace bytes, query heads per workgroup, chunks, keys per chunk) of the decode call's plan.  Host only."""
    sh = _shape(batch, q_heads, kv_heads, n, d, m, _DTYPE_TAG[dtype])
    out = (ctypes.c_int32 * 3)()
    total = int(lib().qjl_decode_plan(ctypes.byref(sh), m_out, splits, out))
    return total, int(out[0]), int(out[1]), int(out[2])


def qjl_decode_attention(Q: torch.Tensor, S: torch.Tensor, bits: torch.Tensor, norms: torch.Tensor,
                         V: torch.Tensor, scale: float = 1.0, out: Optional[torch.Tensor] = None,
                         workspace: Optional[torch.Tensor] = None,
                         events: Optional[Tuple[int, int]] = None, splits: int = 0) -> torch.Tensor:
    """One decode step: Q[B,Hq,d], S[m,d], bits, norms, V[B,Hkv,n,d] -> float32 [B,Hq,d].
    `events` = (hipEvent_t before, hipEvent_t after) as integers selects
    qjl_decode_attention_timed; `splits` > 0 selects qjl_decode_attention_splits."""
    B, Hq, d = Q.shape
    _, Hkv, n, _ = V.shape
    m = S.shape[0]
    if V.dtype != Q.dtype or S.dtype != Q.dtype:
        raise ValueError("Q, S and V must share one dtype")
    if tuple(bits.shape) != (B, Hkv, n, m // 8) or tuple(norms.shape) != (B, Hkv, n):
        raise ValueError("bits/norms do not match V and S")
    need = qjl_decode_plan(B, Hq, Hkv, n, d, m, 0, splits, Q.dtype)[0]
    if workspace is None:
        workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=Q.device)
    if out is None:
        out = torch.empty((B, Hq, d), dtype=torch.float32, device=Q.device)
    sh = _shape(B, Hq, Hkv, n, d, m, _tag(Q), scale)
    args = (ctypes.byref(sh), _dev(Q, "Q"), _dev(S, "S"), _dev(bits, "bits"), _dev(norms, "norms"),
            _dev(V, "V"), _dev(out, "out"), _dev(workspace, "workspace"),
            workspace.numel() * workspace.element_size(), _stream(Q))
    if splits > 0:
        _check("qjl_decode_attention_splits", lib().qjl_decode_attention_splits(args[0], splits, *args[1:]))
    elif events is None:
        _check("qjl_decode_attention", lib().qjl_decode_attention(*args))
    else:
        _check("qjl_decode_attention_timed", lib().qjl_decode_attention_timed(*args, events[0], events[1]))
    return out


def qjl_decode_attention_noalloc(Q: torch.Tensor, S: torch.Tensor, bits: torch.Tensor, norms: torch.Tensor,
                                 V: torch.Tensor, scale: float, out: torch.Tensor) -> torch.Tensor:
    """qjl_decode_attention into a caller-provided `out`, with the per-chunk records in the library's own device
    array: neither this wrapper nor the call allocates."""
    B, Hq, d = Q.shape
    _, Hkv, n, _ = V.shape
    m = S.shape[0]
    if V.dtype != Q.dtype or S.dtype != Q.dtype:
        raise ValueError("Q, S and V must share one dtype")
    if tuple(bits.shape) != (B, Hkv, n, m // 8) or tuple(norms.shape) != (B, Hkv, n):
        raise ValueError("bits/norms do not match V and S")
    if tuple(out.shape) != (B, Hq, d) or out.dtype != torch.float32:
        raise ValueError("out must be float32 [B,Hq,d]")
    sh = _shape(B, Hq, Hkv, n, d, m, _tag(Q), scale)
    _check("qjl_decode_attention_noalloc",
           lib().qjl_decode_attention_noalloc(ctypes.byref(sh), _dev(Q, "Q"), _dev(S, "S"), _dev(bits, "bits"),
                                              _dev(norms, "norms"), _dev(V, "V"), _dev(out, "out"), _stream(Q)))
    return out


# ---- outlier channels (Section 4.1): two quantizers per key
def qjl_select_outliers(K: torch.Tensor, count: int, channels: Optional[torch.Tensor] = None,
                        workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """K[B,Hkv,n,d] -> int32 [B,Hkv,count]: channels with the largest mean |k|, largest first."""
    B, Hkv, n, d = K.shape
    sh = _shape(B, Hkv, Hkv, n, d, 32, _tag(K))
    need = int(lib().qjl_outlier_workspace_bytes(ctypes.byref(sh)))
    if workspace is None:
        workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=K.device)
    if channels is None:
        channels = torch.empty((B, Hkv, count), dtype=torch.int32, device=K.device)
    if tuple(channels.shape) != (B, Hkv, count) or channels.dtype != torch.int32:
        raise ValueError("channels must be int32 [B,Hkv,count]")
    _check("qjl_select_outliers",
           lib().qjl_select_outliers(ctypes.byref(sh), _dev(K, "K"), count, _dev(channels, "channels"),
                                     _dev(workspace, "workspace"),
                                     workspace.numel() * workspace.element_size(), _stream(K)))
    return channels


def qjl_make_dual_sketch(S_in: torch.Tensor, S_out: torch.Tensor, channels: torch.Tensor,
                         S_dual: Optional[torch.Tensor] = None) -> torch.Tensor:
    """S_in[m,d], S_out[m_out,d], channels int32 [B,Hkv,count] -> S_dual[B,Hkv,m+m_out,d]."""
    m, d = S_in.shape
    m_out = S_out.shape[0]
    B, Hkv, count = channels.shape
    if S_out.shape[1] != d or S_out.dtype != S_in.dtype or channels.dtype != torch.int32:
        raise ValueError("S_out must be [m_out,d] with the dtype of S_in; channels int32")
    if S_dual is None:
        S_dual = torch.empty((B, Hkv, m + m_out, d), dtype=S_in.dtype, device=S_in.device)
    sh = _shape(B, Hkv, Hkv, 1, d, m, _tag(S_in))
    _check("qjl_make_dual_sketch",
           lib().qjl_make_dual_sketch(ctypes.byref(sh), m_out, _dev(S_in, "S_in"), _dev(S_out, "S_out"),
                                      _dev(channels, "channels"), count, _dev(S_dual, "S_dual"),
                                      _stream(S_in)))
    return S_dual


def qjl_quantize_keys_dual(K: torch.Tensor, S_dual: torch.Tensor, channels: torch.Tensor, m_out: int,
                           bits: Optional[torch.Tensor] = None, norms_in: Optional[torch.Tensor] = None,
                           norms_out: Optional[torch.Tensor] = None):
    """K[B,Hkv,n,d], S_dual[B,Hkv,m+m_out,d] -> (bits uint8 [B,Hkv,n,(m+m_out)/8], norms_in, norms_out)."""
    B, Hkv, n, d = K.shape
    mt = S_dual.shape[2]
    count = channels.shape[2]
    if tuple(S_dual.shape) != (B, Hkv, mt, d) or S_dual.dtype != K.dtype or not 0 < m_out < mt:
        raise ValueError("S_dual must be [B,Hkv,m+m_out,d] with the dtype of K")
    if tuple(channels.shape) != (B, Hkv, count) or channels.dtype != torch.int32:
        raise ValueError("channels must be int32 [B,Hkv,count]")
    if bits is None:
        bits = torch.empty((B, Hkv, n, mt // 8), dtype=torch.uint8, device=K.device)
    if norms_in is None:
        norms_in = torch.empty((B, Hkv, n), dtype=torch.float16, device=K.device)
    if norms_out is None:
        norms_out = torch.empty((B, Hkv, n), dtype=torch.float16, device=K.device)
    sh = _shape(B, Hkv, Hkv, n, d, mt - m_out, _tag(K))
    _check("qjl_quantize_keys_dual",
           lib().qjl_quantize_keys_dual(ctypes.byref(sh), m_out, _dev(K, "K"), _dev(S_dual, "S_dual"),
                                        _dev(channels, "channels"), count, _dev(bits, "bits"),
                                        _dev(norms_in, "norms_in"), _dev(norms_out, "norms_out"),
                                        _stream(K)))
    return bits, norms_in, norms_out


def qjl_decode_dual_workspace_bytes(batch: int, q_heads: int, kv_heads: int, n: int, d: int, m: int,
                                    m_out: int, dtype: torch.dtype = torch.bfloat16) -> int:
    sh = _shape(batch, q_heads, kv_heads, n, d, m, _DTYPE_TAG[dtype])
    return int(lib().qjl_decode_dual_workspace_bytes(ctypes.byref(sh), m_out))


def qjl_decode_attention_dual(Q: torch.Tensor, S_dual: torch.Tensor, bits: torch.Tensor,
                              norms_in: torch.Tensor, norms_out: torch.Tensor, V: torch.Tensor,
                              m_out: int, scale: float = 1.0, out: Optional[torch.Tensor] = None,
                              workspace: Optional[torch.Tensor] = None,
                              events: Optional[Tuple[int, int]] = None) -> torch.Tensor:
    """One decode step on a two-part cache: -> float32 [B,Hq,d].  `events` as in qjl_decode_attention."""
    B, Hq, d = Q.shape
    _, Hkv, n, _ = V.shape
    mt = S_dual.shape[2]
    m = mt - m_out
    if V.dtype != Q.dtype or S_dual.dtype != Q.dtype:
        raise ValueError("Q, S_dual and V must share one dtype")
    if tuple(S_dual.shape) != (B, Hkv, mt, d) or tuple(bits.shape) != (B, Hkv, n, mt // 8):
        raise ValueError("S_dual/bits do not match V")
    if tuple(norms_in.shape) != (B, Hkv, n) or tuple(norms_out.shape) != (B, Hkv, n):
        raise ValueError("norms do not match V")
    need = qjl_decode_dual_workspace_bytes(B, Hq, Hkv, n, d, m, m_out, Q.dtype)
    if workspace is None:
        workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=Q.device)
    if out is None:
        out = torch.empty((B, Hq, d), dtype=torch.float32, device=Q.device)
    sh = _shape(B, Hq, Hkv, n, d, m, _tag(Q), scale)
    _check("qjl_decode_attention_dual",
           lib().qjl_decode_attention_dual(ctypes.byref(sh), m_out, _dev(Q, "Q"), _dev(S_dual, "S_dual"),
                                           _dev(bits, "bits"), _dev(norms_in, "norms_in"),
                                           _dev(norms_out, "norms_out"), _dev(V, "V"), _dev(out, "out"),
                                           _dev(workspace, "workspace"),
                                           workspace.numel() * workspace.element_size(), _stream(Q),
                                           events[0] if events else None, events[1] if events else None))
    return out


# ---- value cache quantization (Section 3.2)
def qjl_quantize_values(V: torch.Tensor, vbits: int = 4, vcodes: Optional[torch.Tensor] = None,
                        vscale: Optional[torch.Tensor] = None, vzero: Optional[torch.Tensor] = None):
    """V[B,Hkv,n,d] -> (codes uint8 [B,Hkv,n,d*vbits/8], scale float16 [B,Hkv,n], zero float16 [B,Hkv,n])."""
    B, Hkv, n, d = V.shape
    if vcodes is None:
        vcodes = torch.empty((B, Hkv, n, d * vbits // 8), dtype=torch.uint8, device=V.device)
    if vscale is None:
        vscale = torch.empty((B, Hkv, n), dtype=torch.float16, device=V.device)
    if vzero is None:
        vzero = torch.empty((B, Hkv, n), dtype=torch.float16, device=V.device)
    if tuple(vcodes.shape) != (B, Hkv, n, d * vbits // 8) or vcodes.dtype != torch.uint8:
        raise ValueError("vcodes must be uint8 [B,Hkv,n,d*vbits/8]")
    sh = _shape(B, Hkv, Hkv, n, d, 32, _tag(V))
    _check("qjl_quantize_values",
           lib().qjl_quantize_values(ctypes.byref(sh), vbits, _dev(V, "V"), _dev(vcodes, "vcodes"),
                                     _dev(vscale, "vscale"), _dev(vzero, "vzero"), _stream(V)))
    return vcodes, vscale, vzero


def qjl_decode_attention_vq(Q: torch.Tensor, S: torch.Tensor, bits: torch.Tensor, norms: torch.Tensor,
                            vcodes: torch.Tensor, vscale: torch.Tensor, vzero: torch.Tensor, vbits: int = 4,
                            scale: float = 1.0, out: Optional[torch.Tensor] = None,
                            workspace: Optional[torch.Tensor] = None,
                            events: Optional[Tuple[int, int]] = None) -> torch.Tensor:
    """One decode step with quantized keys and values -> float32 [B,Hq,d]."""
    B, Hq, d = Q.shape
    _, Hkv, n, vb = vcodes.shape
    m = S.shape[0]
    if S.dtype != Q.dtype or vb * 8 != d * vbits:
        raise ValueError("S must have the dtype of Q; vcodes must be [B,Hkv,n,d*vbits/8]")
    if tuple(bits.shape) != (B, Hkv, n, m // 8) or tuple(norms.shape) != (B, Hkv, n):
        raise ValueError("bits/norms do not match the value cache and S")
    if tuple(vscale.shape) != (B, Hkv, n) or tuple(vzero.shape) != (B, Hkv, n):
        raise ValueError("vscale/vzero must be [B,Hkv,n]")
    need = qjl_decode_workspace_bytes(B, Hq, Hkv, n, d, m, Q.dtype)
    if workspace is None:
        workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=Q.device)
    if out is None:
        out = torch.empty((B, Hq, d), dtype=torch.float32, device=Q.device)
    sh = _shape(B, Hq, Hkv, n, d, m, _tag(Q), scale)
    _check("qjl_decode_attention_vq",
           lib().qjl_decode_attention_vq(ctypes.byref(sh), vbits, _dev(Q, "Q"), _dev(S, "S"), _dev(bits, "bits"),
                                         _dev(norms, "norms"), _dev(vcodes, "vcodes"), _dev(vscale, "vscale"),
                                         _dev(vzero, "vzero"), _dev(out, "out"), _dev(workspace, "workspace"),
                                         workspace.numel() * workspace.element_size(), _stream(Q),
                                         events[0] if events else None, events[1] if events else None))
    return out


# ---- streaming (Algorithm 1 as a loop over the token stream)
def qjl_append_keys(K_new: torch.Tensor, S: torch.Tensor, bits: torch.Tensor, norms: torch.Tensor, pos: int) -> None:
    """K_new[B,Hkv,t,d] -> rows pos..pos+t-1 of bits[B,Hkv,cap,m/8], norms[B,Hkv,cap] (in place)."""
    B, Hkv, t, d = K_new.shape
    m = S.shape[0]
    cap = bits.shape[2]
    if tuple(bits.shape) != (B, Hkv, cap, m // 8) or tuple(norms.shape) != (B, Hkv, cap) or S.dtype != K_new.dtype:
        raise ValueError("caches do not match K_new and S")
    sh = _shape(B, Hkv, Hkv, cap, d, m, _tag(K_new))
    _check("qjl_append_keys",
           lib().qjl_append_keys(ctypes.byref(sh), pos, t, _dev(K_new, "K_new"), _dev(S, "S"), _dev(bits, "bits"),
                                 _dev(norms, "norms"), _stream(K_new)))


def qjl_decode_step(Q: torch.Tensor, K_new: torch.Tensor, S: torch.Tensor, bits: torch.Tensor, norms: torch.Tensor,
                    V: torch.Tensor, pos: int, scale: float = 1.0, out: Optional[torch.Tensor] = None,
                    workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Append K_new[B,Hkv,1,d] at row pos, then attention of Q[B,Hq,d] over rows 0..pos -> float32 [B,Hq,d]."""
    B, Hq, d = Q.shape
    _, Hkv, cap, _ = V.shape
    m = S.shape[0]
    if tuple(K_new.shape) != (B, Hkv, 1, d) or tuple(bits.shape) != (B, Hkv, cap, m // 8):
        raise ValueError("K_new must be [B,Hkv,1,d]; bits [B,Hkv,cap,m/8]")
    need = qjl_decode_workspace_bytes(B, Hq, Hkv, cap, d, m, Q.dtype)
    if workspace is None:
        workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=Q.device)
    if out is None:
        out = torch.empty((B, Hq, d), dtype=torch.float32, device=Q.device)
    sh = _shape(B, Hq, Hkv, cap, d, m, _tag(Q), scale)
    _check("qjl_decode_step",
           lib().qjl_decode_step(ctypes.byref(sh), pos, _dev(K_new, "K_new"), _dev(Q, "Q"), _dev(S, "S"),
                                 _dev(bits, "bits"), _dev(norms, "norms"), _dev(V, "V"), _dev(out, "out"),
                                 _dev(workspace, "workspace"), workspace.numel() * workspace.element_size(),
                                 _stream(Q)))
    return out


# ---- the paper's operating point: two-part key codes + quantized values (+ the stream)
def qjl_decode_attention_dual_vq(Q: torch.Tensor, S_dual: torch.Tensor, bits: torch.Tensor, norms_in: torch.Tensor,
                                 norms_out: torch.Tensor, vcodes: torch.Tensor, vscale: torch.Tensor,
                                 vzero: torch.Tensor, m_out: int, vbits: int = 4, scale: float = 1.0,
                                 out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                                 events: Optional[Tuple[int, int]] = None) -> torch.Tensor:
    """One decode step on two-part key codes and quantized values -> float32 [B,Hq,d]."""
    B, Hq, d = Q.shape
    _, Hkv, n, vb = vcodes.shape
    mt = S_dual.shape[2]
    m = mt - m_out
    if S_dual.dtype != Q.dtype or vb * 8 != d * vbits or tuple(S_dual.shape) != (B, Hkv, mt, d):
        raise ValueError("S_dual must be [B,Hkv,m+m_out,d] with the dtype of Q; vcodes [B,Hkv,n,d*vbits/8]")
    if tuple(bits.shape) != (B, Hkv, n, mt // 8):
        raise ValueError("bits do not match the value cache and S_dual")
    for t in (norms_in, norms_out, vscale, vzero):
        if tuple(t.shape) != (B, Hkv, n):
            raise ValueError("norms / vscale / vzero must be [B,Hkv,n]")
    need = qjl_decode_dual_workspace_bytes(B, Hq, Hkv, n, d, m, m_out, Q.dtype)
    if workspace is None:
        workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=Q.device)
    if out is None:
        out = torch.empty((B, Hq, d), dtype=torch.float32, device=Q.device)
    sh = _shape(B, Hq, Hkv, n, d, m, _tag(Q), scale)
    _check("qjl_decode_attention_dual_vq",
           lib().qjl_decode_attention_dual_vq(ctypes.byref(sh), m_out, vbits, _dev(Q, "Q"), _dev(S_dual, "S_dual"),
                                              _dev(bits, "bits"), _dev(norms_in, "norms_in"),
                                              _dev(norms_out, "norms_out"), _dev(vcodes, "vcodes"),
                                              _dev(vscale, "vscale"), _dev(vzero, "vzero"), _dev(out, "out"),
                                              _dev(workspace, "workspace"),
                                              workspace.numel() * workspace.element_size(), _stream(Q),
                                              events[0] if events else None, events[1] if events else None))
    return out


def qjl_generation_step(Q: torch.Tensor, K_new: torch.Tensor, V_new: torch.Tensor, S_dual: torch.Tensor,
                        channels: torch.Tensor, bits: torch.Tensor, norms_in: torch.Tensor, norms_out: torch.Tensor,
                        vcodes: torch.Tensor, vscale: torch.Tensor, vzero: torch.Tensor, pos, m_out: int,
                        vbits: int = 4, scale: float = 1.0, out: Optional[torch.Tensor] = None,
                        workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Append the new token (K_new, V_new [B,Hkv,1,d]) at row pos of the six cache arrays, then attention of
    Q[B,Hq,d] over rows 0..pos -> float32 [B,Hq,d].  pos: an int, or a one-element int32 device tensor that the
    kernel reads (qjl_generation_step_devpos: for steps replayed from a graph)."""
    B, Hq, d = Q.shape
    _, Hkv, cap, vb = vcodes.shape
    mt = S_dual.shape[2]
    m = mt - m_out
    count = channels.shape[2]
    if tuple(K_new.shape) != (B, Hkv, 1, d) or tuple(V_new.shape) != (B, Hkv, 1, d) or K_new.dtype != Q.dtype or \
            V_new.dtype != Q.dtype:
        raise ValueError("K_new and V_new must be [B,Hkv,1,d] with the dtype of Q")
    if S_dual.dtype != Q.dtype or vb * 8 != d * vbits or tuple(S_dual.shape) != (B, Hkv, mt, d):
        raise ValueError("S_dual must be [B,Hkv,m+m_out,d] with the dtype of Q; vcodes [B,Hkv,cap,d*vbits/8]")
    if tuple(bits.shape) != (B, Hkv, cap, mt // 8) or tuple(channels.shape) != (B, Hkv, count) or \
            channels.dtype != torch.int32:
        raise ValueError("bits [B,Hkv,cap,(m+m_out)/8]; channels int32 [B,Hkv,count]")
    for t in (norms_in, norms_out, vscale, vzero):
        if tuple(t.shape) != (B, Hkv, cap):
            raise ValueError("norms / vscale / vzero must be [B,Hkv,cap]")
    need = qjl_decode_dual_workspace_bytes(B, Hq, Hkv, cap, d, m, m_out, Q.dtype)
    if workspace is None:
        workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=Q.device)
    if out is None:
        out = torch.empty((B, Hq, d), dtype=torch.float32, device=Q.device)
    sh = _shape(B, Hq, Hkv, cap, d, m, _tag(Q), scale)
    if isinstance(pos, torch.Tensor):               # position in device memory (int32, one element): graph-replayable
        if pos.dtype != torch.int32 or pos.numel() != 1:
            raise ValueError("a device position must be one int32")
        _check("qjl_generation_step_devpos",
               lib().qjl_generation_step_devpos(ctypes.byref(sh), m_out, vbits, _dev(pos, "pos"), _dev(K_new, "K_new"),
                                                _dev(V_new, "V_new"), _dev(Q, "Q"), _dev(S_dual, "S_dual"),
                                                _dev(channels, "channels"), count, _dev(bits, "bits"),
                                                _dev(norms_in, "norms_in"), _dev(norms_out, "norms_out"),
                                                _dev(vcodes, "vcodes"), _dev(vscale, "vscale"), _dev(vzero, "vzero"),
                                                _dev(out, "out"), _dev(workspace, "workspace"),
                                                workspace.numel() * workspace.element_size(), _stream(Q)))
        return out
    _check("qjl_generation_step",
           lib().qjl_generation_step(ctypes.byref(sh), m_out, vbits, pos, _dev(K_new, "K_new"), _dev(V_new, "V_new"),
                                     _dev(Q, "Q"), _dev(S_dual, "S_dual"), _dev(channels, "channels"), count,
                                     _dev(bits, "bits"), _dev(norms_in, "norms_in"), _dev(norms_out, "norms_out"),
                                     _dev(vcodes, "vcodes"), _dev(vscale, "vscale"), _dev(vzero, "vzero"),
                                     _dev(out, "out"), _dev(workspace, "workspace"),
                                     workspace.numel() * workspace.element_size(), _stream(Q)))
    return out
