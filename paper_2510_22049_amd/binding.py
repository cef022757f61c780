"""ctypes binding of libvista.so: argument marshalling only.

The functions carry the names of the C entry points declared in
include/vista.h and do nothing but turn torch tensors (device memory) and the
current torch stream into the pointers the C ABI takes.  Every step of the
computation runs inside the library's HIP kernels; when the library is absent
or fails to load, importing this module's entry points raises -- there is no
CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libvista.so")

VISTA_OK = 0
VISTA_ERR_NULL, VISTA_ERR_SHAPE, VISTA_ERR_OFFSETS = 1, 2, 3
VISTA_ERR_UNSUPPORTED, VISTA_ERR_WORKSPACE, VISTA_ERR_HIP, VISTA_ERR_SCRATCH = 4, 5, 6, 7
VISTA_STATIC_SCRATCH_BYTES = 64 << 20
VISTA_F32, VISTA_BF16 = 0, 1
VISTA_ATTN_SOFTMAX, VISTA_ATTN_SILU, VISTA_ATTN_QLA = 0, 1, 2
VISTA_FLAG_SELF_TERM = 1

EXPORTS = (
    "vista_status_string",
    "vista_summarize_segment_items",
    "vista_summarize_workspace_bytes",
    "vista_summarize_schedule",
    "vista_summarize",
    "vista_summarize_static",
    "vista_target_attend",
    "vista_target_attend_q8",
    "vista_quantize_summaries",
    "vista_summarize_q8",
    "vista_qla_backward_workspace_bytes",
    "vista_qla_backward",
    "vista_sglu_ffn",
)


class SummarizeDesc(C.Structure):
    _fields_ = [("B", C.c_int32), ("S", C.c_int32), ("d", C.c_int32), ("H", C.c_int32),
                ("dtype", C.c_int32), ("attn", C.c_int32), ("scale", C.c_float),
                ("segment_items", C.c_int32), ("total_items", C.c_int64),
                ("q_user_stride", C.c_int64), ("flags", C.c_int32), ("reserved", C.c_int32)]


class AttendDesc(C.Structure):
    _fields_ = [("B", C.c_int32), ("C", C.c_int32), ("S", C.c_int32), ("d", C.c_int32),
                ("H", C.c_int32), ("dtype", C.c_int32), ("scale", C.c_float), ("flags", C.c_int32)]


class CodecDesc(C.Structure):
    _fields_ = [("rows", C.c_int64), ("d", C.c_int32), ("H", C.c_int32), ("dtype", C.c_int32)]


class FfnDesc(C.Structure):
    _fields_ = [("rows", C.c_int64), ("d", C.c_int32), ("d_ff", C.c_int32),
                ("dtype", C.c_int32), ("eps", C.c_float)]


class VistaError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(lib().vista_status_string(status).decode())


_lib = None


def lib() -> C.CDLL:
    """Loads libvista.so (built by ``python -m paper_2510_22049_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: run `python -m paper_2510_22049_amd.build` first; "
            "there is no fallback path")
    L = C.CDLL(LIB_PATH)
    vp, i64p = C.c_void_p, C.POINTER(C.c_int64)
    L.vista_status_string.restype = C.c_char_p
    L.vista_status_string.argtypes = [C.c_int]
    L.vista_summarize_segment_items.restype = C.c_int32
    L.vista_summarize_segment_items.argtypes = [C.POINTER(SummarizeDesc)]
    L.vista_summarize_workspace_bytes.restype = C.c_size_t
    L.vista_summarize_workspace_bytes.argtypes = [C.POINTER(SummarizeDesc)]
    L.vista_summarize_schedule.restype = C.c_int64
    L.vista_summarize_schedule.argtypes = [C.POINTER(SummarizeDesc), i64p, i64p, C.c_int64]
    L.vista_summarize.restype = C.c_int
    L.vista_summarize.argtypes = [C.POINTER(SummarizeDesc), vp, vp, vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
    L.vista_summarize_static.restype = C.c_int
    L.vista_summarize_static.argtypes = [C.POINTER(SummarizeDesc), vp, vp, vp, vp, vp, vp, vp, vp]
    L.vista_summarize_q8.restype = C.c_int
    L.vista_summarize_q8.argtypes = [C.POINTER(SummarizeDesc), vp, vp, vp, vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
    L.vista_qla_backward_workspace_bytes.restype = C.c_size_t
    L.vista_qla_backward_workspace_bytes.argtypes = [C.POINTER(SummarizeDesc)]
    L.vista_qla_backward.restype = C.c_int
    L.vista_qla_backward.argtypes = [C.POINTER(SummarizeDesc)] + [vp] * 13 + [C.c_size_t, vp]
    L.vista_quantize_summaries.restype = C.c_int
    L.vista_quantize_summaries.argtypes = [C.POINTER(CodecDesc), vp, vp, vp, vp]
    L.vista_target_attend_q8.restype = C.c_int
    L.vista_target_attend_q8.argtypes = [C.POINTER(AttendDesc), vp, vp, vp, vp, vp]
    L.vista_target_attend.restype = C.c_int
    L.vista_target_attend.argtypes = [C.POINTER(AttendDesc), vp, vp, vp, vp]
    L.vista_sglu_ffn.restype = C.c_int
    L.vista_sglu_ffn.argtypes = [C.POINTER(FfnDesc), vp, vp, vp, vp, vp, vp]
    _lib = L
    return L


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return VISTA_F32
    if t.dtype == torch.bfloat16:
        return VISTA_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _dev(t: torch.Tensor, name: str) -> int:
    if not t.is_cuda:
        raise ValueError(f"{name} must live in device memory")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def summarize_desc(B, S, d, H, dtype, total_items, per_user_q=False, scale=0.0, segment_items=0,
                   attn=VISTA_ATTN_SOFTMAX, self_term=False):
    return SummarizeDesc(B=B, S=S, d=d, H=H, dtype=dtype, attn=attn, scale=scale,
                         segment_items=segment_items, total_items=total_items,
                         q_user_stride=S * d if per_user_q else 0,
                         flags=VISTA_FLAG_SELF_TERM if self_term else 0, reserved=0)


def vista_summarize_segment_items(desc: SummarizeDesc) -> int:
    return lib().vista_summarize_segment_items(C.byref(desc))


def vista_summarize_workspace_bytes(desc: SummarizeDesc) -> int:
    return lib().vista_summarize_workspace_bytes(C.byref(desc))


def vista_summarize_schedule(desc: SummarizeDesc, offsets_host):
    """The tiles the kernels visit, int64 [n, 4] = (segment, user, first row, rows); host only.
    ``offsets_host`` is a numpy int64 array of B + 1 entries (not validated by the call)."""
    import numpy as np
    off = np.ascontiguousarray(offsets_host, dtype=np.int64)
    if off.size != desc.B + 1:
        raise ValueError("offsets_host must hold B + 1 entries")
    ptr = off.ctypes.data_as(C.POINTER(C.c_int64))
    n = lib().vista_summarize_schedule(C.byref(desc), ptr, None, 0)
    if n < 0:
        raise VistaError(VISTA_ERR_SHAPE)
    tiles = np.empty((n, 4), dtype=np.int64)
    lib().vista_summarize_schedule(C.byref(desc), ptr, tiles.ctypes.data_as(C.POINTER(C.c_int64)), n)
    return tiles


def vista_summarize(history_emb, offsets, virtual_queries, W_k, W_v, out, *, H, scale=0.0,
                    segment_items=0, offsets_host=None, workspace=None, attn=VISTA_ATTN_SOFTMAX,
                    self_term=False):
    """Stage 1.  history_emb [N,d], offsets int64 [B+1] (device), virtual_queries
    [S,d] or [B,S,d], W_k/W_v [d,d], out [B,S,d]; all on the GPU, same dtype.
    ``workspace`` is a uint8 device tensor (allocated here when None, by torch)."""
    B = offsets.numel() - 1
    S, d = virtual_queries.shape[-2:]
    N = history_emb.shape[0]
    desc = summarize_desc(B, S, d, H, _dtype_code(history_emb), N, virtual_queries.dim() == 3, scale,
                          segment_items, attn, self_term)
    need = vista_summarize_workspace_bytes(desc)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=history_emb.device)
    host = None
    if offsets_host is not None:
        if offsets_host.is_cuda or offsets_host.dtype != torch.int64:
            raise ValueError("offsets_host must be a CPU int64 tensor")
        host = offsets_host.contiguous().data_ptr()
    if offsets.dtype != torch.int64:
        raise TypeError("offsets must be int64")
    st = lib().vista_summarize(C.byref(desc), _dev(history_emb, "history_emb") if N else None,
                               _dev(offsets, "offsets"), host, _dev(virtual_queries, "virtual_queries"),
                               _dev(W_k, "W_k"), _dev(W_v, "W_v"), _dev(out, "out"),
                               _dev(workspace, "workspace"), workspace.numel(), _stream())
    if st != VISTA_OK:
        raise VistaError(st)
    return workspace


def vista_summarize_q8(history_emb, offsets, virtual_queries, W_k, W_v, out_codes, out_scales, *, H, scale=0.0,
                       segment_items=0, offsets_host=None, workspace=None, attn=VISTA_ATTN_SOFTMAX, self_term=False):
    """Stage 1 with the cache codec fused: out_codes int8 [B,S,d], out_scales float32 [B,S,H]."""
    B = offsets.numel() - 1
    S, d = virtual_queries.shape[-2:]
    N = history_emb.shape[0]
    desc = summarize_desc(B, S, d, H, _dtype_code(history_emb), N, virtual_queries.dim() == 3, scale,
                          segment_items, attn, self_term)
    need = vista_summarize_workspace_bytes(desc)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=history_emb.device)
    if out_codes.dtype != torch.int8 or out_scales.dtype != torch.float32:
        raise TypeError("out_codes must be int8 and out_scales float32")
    host = offsets_host.contiguous().data_ptr() if offsets_host is not None else None
    st = lib().vista_summarize_q8(C.byref(desc), _dev(history_emb, "history_emb") if N else None,
                                  _dev(offsets, "offsets"), host, _dev(virtual_queries, "virtual_queries"),
                                  _dev(W_k, "W_k"), _dev(W_v, "W_v"), _dev(out_codes, "out_codes"),
                                  _dev(out_scales, "out_scales"), _dev(workspace, "workspace"), workspace.numel(),
                                  _stream())
    if st != VISTA_OK:
        raise VistaError(st)
    return workspace


def vista_qla_backward(history_emb, offsets, virtual_queries, W_k, W_v, d_out, d_queries, d_keys, d_values, *, H,
                       segment_items=0, offsets_host=None, workspace=None, d_self_keys=None, d_self_values=None):
    """Gradients of quasi-linear attention: d_out [B,S,d] -> d_queries [B,S,d], d_keys / d_values [N,d];
    with d_self_keys / d_self_values [B,S,d] given, the forward had the self term and its gradients
    are formed as well."""
    B = offsets.numel() - 1
    S, d = virtual_queries.shape[-2:]
    N = history_emb.shape[0]
    self_term = d_self_keys is not None or d_self_values is not None
    desc = summarize_desc(B, S, d, H, _dtype_code(history_emb), N, virtual_queries.dim() == 3, 0.0,
                          segment_items, VISTA_ATTN_QLA, self_term)
    need = lib().vista_qla_backward_workspace_bytes(C.byref(desc))
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=history_emb.device)
    host = offsets_host.contiguous().data_ptr() if offsets_host is not None else None
    st = lib().vista_qla_backward(C.byref(desc), _dev(history_emb, "history_emb") if N else None,
                                  _dev(offsets, "offsets"), host, _dev(virtual_queries, "virtual_queries"),
                                  _dev(W_k, "W_k"), _dev(W_v, "W_v"), _dev(d_out, "d_out"),
                                  _dev(d_queries, "d_queries"), _dev(d_keys, "d_keys") if N else None,
                                  _dev(d_values, "d_values") if N else None,
                                  _dev(d_self_keys, "d_self_keys") if d_self_keys is not None else None,
                                  _dev(d_self_values, "d_self_values") if d_self_values is not None else None,
                                  _dev(workspace, "workspace"), workspace.numel(), _stream())
    if st != VISTA_OK:
        raise VistaError(st)
    return workspace


def vista_quantize_summaries(y, codes, scales, *, H):
    """Cache codec: y [..., d] -> codes int8 [..., d], scales float32 [..., H] (device tensors)."""
    d = y.shape[-1]
    desc = CodecDesc(rows=y.numel() // d, d=d, H=H, dtype=_dtype_code(y))
    if codes.dtype != torch.int8 or scales.dtype != torch.float32:
        raise TypeError("codes must be int8 and scales float32")
    st = lib().vista_quantize_summaries(C.byref(desc), _dev(y, "y"), _dev(codes, "codes"), _dev(scales, "scales"),
                                        _stream())
    if st != VISTA_OK:
        raise VistaError(st)


def vista_target_attend_q8(candidates, codes, scales, out, *, H, scale=0.0, self_term=False):
    """Stage 2 on quantized summaries: codes int8 [B,S,d], scales float32 [B,S,H]."""
    B, Cn, d = candidates.shape
    S = codes.shape[1]
    desc = AttendDesc(B=B, C=Cn, S=S, d=d, H=H, dtype=_dtype_code(candidates), scale=scale,
                      flags=VISTA_FLAG_SELF_TERM if self_term else 0)
    if codes.dtype != torch.int8 or scales.dtype != torch.float32:
        raise TypeError("codes must be int8 and scales float32")
    st = lib().vista_target_attend_q8(C.byref(desc), _dev(candidates, "candidates"), _dev(codes, "codes"),
                                      _dev(scales, "scales"), _dev(out, "out"), _stream())
    if st != VISTA_OK:
        raise VistaError(st)


def vista_summarize_static(history_emb, offsets, virtual_queries, W_k, W_v, out, *, H, scale=0.0,
                           segment_items=0, offsets_host=None, attn=VISTA_ATTN_SOFTMAX, self_term=False):
    """Stage 1 on the library's static scratch: no workspace argument, nothing allocated."""
    B = offsets.numel() - 1
    S, d = virtual_queries.shape[-2:]
    N = history_emb.shape[0]
    desc = summarize_desc(B, S, d, H, _dtype_code(history_emb), N, virtual_queries.dim() == 3, scale,
                          segment_items, attn, self_term)
    host = None
    if offsets_host is not None:
        if offsets_host.is_cuda or offsets_host.dtype != torch.int64:
            raise ValueError("offsets_host must be a CPU int64 tensor")
        host = offsets_host.contiguous().data_ptr()
    if offsets.dtype != torch.int64:
        raise TypeError("offsets must be int64")
    st = lib().vista_summarize_static(C.byref(desc), _dev(history_emb, "history_emb") if N else None,
                                      _dev(offsets, "offsets"), host, _dev(virtual_queries, "virtual_queries"),
                                      _dev(W_k, "W_k"), _dev(W_v, "W_v"), _dev(out, "out"), _stream())
    if st != VISTA_OK:
        raise VistaError(st)


def vista_target_attend(candidates, summaries, out, *, H, scale=0.0, self_term=False):
    """Stage 2.  candidates [B,C,d], summaries [B,S,d], out [B,C,d]; device, same dtype."""
    B, Cn, d = candidates.shape
    S = summaries.shape[1]
    desc = AttendDesc(B=B, C=Cn, S=S, d=d, H=H, dtype=_dtype_code(candidates), scale=scale,
                      flags=VISTA_FLAG_SELF_TERM if self_term else 0)
    st = lib().vista_target_attend(C.byref(desc), _dev(candidates, "candidates"),
                                   _dev(summaries, "summaries"), _dev(out, "out"), _stream())
    if st != VISTA_OK:
        raise VistaError(st)


def vista_sglu_ffn(y, W_g, W_u, W_o, out, *, eps=0.0):
    """Gated block between layers.  y [rows,d] (any leading shape), W_g/W_u [d,d_ff], W_o [d_ff,d]."""
    d = y.shape[-1]
    rows = y.numel() // d
    desc = FfnDesc(rows=rows, d=d, d_ff=W_g.shape[1], dtype=_dtype_code(y), eps=eps)
    st = lib().vista_sglu_ffn(C.byref(desc), _dev(y, "y"), _dev(W_g, "W_g"), _dev(W_u, "W_u"),
                              _dev(W_o, "W_o"), _dev(out, "out"), _stream())
    if st != VISTA_OK:
        raise VistaError(st)
