"""Host-only checks of the C ABI: the library loads, exports every symbol the
header declares, and rejects bad descriptors and offsets before any launch."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2510_22049_amd import binding as V

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "vista.h")).read()
    declared = set(re.findall(r"\b(vista_[a-z0-9_]+)\s*\(", header))
    assert declared == set(V.EXPORTS)
    L = V.lib()
    for name in declared:
        assert getattr(L, name) is not None


def test_calibration_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "vista_calibrate.h")).read()
    declared = set(re.findall(r"\b(vista_calibrate_[a-z0-9_]+)\s*\(", header))
    assert declared == {"vista_calibrate_issue", "vista_calibrate_lds_read", "vista_calibrate_stream_read"}
    L = C.CDLL(os.path.join(ROOT, "paper_2510_22049_amd", "libvista_calibrate.so"))
    for name in declared:
        assert getattr(L, name) is not None


def test_status_strings():
    L = V.lib()
    assert L.vista_status_string(0) == b"VISTA_OK"
    for code in range(1, 8):
        assert L.vista_status_string(code).startswith(b"VISTA_ERR_")
    assert b"unknown" in L.vista_status_string(99)


def desc(**kw):
    base = dict(B=2, S=16, d=64, H=1, dtype=V.VISTA_F32, total_items=100)
    base.update(kw)
    return V.summarize_desc(**base)


def test_segment_default_is_a_function_of_total_items_only():
    assert V.vista_summarize_segment_items(desc(total_items=1024)) == 256
    assert V.vista_summarize_segment_items(desc(total_items=768597, B=64)) == 3008      # 256 segments
    assert V.vista_summarize_segment_items(desc(total_items=8_000_000, B=8)) == 7840     # 4 x 256 segments
    assert V.vista_summarize_segment_items(desc(segment_items=64)) == 64
    assert V.vista_summarize_segment_items(desc(segment_items=48)) == 0      # not a multiple of 32
    assert V.vista_summarize_workspace_bytes(desc()) > 0


@pytest.mark.parametrize("kw,code", [
    (dict(B=0), V.VISTA_ERR_SHAPE),
    (dict(d=66, H=4), V.VISTA_ERR_SHAPE),
    (dict(S=513), V.VISTA_ERR_UNSUPPORTED),
    (dict(d=512, H=4), V.VISTA_ERR_UNSUPPORTED),
    (dict(dtype=7), V.VISTA_ERR_UNSUPPORTED),
    (dict(scale=-1.0), V.VISTA_ERR_SHAPE),
])
def test_summarize_rejects_bad_descriptors(kw, code):
    d = desc(**kw)
    one = C.c_void_p(256)                  # never dereferenced: the descriptor fails first
    st = V.lib().vista_summarize(C.byref(d), one, one, None, one, one, one, one, one, 1 << 30, None)
    assert st == code
    assert V.vista_summarize_workspace_bytes(d) == 0


def test_summarize_rejects_null_bad_offsets_and_small_workspace():
    d = desc()
    L = V.lib()
    one = C.c_void_p(256)
    assert L.vista_summarize(C.byref(d), one, None, None, one, one, one, one, one, 1 << 30, None) == V.VISTA_ERR_NULL
    assert L.vista_summarize(None, one, one, None, one, one, one, one, one, 1 << 30, None) == V.VISTA_ERR_NULL
    for bad in ([1, 50, 100], [0, 60, 50], [0, 50, 99]):
        off = np.array(bad, dtype=np.int64)
        st = L.vista_summarize(C.byref(d), one, one, off.ctypes.data, one, one, one, one, one, 1 << 30, None)
        assert st == V.VISTA_ERR_OFFSETS
    good = np.array([0, 50, 100], dtype=np.int64)
    need = V.vista_summarize_workspace_bytes(d)
    args = (C.byref(d), one, one, good.ctypes.data, one, one, one, one)
    assert L.vista_summarize(*args, one, need - 1, None) == V.VISTA_ERR_WORKSPACE
    assert L.vista_summarize(*args, None, need, None) == V.VISTA_ERR_WORKSPACE
    assert L.vista_summarize(*args, C.c_void_p(264), need, None) == V.VISTA_ERR_WORKSPACE   # misaligned


def test_attend_and_ffn_reject_bad_arguments():
    L = V.lib()
    one = C.c_void_p(256)
    a = V.AttendDesc(B=1, C=4, S=8, d=64, H=3, dtype=V.VISTA_F32, scale=0.0)
    assert L.vista_target_attend(C.byref(a), one, one, one, None) == V.VISTA_ERR_SHAPE
    a = V.AttendDesc(B=1, C=4, S=1024, d=64, H=1, dtype=V.VISTA_F32, scale=0.0)
    assert L.vista_target_attend(C.byref(a), one, one, one, None) == V.VISTA_ERR_UNSUPPORTED
    a = V.AttendDesc(B=1, C=4, S=8, d=64, H=1, dtype=V.VISTA_F32, scale=0.0)
    assert L.vista_target_attend(C.byref(a), None, one, one, None) == V.VISTA_ERR_NULL
    f = V.FfnDesc(rows=4, d=48, d_ff=64, dtype=V.VISTA_BF16, eps=0.0)
    assert L.vista_sglu_ffn(C.byref(f), one, one, one, one, one, None) == V.VISTA_ERR_UNSUPPORTED
    f = V.FfnDesc(rows=0, d=64, d_ff=64, dtype=V.VISTA_BF16, eps=0.0)
    assert L.vista_sglu_ffn(C.byref(f), one, one, one, one, one, None) == V.VISTA_ERR_SHAPE


def test_forms_and_flags_are_validated():
    L = V.lib()
    one = C.c_void_p(256)
    call = lambda d: L.vista_summarize(C.byref(d), one, one, None, one, one, one, one, one, 1 << 30, None)
    assert call(desc(attn=3)) == V.VISTA_ERR_UNSUPPORTED             # no such form
    assert call(desc(attn=-1)) == V.VISTA_ERR_UNSUPPORTED
    d = desc()
    d.flags = 2                                                       # unknown flag bit
    assert call(d) == V.VISTA_ERR_SHAPE
    d = desc()
    d.reserved = 1
    assert call(d) == V.VISTA_ERR_SHAPE
    assert call(desc(attn=V.VISTA_ATTN_QLA, scale=0.5)) == V.VISTA_ERR_SHAPE   # the quasi-linear form has no score scale
    # segment default of the quasi-linear form: four times finer
    assert V.vista_summarize_segment_items(desc(total_items=768597, B=64, attn=V.VISTA_ATTN_QLA)) == 768


def test_codec_entry_points_reject_bad_arguments():
    L = V.lib()
    one = C.c_void_p(256)
    c = V.CodecDesc(rows=4, d=64, H=3, dtype=V.VISTA_BF16)
    assert L.vista_quantize_summaries(C.byref(c), one, one, one, None) == V.VISTA_ERR_SHAPE
    c = V.CodecDesc(rows=0, d=64, H=2, dtype=V.VISTA_BF16)
    assert L.vista_quantize_summaries(C.byref(c), one, one, one, None) == V.VISTA_ERR_SHAPE
    c = V.CodecDesc(rows=4, d=256, H=2, dtype=V.VISTA_BF16)            # heads wider than 64
    assert L.vista_quantize_summaries(C.byref(c), one, one, one, None) == V.VISTA_ERR_UNSUPPORTED
    c = V.CodecDesc(rows=4, d=64, H=2, dtype=V.VISTA_BF16)
    assert L.vista_quantize_summaries(C.byref(c), one, None, one, None) == V.VISTA_ERR_NULL
    assert L.vista_quantize_summaries(None, one, one, one, None) == V.VISTA_ERR_NULL
    # summaries as codes: both the codes and their scales are required
    a = V.AttendDesc(B=1, C=4, S=32, d=128, H=4, dtype=V.VISTA_BF16, scale=0.0)
    assert L.vista_target_attend_q8(C.byref(a), one, None, one, one, None) == V.VISTA_ERR_NULL
    assert L.vista_target_attend_q8(C.byref(a), one, one, None, one, None) == V.VISTA_ERR_NULL
    a.flags = 4
    assert L.vista_target_attend_q8(C.byref(a), one, one, one, one, None) == V.VISTA_ERR_SHAPE
    # the fused codec exists for the matrix-core shapes only
    d = desc(dtype=V.VISTA_F32)
    st = L.vista_summarize_q8(C.byref(d), one, one, None, one, one, one, one, one, one, 1 << 30, None)
    assert st == V.VISTA_ERR_UNSUPPORTED
    d = V.summarize_desc(B=2, S=256, d=128, H=4, dtype=V.VISTA_BF16, total_items=100)
    st = L.vista_summarize_q8(C.byref(d), one, one, None, one, one, one, one, None, one, 1 << 30, None)
    assert st == V.VISTA_ERR_NULL


def test_qla_backward_rejects_bad_arguments():
    L = V.lib()
    one = C.c_void_p(256)
    args = lambda d, **kw: [C.byref(d)] + [kw.get(k, one) for k in
                                            ("x", "off", "off_host", "q", "wk", "wv", "do", "dq", "dk", "dv", "dks", "dvs",
                                             "ws")] + \
        [kw.get("bytes", 1 << 30), None]
    d = desc()                                                          # softmax form: no gradients here
    assert L.vista_qla_backward(*args(d, off_host=None)) == V.VISTA_ERR_UNSUPPORTED
    assert V.lib().vista_qla_backward_workspace_bytes(C.byref(d)) == 0
    d = desc(attn=V.VISTA_ATTN_QLA)
    assert L.vista_qla_backward(*args(d, off_host=None, do=None)) == V.VISTA_ERR_NULL
    assert L.vista_qla_backward(*args(d, off_host=None, dk=None)) == V.VISTA_ERR_NULL
    bad = np.array([0, 60, 50], dtype=np.int64)
    assert L.vista_qla_backward(*args(d, off_host=bad.ctypes.data)) == V.VISTA_ERR_OFFSETS
    good = np.array([0, 50, 100], dtype=np.int64)
    need = L.vista_qla_backward_workspace_bytes(C.byref(d))
    assert need > V.vista_summarize_workspace_bytes(d) > 0
    assert L.vista_qla_backward(*args(d, off_host=good.ctypes.data, bytes=need - 1)) == V.VISTA_ERR_WORKSPACE
    d.flags = V.VISTA_FLAG_SELF_TERM                                    # the self term needs its two outputs
    assert L.vista_qla_backward_workspace_bytes(C.byref(d)) > need
    assert L.vista_qla_backward(*args(d, off_host=good.ctypes.data, dks=None)) == V.VISTA_ERR_NULL
    assert L.vista_qla_backward(*args(d, off_host=good.ctypes.data, dvs=None)) == V.VISTA_ERR_NULL


def test_static_entry_point_rejects_what_does_not_fit_its_array():
    L = V.lib()
    one = C.c_void_p(256)
    d = V.summarize_desc(B=8, S=256, d=128, H=4, dtype=V.VISTA_BF16, total_items=8_000_000)   # needs ~180 MB
    assert V.vista_summarize_workspace_bytes(d) > V.VISTA_STATIC_SCRATCH_BYTES
    assert L.vista_summarize_static(C.byref(d), one, one, None, one, one, one, one, None) == V.VISTA_ERR_SCRATCH
    assert L.vista_summarize_static(C.byref(desc(B=0)), one, one, None, one, one, one, one, None) == V.VISTA_ERR_SHAPE
