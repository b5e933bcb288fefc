"""ctypes binding of libqadagrad.so: argument marshalling only.

Each function has the name and the argument order of its C entry point in
include/qadagrad.h and takes torch tensors (device memory) where the C call takes device
pointers.  Nothing is computed here and there is no fallback: if the library is missing the
import raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

QA_OK = 0
QA_REQUANT_NONE, QA_REQUANT_BUCKET, QA_REQUANT_GLOBAL = 0, 1, 2
QA_THRESH_GIVEN = 1
QA_THRESH_EXACT = 2
QA_OP_QUANTIZE, QA_OP_STEP, QA_OP_GRAD_CSR, QA_OP_GRAD_DENSE = 1, 2, 3, 4
QA_OP_SELECT, QA_OP_STEP_SELECTED, QA_OP_QUANTIZE_EXACT = 5, 6, 7
QA_DENSE, QA_CSR = 0, 1
QA_METHOD_QCMD, QA_METHOD_QRDA = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))


def lib_path() -> str:
    """In-tree library; QA_LIBRARY may name another build of the same ABI."""
    return os.environ.get("QA_LIBRARY") or os.path.join(_HERE, "libqadagrad.so")


class QaError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {qa_strerror(code)} ({code})")


class Layout(C.Structure):
    """Mirror of qa_layout."""
    _fields_ = [("d", C.c_int64), ("M", C.c_int32), ("bucket", C.c_int32),
                ("thr_coef", C.c_float), ("code_stride", C.c_int64), ("scale_stride", C.c_int64)]

    @staticmethod
    def make(d, M, bucket=4096, thr_coef=0.75, code_stride=None, scale_stride=None):
        W = (d + 15) // 16
        nb = (d + bucket - 1) // bucket if bucket else 1
        return Layout(d, M, bucket, thr_coef, code_stride or W, scale_stride or nb)

    @staticmethod
    def spaced_code_stride(d):
        """A code_stride (in words) for large d: every worker's row starts on a 1 KiB boundary,
        3 KiB (mod 16 KiB) after the previous one.  Rows a power of two apart send the M code
        streams of a tile to the same memory channels (see the note on qa_layout in the header)."""
        stride = (d + 15) // 16
        stride += (-stride) % 256
        return stride + 256 * ((3 - stride // 256) % 16)

    @property
    def words(self):
        return (self.d + 15) // 16

    @property
    def n_buckets(self):
        return (self.d + self.bucket - 1) // self.bucket if self.bucket else 1


class SegmentPlan(C.Structure):
    """Mirror of qa_segment_plan; `keep` holds the tensor that owns the device table."""
    _fields_ = [("d", C.c_int64), ("n_seg", C.c_int64), ("n_pieces", C.c_int64), ("table", C.c_void_p)]
    keep = None


if not os.path.exists(lib_path()):
    raise ImportError(
        f"{lib_path()} not found: build it first (python -c 'import __graft_entry__ as g; g.build()')")

_lib = C.CDLL(lib_path())
_vp, _sz = C.c_void_p, C.c_size_t
_lib.qa_version.restype = C.c_int
_lib.qa_strerror.restype = C.c_char_p
_lib.qa_strerror.argtypes = [C.c_int]
_lib.qa_workspace_bytes.restype = _sz
_lib.qa_workspace_bytes.argtypes = [C.POINTER(Layout), C.c_int]
_lib.qa_local_grad.argtypes = [C.c_int, _vp, _vp, _vp, C.c_int64, C.c_int64, _vp, _vp, C.c_int32,
                               _vp, _vp, _vp, _vp, _sz, _vp]
_lib.qa_local_grad_batched.argtypes = [C.c_int, _vp, _vp, _vp, C.c_int64, C.c_int64, _vp, _vp, C.c_int32,
                                       C.c_int32, _vp, _vp, C.c_int64, _vp, _vp, _sz, _vp]
_lib.qa_quantize_pack.argtypes = [C.POINTER(Layout), _vp, C.c_int64, _vp, _vp, _vp, C.c_uint32,
                                  _vp, _sz, _vp]
_lib.qa_aggregate_unpack.argtypes = [C.POINTER(Layout), _vp, _vp, _vp, _vp]
_lib.qa_step_qcmd.argtypes = [C.POINTER(Layout), _vp, _vp, _vp, _vp, _vp, C.c_float, C.c_float,
                              C.c_float, C.c_int, _vp, _sz, _vp]
_lib.qa_step_qrda.argtypes = [C.POINTER(Layout), _vp, _vp, _vp, _vp, _vp, C.c_int64, C.c_float,
                              C.c_float, C.c_float, C.c_int, _vp, _sz, _vp]
_lib.qa_indicator.argtypes = [C.POINTER(Layout), C.c_int, _vp, C.c_int64, _vp, _vp, _vp, C.c_int64,
                              C.c_float, C.c_float, C.c_float, _vp, C.c_int64, _vp]
_lib.qa_indicator_or.argtypes = [C.POINTER(Layout), _vp, C.c_int64, _vp, _vp]
_lib.qa_quantize_pack_selected.argtypes = [C.POINTER(Layout), _vp, C.c_int64, _vp, C.c_int64, _vp, _vp,
                                           _vp, _vp, _vp, _sz, _vp]
_lib.qa_decode_selected.argtypes = [C.POINTER(Layout), _vp, C.c_int64, _vp, _vp, _vp, _sz, _vp]
_lib.qa_quantize_pack_stochastic.argtypes = [C.POINTER(Layout), _vp, C.c_int64, _vp, _vp, C.c_uint64,
                                             C.c_uint32, _vp]
_lib.qa_segment_plan_bytes.restype = _sz
_lib.qa_segment_plan_bytes.argtypes = [C.c_int64, C.c_int64]
_lib.qa_segment_workspace_bytes.restype = _sz


def _p(t):
    return None if t is None else t.data_ptr()


def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream
    return int(stream)


def _check(rc, where):
    if rc != QA_OK:
        raise QaError(rc, where)


def qa_version() -> int:
    return _lib.qa_version()


def qa_strerror(code: int) -> str:
    return _lib.qa_strerror(code).decode()


def qa_workspace_bytes(layout: Layout, op: int) -> int:
    return int(_lib.qa_workspace_bytes(C.byref(layout), op))


def qa_local_grad(fmt, A_or_vals, indptr, indices, n_rows, d, y, batch_rows, B, x, g_out, loss_out,
                  ws, stream=None):
    _check(_lib.qa_local_grad(fmt, _p(A_or_vals), _p(indptr), _p(indices), n_rows, d, _p(y),
                              _p(batch_rows), B, _p(x), _p(g_out), _p(loss_out), _p(ws), _nbytes(ws),
                              _stream(stream)), "qa_local_grad")


def qa_local_grad_batched(fmt, A_or_vals, indptr, indices, n_rows, d, y, batch_rows, B, M, x, g_out,
                          g_stride, loss_out, ws, stream=None):
    _check(_lib.qa_local_grad_batched(fmt, _p(A_or_vals), _p(indptr), _p(indices), n_rows, d, _p(y),
                                      _p(batch_rows), B, M, _p(x), _p(g_out), g_stride, _p(loss_out),
                                      _p(ws), _nbytes(ws), _stream(stream)), "qa_local_grad_batched")


def qa_quantize_pack(layout, g, g_stride, codes, scales, thresholds, flags, ws, stream=None):
    _check(_lib.qa_quantize_pack(C.byref(layout), _p(g), g_stride, _p(codes), _p(scales),
                                 _p(thresholds), flags, _p(ws), _nbytes(ws), _stream(stream)),
           "qa_quantize_pack")


def qa_quantize_pack_static(layout, g, g_stride, codes, scales, thresholds, flags, stream=None):
    _lib.qa_quantize_pack_static.argtypes = [C.POINTER(Layout), _vp, C.c_int64, _vp, _vp, _vp,
                                             C.c_uint32, _vp]
    _check(_lib.qa_quantize_pack_static(C.byref(layout), _p(g), g_stride, _p(codes), _p(scales),
                                        _p(thresholds), flags, _stream(stream)),
           "qa_quantize_pack_static")


def qa_aggregate_unpack(layout, codes, scales, gbar_out, stream=None):
    _check(_lib.qa_aggregate_unpack(C.byref(layout), _p(codes), _p(scales), _p(gbar_out),
                                    _stream(stream)), "qa_aggregate_unpack")


def qa_step_qcmd(layout, codes, scales, x, G, z_or_null, eta, lam, delta, requant, ws, stream=None):
    _check(_lib.qa_step_qcmd(C.byref(layout), _p(codes), _p(scales), _p(x), _p(G), _p(z_or_null),
                             eta, lam, delta, requant, _p(ws), _nbytes(ws), _stream(stream)),
           "qa_step_qcmd")


def qa_step_qrda(layout, codes, scales, x, G, z, t, eta, lam, delta, requant, ws, stream=None):
    _check(_lib.qa_step_qrda(C.byref(layout), _p(codes), _p(scales), _p(x), _p(G), _p(z), t, eta,
                             lam, delta, requant, _p(ws), _nbytes(ws), _stream(stream)),
           "qa_step_qrda")


def qa_indicator(layout, method, g, g_stride, x, G, z, t, eta, lam, delta, ind_out, ind_stride,
                 stream=None):
    _check(_lib.qa_indicator(C.byref(layout), method, _p(g), g_stride, _p(x), _p(G), _p(z), t, eta, lam,
                             delta, _p(ind_out), ind_stride, _stream(stream)), "qa_indicator")


def qa_indicator_or(layout, ind, ind_stride, ind_syn_out, stream=None):
    _check(_lib.qa_indicator_or(C.byref(layout), _p(ind), ind_stride, _p(ind_syn_out), _stream(stream)),
           "qa_indicator_or")


def qa_quantize_pack_selected(layout, g, g_stride, ind, ind_stride, sel_codes, counts, scales,
                              thresholds, ws=None, stream=None):
    _check(_lib.qa_quantize_pack_selected(C.byref(layout), _p(g), g_stride, _p(ind), ind_stride,
                                          _p(sel_codes), _p(counts), _p(scales), _p(thresholds),
                                          _p(ws), _nbytes(ws), _stream(stream)),
           "qa_quantize_pack_selected")


def qa_decode_selected(layout, ind, ind_stride, sel_codes, codes_out, ws=None, stream=None):
    _check(_lib.qa_decode_selected(C.byref(layout), _p(ind), ind_stride, _p(sel_codes), _p(codes_out),
                                   _p(ws), _nbytes(ws), _stream(stream)), "qa_decode_selected")


def qa_quantize_pack_stochastic(layout, g, g_stride, codes, scales, seed, step, stream=None):
    _check(_lib.qa_quantize_pack_stochastic(C.byref(layout), _p(g), g_stride, _p(codes), _p(scales),
                                            seed, step, _stream(stream)), "qa_quantize_pack_stochastic")


def qa_segment_plan_bytes(d: int, n_seg: int) -> int:
    return int(_lib.qa_segment_plan_bytes(d, n_seg))


def qa_segment_plan_init(d, begin, length, table, stream=None) -> SegmentPlan:
    """begin, length: host sequences of ints; table: device tensor of at least
    qa_segment_plan_bytes(d, len(begin)) bytes, kept alive by the returned plan."""
    n = len(begin)
    assert len(length) == n
    b = (C.c_int64 * max(n, 1))(*[int(v) for v in begin])
    l = (C.c_int64 * max(n, 1))(*[int(v) for v in length])
    plan = SegmentPlan()
    _lib.qa_segment_plan_init.argtypes = [C.c_int64, C.c_int64, C.POINTER(C.c_int64),
                                          C.POINTER(C.c_int64), _vp, _sz, C.POINTER(SegmentPlan), _vp]
    _check(_lib.qa_segment_plan_init(d, n, b, l, _p(table), _nbytes(table), C.byref(plan),
                                     _stream(stream)), "qa_segment_plan_init")
    plan.keep = table
    return plan


def qa_segment_workspace_bytes(plan: SegmentPlan, M: int, op: int) -> int:
    _lib.qa_segment_workspace_bytes.argtypes = [C.POINTER(SegmentPlan), C.c_int32, C.c_int]
    return int(_lib.qa_segment_workspace_bytes(C.byref(plan), M, op))


def qa_quantize_pack_segments(layout, plan, g, g_stride, codes, scales, thresholds, ws, stream=None):
    _lib.qa_quantize_pack_segments.argtypes = [C.POINTER(Layout), C.POINTER(SegmentPlan), _vp, C.c_int64,
                                               _vp, _vp, _vp, _vp, _sz, _vp]
    _check(_lib.qa_quantize_pack_segments(C.byref(layout), C.byref(plan), _p(g), g_stride, _p(codes),
                                          _p(scales), _p(thresholds), _p(ws), _nbytes(ws),
                                          _stream(stream)), "qa_quantize_pack_segments")


def qa_step_qcmd_segments(layout, plan, codes, scales, x, G, z_or_null, eta, lam, delta, requant, ws,
                          stream=None):
    _lib.qa_step_qcmd_segments.argtypes = [C.POINTER(Layout), C.POINTER(SegmentPlan), _vp, _vp, _vp, _vp,
                                           _vp, C.c_float, C.c_float, C.c_float, C.c_int, _vp, _sz, _vp]
    _check(_lib.qa_step_qcmd_segments(C.byref(layout), C.byref(plan), _p(codes), _p(scales), _p(x),
                                      _p(G), _p(z_or_null), eta, lam, delta, requant, _p(ws),
                                      _nbytes(ws), _stream(stream)), "qa_step_qcmd_segments")


def qa_step_qrda_segments(layout, plan, codes, scales, x, G, z, t, eta, lam, delta, requant, ws,
                          stream=None):
    _lib.qa_step_qrda_segments.argtypes = [C.POINTER(Layout), C.POINTER(SegmentPlan), _vp, _vp, _vp, _vp,
                                           _vp, C.c_int64, C.c_float, C.c_float, C.c_float, C.c_int,
                                           _vp, _sz, _vp]
    _check(_lib.qa_step_qrda_segments(C.byref(layout), C.byref(plan), _p(codes), _p(scales), _p(x),
                                      _p(G), _p(z), t, eta, lam, delta, requant, _p(ws), _nbytes(ws),
                                      _stream(stream)), "qa_step_qrda_segments")


def qa_select_codes(layout, codes, ind, ind_stride, sel_codes, counts, ws=None, stream=None):
    _lib.qa_select_codes.argtypes = [C.POINTER(Layout), _vp, _vp, C.c_int64, _vp, _vp, _vp, _sz, _vp]
    _check(_lib.qa_select_codes(C.byref(layout), _p(codes), _p(ind), ind_stride, _p(sel_codes),
                                _p(counts), _p(ws), _nbytes(ws), _stream(stream)), "qa_select_codes")


def qa_step_qcmd_selected(layout, ind, ind_stride, sel_codes, scales, x, G, z_or_null, eta, lam, delta,
                          requant, ws, stream=None):
    _lib.qa_step_qcmd_selected.argtypes = [C.POINTER(Layout), _vp, C.c_int64, _vp, _vp, _vp, _vp, _vp,
                                           C.c_float, C.c_float, C.c_float, C.c_int, _vp, _sz, _vp]
    _check(_lib.qa_step_qcmd_selected(C.byref(layout), _p(ind), ind_stride, _p(sel_codes), _p(scales),
                                      _p(x), _p(G), _p(z_or_null), eta, lam, delta, requant, _p(ws),
                                      _nbytes(ws), _stream(stream)), "qa_step_qcmd_selected")


def qa_step_qrda_selected(layout, ind, ind_stride, sel_codes, scales, x, G, z, t, eta, lam, delta,
                          requant, ws, stream=None):
    _lib.qa_step_qrda_selected.argtypes = [C.POINTER(Layout), _vp, C.c_int64, _vp, _vp, _vp, _vp, _vp,
                                           C.c_int64, C.c_float, C.c_float, C.c_float, C.c_int, _vp,
                                           _sz, _vp]
    _check(_lib.qa_step_qrda_selected(C.byref(layout), _p(ind), ind_stride, _p(sel_codes), _p(scales),
                                      _p(x), _p(G), _p(z), t, eta, lam, delta, requant, _p(ws),
                                      _nbytes(ws), _stream(stream)), "qa_step_qrda_selected")


def qa_aggregate_quantize(layout, codes, scales, requant, q_codes, q_scales, q_thresholds, ws, stream=None):
    _lib.qa_aggregate_quantize.argtypes = [C.POINTER(Layout), _vp, _vp, C.c_int, _vp, _vp, _vp, _vp, _sz, _vp]
    _check(_lib.qa_aggregate_quantize(C.byref(layout), _p(codes), _p(scales), requant, _p(q_codes),
                                      _p(q_scales), _p(q_thresholds), _p(ws), _nbytes(ws),
                                      _stream(stream)), "qa_aggregate_quantize")


def qa_aggregate_quantize_selected(layout, ind, ind_stride, sel_codes, scales, requant, q_codes, q_scales,
                                   q_thresholds, ind_syn_out, ws, stream=None):
    _lib.qa_aggregate_quantize_selected.argtypes = [C.POINTER(Layout), _vp, C.c_int64, _vp, _vp, C.c_int,
                                                    _vp, _vp, _vp, _vp, _vp, _sz, _vp]
    _check(_lib.qa_aggregate_quantize_selected(C.byref(layout), _p(ind), ind_stride, _p(sel_codes),
                                               _p(scales), requant, _p(q_codes), _p(q_scales),
                                               _p(q_thresholds), _p(ind_syn_out), _p(ws), _nbytes(ws),
                                               _stream(stream)),
           "qa_aggregate_quantize_selected")


def qa_segment_plan_host(d, begin, length):
    """Host-only validation and table of a tensor list -> (n_pieces, table as a list of int64)."""
    n = len(begin)
    nwords = qa_segment_plan_bytes(d, n) // 8
    table = (C.c_int64 * max(nwords, 1))()
    npieces = C.c_int64(0)
    _lib.qa_segment_plan_host.argtypes = [C.c_int64, C.c_int64, C.POINTER(C.c_int64), C.POINTER(C.c_int64),
                                          C.POINTER(C.c_int64), _sz, C.POINTER(C.c_int64)]
    _check(_lib.qa_segment_plan_host(d, n, (C.c_int64 * max(n, 1))(*[int(v) for v in begin]),
                                     (C.c_int64 * max(n, 1))(*[int(v) for v in length]), table,
                                     nwords * 8, C.byref(npieces)), "qa_segment_plan_host")
    return npieces.value, list(table)
