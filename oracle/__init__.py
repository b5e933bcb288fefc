"""ctypes access to the CPU oracle (oracle/qa_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
cpu_baseline leg.  Nothing in the product package imports this module, and this module
imports nothing from the product package.

Every wrapper takes and returns numpy arrays; all arithmetic happens in the C++ file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "qa_oracle.cpp")
_LIB = os.path.join(_HERE, "liboracle.so")

REQUANT_NONE, REQUANT_BUCKET, REQUANT_GLOBAL = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the oracle with the host compiler.  No fused multiply-add, no fast-math."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-std=c++17", "-O2", "-ffp-contract=off", "-fPIC", "-shared",
               _SRC, "-o", _LIB]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    """The compiled oracle.  QA_ORACLE_LIB may name another build of the same source (the
    mutation test points it at deliberately broken copies to show that the pins notice)."""
    global _lib
    if _lib is None:
        _lib = C.CDLL(os.environ.get("QA_ORACLE_LIB") or build())
        _declare(_lib)
    return _lib


_f32p = np.ctypeslib.ndpointer(np.float32, flags="C_CONTIGUOUS")
_f64p = np.ctypeslib.ndpointer(np.float64, flags="C_CONTIGUOUS")
_i8p = np.ctypeslib.ndpointer(np.int8, flags="C_CONTIGUOUS")
_u32p = np.ctypeslib.ndpointer(np.uint32, flags="C_CONTIGUOUS")
_i32p = np.ctypeslib.ndpointer(np.int32, flags="C_CONTIGUOUS")
_i64p = np.ctypeslib.ndpointer(np.int64, flags="C_CONTIGUOUS")
_i64, _i32, _f32, _f64, _vp = C.c_int64, C.c_int, C.c_float, C.c_double, C.c_void_p


def _declare(L):
    L.orc_threshold_scale.argtypes = [_f32p, _i64, _f32, C.POINTER(_f32), C.POINTER(_f32),
                                      C.POINTER(_i64)]
    L.orc_scale_for_threshold.argtypes = [_f32p, _i64, _f32, C.POINTER(_f32), C.POINTER(_i64)]
    L.orc_quantize.argtypes = [_f32p, _i64, _i64, _f32, _i8p, _f32p, _vp, _vp]
    L.orc_exact_threshold.argtypes = [_f32p, _i64, C.POINTER(_f64), C.POINTER(_f64),
                                      C.POINTER(_f64), C.POINTER(_i64)]
    L.orc_exact_thresholds.argtypes = [_f32p, _i64, _i64, _f32p]
    L.orc_pack.argtypes = [_i8p, _i64, _u32p]
    L.orc_unpack.argtypes = [_u32p, _i64, _i8p]
    L.orc_quantize_pack.argtypes = [_f32p, _i64, _i64, _i32, _i64, _f32, _u32p, _i64, _f32p,
                                    _vp, _i64, _i32]
    L.orc_aggregate.argtypes = [_u32p, _i64, _f32p, _i64, _i64, _i32, _i64, _f32p]
    L.orc_requantize.argtypes = [_f32p, _i64, _i64, _f32, _f32p]
    L.orc_update_qcmd.argtypes = [_f32p, _i64, _f32p, _f32p, _vp, _f32, _f32, _f32]
    L.orc_update_qrda.argtypes = [_f32p, _i64, _f32p, _f32p, _f32p, _i64, _f32, _f32, _f32]
    L.orc_qrda_literal_f64.argtypes = [_f64p, _f64p, _i64, _i64, _f64, _f64, _f64p]
    L.orc_step_qcmd.argtypes = [_u32p, _i64, _f32p, _i64, _i64, _i32, _i64, _f32, _f32p, _f32p,
                                _vp, _f32, _f32, _f32, _i32]
    L.orc_step_qrda.argtypes = [_u32p, _i64, _f32p, _i64, _i64, _i32, _i64, _f32, _f32p, _f32p,
                                _f32p, _i64, _f32, _f32, _f32, _i32]
    L.orc_quantize_pack_segments.argtypes = [_f32p, _i64, _i64, _i32, _i64, _i64p, _i64p, _f32,
                                             _u32p, _i64, _f32p, _vp, _i64]
    L.orc_step_segments.argtypes = [_i32, _u32p, _i64, _f32p, _i64, _i64, _i32, _i64, _i64p, _i64p,
                                    _f32, _f32p, _f32p, _vp, _i64, _f32, _f32, _f32, _i32]
    L.orc_indicator.argtypes = [_i32, _f32p, _i64, _f32p, _f32p, _vp, _i64, _f32, _f32, _f32, _u32p]
    L.orc_indicator_or.argtypes = [_u32p, _i64, _i32, _i64, _u32p]
    L.orc_quantize_selected.argtypes = [_f32p, _u32p, _i64, _i64, _f32, _u32p, _u32p, _f32p, _f32p]
    L.orc_decode_selected.argtypes = [_u32p, _u32p, _i64, _i64, _u32p]
    L.orc_select_codes.argtypes = [_u32p, _u32p, _i64, _i64, _u32p, _u32p]
    L.orc_philox4x32_10.argtypes = [_u32p, _u32p, _u32p]
    L.orc_uniform.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, _i64]
    L.orc_uniform.restype = _f32
    L.orc_quantize_stochastic.argtypes = [_f32p, _i64, _i64, C.c_uint64, C.c_uint32, C.c_uint32, _i8p,
                                          _f32p]
    L.orc_local_grad_dense.argtypes = [_f32p, _i64, _i64, _f32p, _i32p, _i32, _f32p, _f32p,
                                       C.POINTER(_f32)]
    L.orc_local_grad_csr.argtypes = [_f32p, _i64p, _i32p, _i64, _i64, _f32p, _i32p, _i32, _f32p,
                                     _f32p, C.POINTER(_f32)]


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def n_buckets(d: int, bucket: int) -> int:
    b = bucket if bucket > 0 else d
    return (d + b - 1) // b


def n_words(d: int) -> int:
    return (d + 15) // 16


# ---- quantizer -------------------------------------------------------------------

def threshold_scale(v, thr_coef=0.75):
    v = np.ascontiguousarray(v, np.float32)
    D, s, c = _f32(), _f32(), _i64()
    lib().orc_threshold_scale(v, v.size, thr_coef, C.byref(D), C.byref(s), C.byref(c))
    return D.value, s.value, c.value


def scale_for_threshold(v, Delta):
    v = np.ascontiguousarray(v, np.float32)
    s, c = _f32(), _i64()
    lib().orc_scale_for_threshold(v, v.size, Delta, C.byref(s), C.byref(c))
    return s.value, c.value


def quantize(v, bucket=0, thr_coef=0.75, thresholds=None):
    """-> (codes int8[d], scales f32[nb], thresholds f32[nb])"""
    v = np.ascontiguousarray(v, np.float32)
    d = v.size
    nb = n_buckets(d, bucket)
    code = np.empty(d, np.int8)
    sc = np.empty(nb, np.float32)
    th = np.empty(nb, np.float32)
    tin = None
    if thresholds is not None:
        tin = np.ascontiguousarray(thresholds, np.float32)
        assert tin.size == nb
    lib().orc_quantize(v, d, bucket, thr_coef, code, sc, _ptr(th), _ptr(tin))
    return code, sc, th


def exact_threshold(v):
    """-> (smallest kept magnitude, scale, objective (sum kept)^2/k, kept count)"""
    v = np.ascontiguousarray(v, np.float32)
    a, s, o, k = _f64(), _f64(), _f64(), _i64()
    lib().orc_exact_threshold(v, v.size, C.byref(a), C.byref(s), C.byref(o), C.byref(k))
    return a.value, s.value, o.value, k.value


def exact_thresholds(v, bucket=0):
    """Per bucket, the strict threshold whose kept set {|v| > Delta} is the least-squares optimum."""
    v = np.ascontiguousarray(v, np.float32)
    th = np.empty(n_buckets(v.size, bucket), np.float32)
    lib().orc_exact_thresholds(v, v.size, bucket, th)
    return th


def pack(code):
    code = np.ascontiguousarray(code, np.int8)
    words = np.empty(n_words(code.size), np.uint32)
    lib().orc_pack(code, code.size, words)
    return words


def unpack(words, d):
    words = np.ascontiguousarray(words, np.uint32)
    assert words.size >= n_words(d)
    code = np.empty(d, np.int8)
    lib().orc_unpack(words, d, code)
    return code


def quantize_pack(g, bucket=0, thr_coef=0.75, thresholds=None, code_stride=None,
                  scale_stride=None):
    """g: f32[M, d] -> (codes u32[M, code_stride], scales f32[M, scale_stride],
    thresholds f32[M, scale_stride])"""
    g = np.ascontiguousarray(g, np.float32)
    M, d = g.shape
    W, nb = n_words(d), n_buckets(d, bucket)
    cs = code_stride or W
    ss = scale_stride or nb
    codes = np.zeros((M, cs), np.uint32)
    scales = np.zeros((M, ss), np.float32)
    given = thresholds is not None
    th = np.zeros((M, ss), np.float32)
    if given:
        th[:, :nb] = np.asarray(thresholds, np.float32).reshape(M, -1)[:, :nb]
    lib().orc_quantize_pack(g, d, d, M, bucket, thr_coef, codes, cs, scales, _ptr(th), ss,
                            1 if given else 0)
    return codes, scales, th


# ---- server ------------------------------------------------------------------------

def aggregate(codes, scales, d, bucket=0):
    codes = np.ascontiguousarray(codes, np.uint32)
    scales = np.ascontiguousarray(scales, np.float32)
    M = codes.shape[0]
    out = np.empty(d, np.float32)
    lib().orc_aggregate(codes, codes.shape[1], scales, scales.shape[1], d, M, bucket, out)
    return out


def requantize(gbar, bucket=0, thr_coef=0.75):
    gbar = np.ascontiguousarray(gbar, np.float32)
    q = np.empty_like(gbar)
    lib().orc_requantize(gbar, gbar.size, bucket, thr_coef, q)
    return q


# ---- updates (in place on x, G, z) ---------------------------------------------------

def _chk_state(*arrs):
    for a in arrs:
        if a is not None:
            assert a.dtype == np.float32 and a.flags.c_contiguous


def update_qcmd(q, x, G, z, eta, lam, delta):
    q = np.ascontiguousarray(q, np.float32)
    _chk_state(x, G, z)
    lib().orc_update_qcmd(q, q.size, x, G, _ptr(z), eta, lam, delta)


def update_qrda(q, x, G, z, t, eta, lam, delta):
    q = np.ascontiguousarray(q, np.float32)
    _chk_state(x, G, z)
    lib().orc_update_qrda(q, q.size, x, G, z, t, eta, lam, delta)


def qrda_literal_f64(z, H, t, eta, lam):
    z = np.ascontiguousarray(z, np.float64)
    H = np.ascontiguousarray(H, np.float64)
    out = np.empty_like(z)
    lib().orc_qrda_literal_f64(z, H, z.size, t, eta, lam, out)
    return out


def step_qcmd(codes, scales, d, bucket, x, G, z, eta, lam, delta, requant=REQUANT_NONE,
              thr_coef=0.75):
    codes = np.ascontiguousarray(codes, np.uint32)
    scales = np.ascontiguousarray(scales, np.float32)
    _chk_state(x, G, z)
    lib().orc_step_qcmd(codes, codes.shape[1], scales, scales.shape[1], d, codes.shape[0],
                        bucket, thr_coef, x, G, _ptr(z), eta, lam, delta, requant)


def step_qrda(codes, scales, d, bucket, x, G, z, t, eta, lam, delta, requant=REQUANT_NONE,
              thr_coef=0.75):
    codes = np.ascontiguousarray(codes, np.uint32)
    scales = np.ascontiguousarray(scales, np.float32)
    _chk_state(x, G, z)
    lib().orc_step_qrda(codes, codes.shape[1], scales, scales.shape[1], d, codes.shape[0],
                        bucket, thr_coef, x, G, z, t, eta, lam, delta, requant)


# ---- a list of tensors in one flat vector -------------------------------------------------

def quantize_pack_segments(g, begin, length, thr_coef=0.75):
    """g: f32[M, d]; tensor s = coordinates [begin[s], begin[s]+length[s]) ->
    (codes u32[M, ceil(d/16)] with untouched words 0, scales f32[M, n_seg], thresholds)"""
    g = np.ascontiguousarray(g, np.float32)
    begin = np.ascontiguousarray(begin, np.int64)
    length = np.ascontiguousarray(length, np.int64)
    M, d = g.shape
    codes = np.zeros((M, n_words(d)), np.uint32)
    scales = np.zeros((M, max(begin.size, 1)), np.float32)
    th = np.zeros_like(scales)
    lib().orc_quantize_pack_segments(g, d, d, M, begin.size, begin, length, thr_coef, codes,
                                     codes.shape[1], scales, _ptr(th), scales.shape[1])
    return codes, scales, th


def step_segments(method, codes, scales, d, begin, length, x, G, z, t, eta, lam, delta,
                  requant=False, thr_coef=0.75):
    codes = np.ascontiguousarray(codes, np.uint32)
    scales = np.ascontiguousarray(scales, np.float32)
    begin = np.ascontiguousarray(begin, np.int64)
    length = np.ascontiguousarray(length, np.int64)
    _chk_state(x, G, z)
    lib().orc_step_segments(method, codes, codes.shape[1], scales, scales.shape[1], d,
                            codes.shape[0], begin.size, begin, length, thr_coef, x, G, _ptr(z),
                            t, eta, lam, delta, 1 if requant else 0)


# ---- local gradient --------------------------------------------------------------------

def local_grad_dense(A, y, batch_rows, x):
    A = np.ascontiguousarray(A, np.float32)
    y = np.ascontiguousarray(y, np.float32)
    rows = np.ascontiguousarray(batch_rows, np.int32)
    x = np.ascontiguousarray(x, np.float32)
    n, d = A.shape
    g = np.empty(d, np.float32)
    loss = _f32()
    lib().orc_local_grad_dense(A, n, d, y, rows, rows.size, x, g, C.byref(loss))
    return g, loss.value


def local_grad_csr(vals, indptr, indices, d, y, batch_rows, x):
    vals = np.ascontiguousarray(vals, np.float32)
    indptr = np.ascontiguousarray(indptr, np.int64)
    indices = np.ascontiguousarray(indices, np.int32)
    y = np.ascontiguousarray(y, np.float32)
    rows = np.ascontiguousarray(batch_rows, np.int32)
    x = np.ascontiguousarray(x, np.float32)
    g = np.empty(d, np.float32)
    loss = _f32()
    lib().orc_local_grad_csr(vals, indptr, indices, indptr.size - 1, d, y, rows, rows.size, x, g,
                             C.byref(loss))
    return g, loss.value


# ---- indicator / selection / sparse encoding ---------------------------------------------

QCMD, QRDA = 0, 1


def n_ind_words(d: int) -> int:
    return (d + 31) // 32


def indicator(method, g, x, G, z, t, eta, lam, delta):
    """-> u32[ceil(d/32)]: bit i set iff x_i != 0 or the worker's own update of x_i is != 0."""
    g = np.ascontiguousarray(g, np.float32)
    _chk_state(x, G, z)
    out = np.empty(n_ind_words(g.size), np.uint32)
    lib().orc_indicator(method, g, g.size, x, G, _ptr(z), t, eta, lam, delta, out)
    return out


def indicator_or(ind, d):
    ind = np.ascontiguousarray(ind, np.uint32)
    out = np.empty(n_ind_words(d), np.uint32)
    lib().orc_indicator_or(ind, ind.shape[1], ind.shape[0], d, out)
    return out


def quantize_selected(g, ind, bucket=0, thr_coef=0.75):
    """-> (sel_codes u32[nb*area], counts u32[nb], scales f32[nb], thresholds f32[nb]);
    area = ceil(bucket_len/16) words per bucket, only the first ceil(count/16) are written."""
    g = np.ascontiguousarray(g, np.float32)
    ind = np.ascontiguousarray(ind, np.uint32)
    d = g.size
    nb = n_buckets(d, bucket)
    b = bucket if bucket > 0 else d
    area = (b + 15) // 16
    sel = np.zeros(nb * area, np.uint32)
    cnt = np.zeros(nb, np.uint32)
    sc = np.zeros(nb, np.float32)
    th = np.zeros(nb, np.float32)
    lib().orc_quantize_selected(g, ind, d, bucket, thr_coef, sel, cnt, sc, th)
    return sel, cnt, sc, th


def select_codes(dense_words, ind, d, bucket=0):
    """Codes of the marked components of one dense message -> (sel_codes u32[nb*area], counts)."""
    dense_words = np.ascontiguousarray(dense_words, np.uint32)
    ind = np.ascontiguousarray(ind, np.uint32)
    nb = n_buckets(d, bucket)
    b = bucket if bucket > 0 else d
    area = (b + 15) // 16
    sel = np.zeros(nb * area, np.uint32)
    cnt = np.zeros(nb, np.uint32)
    lib().orc_select_codes(dense_words, ind, d, bucket, sel, cnt)
    return sel, cnt


def decode_selected(ind, sel_codes, d, bucket=0):
    ind = np.ascontiguousarray(ind, np.uint32)
    sel_codes = np.ascontiguousarray(sel_codes, np.uint32)
    out = np.empty(n_words(d), np.uint32)
    lib().orc_decode_selected(ind, sel_codes, d, bucket, out)
    return out


# ---- stochastic ternary quantizer ---------------------------------------------------------

def philox4x32_10(ctr, key):
    out = np.empty(4, np.uint32)
    lib().orc_philox4x32_10(np.asarray(ctr, np.uint32), np.asarray(key, np.uint32), out)
    return out


def uniform(seed, step, m, i):
    return float(lib().orc_uniform(seed, step, m, i))


def quantize_stochastic(v, bucket=0, seed=0, step=0, m=0):
    """-> (codes int8[d], scales f32[nb]) of the max-norm stochastic ternary quantizer."""
    v = np.ascontiguousarray(v, np.float32)
    code = np.empty(v.size, np.int8)
    sc = np.empty(n_buckets(v.size, bucket), np.float32)
    lib().orc_quantize_stochastic(v, v.size, bucket, seed, step, m, code, sc)
    return code, sc


def quantize_pack_stochastic(g, bucket=0, seed=0, step=0):
    g = np.ascontiguousarray(g, np.float32)
    M, d = g.shape
    codes = np.zeros((M, n_words(d)), np.uint32)
    scales = np.zeros((M, n_buckets(d, bucket)), np.float32)
    for m in range(M):
        c, s = quantize_stochastic(g[m], bucket, seed, step, m)
        codes[m] = pack(c)
        scales[m] = s
    return codes, scales
