"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, sizes workspaces, and rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
qa = pytest.importorskip("paper_2208_05631_amd", reason="libqadagrad.so not built")
from paper_2208_05631_amd import binding as B  # noqa: E402


def test_every_declared_symbol_is_exported():
    hdr = open(os.path.join(ROOT, "include", "qadagrad.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(qa_[a-z_]+)\s*\(", hdr))
    assert {"qa_local_grad", "qa_local_grad_batched", "qa_quantize_pack", "qa_aggregate_unpack", "qa_step_qcmd",
            "qa_step_qrda", "qa_workspace_bytes", "qa_strerror", "qa_version"} <= names
    lib = C.CDLL(B.lib_path())
    for n in names:
        assert hasattr(lib, n), n
    assert qa.qa_version() == 100


def test_binding_mirrors_the_header_names():
    for n in ("qa_local_grad", "qa_quantize_pack", "qa_aggregate_unpack", "qa_step_qcmd",
              "qa_step_qrda", "qa_workspace_bytes", "qa_strerror", "qa_version"):
        assert callable(getattr(qa, n))


def test_error_strings():
    for code in range(0, -6, -1):
        assert "unknown" not in qa.qa_strerror(code)
    assert "unknown" in qa.qa_strerror(-99)


def test_workspace_sizes():
    L = qa.Layout.make(10**6, 8, 4096)
    assert qa.qa_workspace_bytes(L, qa.QA_OP_QUANTIZE) == 0          # single pass, no scratch
    Lg = qa.Layout.make(10**6, 8, 0)
    nt = (10**6 + 4095) // 4096
    assert qa.qa_workspace_bytes(Lg, qa.QA_OP_QUANTIZE) >= 8 * nt * 12
    # the exact threshold: nothing more for buckets inside a tile; a sort's worth of scratch
    # (two buffers of 64-bit keys, independent of the worker count) for buckets that span tiles
    assert qa.qa_workspace_bytes(L, qa.QA_OP_QUANTIZE_EXACT) == 0
    more = qa.qa_workspace_bytes(Lg, qa.QA_OP_QUANTIZE_EXACT) - qa.qa_workspace_bytes(Lg, qa.QA_OP_QUANTIZE)
    assert 16 * 10**6 <= more <= 22 * 10**6
    assert qa.qa_workspace_bytes(L, qa.QA_OP_STEP) >= 4 * 10**6       # averaged vector for GLOBAL
    assert qa.qa_workspace_bytes(L, qa.QA_OP_GRAD_CSR) >= 8 * 8 * 10**6      # M = 8 accumulators
    assert 0 < qa.qa_workspace_bytes(L, qa.QA_OP_GRAD_DENSE) < 8 * 10**6
    bad = qa.Layout.make(10**6, 8, 100)                               # not a power of two
    assert qa.qa_workspace_bytes(bad, qa.QA_OP_STEP) == 0


FAKE = 0x10000        # non-null, 16-byte aligned, never dereferenced: checks fail first


def _step(L, codes=FAKE, scales=FAKE, x=FAKE, G=FAKE, z=None, eta=0.1, lam=0.0, delta=1e-8,
          requant=0, ws=None, wsb=0):
    return B._lib.qa_step_qcmd(C.byref(L), codes, scales, x, G, z, eta, lam, delta, requant, ws, wsb,
                               None)


def test_step_argument_checks():
    ok = qa.Layout.make(1000, 4, 0)
    assert _step(ok, codes=None) == -1
    assert _step(ok, x=None) == -1
    assert _step(ok, eta=0.0) == -1
    assert _step(ok, lam=-1.0) == -1
    assert _step(ok, delta=0.0) == -1
    assert _step(ok, requant=7) == -1
    assert _step(ok, requant=qa.QA_REQUANT_BUCKET) == -1             # no buckets in this layout
    assert _step(ok, x=FAKE + 4) == -2
    big = qa.Layout.make(10000, 4, 0)                                # more than one tile
    assert _step(big, requant=qa.QA_REQUANT_GLOBAL) == -3            # needs a workspace
    assert _step(big, requant=qa.QA_REQUANT_GLOBAL, ws=FAKE, wsb=16) == -3
    for bad in (qa.Layout.make(0, 4, 0), qa.Layout.make(1000, 0, 0), qa.Layout.make(1000, 4, 100),
                qa.Layout.make(1000, 4, 32), qa.Layout.make(1000, 4, 0, code_stride=10),
                qa.Layout.make(1000, 4, 64, scale_stride=3), qa.Layout.make(1000, 4, 0, thr_coef=0.0)):
        assert _step(bad) == -1
    assert B._lib.qa_step_qrda(C.byref(ok), FAKE, FAKE, FAKE, FAKE, None, 1, 0.1, 0.0, 1e-8, 0, None,
                               0, None) == -1                        # z is required
    assert B._lib.qa_step_qrda(C.byref(ok), FAKE, FAKE, FAKE, FAKE, FAKE, 0, 0.1, 0.0, 1e-8, 0, None,
                               0, None) == -1                        # t >= 1


def test_quantize_and_aggregate_argument_checks():
    ok = qa.Layout.make(1000, 4, 0)
    q = B._lib.qa_quantize_pack
    assert q(C.byref(ok), None, 1000, FAKE, FAKE, None, 0, FAKE, 1 << 20, None) == -1
    assert q(C.byref(ok), FAKE, 999, FAKE, FAKE, None, 0, FAKE, 1 << 20, None) == -1    # stride < d
    assert q(C.byref(ok), FAKE, 1002, FAKE, FAKE, None, 0, FAKE, 1 << 20, None) == -1   # not % 4
    assert q(C.byref(ok), FAKE, 1000, FAKE, FAKE, None, 1, FAKE, 1 << 20, None) == -1   # given, null
    assert q(C.byref(ok), FAKE, 1000, FAKE, FAKE, None, 4, FAKE, 1 << 20, None) == -1   # unknown flag
    assert q(C.byref(ok), FAKE, 1000, FAKE, FAKE, None, 2, FAKE, 1 << 20, None) == -1   # exact, null
    assert q(C.byref(ok), FAKE, 1000, FAKE, FAKE, FAKE, 3, FAKE, 1 << 20, None) == -1   # given and exact
    assert q(C.byref(ok), FAKE + 4, 1000, FAKE, FAKE, None, 0, FAKE, 1 << 20, None) == -2
    big = qa.Layout.make(10000, 4, 0)                                # more than one tile: two passes
    assert q(C.byref(big), FAKE, 10000, FAKE, FAKE, None, 0, None, 0, None) == -3
    assert B._lib.qa_aggregate_unpack(C.byref(ok), FAKE, FAKE, None, None) == -1
    assert B._lib.qa_aggregate_unpack(C.byref(ok), FAKE, FAKE, FAKE + 8, None) == -2


def test_local_grad_argument_checks():
    f = B._lib.qa_local_grad
    assert f(5, FAKE, None, None, 10, 10, FAKE, FAKE, 4, FAKE, FAKE, None, FAKE, 1 << 30, None) == -1
    assert f(1, FAKE, None, None, 10, 10, FAKE, FAKE, 4, FAKE, FAKE, None, FAKE, 1 << 30, None) == -1
    assert f(0, FAKE, None, None, 10, 10, FAKE, FAKE, 0, FAKE, FAKE, None, FAKE, 1 << 30, None) == -1
    assert f(0, FAKE, None, None, 10, 10, FAKE, FAKE, 4, FAKE, FAKE, None, None, 0, None) == -3
    assert f(0, FAKE, None, None, 10, 10, FAKE, FAKE, 4, FAKE, FAKE + 4, None, FAKE, 1 << 30, None) == -2


def test_segment_plan_argument_checks():
    """The tensor table is validated on the host before anything is copied to the device."""
    init = B._lib.qa_segment_plan_init
    init.argtypes = [C.c_int64, C.c_int64, C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.c_void_p,
                     C.c_size_t, C.POINTER(B.SegmentPlan), C.c_void_p]
    plan = B.SegmentPlan()

    def run(d, begin, length, table=FAKE, nbytes=1 << 20):
        n = len(begin)
        return init(d, n, (C.c_int64 * max(n, 1))(*begin), (C.c_int64 * max(n, 1))(*length), table,
                    nbytes, C.byref(plan), None)

    assert run(1000, [0, 8], [4, 4]) == -1              # begin not a multiple of 16
    assert run(1000, [0, 16], [20, 4]) == -1            # overlap
    assert run(1000, [32, 0], [4, 4]) == -1             # not ascending
    assert run(1000, [0, 992], [4, 9]) == -1            # runs past d
    assert run(1000, [0], [-1]) == -1
    assert run(0, [0], [0]) == -1
    assert run(1000, [], []) == -1                      # at least one tensor
    assert run(1000, [0], [4], table=None) == -1
    assert run(1000, [0], [4], table=FAKE + 4) == -2
    assert run(1 << 20, [0], [1 << 20], nbytes=64) == -3
    assert qa.qa_segment_plan_bytes(1 << 20, 10) == 8 * (4 + 20 + 11 + 2 * (256 + 10))
    assert qa.qa_segment_plan_bytes(0, 10) == 0 and qa.qa_segment_plan_bytes(100, 0) == 0
    bad = B.SegmentPlan(1000, 1, 1, None)
    assert qa.qa_segment_workspace_bytes(B.SegmentPlan(1000, 3, 3, FAKE), 4, qa.QA_OP_QUANTIZE) > 0
    ok = qa.Layout.make(1000, 4, 0)
    B._lib.qa_quantize_pack_segments.argtypes = [C.POINTER(qa.Layout), C.POINTER(B.SegmentPlan), C.c_void_p,
                                                 C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                                 C.c_size_t, C.c_void_p]
    assert B._lib.qa_quantize_pack_segments(C.byref(ok), C.byref(bad), FAKE, 1000, FAKE, FAKE, None, FAKE,
                                            1 << 20, None) == -1            # plan without table


def _plan_host(d, begin, length):
    f = B._lib.qa_segment_plan_host
    f.argtypes = [C.c_int64, C.c_int64, C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.POINTER(C.c_int64),
                  C.c_size_t, C.POINTER(C.c_int64)]
    n = len(begin)
    nbytes = qa.qa_segment_plan_bytes(d, n)
    table = (C.c_int64 * (nbytes // 8))()
    npieces = C.c_int64(-1)
    rc = f(d, n, (C.c_int64 * max(n, 1))(*begin), (C.c_int64 * max(n, 1))(*length), table, nbytes,
           C.byref(npieces))
    return rc, npieces.value, list(table)


def test_segment_table_against_a_python_reference():
    """The piece table (built on the host, the same words that are copied to the device): every
    (4096-tile, tensor) intersection exactly once, in order, for seeded random tensor lists."""
    import random
    rnd = random.Random(12)
    for _ in range(200):
        n = rnd.randint(1, 12)
        begin, length, pos = [], [], rnd.choice([0, 16, 4096, 4080])
        for _ in range(n):
            begin.append(pos)
            ln = rnd.choice([0, 1, 15, 16, 17, 4095, 4096, 4097, rnd.randint(0, 30000)])
            length.append(ln)
            pos = (pos + ln + 15) // 16 * 16 + 16 * rnd.choice([0, 0, 1, 300])
        d = pos + rnd.randint(0, 5) if pos > 0 else 1
        rc, npieces, t = _plan_host(d, begin, length)
        assert rc == 0
        want = [(T, s) for s in range(n) if length[s] > 0
                for T in range(begin[s] // 4096, (begin[s] + length[s] - 1) // 4096 + 1)]
        assert npieces == len(want) and npieces <= (d + 4095) // 4096 + n
        assert t[1:4] == [d, n, npieces]
        o = 4
        assert t[o:o + n] == begin and t[o + n:o + 2 * n] == length
        first = t[o + 2 * n:o + 3 * n + 1]
        tiles = t[o + 3 * n + 1:o + 3 * n + 1 + npieces]
        segs = t[o + 3 * n + 1 + npieces:o + 3 * n + 1 + 2 * npieces]
        assert list(zip(tiles, segs)) == want
        for s in range(n):
            assert segs[first[s]:first[s + 1]] == [s] * (first[s + 1] - first[s])
        assert first[0] == 0 and first[n] == npieces
    assert _plan_host(1000, [0, 8], [4, 4])[0] == -1
