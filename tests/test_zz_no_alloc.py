"""The entry point that allocates nothing (qa_quantize_pack_static: the multi-pass quantizer with
its partial sums in the library's own static device array) against qa_quantize_pack with a
caller's workspace: bit for bit, on two calls in a row, the second on a smaller input, so that
whatever the first call left in the shared array must not leak into the second."""
import ctypes as C

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2208_05631_amd as qa
    from paper_2208_05631_amd import binding as B
    from gpu_util import DEV, dev, host, workspace


def both_ways(g, bucket, flags=0, thresholds=None):
    M, d = g.shape
    L = qa.Layout.make(d, M, bucket)
    gs = ((d + 3) // 4) * 4
    gp = np.zeros((M, gs), np.float32)
    gp[:, :d] = g
    gd = dev(gp)
    out = []
    for static in (False, True):
        codes = torch.full((M, L.code_stride), -1, dtype=torch.int32, device=DEV)
        scales = torch.full((M, L.scale_stride), -7.0, dtype=torch.float32, device=DEV)
        th = torch.full((M, L.scale_stride), -7.0, dtype=torch.float32, device=DEV)
        if thresholds is not None:
            th.copy_(dev(thresholds))
        if static:
            qa.qa_quantize_pack_static(L, gd, gs, codes, scales, th, flags)
        else:
            ws = workspace(qa.qa_workspace_bytes(L, qa.QA_OP_QUANTIZE))
            qa.qa_quantize_pack(L, gd, gs, codes, scales, th, flags, ws)
        torch.cuda.synchronize()
        out.append((host(codes).view(np.uint32), host(scales), host(th)))
    return out


@pytest.mark.parametrize("bucket", [0, 16384])
def test_static_scratch_quantizer_equals_the_workspace_one_on_two_calls_in_a_row(bucket):
    rng = np.random.default_rng(31)
    # first call: 3 workers x 18 tiles (ragged tail); second call: smaller in both dimensions
    for M, d in ((3, 70001), (2, 20011)):
        g = (rng.standard_normal((M, d)) * 1e-2 * (rng.random((M, d)) < 0.4)).astype(np.float32)
        assert qa.qa_workspace_bytes(qa.Layout.make(d, M, bucket), qa.QA_OP_QUANTIZE) > 0
        (c0, s0, t0), (c1, s1, t1) = both_ways(g, bucket)
        assert c0.any() and s0[:, 0].all()
        assert np.array_equal(c0, c1), (M, d)
        assert np.array_equal(s0.view(np.uint32), s1.view(np.uint32)), (M, d)
        assert np.array_equal(t0.view(np.uint32), t1.view(np.uint32)), (M, d)
    # thresholds given by the caller: the array's threshold slots are not used at all
    nb = qa.Layout.make(20011, 2, bucket).n_buckets
    thr = np.full((2, nb), 3e-3, np.float32)
    (c0, s0, _), (c1, s1, _) = both_ways(g, bucket, qa.QA_THRESH_GIVEN, thr)
    assert np.array_equal(c0, c1) and np.array_equal(s0.view(np.uint32), s1.view(np.uint32))


def test_static_scratch_quantizer_without_scratch_and_beyond_its_limit():
    # single-pass layouts use no scratch and have no size limit
    rng = np.random.default_rng(32)
    g = (rng.standard_normal((2, 9000)) * 1e-2).astype(np.float32)
    for bucket in (4096, 256):
        (c0, s0, t0), (c1, s1, t1) = both_ways(g, bucket)
        assert np.array_equal(c0, c1) and np.array_equal(s0.view(np.uint32), s1.view(np.uint32))
    # more partials than the array holds: refused before anything is launched or touched
    big = qa.Layout.make(1 << 31, 1, 0)
    assert qa.qa_workspace_bytes(big, qa.QA_OP_QUANTIZE) > 4 << 20
    fake = 0x10000
    rc = B._lib.qa_quantize_pack_static(C.byref(big), fake, 1 << 31, fake, fake, None, 0, None)
    assert rc == -6 and "static" in qa.qa_strerror(rc)
