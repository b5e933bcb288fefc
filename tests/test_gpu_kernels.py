"""Parity of each HIP kernel with the CPU oracle on identical seeded inputs, element by
element, through the C ABI.  Integer work (codes, zero sets) must be bit-exact; binary32
state is expected bit-exact too (both sides follow the same arithmetic contract) and is
asserted within the stated tolerance of 1e-5 max relative error, with exactness reported."""
import numpy as np
import pytest
import torch

import oracle
from paper_2208_05631_amd import synth

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2208_05631_amd as qa
    from gpu_util import DEV, GpuState, dev, gpu_quantize_pack, host, quantizer_parity, ulp_distance, workspace

RTOL = 1e-5


def make_grad(kind, M, d, seed):
    rng = np.random.default_rng(seed)
    if kind == "gauss":
        g = rng.standard_normal((M, d)) * 1e-2 + rng.standard_normal((M, 1)) * 3e-3
    elif kind == "laplace_sparse":
        g = rng.laplace(0, 1e-3, (M, d)) * (rng.random((M, d)) < 0.05)
    elif kind == "student":
        g = rng.standard_t(3, (M, d)) * 1e-2 * (rng.random((M, d)) < 0.1)
    elif kind == "mixed_scale":
        g = rng.standard_normal((M, d)) * (10.0 ** rng.integers(-6, 3, (M, 1)))
    elif kind == "zeros":
        g = np.zeros((M, d))
    else:
        raise ValueError(kind)
    return g.astype(np.float32)


def assert_close(a, b, what):
    assert a.shape == b.shape, what
    if np.array_equal(a, b):
        return
    denom = np.maximum(np.abs(b), 1e-30)
    err = np.max(np.abs(a.astype(np.float64) - b) / denom)
    assert err <= RTOL, f"{what}: max rel err {err}"


# ------------------------------------------------------------------ quantize + pack

QP_CASES = [
    # d, M, bucket
    (1, 1, 0), (15, 2, 0), (16, 1, 64), (17, 3, 64), (1000, 4, 0), (1000, 2, 256),
    (4096, 2, 4096), (4097, 2, 4096), (10000, 3, 1024), (10000, 3, 2048), (12289, 2, 512),
    (70001, 2, 4096), (70001, 2, 8192), (70001, 2, 65536), (70001, 3, 0), (300000, 2, 128),
]


@pytest.mark.parametrize("d,M,bucket", QP_CASES)
@pytest.mark.parametrize("kind", ["gauss", "laplace_sparse"])
def test_quantize_pack_matches_oracle(d, M, bucket, kind):
    g = make_grad(kind, M, d, seed=d * 7 + M)
    oc, osc, oth = oracle.quantize_pack(g, bucket=bucket)
    codes, scales, th, L = gpu_quantize_pack(g, bucket)
    # bit-identical, or (about once in 2^29 sums) a threshold / scale one ulp off with codes that
    # are exact for the GPU's own threshold
    assert quantizer_parity(g, bucket, codes, scales, th) <= 1


_MID = []


def mid_size_gradient():
    """4 workers x 2^26 coordinates, 30 % non-zero, Laplace(0, 1e-3) magnitudes; drawn on the
    device by the seeded input generator and copied to the host once."""
    if not _MID:
        _MID.append(np.stack([host(synth.grad_laplace_sparse(1 << 26, m, 1, seed=2024, keep=0.3,
                                                             device=DEV)) for m in range(4)]))
    return _MID[0]


@pytest.mark.parametrize("bucket", [4096, 256, 0])
def test_every_threshold_and_scale_at_a_mid_size(bucket):
    """All buckets of a 2^26-coordinate message from each of 4 workers (2 x 65 536 sums per worker
    at bucket 4096, 16 times that at 256): thresholds, scales and codes against the oracle.  The
    two sides add the same binary64 terms in different orders, so a rounded sum may differ in its
    last binary32 bit about once in 2^29 sums: the count of such buckets is reported, each must
    lie within one ulp, and the codes must be exact for the GPU's own thresholds."""
    g = mid_size_gradient()
    M, d = g.shape
    codes, scales, th, L = gpu_quantize_pack(g, bucket)
    off = quantizer_parity(g, bucket, codes, scales, th)
    print(f"bucket {bucket}: {off} of {M * L.n_buckets} (worker, bucket) pairs not bit-identical")
    assert off <= 4


@pytest.mark.parametrize("bucket", [4096, 1024, 0])
def test_quantizer_on_magnitudes_spread_over_many_binades(bucket):
    """Partial sums of a bucket are exact in binary64 only while the magnitudes span few enough
    binades (span + log2 n + 24 <= 53); beyond that each side rounds its own partial sums.  With
    magnitudes over 60 binades the results may therefore differ, but only in the last bit."""
    d, M = 50000, 3
    rng = np.random.default_rng(77)
    g = (rng.standard_normal((M, d)) * np.exp2(rng.integers(-40, 20, (M, d)))).astype(np.float32)
    codes, scales, th, L = gpu_quantize_pack(g, bucket)
    off = quantizer_parity(g, bucket, codes, scales, th)
    print(f"bucket {bucket}: {off} of {M * L.n_buckets} (worker, bucket) pairs not bit-identical")


def test_quantize_pack_strides_and_untouched_padding():
    d, M, b = 5000, 3, 1024
    g = make_grad("gauss", M, d, 5)
    codes, scales, th, L = gpu_quantize_pack(g, b, code_stride=400, scale_stride=9, g_stride=5008)
    oc, osc, oth = oracle.quantize_pack(g, bucket=b, code_stride=400, scale_stride=9)
    W, nb = L.words, L.n_buckets
    assert np.array_equal(codes[:, :W], oc[:, :W]) and np.array_equal(scales[:, :nb], osc[:, :nb])
    assert np.all(codes[:, W:] == 0xFFFFFFFF) and np.all(scales[:, nb:] == -7.0)   # not written


@pytest.mark.parametrize("bucket", [0, 256, 4096, 16384])
def test_quantize_pack_with_given_thresholds(bucket):
    d, M = 40000, 2
    g = make_grad("gauss", M, d, 11)
    nb = oracle.n_buckets(d, bucket)
    rng = np.random.default_rng(1)
    thr = (rng.random((M, nb)) * 1e-2).astype(np.float32)
    oc, osc, _ = oracle.quantize_pack(g, bucket=bucket, thresholds=thr)
    codes, scales, th, L = gpu_quantize_pack(g, bucket, thresholds=thr)
    assert np.array_equal(codes, oc) and np.array_equal(scales[:, :nb], osc[:, :nb])
    assert np.array_equal(th[:, :nb], thr)                                          # left as given


@pytest.mark.parametrize("bucket", [0, 64, 4096])
def test_quantize_degenerate_inputs(bucket):
    d, M = 9000, 2
    g = make_grad("zeros", M, d, 0)
    g[1, 100] = np.nan            # poisons its bucket only: threshold NaN, codes 0, scale 0
    g[1, 8000:] = 0.5
    oc, osc, oth = oracle.quantize_pack(g, bucket=bucket)
    codes, scales, th, L = gpu_quantize_pack(g, bucket)
    nb = L.n_buckets
    assert np.array_equal(codes, oc)
    assert np.array_equal(scales[:, :nb], osc[:, :nb])
    assert np.array_equal(np.isnan(th[:, :nb]), np.isnan(oth[:, :nb]))
    assert np.array_equal(np.nan_to_num(th[:, :nb]), np.nan_to_num(oth[:, :nb]))
    assert not codes[0].any() and not scales[0, :nb].any()


# ------------------------------------------------------------------ aggregate

@pytest.mark.parametrize("d,M,bucket", [(1, 1, 0), (1000, 4, 0), (5000, 3, 64), (70001, 6, 4096),
                                        (70001, 64, 4096), (33333, 7, 16384), (20000, 33, 1024),
                                        # complete chunks of 16 and of 8 workers whose last tile ends
                                        # inside a 16-byte group of a row of code words
                                        (9000, 48, 4096), (8192 + 16 * 5 + 3, 8, 4096), (70001, 24, 0),
                                        (4096 + 16 * 62 + 1, 32, 8192)])
def test_aggregate_matches_oracle(d, M, bucket):
    g = make_grad("mixed_scale" if M <= 7 else "gauss", M, d, seed=M + d)
    oc, osc, _ = oracle.quantize_pack(g, bucket=bucket)
    L = qa.Layout.make(d, M, bucket)
    out = torch.full((d,), 9.0, dtype=torch.float32, device=DEV)
    qa.qa_aggregate_unpack(L, dev(oc.view(np.int32)), dev(osc), out)
    torch.cuda.synchronize()
    assert np.array_equal(host(out), oracle.aggregate(oc, osc, d, bucket=bucket))


@pytest.mark.parametrize("d,M,bucket", [(70001, 64, 4096), (50000, 130, 8192), (9000, 70, 0),
                                        (20000, 5, 4096)])
def test_aggregate_with_widely_spread_scales_takes_the_ordered_path(d, M, bucket):
    """Scales spanning > 29 - log2(M) binades inside a bucket: the sum is no longer exact in
    binary64, so only worker order reproduces the oracle's rounding."""
    rng = np.random.default_rng(M)
    g = rng.standard_normal((M, d)).astype(np.float32) * (2.0 ** rng.integers(-40, 40, (M, 1))).astype(np.float32)
    oc, osc, _ = oracle.quantize_pack(g, bucket=bucket)
    L = qa.Layout.make(d, M, bucket)
    out = torch.zeros(d, dtype=torch.float32, device=DEV)
    qa.qa_aggregate_unpack(L, dev(oc.view(np.int32)), dev(osc), out)
    torch.cuda.synchronize()
    ref = oracle.aggregate(oc, osc, d, bucket=bucket)
    assert np.array_equal(host(out), ref)
    # half the buckets get narrow spans again: both paths inside one launch
    nb = L.n_buckets
    osc2 = osc.copy()
    osc2[:, : max(1, nb // 2)] = (1e-3 * (1 + rng.random((M, max(1, nb // 2))))).astype(np.float32)
    qa.qa_aggregate_unpack(L, dev(oc.view(np.int32)), dev(osc2), out)
    torch.cuda.synchronize()
    assert np.array_equal(host(out), oracle.aggregate(oc, osc2, d, bucket=bucket))


def test_aggregate_with_nonfinite_scale_matches_oracle():
    d, M, b = 10000, 8, 4096
    g = make_grad("gauss", M, d, 9)
    oc, osc, _ = oracle.quantize_pack(g, bucket=b)
    osc[3, 1] = np.inf                      # inf * 0 = NaN, inf * +-1 = +-inf: bucket 1 is poisoned
    out = torch.zeros(d, dtype=torch.float32, device=DEV)
    qa.qa_aggregate_unpack(qa.Layout.make(d, M, b), dev(oc.view(np.int32)), dev(osc), out)
    torch.cuda.synchronize()
    ref = oracle.aggregate(oc, osc, d, bucket=b)
    assert not np.isfinite(ref[4096:8192]).any() and np.isfinite(ref[:4096]).all()
    assert np.array_equal(host(out), ref, equal_nan=True)


def test_aggregate_reads_reserved_pattern_as_zero_and_ignores_tail_bits():
    d, M = 40, 2
    rng = np.random.default_rng(3)
    words = rng.integers(0, 2 ** 32, (M, 3), dtype=np.uint64).astype(np.uint32)   # all 4 patterns
    scales = np.array([[0.5], [0.25]], np.float32)
    for bucket in (0, 64):                 # table-driven sum / worker-ordered sum
        L = qa.Layout.make(d, M, bucket)
        out = torch.zeros(d, dtype=torch.float32, device=DEV)
        qa.qa_aggregate_unpack(L, dev(words.view(np.int32)), dev(scales), out)
        torch.cuda.synchronize()
        assert np.array_equal(host(out), oracle.aggregate(words, scales, d, bucket=bucket))


# ------------------------------------------------------------------ fused steps

STEP_CASES = [
    # d, M, bucket, requant
    (1, 1, 0, 0), (1000, 4, 0, 0), (1000, 4, 0, 2), (4096, 8, 4096, 0), (4097, 8, 4096, 1),
    (10000, 3, 64, 1), (10000, 5, 256, 1), (10000, 16, 1024, 1), (10000, 2, 2048, 1),
    (70001, 64, 4096, 0), (70001, 32, 4096, 1), (70001, 6, 4096, 2), (70001, 4, 16384, 1),
    (70001, 4, 16384, 0), (300001, 8, 4096, 0), (50001, 130, 4096, 0), (50001, 67, 4096, 1),
    (20000, 128, 4096, 1),
    # chunking of the table-driven kernel: 3 chunks of 8, 3 chunks of 16, guarded chunks (20 = 16 + 4, 12)
    (9000, 24, 4096, 0), (9000, 48, 4096, 1), (9000, 20, 0, 0), (9000, 12, 4096, 2), (9000, 40, 8192, 0),
    # buckets smaller than the tile without in-kernel second quantization: per-thread scales
    (10000, 3, 64, 0), (10000, 9, 256, 0), (70001, 16, 1024, 0), (70001, 64, 2048, 2), (4100, 8, 512, 2),
    # the largest worker count the layout accepts, and a large odd one
    (5000, 4096, 4096, 0), (3000, 1001, 0, 2),
    # second quantization over buckets that span tiles: few workers (the average is formed from the
    # messages in every pass) with chunks of 16, 8, 4 and guarded chunks; many workers (the average
    # is written to the workspace once)
    (70001, 16, 0, 2), (70001, 8, 8192, 1), (70001, 3, 0, 2), (70001, 13, 16384, 1), (9000, 16, 64, 2),
    (70001, 24, 0, 2), (70001, 20, 16384, 1),
    # ... and where that second quantization is a one-pass one although it is not formed in the
    # step kernel (single tile, messages with smaller buckets), or spans "several" tiles of one
    (3000, 4, 64, 2), (4096, 8, 1024, 2), (50, 3, 8192, 1),
]


@pytest.mark.parametrize("d,M,bucket,requant", STEP_CASES)
def test_fused_steps_match_oracle_over_several_steps(d, M, bucket, requant):
    eta, lam, delta = 0.1, 2e-4, 1e-8
    rng = np.random.default_rng(d + M)
    x0 = (rng.standard_normal(d) * 1e-2 * (rng.random(d) < 0.5)).astype(np.float32)
    ox, oG, oz = x0.copy(), np.zeros(d, np.float32), np.zeros(d, np.float32)
    L = qa.Layout.make(d, M, bucket)
    st = None
    T = 6
    for t in range(1, T + 1):
        g = make_grad("gauss" if t % 2 else "laplace_sparse", M, d, seed=1000 * t + d)
        oc, osc, _ = oracle.quantize_pack(g, bucket=bucket)
        if st is None:
            st = GpuState(L, oc, osc, ox, oG, oz)
        else:
            st.codes.copy_(dev(oc.view(np.int32)))
            st.scales.copy_(dev(osc))
        if t % 3 == 0:                       # QRDA steps overwrite x from (z, G, t)
            oracle.step_qrda(oc, osc, d, bucket, ox, oG, oz, t, eta, lam, delta, requant)
            st.qrda(t, eta, lam, delta, requant)
        else:                                # QCMD steps keep z current
            oracle.step_qcmd(oc, osc, d, bucket, ox, oG, oz, eta, lam, delta, requant)
            st.qcmd(eta, lam, delta, requant, track_z=True)
        x, G, z = st.get()
        assert np.array_equal(x == 0, ox == 0), f"zero set differs at step {t}"
        assert_close(G, oG, f"G step {t}")
        assert_close(z, oz, f"z step {t}")
        assert_close(x, ox, f"x step {t}")
    assert np.array_equal(x, ox) and np.array_equal(G, oG) and np.array_equal(z, oz), \
        "within tolerance but not bit-identical"


@pytest.mark.parametrize("method", ["qcmd", "qcmd_z", "qrda"])
@pytest.mark.parametrize("requant", [0, 1])
def test_update_with_state_and_scalars_at_the_ends_of_the_exponent_range(method, requant):
    """For tiles whose scales lie in a safe exponent window the kernel takes short forms of the
    correctly rounded sqrt and division, and falls back to the full forms for any group of lanes
    whose accumulator (or, for QRDA, |z| - t*lambda) leaves the window.  State planted with tiny,
    huge, zero, negative-zero and non-finite values next to ordinary ones, and hyper-parameters
    inside and outside the window, must all give the oracle's bits."""
    d, M, bucket = 5 * 4096, 16, 4096
    rng = np.random.default_rng(404)
    g = make_grad("laplace_sparse", M, d, seed=5)
    oc, osc, _ = oracle.quantize_pack(g, bucket=bucket)
    L = qa.Layout.make(d, M, bucket)
    pool = np.array([0.0, -0.0, 1e-45, 1e-40, 3e-39, 1e-35, 1e-30, 1.2e-29, 1.3e-29, 1e-20, 1e-6, 1.0,
                     1e20, 8e37, 9e37, 3e38, np.inf, np.nan], np.float32)
    for case, (eta, lam, delta, t) in enumerate([(0.1, 2e-4, 1e-8, 3), (0.1, 0.0, 1e-8, 1),
                                                 (1e-20, 1e-3, 1e-8, 2), (0.1, 2e-4, 1e-30, 5),
                                                 (3e3, 1e-38, 1e10, 7), (0.1, 1e30, 1e-8, 4)]):
        x0 = (rng.standard_normal(d) * 1e-2 * (rng.random(d) < 0.5)).astype(np.float32)
        G0 = (rng.random(d) * 1e-5).astype(np.float32)
        z0 = (rng.standard_normal(d) * 1e-3).astype(np.float32)
        where = rng.random(d) < 0.02                       # a few lanes per wave
        G0[where] = np.abs(rng.choice(pool, int(where.sum())))
        where = rng.random(d) < 0.02
        z0[where] = rng.choice(pool, int(where.sum())) * rng.choice([-1, 1], int(where.sum()))
        tl = np.float32(t) * np.float32(lam)
        where = rng.random(d) < 0.02                       # |z| - t*lambda just above / below zero
        z0[where] = (tl * (1 + rng.integers(-3, 4, int(where.sum())) * 2.0 ** -23)).astype(np.float32)
        where = rng.random(d) < 0.01
        x0[where] = rng.choice(pool, int(where.sum())) * rng.choice([-1, 1], int(where.sum()))
        ox, oG, oz = x0.copy(), G0.copy(), z0.copy()
        st = GpuState(L, oc, osc, x0, G0, z0)
        if method == "qrda":
            oracle.step_qrda(oc, osc, d, bucket, ox, oG, oz, t, eta, lam, delta, requant)
            st.qrda(t, eta, lam, delta, requant)
        else:
            tz = method == "qcmd_z"
            oracle.step_qcmd(oc, osc, d, bucket, ox, oG, oz if tz else None, eta, lam, delta, requant)
            st.qcmd(eta, lam, delta, requant, track_z=tz)
        x, G, z = st.get()
        for name, a, o in (("x", x, ox), ("G", G, oG), ("z", z, oz)):
            same = (a.view(np.uint32) == o.view(np.uint32)) | (np.isnan(a) & np.isnan(o))
            assert same.all(), (case, name, int((~same).sum()), a[~same][:4], o[~same][:4])


def test_qcmd_without_z_leaves_z_alone():
    d, M, b = 9000, 4, 4096
    g = make_grad("gauss", M, d, 77)
    oc, osc, _ = oracle.quantize_pack(g, bucket=b)
    ox, oG = np.zeros(d, np.float32), np.zeros(d, np.float32)
    z0 = np.full(d, 3.0, np.float32)
    st = GpuState(qa.Layout.make(d, M, b), oc, osc, ox, oG, z0)
    oracle.step_qcmd(oc, osc, d, b, ox, oG, None, 0.1, 1e-4, 1e-8)
    st.qcmd(0.1, 1e-4, 1e-8, 0, track_z=False)
    x, G, z = st.get()
    assert np.array_equal(x, ox) and np.array_equal(G, oG) and np.array_equal(z, z0)


def test_checkpoint_resume_is_bit_identical():
    """State is three tensors and t: T steps in one go == T/2, copy out, copy in, T/2."""
    d, M, b = 20000, 4, 4096
    L = qa.Layout.make(d, M, b)
    msgs = [oracle.quantize_pack(make_grad("gauss", M, d, 300 + t), bucket=b)[:2] for t in range(6)]
    zero = np.zeros(d, np.float32)

    def run(st, ts):
        for t in ts:
            st.codes.copy_(dev(msgs[t - 1][0].view(np.int32)))
            st.scales.copy_(dev(msgs[t - 1][1]))
            st.qrda(t, 0.1, 1e-4, 1e-8) if t % 2 == 0 else st.qcmd(0.1, 1e-4, 1e-8)
        return st.get()

    full = run(GpuState(L, msgs[0][0], msgs[0][1], zero, zero, zero), range(1, 7))
    half = run(GpuState(L, msgs[0][0], msgs[0][1], zero, zero, zero), range(1, 4))
    resumed = run(GpuState(L, msgs[0][0], msgs[0][1], *half), range(4, 7))
    for a, c in zip(full, resumed):
        assert np.array_equal(a, c)


# ------------------------------------------------------------------ local gradient

@pytest.mark.parametrize("d,B", [(1000, 64), (1003, 64), (4100, 13), (6144, 1), (257, 50)])
def test_local_grad_dense_matches_oracle(d, B):
    rng = np.random.default_rng(5)
    n = 512
    A = rng.standard_normal((n, d)).astype(np.float32)
    y = np.where(rng.random(n) < 0.5, -1.0, 1.0).astype(np.float32)
    rows = rng.integers(0, n, B).astype(np.int32)
    x = (rng.standard_normal(d) * 0.05).astype(np.float32)
    og, ol = oracle.local_grad_dense(A, y, rows, x)
    L = qa.Layout.make(d, 1, 0)
    ws = workspace(qa.qa_workspace_bytes(L, qa.QA_OP_GRAD_DENSE))
    g = torch.full((d,), 5.0, dtype=torch.float32, device=DEV)
    loss = torch.zeros(1, dtype=torch.float32, device=DEV)
    qa.qa_local_grad(qa.QA_DENSE, dev(A), None, None, n, d, dev(y), dev(rows), B, dev(x), g, loss, ws)
    torch.cuda.synchronize()
    gg = host(g)
    assert np.allclose(gg, og, rtol=1e-6, atol=1e-12)
    assert host(loss)[0] == pytest.approx(ol, rel=1e-6)
    print("dense grad bit-identical entries:", (gg == og).mean())
    assert (gg == og).mean() > 0.999


def _random_csr(rng, n, d, k):
    idx = np.stack([np.sort(rng.choice(d, k, replace=False)) for _ in range(n)]).astype(np.int32)
    vals = rng.standard_normal((n, k)).astype(np.float32)
    indptr = (np.arange(n + 1) * k).astype(np.int64)
    return vals.reshape(-1), indptr, idx.reshape(-1)


def test_local_grad_csr_matches_oracle():
    rng = np.random.default_rng(6)
    n, d, k, B = 300, 5000, 40, 128          # many column collisions -> atomics are exercised
    vals, indptr, idx = _random_csr(rng, n, d, k)
    idx = (idx % 200).astype(np.int32)       # hot columns (duplicates inside a row are summed too)
    y = np.where(rng.random(n) < 0.5, -1.0, 1.0).astype(np.float32)
    rows = rng.integers(0, n, B).astype(np.int32)
    x = (rng.standard_normal(d) * 0.1).astype(np.float32)
    og, ol = oracle.local_grad_csr(vals, indptr, idx, d, y, rows, x)
    L = qa.Layout.make(d, 1, 0)
    ws = workspace(qa.qa_workspace_bytes(L, qa.QA_OP_GRAD_CSR))
    ws.fill_(0xAB)                            # contents on entry must not matter
    g = torch.full((d,), 5.0, dtype=torch.float32, device=DEV)
    loss = torch.zeros(1, dtype=torch.float32, device=DEV)
    for _ in range(2):                        # second call reuses the dirty workspace
        qa.qa_local_grad(qa.QA_CSR, dev(vals), dev(indptr), dev(idx), n, d, dev(y), dev(rows), B,
                         dev(x), g, loss, ws)
    torch.cuda.synchronize()
    gg = host(g)
    assert np.array_equal(gg != 0, og != 0), "CSR indexing: non-zero set differs"
    assert np.allclose(gg, og, rtol=1e-6, atol=1e-12)
    assert host(loss)[0] == pytest.approx(ol, rel=1e-6)
    assert (gg == og).mean() > 0.999


@pytest.mark.parametrize("csr,shape", [(False, (400, 3000, 30, 48, 5)), (True, (400, 3000, 30, 48, 5)),
                                       # large batches, heavy collisions on a few columns, a ragged last row group
                                       (True, (600, 5000, 30, 301, 7)), (True, (600, 1500, 20, 256, 8))])
def test_local_grad_batched_equals_per_worker_calls_and_oracle(csr, shape):
    rng = np.random.default_rng(8)
    n, d, k, B, M = shape
    y = np.where(rng.random(n) < 0.5, -1.0, 1.0).astype(np.float32)
    x = (rng.standard_normal(d) * 0.1).astype(np.float32)
    rows = rng.integers(0, n, (M, B)).astype(np.int32)
    if csr:
        vals, indptr, idx = _random_csr(rng, n, d, k)
        if B > 100:
            idx = np.where(rng.random(idx.size) < 0.6, idx % 37, idx).astype(np.int32)   # hot columns
        A_d, ip_d, ix_d = dev(vals), dev(indptr), dev(idx)
        ref = [oracle.local_grad_csr(vals, indptr, idx, d, y, rows[m], x) for m in range(M)]
        fmt, op = qa.QA_CSR, qa.QA_OP_GRAD_CSR
    else:
        A = rng.standard_normal((n, d)).astype(np.float32)
        A_d, ip_d, ix_d = dev(A), None, None
        ref = [oracle.local_grad_dense(A, y, rows[m], x) for m in range(M)]
        fmt, op = qa.QA_DENSE, qa.QA_OP_GRAD_DENSE
    gs = d + 8
    ws = workspace(qa.qa_workspace_bytes(qa.Layout.make(d, M, 0), op))
    g = torch.full((M, gs), 5.0, dtype=torch.float32, device=DEV)
    loss = torch.zeros(M, dtype=torch.float32, device=DEV)
    qa.qa_local_grad_batched(fmt, A_d, ip_d, ix_d, n, d, dev(y), dev(rows), B, M, dev(x), g, gs, loss, ws)
    torch.cuda.synchronize()
    gg, ll = host(g), host(loss)
    assert np.all(gg[:, d:] == 5.0)                      # padding between workers untouched
    for m in range(M):
        assert np.array_equal(gg[m, :d] != 0, ref[m][0] != 0)
        assert np.allclose(gg[m, :d], ref[m][0], rtol=1e-6, atol=1e-12)
        assert ll[m] == pytest.approx(ref[m][1], rel=1e-6)
    assert (gg[:, :d] == np.stack([r[0] for r in ref])).mean() > 0.999


# ------------------------------------------------------------------ stochastic ternary quantizer

@pytest.mark.parametrize("d,M,bucket", [(1, 1, 0), (1000, 3, 0), (4096, 2, 4096), (70001, 3, 4096),
                                        (70001, 2, 16384), (70001, 2, 0), (300001, 2, 4096),
                                        (70001, 2, 64), (12289, 3, 256), (70001, 2, 1024), (70001, 2, 2048),
                                        (100, 2, 512)])
def test_stochastic_quantizer_matches_oracle(d, M, bucket):
    g = make_grad("gauss" if d % 2 else "laplace_sparse", M, d, seed=d + 3)
    if d > 9000:
        g[0, 4096:8192] = 0.0                       # an all-zero tile: scale 0, nothing kept
    seed, step = 0x1234567811223344, 17
    oc, osc = oracle.quantize_pack_stochastic(g, bucket=bucket, seed=seed, step=step)
    L = qa.Layout.make(d, M, bucket)
    gs = ((d + 3) // 4) * 4
    gp = np.zeros((M, gs), np.float32); gp[:, :d] = g
    codes = torch.full((M, L.code_stride), -1, dtype=torch.int32, device=DEV)
    scales = torch.full((M, L.scale_stride), -7.0, dtype=torch.float32, device=DEV)
    qa.qa_quantize_pack_stochastic(L, dev(gp), gs, codes, scales, seed, step)
    torch.cuda.synchronize()
    assert np.array_equal(host(scales)[:, :L.n_buckets], osc)
    assert np.array_equal(host(codes).view(np.uint32)[:, :L.words], oc)
    c2 = torch.zeros_like(codes)
    qa.qa_quantize_pack_stochastic(L, dev(gp), gs, c2, scales, seed, step + 1)
    torch.cuda.synchronize()
    assert d < 100 or not torch.equal(c2, codes)    # another step, other draws


# ---- the server's call: messages in, q_t = Q(SynQ_t) out as a message ---------------------------

AGGQ_CASES = [
    # d, M, bucket, requant (1 = per bucket, 2 = one scale for the vector)
    (1, 1, 0, 2), (1000, 4, 0, 2), (4096, 8, 4096, 1), (4097, 8, 4096, 1), (70001, 16, 4096, 1),
    (70001, 20, 4096, 2), (10000, 3, 64, 1), (10000, 5, 256, 1), (70001, 6, 2048, 1),
    (70001, 4, 16384, 1), (70001, 4, 0, 2), (9000, 48, 4096, 1), (4100, 8, 512, 2),
    (70001, 16, 0, 2), (70001, 8, 8192, 1), (70001, 13, 0, 2), (70001, 24, 16384, 1),
    # one scale everywhere, up to 8 workers: three passes of the kernel that walks several tiles
    (70001, 8, 0, 2), (70001, 7, 0, 2), (4096 * 16400 + 5, 2, 0, 2), (4097, 1, 0, 2),
    # complete chunks of 16 and of 8 workers, one to four of them, rows ending inside a 16-byte group
    (70001, 32, 4096, 1), (70001, 64, 4096, 1), (9000, 24, 4096, 1), (8192 + 16 * 7 + 5, 40, 4096, 1),
]


@pytest.mark.parametrize("M", [3, 8, 24])
@pytest.mark.parametrize("spread", [30, 60, 100])
def test_one_scale_for_the_average_when_buckets_lie_far_apart(M, spread):
    """Messages with a scale per 4096-bucket whose magnitudes differ by up to 2^spread from bucket
    to bucket, and ONE scale for Q(SynQ): that scale is set by the largest buckets, so in most
    tiles q = +-s lies far outside the range of the tile's own scales (which is what decides
    whether the update may use the short forms of its division)."""
    d, bucket = 70001, 4096
    rng = np.random.default_rng(M * 1000 + spread)
    nb = (d + bucket - 1) // bucket
    g = make_grad("gauss", M, d, seed=M + spread)
    factor = np.exp2(rng.integers(-spread, spread // 3, nb)).astype(np.float32)
    g = g * np.repeat(factor, bucket)[:d][None, :]
    oc, osc, _ = oracle.quantize_pack(g, bucket=bucket)
    L = qa.Layout.make(d, M, bucket)
    x0 = (rng.standard_normal(d) * 1e-2 * (rng.random(d) < 0.5)).astype(np.float32)
    G0 = (rng.random(d) * 1e-4).astype(np.float32)
    z0 = (rng.standard_normal(d) * 1e-3).astype(np.float32)
    for method in ("qcmd", "qcmd_z", "qrda"):
        ox, oG, oz = x0.copy(), G0.copy(), z0.copy()
        st = GpuState(L, oc, osc, x0, G0, z0)
        with np.errstate(all="ignore"):
            if method == "qrda":
                oracle.step_qrda(oc, osc, d, bucket, ox, oG, oz, 2, 0.1, 1e-4, 1e-8, 2)
                st.qrda(2, 0.1, 1e-4, 1e-8, 2)
            else:
                oracle.step_qcmd(oc, osc, d, bucket, ox, oG, oz if method == "qcmd_z" else None, 0.1, 1e-4, 1e-8, 2)
                st.qcmd(0.1, 1e-4, 1e-8, 2, track_z=method == "qcmd_z")
        x, G, z = st.get()
        for got, want, name in ((x, ox, "x"), (G, oG, "G"), (z, oz, "z")):
            same = (got.view(np.uint32) == want.view(np.uint32)) | (np.isnan(got) & np.isnan(want))
            assert same.all(), (method, name, int((~same).sum()))


ONE_SCALE_CASES = [(d, M, kind) for d, M in ((70001, 8), (70001, 6), (9000, 1), (4097, 2))
                   for kind in ("close", "wide", "inf")] + \
                  [(4096 * 4100 + 3, 5, "close"), (4096 * 8200 + 17, 4, "close"),
                   (4096 * 16400 + 5, 2, "close")]                             # 2, 4 and 8 tiles per group


@pytest.mark.parametrize("d,M,scales", ONE_SCALE_CASES)
def test_steps_with_one_scale_everywhere_match_oracle(d, M, scales):
    """One scale per message, one for Q(SynQ), few workers: the two sums behind Q(SynQ) come from a
    kernel of their own that builds its tables once per work-group and walks 1, 2, 4 or 8 tiles (by
    the vector's length).  Scales close together take its tables, scales spread over 80 binades
    its worker-ordered sum, an infinite scale poisons the sums; fields of the last code word beyond
    d hold garbage and must not count."""
    rng = np.random.default_rng(d + M)
    g = make_grad("laplace_sparse" if d > 10 ** 6 else "gauss", M, d, seed=7 * d + M)
    if scales != "close":
        g = g * (2.0 ** rng.integers(-40, 40, (M, 1))).astype(np.float32)
    oc, osc, _ = oracle.quantize_pack(g, bucket=0)
    if scales == "inf":
        osc[M // 2, 0] = np.inf
    if d % 16:
        oc[:, -1] |= np.uint32((0xFFFFFFFF << (2 * (d % 16))) & 0xFFFFFFFF)      # garbage past d
    L = qa.Layout.make(d, M, 0)
    x0 = (rng.standard_normal(d) * 1e-2 * (rng.random(d) < 0.5)).astype(np.float32)
    G0 = (rng.random(d) * 1e-4).astype(np.float32)
    z0 = (rng.standard_normal(d) * 1e-3).astype(np.float32)
    for method in ("qcmd", "qcmd_z", "qrda"):
        ox, oG, oz = x0.copy(), G0.copy(), z0.copy()
        st = GpuState(L, oc, osc, x0, G0, z0)
        with np.errstate(all="ignore"):
            if method == "qrda":
                oracle.step_qrda(oc, osc, d, 0, ox, oG, oz, 3, 0.1, 1e-4, 1e-8, 2)
                st.qrda(3, 0.1, 1e-4, 1e-8, 2)
            else:
                oracle.step_qcmd(oc, osc, d, 0, ox, oG, oz if method == "qcmd_z" else None, 0.1, 1e-4, 1e-8, 2)
                st.qcmd(0.1, 1e-4, 1e-8, 2, track_z=method == "qcmd_z")
        x, G, z = st.get()
        for got, want, name in ((x, ox, "x"), (G, oG, "G"), (z, oz, "z")):
            same = (got.view(np.uint32) == want.view(np.uint32)) | (np.isnan(got) & np.isnan(want))
            assert same.all(), (method, name, int((~same).sum()))


@pytest.mark.parametrize("d,M,bucket,requant", AGGQ_CASES)
def test_aggregate_quantize_matches_oracle_and_the_fused_step(d, M, bucket, requant):
    g = make_grad("gauss", M, d, seed=31 * d + M)
    oc, osc, _ = oracle.quantize_pack(g, bucket=bucket)
    L = qa.Layout.make(d, M, bucket)
    bq = bucket if requant == 1 else 0
    L1 = qa.Layout.make(d, 1, bq)
    # oracle: the average, then the quantizer on it as a one-worker message
    gbar = oracle.aggregate(oc, osc, d, bucket)
    qc_ref, qs_ref, qt_ref = oracle.quantize_pack(gbar[None, :], bucket=bq)
    codes, scales = dev(oc.view(np.int32)), dev(osc)
    qc = torch.full((1, L1.code_stride), -1, dtype=torch.int32, device=DEV)
    qs = torch.full((1, L1.scale_stride), -7.0, dtype=torch.float32, device=DEV)
    qt = torch.full((1, L1.scale_stride), -7.0, dtype=torch.float32, device=DEV)
    ws = workspace(qa.qa_workspace_bytes(L, qa.QA_OP_STEP))
    qa.qa_aggregate_quantize(L, codes, scales, requant, qc, qs, qt, ws)
    torch.cuda.synchronize()
    assert np.array_equal(host(qc).view(np.uint32)[:, :L1.words], qc_ref)
    assert np.array_equal(host(qs)[:, :L1.n_buckets].view(np.uint32), qs_ref.view(np.uint32))
    assert np.array_equal(host(qt)[:, :L1.n_buckets].view(np.uint32), qt_ref.view(np.uint32))
    # stepping from the message == the fused step with the same second quantization
    rng = np.random.default_rng(d)
    x0 = (rng.standard_normal(d) * 1e-2 * (rng.random(d) < 0.5)).astype(np.float32)
    G0 = (rng.random(d) * 1e-4).astype(np.float32)
    z0 = (rng.standard_normal(d) * 1e-3).astype(np.float32)
    xa, Ga, za = dev(x0), dev(G0), dev(z0)
    xb, Gb, zb = dev(x0), dev(G0), dev(z0)
    qa.qa_step_qrda(L, codes, scales, xa, Ga, za, 3, 0.1, 2e-4, 1e-8, requant, ws)
    qa.qa_step_qrda(L1, qc, qs, xb, Gb, zb, 3, 0.1, 2e-4, 1e-8, qa.QA_REQUANT_NONE, None)
    torch.cuda.synchronize()
    for u, v in ((xa, xb), (Ga, Gb), (za, zb)):
        assert np.array_equal(host(u).view(np.uint32), host(v).view(np.uint32))


def test_aggregate_quantize_checks_its_arguments():
    L = qa.Layout.make(100000, 2, 4096)
    t = torch.zeros(8, dtype=torch.int32, device=DEV)
    f = torch.zeros(8, dtype=torch.float32, device=DEV)
    with pytest.raises(qa.QaError) as e:                 # NONE is not a quantization
        qa.qa_aggregate_quantize(L, t, f, qa.QA_REQUANT_NONE, t, f, None, None)
    assert e.value.code == -1
    with pytest.raises(qa.QaError) as e:                 # one scale for 100000 components needs the workspace
        qa.qa_aggregate_quantize(L, t, f, qa.QA_REQUANT_GLOBAL, t, f, None, None)
    assert e.value.code == -3
    L0 = qa.Layout.make(100000, 2, 0)
    with pytest.raises(qa.QaError) as e:                 # per-bucket needs buckets
        qa.qa_aggregate_quantize(L0, t, f, qa.QA_REQUANT_BUCKET, t, f, None, None)
    assert e.value.code == -1


# ---- exact least-squares threshold by ranking (Section 3.4) ------------------------------------

@pytest.mark.parametrize("d,M,bucket", [(4096, 1, 0), (1000, 2, 0), (3, 1, 0), (4096 * 5, 3, 4096),
                                        (4096 * 7 + 1234, 4, 4096), (4096 * 3 + 1, 2, 4096),
                                        # buckets smaller than the tile: the network stops early
                                        (10000, 2, 64), (10000, 2, 128), (9001, 3, 256), (12289, 2, 512),
                                        (10000, 2, 1024), (4096 * 3 + 77, 3, 2048), (70, 1, 64)])
@pytest.mark.parametrize("kind", ["gauss", "student", "laplace_sparse"])
def test_exact_threshold_quantizer_matches_oracle(d, M, bucket, kind):
    g = make_grad(kind, M, d, seed=d % 977 + M)
    th_ref = np.stack([oracle.exact_thresholds(g[m], bucket) for m in range(M)])
    c_ref, s_ref, _ = oracle.quantize_pack(g, bucket, thresholds=th_ref)
    c, s, th, L = gpu_quantize_pack(g, bucket, exact=True)
    nb = L.n_buckets
    assert np.array_equal(th[:, :nb].view(np.uint32), th_ref.view(np.uint32))
    assert np.array_equal(c[:, :L.words], c_ref)
    assert np.array_equal(s[:, :nb].view(np.uint32), s_ref.view(np.uint32))


@pytest.mark.parametrize("bucket", [4096, 256, 64])
def test_exact_threshold_never_splits_equal_magnitudes_and_handles_zeros(bucket):
    rng = np.random.default_rng(5)
    d = 4096 * 3
    g = np.zeros((3, d), np.float32)
    g[0] = rng.integers(-3, 4, d)                       # many ties, many zeros, sums exact
    g[1, ::7] = 2.5                                      # all kept magnitudes equal
    g[2, :4096] = rng.standard_normal(4096)              # all-zero buckets after the first tile
    th_ref = np.stack([oracle.exact_thresholds(g[m], bucket) for m in range(3)])
    c_ref, s_ref, _ = oracle.quantize_pack(g, bucket, thresholds=th_ref)
    c, s, th, L = gpu_quantize_pack(g, bucket, exact=True)
    assert np.array_equal(th.view(np.uint32), th_ref.view(np.uint32))
    assert np.array_equal(c, c_ref)
    assert np.array_equal(s.view(np.uint32), s_ref.view(np.uint32))
    first_empty = 4096 // bucket
    assert th[2, first_empty] == 0 and s[2, first_empty] == 0 and not c[2, 256:].any()


# buckets longer than one tile, and one threshold for a long vector: device-wide ranking
@pytest.mark.parametrize("d,M,bucket", [(70001, 2, 0), (70001, 2, 8192), (4096 * 5 + 1, 3, 16384),
                                        (4097, 1, 0), (300001, 1, 0), (8192 * 3, 2, 8192),
                                        ((1 << 20) + 17, 1, 65536),
                                        # one bucket that is longer than the vector, buckets ending one
                                        # past a tile, several workers with a padded gradient stride
                                        (5000, 2, 8192), (8193, 3, 8192), (4097, 2, 16384)])
@pytest.mark.parametrize("kind", ["gauss", "student", "laplace_sparse"])
def test_exact_threshold_over_several_tiles_matches_oracle(d, M, bucket, kind):
    """Section 3.4's optimum over a bucket (or a whole gradient) of many tiles.  At these sizes the
    objectives of neighbouring k differ by far more than the rounding of the binary64 sums, so
    the k, and with it threshold, codes and scale, must be the oracle's."""
    g = make_grad(kind, M, d, seed=d % 977 + M)
    th_ref = np.stack([oracle.exact_thresholds(g[m], bucket) for m in range(M)])
    c_ref, s_ref, _ = oracle.quantize_pack(g, bucket, thresholds=th_ref)
    c, s, th, L = gpu_quantize_pack(g, bucket, exact=True)
    nb = L.n_buckets
    assert np.array_equal(th[:, :nb].view(np.uint32), th_ref.view(np.uint32))
    assert np.array_equal(c[:, :L.words], c_ref)
    assert int(ulp_distance(s[:, :nb], s_ref).max()) <= 1   # binary64 sums over many tiles, rounded once


@pytest.mark.parametrize("bucket", [0, 8192])
def test_exact_threshold_over_several_tiles_with_ties_zeros_and_a_ramp(bucket):
    rng = np.random.default_rng(11)
    d = 8192 * 4 + 300
    g = np.zeros((4, d), np.float32)
    g[0] = rng.integers(-3, 4, d)                       # many ties, many zeros, sums exact
    g[1, ::7] = 2.5                                      # all kept magnitudes equal
    g[2, :5000] = rng.standard_normal(5000)              # all-zero buckets after the first
    g[3] = rng.permutation(np.arange(1, d + 1))          # a ramp: the closed form of the pin
    th_ref = np.stack([oracle.exact_thresholds(g[m], bucket) for m in range(4)])
    c_ref, s_ref, _ = oracle.quantize_pack(g, bucket, thresholds=th_ref)
    c, s, th, L = gpu_quantize_pack(g, bucket, exact=True)
    assert np.array_equal(th.view(np.uint32), th_ref.view(np.uint32))
    assert np.array_equal(c, c_ref)
    assert np.array_equal(s.view(np.uint32), s_ref.view(np.uint32))
    if bucket:
        assert th[2, 1] == 0 and s[2, 1] == 0 and not c[2, 512:].any()


def test_exact_threshold_of_a_long_vector_is_optimal_to_binary64_resolution():
    """Beyond some 1e7 components the objectives of neighbouring k near the optimum agree to
    binary64 rounding and the association of the sums may decide between them; what must hold
    at any size: the GPU's kept set is {|v| > its threshold}, no candidate the oracle finds is
    better than it by more than that rounding, and codes and scale follow from the threshold."""
    d, M = (1 << 24) + 12345, 1
    g = np.empty((M, d), np.float32)
    g[0] = host(synth.grad_laplace_sparse(d, 0, 1, device=DEV, seed=77, keep=0.5))
    c, s, th, L = gpu_quantize_pack(g, 0, exact=True)
    a = np.abs(g[0].astype(np.float64))
    kept = a > float(th[0, 0])
    k = int(kept.sum())
    assert k > 0 and (th[0, 0] == 0 or (a == float(th[0, 0])).any())      # an actual magnitude
    obj_gpu = a[kept].sum() ** 2 / k
    _, _, obj_ref, k_ref = oracle.exact_threshold(g[0])
    assert obj_gpu >= obj_ref * (1 - 1e-12)
    print(f"\n[exact, d=2^24] kept {k} (oracle {k_ref}), objective ratio - 1 = {obj_gpu / obj_ref - 1:.2e}")
    c_ref, s_ref, _ = oracle.quantize_pack(g, 0, thresholds=th[:, :1])
    assert np.array_equal(c[:, :L.words], c_ref)
    assert int(ulp_distance(s[:, :1], s_ref[:, :1]).max()) <= 1


def test_exact_threshold_checks_workspace_and_missing_output():
    g = dev(np.ones((1, 8192), np.float32))
    codes = torch.zeros((1, 512), dtype=torch.int32, device=DEV)
    scales = torch.zeros((1, 128), dtype=torch.float32, device=DEV)
    th = torch.zeros((1, 128), dtype=torch.float32, device=DEV)
    for bucket in (8192, 0):                            # buckets beyond one tile need the larger workspace
        L = qa.Layout.make(8192, 1, bucket)
        assert qa.qa_workspace_bytes(L, qa.QA_OP_QUANTIZE_EXACT) > qa.qa_workspace_bytes(L, qa.QA_OP_QUANTIZE)
        ws = workspace(qa.qa_workspace_bytes(L, qa.QA_OP_QUANTIZE))
        with pytest.raises(qa.QaError) as e:
            qa.qa_quantize_pack(L, g, 8192, codes, scales, th, qa.QA_THRESH_EXACT, ws)
        assert e.value.code == -3
        with pytest.raises(qa.QaError) as e:            # and are refused without it
            qa.qa_quantize_pack_static(L, g, 8192, codes, scales, th, qa.QA_THRESH_EXACT)
        assert e.value.code == -6
    L = qa.Layout.make(8192, 1, 4096)
    assert qa.qa_workspace_bytes(L, qa.QA_OP_QUANTIZE_EXACT) == qa.qa_workspace_bytes(L, qa.QA_OP_QUANTIZE)
    with pytest.raises(qa.QaError) as e:
        qa.qa_quantize_pack(L, g, 8192, codes, scales, None, qa.QA_THRESH_EXACT, None)
    assert e.value.code == -1
    with pytest.raises(qa.QaError) as e:
        qa.qa_quantize_pack(L, g, 8192, codes, scales, th,
                            qa.QA_THRESH_EXACT | qa.QA_THRESH_GIVEN, None)
    assert e.value.code == -1
