"""Parity of the indicator / selection / sparse-encoding kernels with the oracle (bit-exact:
indicator bits, counts, compact codes, decoded dense codes; scales and thresholds equal), and
an end-to-end run of Algorithm 1 WITH selection on the sparse synthetic problem, where the
message size 32*nb + d + 2k bits is accounted."""
import numpy as np
import pytest
import torch

import oracle
from paper_2208_05631_amd import synth

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2208_05631_amd as qa
    from gpu_util import DEV, dev, host, workspace


def rand_state(rng, d, nz=0.3):
    x = (rng.standard_normal(d) * 0.1 * (rng.random(d) < nz)).astype(np.float32)
    G = (rng.random(d) * 1e-3).astype(np.float32)
    z = (rng.standard_normal(d) * 0.05).astype(np.float32)
    return x, G, z


@pytest.mark.parametrize("method", [0, 1])
@pytest.mark.parametrize("d,M", [(1, 1), (33, 2), (1000, 3), (4096, 2), (70001, 4), (70004, 3)])
def test_indicator_matches_oracle(method, d, M):
    rng = np.random.default_rng(d + M + method)
    x, G, z = rand_state(rng, d)
    g = (rng.standard_normal((M, d)) * rng.choice([1e-3, 0.05], (M, d))).astype(np.float32)
    eta, lam, delta, t = 0.1, 0.01, 1e-8, 5
    NW = (d + 31) // 32
    ind = torch.full((M, NW + 3), -1, dtype=torch.int32, device=DEV)
    L = qa.Layout.make(d, M, 0 if d <= 4096 else 4096)
    qa.qa_indicator(L, method, dev(g), d, dev(x), dev(G), dev(z), t, eta, lam, delta, ind, NW + 3)
    syn = torch.zeros(NW, dtype=torch.int32, device=DEV)
    qa.qa_indicator_or(L, ind, NW + 3, syn)
    torch.cuda.synchronize()
    got = host(ind).view(np.uint32)
    ref = np.stack([oracle.indicator(method, g[m], x, G, z, t, eta, lam, delta) for m in range(M)])
    assert np.array_equal(got[:, :NW], ref)
    assert np.all(got[:, NW:] == 0xFFFFFFFF)                         # padding untouched
    assert np.array_equal(host(syn).view(np.uint32), oracle.indicator_or(ref, d))
    frac = np.unpackbits(ref.view(np.uint8)).mean()
    assert d < 100 or 0.02 < frac < 0.98


@pytest.mark.parametrize("method", [0, 1])
@pytest.mark.parametrize("lam", [0.0, 0.01])
def test_indicator_at_decision_boundaries_matches_oracle(method, lam):
    """Gradients within a few ulps of the zero/non-zero boundary of the worker's own update,
    huge accumulators (quotients underflow), non-finite values: the division-free decision
    must hand these to the closed form."""
    rng = np.random.default_rng(3 + method)
    d, M, eta, delta, t = 8192, 2, 0.1, 1e-8, 7
    x = np.zeros(d, np.float32)
    x[::97] = 0.5
    G = (rng.random(d) * 1e-3).astype(np.float32)
    G[1::5] = np.float32(1e30)
    G[2::11] = np.float32(3e38)
    z = (rng.standard_normal(d) * 0.05).astype(np.float32)
    g = np.empty((M, d), np.float32)
    for m in range(M):
        if method == 0:
            base = np.full(d, lam, np.float32)                       # |eta*g| ~ lambda*eta
        else:
            base = (np.sign(rng.standard_normal(d)) * (t * lam) - z).astype(np.float32)   # |z+g| ~ t*lambda
        ulps = rng.integers(-3, 4, d)
        v = base.copy()
        for k in range(1, 4):
            v = np.where(ulps >= k, np.nextafter(v, np.float32(np.inf)), v)
            v = np.where(ulps <= -k, np.nextafter(v, np.float32(-np.inf)), v)
        v[3::13] *= rng.choice([-1.0, 1.0], v[3::13].size).astype(np.float32)
        v[5::101] = np.float32(1e-38)
        v[7::211] = np.nan
        v[9::223] = np.inf
        v[11::227] = np.float32(1e20)
        g[m] = v
    NW = d // 32
    L = qa.Layout.make(d, M, 4096)
    ind = torch.zeros((M, NW), dtype=torch.int32, device=DEV)
    qa.qa_indicator(L, method, dev(g), d, dev(x), dev(G), dev(z), t, eta, lam, delta, ind, NW)
    torch.cuda.synchronize()
    ref = np.stack([oracle.indicator(method, g[m], x, G, z, t, eta, lam, delta) for m in range(M)])
    assert np.array_equal(host(ind).view(np.uint32), ref)


def random_indicator(rng, M, d, p):
    bits = rng.random((M, d)) < p
    NW = (d + 31) // 32
    ind = np.zeros((M, NW), np.uint32)
    for m in range(M):
        idx = np.nonzero(bits[m])[0]
        np.bitwise_or.at(ind[m], idx // 32, (np.uint32(1) << (idx % 32).astype(np.uint32)))
    return ind


GENERAL_BUCKETS = [
    # one scale per message over many tiles (the 32 + d + 2k bit message), dense / sparse / full / empty
    (70001, 3, 0, 0.2), (300000, 2, 0, 0.004), (70001, 2, 0, 1.0), (20000, 2, 0, 0.0), (4097, 1, 0, 0.5),
    # buckets inside a tile
    (70001, 2, 64, 0.5), (70001, 2, 256, 0.3), (12289, 3, 1024, 0.05), (70001, 2, 2048, 0.1),
    # buckets over several tiles
    (70001, 2, 8192, 0.3), (70001, 3, 16384, 0.02), (5000, 2, 65536, 0.5),
]


def area_words(d, bucket):
    return ((bucket or d) + 15) // 16


@pytest.mark.parametrize("d,M,bucket,p", [(1, 1, 0, 1.0), (1000, 2, 0, 0.3), (4096, 2, 4096, 0.5),
                                          (4097, 2, 4096, 0.01), (70001, 3, 4096, 0.2),
                                          (70001, 2, 4096, 1.0), (20000, 2, 4096, 0.0)] + GENERAL_BUCKETS)
def test_quantize_selected_and_decode_match_oracle(d, M, bucket, p):
    rng = np.random.default_rng(d + M)
    g = (rng.standard_normal((M, d)) * 1e-2).astype(np.float32)
    ind = random_indicator(rng, M, d, p)
    if d > 8192:
        ind[0, 128:256] = 0                                          # an empty bucket
    L = qa.Layout.make(d, M, bucket)
    nb, W, NW = L.n_buckets, L.words, (d + 31) // 32
    gs = ((d + 3) // 4) * 4
    gp = np.zeros((M, gs), np.float32); gp[:, :d] = g
    sel = torch.full((M, L.code_stride), 0x5A5A5A5A, dtype=torch.int32, device=DEV)
    cnt = torch.zeros((M, nb), dtype=torch.int32, device=DEV)
    sc = torch.full((M, nb), -1.0, dtype=torch.float32, device=DEV)
    th = torch.full((M, nb), -1.0, dtype=torch.float32, device=DEV)
    dense = torch.full((M, L.code_stride), -1, dtype=torch.int32, device=DEV)
    ind_d = dev(ind.view(np.int32))
    ws = workspace(qa.qa_workspace_bytes(L, qa.QA_OP_SELECT))
    qa.qa_quantize_pack_selected(L, dev(gp), gs, ind_d, NW, sel, cnt, sc, th, ws)
    if ws is not None:
        ws.fill_(0x77)                                               # nothing may be carried between calls
    qa.qa_decode_selected(L, ind_d, NW, sel, dense, ws)
    torch.cuda.synchronize()
    sel_h, cnt_h = host(sel).view(np.uint32), host(cnt).view(np.uint32)
    area = area_words(d, bucket)
    for m in range(M):
        o_sel, o_cnt, o_sc, o_th = oracle.quantize_selected(g[m], ind[m], bucket=bucket)
        assert np.array_equal(cnt_h[m], o_cnt)
        assert np.array_equal(host(sc)[m], o_sc) and np.array_equal(host(th)[m], o_th)
        for k in range(nb):
            nwk = (int(o_cnt[k]) + 15) // 16
            lo = k * area
            assert np.array_equal(sel_h[m, lo: lo + nwk], o_sel[lo: lo + nwk]), (m, k)
            untouched = sel_h[m, lo + nwk: min(lo + area, L.code_stride)]
            assert np.all(untouched == 0x5A5A5A5A)                   # only ceil(count/16) words written
        assert np.array_equal(host(dense).view(np.uint32)[m, :W], oracle.decode_selected(ind[m], o_sel, d, bucket=bucket))


@pytest.mark.parametrize("shared", [False, True])
@pytest.mark.parametrize("d,M,bucket,p", [(1, 1, 0, 1.0), (1000, 2, 0, 0.3), (4096, 1, 4096, 0.5),
                                          (4097, 2, 4096, 0.02), (70001, 3, 4096, 0.2),
                                          (70001, 1, 4096, 1.0), (20000, 2, 4096, 0.0)] + GENERAL_BUCKETS)
def test_select_codes_matches_oracle_and_decode_inverts_it(d, M, bucket, p, shared):
    """S(q, I) on coded messages (the server's push): bit-exact with the checker, only the words
    that hold codes are written, and the decoder restores the marked components."""
    rng = np.random.default_rng(7 * d + M)
    L = qa.Layout.make(d, M, bucket)
    nb, W, NW = L.n_buckets, L.words, (d + 31) // 32
    codes = rng.integers(0, 2 ** 32, (M, L.code_stride), dtype=np.uint64).astype(np.uint32)   # incl. pattern 10
    ind = random_indicator(rng, 1 if shared else M, d, p)
    sel = torch.full((M, L.code_stride), 0x5A5A5A5A, dtype=torch.int32, device=DEV)
    cnt = torch.full((M, nb), -1, dtype=torch.int32, device=DEV)
    back = torch.full((M, L.code_stride), -1, dtype=torch.int32, device=DEV)
    codes_d, ind_d = dev(codes.view(np.int32)), dev(ind.view(np.int32))
    ws = workspace(qa.qa_workspace_bytes(L, qa.QA_OP_SELECT))
    qa.qa_select_codes(L, codes_d, ind_d, 0 if shared else NW, sel, cnt, ws)
    if not shared:
        qa.qa_decode_selected(L, ind_d, NW, sel, back, ws)
    torch.cuda.synchronize()
    sel_h, cnt_h = host(sel).view(np.uint32), host(cnt).view(np.uint32)
    area = area_words(d, bucket)
    for m in range(M):
        im = ind[0 if shared else m]
        o_sel, o_cnt = oracle.select_codes(codes[m, :W], im, d, bucket=bucket)
        assert np.array_equal(cnt_h[m], o_cnt)
        for k in range(nb):
            nwk = (int(o_cnt[k]) + 15) // 16
            lo = k * area
            assert np.array_equal(sel_h[m, lo: lo + nwk], o_sel[lo: lo + nwk]), (m, k)
            assert np.all(sel_h[m, lo + nwk: min(lo + area, L.code_stride)] == 0x5A5A5A5A)
        if not shared:
            want = oracle.decode_selected(im, o_sel, d, bucket=bucket)
            assert np.array_equal(host(back).view(np.uint32)[m, :W], want)
            bits = np.unpackbits(im.view(np.uint8), bitorder="little")[:d].astype(bool)
            assert np.array_equal(oracle.unpack(want, d), np.where(bits, oracle.unpack(codes[m, :W], d), 0))


@pytest.mark.parametrize("method", ["qcmd", "qrda"])
def test_pull_direction_through_the_sparse_message_equals_the_fused_step(method):
    """Algorithm 1 end to end on the server's side: decode the workers' sparse messages, average,
    q_t = Q(SynQ_t) as a one-worker message, push S(q_t, I_syn) + I_syn, workers decode and
    update.  Components outside I_syn have q_t = 0, so the result must equal the fused step with
    the same second quantization, bit for bit."""
    rng = np.random.default_rng(11)
    d, M, b = 70001, 4, 4096
    eta, lam, delta, t = 0.1, 1e-3, 1e-8, 3
    L = qa.Layout.make(d, M, b)
    L1 = qa.Layout.make(d, 1, b)
    nb, NW, gs = L.n_buckets, (d + 31) // 32, ((d + 3) // 4) * 4
    x0, G0, z0 = rand_state(rng, d, nz=0.05)
    g = np.zeros((M, gs), np.float32)
    g[:, :d] = rng.standard_normal((M, d)) * rng.choice([1e-4, 0.05], (M, d), p=[0.9, 0.1])
    gd, xd, Gd, zd = dev(g), dev(x0), dev(G0), dev(z0)
    ind = torch.zeros((M, NW), dtype=torch.int32, device=DEV)
    syn = torch.zeros(NW, dtype=torch.int32, device=DEV)
    sel = torch.zeros((M, L.code_stride), dtype=torch.int32, device=DEV)
    cnt = torch.zeros((M, nb), dtype=torch.int32, device=DEV)
    sc = torch.zeros((M, nb), dtype=torch.float32, device=DEV)
    codes = torch.zeros((M, L.code_stride), dtype=torch.int32, device=DEV)
    mth = 0 if method == "qcmd" else 1
    # workers -> server
    qa.qa_indicator(L, mth, gd, gs, xd, Gd, zd, t, eta, lam, delta, ind, NW)
    qa.qa_indicator_or(L, ind, NW, syn)
    qa.qa_quantize_pack_selected(L, gd, gs, ind, NW, sel, cnt, sc, None)
    qa.qa_decode_selected(L, ind, NW, sel, codes)

    def step(LL, c, s, xx, GG, zz, requant):
        if method == "qcmd":
            qa.qa_step_qcmd(LL, c, s, xx, GG, zz, eta, lam, delta, requant, None)
        else:
            qa.qa_step_qrda(LL, c, s, xx, GG, zz, t, eta, lam, delta, requant, None)

    # A: fused step with the per-bucket second quantization
    xa, Ga, za = xd.clone(), Gd.clone(), zd.clone()
    step(L, codes, sc, xa, Ga, za, qa.QA_REQUANT_BUCKET)
    # B: q_t as a message, through the sparse encoding and back
    gbar = torch.zeros(gs, dtype=torch.float32, device=DEV)
    qc = torch.zeros((1, L1.code_stride), dtype=torch.int32, device=DEV)
    qs = torch.zeros((1, nb), dtype=torch.float32, device=DEV)
    qa.qa_aggregate_unpack(L, codes, sc, gbar)
    qa.qa_quantize_pack(L1, gbar, gs, qc, qs, None, 0, None)
    push = torch.zeros((1, L1.code_stride), dtype=torch.int32, device=DEV)
    push_cnt = torch.zeros((1, nb), dtype=torch.int32, device=DEV)
    qa.qa_select_codes(L1, qc, syn, 0, push, push_cnt)
    pulled = torch.full((1, L1.code_stride), -1, dtype=torch.int32, device=DEV)
    qa.qa_decode_selected(L1, syn, NW, push, pulled)
    xb, Gb, zb = xd.clone(), Gd.clone(), zd.clone()
    step(L1, pulled, qs, xb, Gb, zb, qa.QA_REQUANT_NONE)
    torch.cuda.synchronize()
    assert np.array_equal(host(pulled)[0, :L1.words], host(qc)[0, :L1.words])     # nothing lost
    for u, v in ((xa, xb), (Ga, Gb), (za, zb)):
        assert np.array_equal(host(u).view(np.uint32), host(v).view(np.uint32))
    k_syn = int(host(push_cnt).sum())
    assert 0 < k_syn < d                                                         # a sparse message
    assert np.count_nonzero(host(xa)) > 0


@pytest.mark.parametrize("method", ["qcmd", "qrda"])
def test_server_and_worker_roles_as_separate_calls_equal_the_fused_step(method):
    """Algorithm 1 with only sparse messages between the roles: workers send (I_m, Q(S(g, I_m))),
    the server answers with (I_syn, S(q_t, I_syn)) from qa_aggregate_quantize_selected +
    qa_select_codes, a worker updates with qa_step_*_selected on that one message.  Must equal the
    fused step with the per-bucket second quantization on the decoded codes, bit for bit."""
    rng = np.random.default_rng(17)
    d, M, b = 50001, 5, 4096
    eta, lam, delta, t = 0.1, 1e-3, 1e-8, 4
    L, L1 = qa.Layout.make(d, M, b), qa.Layout.make(d, 1, b)
    nb, NW, gs = L.n_buckets, (d + 31) // 32, ((d + 3) // 4) * 4
    x0, G0, z0 = rand_state(rng, d, nz=0.05)
    g = np.zeros((M, gs), np.float32)
    g[:, :d] = rng.standard_normal((M, d)) * rng.choice([1e-4, 0.05], (M, d), p=[0.9, 0.1])
    gd, xd, Gd, zd = dev(g), dev(x0), dev(G0), dev(z0)
    mth = 0 if method == "qcmd" else 1
    # workers
    ind = torch.zeros((M, NW), dtype=torch.int32, device=DEV)
    sel = torch.zeros((M, L.code_stride), dtype=torch.int32, device=DEV)
    cnt = torch.zeros((M, nb), dtype=torch.int32, device=DEV)
    sc = torch.zeros((M, nb), dtype=torch.float32, device=DEV)
    qa.qa_indicator(L, mth, gd, gs, xd, Gd, zd, t, eta, lam, delta, ind, NW)
    qa.qa_quantize_pack_selected(L, gd, gs, ind, NW, sel, cnt, sc, None)
    # server
    syn = torch.zeros(NW, dtype=torch.int32, device=DEV)
    qc = torch.zeros((1, L1.code_stride), dtype=torch.int32, device=DEV)
    qs = torch.zeros((1, nb), dtype=torch.float32, device=DEV)
    push = torch.zeros((1, L1.code_stride), dtype=torch.int32, device=DEV)
    push_cnt = torch.zeros((1, nb), dtype=torch.int32, device=DEV)
    qa.qa_aggregate_quantize_selected(L, ind, NW, sel, sc, qa.QA_REQUANT_BUCKET, qc, qs, None, syn, None)
    qa.qa_select_codes(L1, qc, syn, 0, push, push_cnt)
    # a worker
    xb, Gb, zb = xd.clone(), Gd.clone(), zd.clone()
    if method == "qcmd":
        qa.qa_step_qcmd_selected(L1, syn, 0, push, qs, xb, Gb, zb, eta, lam, delta, 0, None)
    else:
        qa.qa_step_qrda_selected(L1, syn, 0, push, qs, xb, Gb, zb, t, eta, lam, delta, 0, None)
    # everything in one place: decode, fused step with the second quantization
    codes = torch.zeros((M, L.code_stride), dtype=torch.int32, device=DEV)
    qa.qa_decode_selected(L, ind, NW, sel, codes)
    xa, Ga, za = xd.clone(), Gd.clone(), zd.clone()
    if method == "qcmd":
        qa.qa_step_qcmd(L, codes, sc, xa, Ga, za, eta, lam, delta, qa.QA_REQUANT_BUCKET, None)
    else:
        qa.qa_step_qrda(L, codes, sc, xa, Ga, za, t, eta, lam, delta, qa.QA_REQUANT_BUCKET, None)
    torch.cuda.synchronize()
    for u, v in ((xa, xb), (Ga, Gb), (za, zb)):
        assert np.array_equal(host(u).view(np.uint32), host(v).view(np.uint32))
    assert 0 < int(host(push_cnt).sum()) < d and np.count_nonzero(host(xa)) > 0


def test_sparse_encoding_refuses_what_it_cannot_do_before_launching():
    t = torch.zeros(8, dtype=torch.int32, device=DEV)
    # buckets over several tiles need the scan's workspace
    L = qa.Layout.make(100000, 2, 0)
    assert qa.qa_workspace_bytes(L, qa.QA_OP_SELECT) > 0
    with pytest.raises(qa.QaError) as e:
        qa.qa_decode_selected(L, t, 100000, t, t)
    assert e.value.code == -3
    # buckets inside a tile need none
    assert qa.qa_workspace_bytes(qa.Layout.make(100000, 2, 1024), qa.QA_OP_SELECT) == 0
    # a bucket's count is kept in 32 bits
    L = qa.Layout.make(1 << 33, 1, 0)
    with pytest.raises(qa.QaError) as e:
        qa.qa_decode_selected(L, t, 1 << 28, t, t)
    assert e.value.code == -5


SPARSE_STEP_CASES = [
    # d, M, bucket, fraction marked, requant, one indicator for all, scales spread over many binades
    (1, 1, 0, 1.0, 0, False, False), (1000, 3, 0, 0.3, 0, False, False), (1000, 2, 0, 0.3, 2, False, False),
    (4096, 2, 4096, 0.5, 1, False, False), (4097, 5, 4096, 0.05, 0, False, False),
    (70001, 4, 4096, 0.2, 0, False, False), (70001, 16, 4096, 0.3, 1, False, False),
    (70001, 20, 4096, 1.0, 0, False, False), (70001, 40, 4096, 0.1, 0, False, False),
    (70001, 3, 4096, 0.2, 2, False, False), (20000, 2, 4096, 0.0, 0, False, False),
    (70001, 1, 4096, 0.2, 0, True, False), (70001, 4, 4096, 0.2, 1, True, False),
    (70001, 20, 4096, 0.3, 0, False, True), (9000, 4, 4096, 0.4, 1, False, True),
    # other bucket sizes: decoded into the workspace, then the dense step
    (70001, 4, 0, 0.2, 0, False, False), (70001, 3, 0, 0.3, 2, False, False), (70001, 2, 0, 0.2, 0, True, False),
    (70001, 5, 256, 0.3, 1, False, False), (70001, 4, 2048, 0.1, 0, False, False),
    (70001, 3, 16384, 0.2, 1, False, False), (70001, 20, 1024, 0.3, 0, False, True),
]


@pytest.mark.parametrize("d,M,bucket,p,requant,shared,wide", SPARSE_STEP_CASES)
def test_steps_on_sparse_messages_match_oracle_decode_then_step(d, M, bucket, p, requant, shared, wide):
    """qa_step_*_selected against the oracle's decode followed by its step, three steps in a row
    (QCMD with z, QCMD, QRDA).  Words of a bucket's area beyond ceil(count/16) hold garbage and
    must not matter; `wide` scales force the worker-ordered sum."""
    rng = np.random.default_rng(d + 7 * M + requant)
    eta, lam, delta = 0.1, 2e-4, 1e-8
    L = qa.Layout.make(d, M, bucket)
    nb, W, NW = L.n_buckets, L.words, (d + 31) // 32
    ox, oG, oz = rand_state(rng, d)
    xd, Gd, zd = dev(ox), dev(oG), dev(oz)
    ws = workspace(qa.qa_workspace_bytes(L, qa.QA_OP_STEP_SELECTED))
    area = area_words(d, bucket)
    for t in (1, 2, 3):
        g = (rng.standard_normal((M, d)) * rng.choice([1e-3, 0.02], (M, d))).astype(np.float32)
        ind = random_indicator(rng, 1 if shared else M, d, p)
        if d > 8192:
            ind[0, 128:256] = 0                                      # an empty bucket
        sel = np.full((M, L.code_stride), 0x5A5A5A5A, np.uint32)
        sc = np.zeros((M, nb), np.float32)
        dense = np.zeros((M, W), np.uint32)
        for m in range(M):
            im = ind[0 if shared else m]
            o_sel, o_cnt, o_sc, _ = oracle.quantize_selected(g[m], im, bucket=bucket)
            for k in range(nb):
                nwk = (int(o_cnt[k]) + 15) // 16
                lo = k * area
                sel[m, lo: lo + nwk] = o_sel[lo: lo + nwk]
            sc[m] = o_sc
            dense[m] = oracle.decode_selected(im, o_sel, d, bucket=bucket)
        if wide:
            sc = (sc * np.exp2(rng.integers(-30, 31, sc.shape))).astype(np.float32)
            if M > 2:
                sc[1, 0] = np.inf                                    # a non-finite scale: ordered sum too
        ind_d, sel_d, sc_d = dev(ind.view(np.int32)), dev(sel.view(np.int32)), dev(sc)
        stride = 0 if shared else NW
        with np.errstate(invalid="ignore", over="ignore"):
            if t == 3:
                oracle.step_qrda(dense, sc, d, bucket, ox, oG, oz, t, eta, lam, delta, requant)
            else:
                oracle.step_qcmd(dense, sc, d, bucket, ox, oG, oz if t == 1 else None, eta, lam, delta, requant)
        if t == 3:
            qa.qa_step_qrda_selected(L, ind_d, stride, sel_d, sc_d, xd, Gd, zd, t, eta, lam, delta, requant, ws)
        else:
            qa.qa_step_qcmd_selected(L, ind_d, stride, sel_d, sc_d, xd, Gd, zd if t == 1 else None,
                                     eta, lam, delta, requant, ws)
        torch.cuda.synchronize()
        for got, ref, name in ((xd, ox, "x"), (Gd, oG, "G"), (zd, oz, "z")):
            gh = host(got)
            same = (gh.view(np.uint32) == ref.view(np.uint32)) | (np.isnan(gh) & np.isnan(ref))
            assert same.all(), (name, t, int((~same).sum()))
    assert p == 0.0 or wide or np.count_nonzero(ox) > 0


@pytest.mark.parametrize("d,M,bucket,p,requant,shared", [
    (1000, 3, 0, 0.3, 2, False), (4097, 5, 4096, 0.05, 1, False), (70001, 16, 4096, 0.3, 1, False),
    (70001, 3, 4096, 0.2, 2, False), (70001, 4, 4096, 0.2, 1, True), (20000, 2, 4096, 0.0, 1, False),
    (70001, 4, 0, 0.2, 2, False), (70001, 3, 512, 0.3, 1, False), (70001, 3, 8192, 0.3, 1, True)])
def test_server_call_on_sparse_messages_matches_oracle(d, M, bucket, p, requant, shared):
    """qa_aggregate_quantize_selected == oracle decode, average, quantizer on the average; then
    qa_select_codes with the synchronous indicator gives the pushed message."""
    rng = np.random.default_rng(d + M)
    L = qa.Layout.make(d, M, bucket)
    nb, W, NW = L.n_buckets, L.words, (d + 31) // 32
    g = (rng.standard_normal((M, d)) * rng.choice([1e-3, 0.02], (M, d))).astype(np.float32)
    ind = random_indicator(rng, 1 if shared else M, d, p)
    sel = np.full((M, L.code_stride), 0x5A5A5A5A, np.uint32)
    sc = np.zeros((M, nb), np.float32)
    dense = np.zeros((M, W), np.uint32)
    area = area_words(d, bucket)
    for m in range(M):
        im = ind[0 if shared else m]
        o_sel, o_cnt, o_sc, _ = oracle.quantize_selected(g[m], im, bucket=bucket)
        for k in range(nb):
            nwk = (int(o_cnt[k]) + 15) // 16
            lo = k * area
            sel[m, lo: lo + nwk] = o_sel[lo: lo + nwk]
        sc[m] = o_sc
        dense[m] = oracle.decode_selected(im, o_sel, d, bucket=bucket)
    bq = bucket if requant == 1 else 0
    gbar = oracle.aggregate(dense, sc, d, bucket)
    qc_ref, qs_ref, _ = oracle.quantize_pack(gbar[None, :], bucket=bq)
    L1 = qa.Layout.make(d, 1, bq)
    qc = torch.full((1, L1.code_stride), -1, dtype=torch.int32, device=DEV)
    qs = torch.full((1, L1.scale_stride), -7.0, dtype=torch.float32, device=DEV)
    ws = workspace(qa.qa_workspace_bytes(L, qa.QA_OP_STEP_SELECTED))
    ind_d = dev(ind.view(np.int32))
    syn_k = torch.full((NW + 2,), -1, dtype=torch.int32, device=DEV)
    qa.qa_aggregate_quantize_selected(L, ind_d, 0 if shared else NW, dev(sel.view(np.int32)), dev(sc),
                                      requant, qc, qs, None, syn_k, ws)
    torch.cuda.synchronize()
    assert np.array_equal(host(qc).view(np.uint32)[:, :W], qc_ref)
    assert np.array_equal(host(qs)[:, :L1.n_buckets].view(np.uint32), qs_ref.view(np.uint32))
    # the synchronous indicator comes out of the same pass
    assert np.array_equal(host(syn_k).view(np.uint32)[:NW], oracle.indicator_or(ind, d))
    assert np.all(host(syn_k)[NW:] == -1)
    if bq == bucket:                                     # the pushed message S(q_t, I_syn)
        syn = torch.zeros(NW, dtype=torch.int32, device=DEV)
        ind_all = ind_d if not shared else ind_d.repeat(M, 1)
        qa.qa_indicator_or(L, ind_all, NW, syn)
        L1s = qa.Layout.make(d, 1, bucket)
        push = torch.zeros((1, L1s.code_stride), dtype=torch.int32, device=DEV)
        cnt = torch.zeros((1, nb), dtype=torch.int32, device=DEV)
        qa.qa_select_codes(L1s, qc, syn, 0, push, cnt, workspace(qa.qa_workspace_bytes(L1s, qa.QA_OP_SELECT)))
        torch.cuda.synchronize()
        o_push, o_cnt = oracle.select_codes(qc_ref[0], oracle.indicator_or(ind if not shared else np.repeat(ind, M, 0), d), d, bucket)
        assert np.array_equal(host(cnt).view(np.uint32)[0], o_cnt)
        for k in range(nb):
            nwk = (int(o_cnt[k]) + 15) // 16
            assert np.array_equal(host(push).view(np.uint32)[0, k * area: k * area + nwk], o_push[k * area: k * area + nwk])


def test_sparse_steps_check_their_arguments():
    L = qa.Layout.make(100000, 2, 1024)
    t = torch.zeros(8, dtype=torch.int32, device=DEV)
    f = torch.zeros(8, dtype=torch.float32, device=DEV)
    with pytest.raises(qa.QaError) as e:                             # needs room for the decoded codes
        qa.qa_step_qcmd_selected(L, t, 100000, t, f, f, f, None, 0.1, 0.0, 1e-8, 0, None)
    assert e.value.code == -3
    L = qa.Layout.make(100000, 2, 4096)
    with pytest.raises(qa.QaError) as e:                             # indicator rows overlap
        qa.qa_step_qrda_selected(L, t, 5, t, f, f, f, f, 1, 0.1, 0.0, 1e-8, 0, None)
    assert e.value.code == -1
    with pytest.raises(qa.QaError) as e:                             # no indicator
        qa.qa_step_qrda_selected(L, None, 0, t, f, f, f, f, 1, 0.1, 0.0, 1e-8, 0, None)
    assert e.value.code == -1


@pytest.mark.parametrize("b", [4096, 0])
@pytest.mark.parametrize("method", ["qcmd", "qrda"])
def test_training_with_selection_matches_oracle(method, b):
    """Algorithm 1 with the indicator: local gradients -> indicator -> Q(S(g, I)) -> decode ->
    fused step (alternating with the step that takes the sparse messages), on the CSR stand-in
    (d = 2^18 here), T = 25.  Both sides run the whole loop.  b = 0 is the paper's own message:
    one scale, d indicator bits and 2k code bits per worker."""
    d, M, B, T = 1 << 18, 8, 128, 25
    eta, lam, delta = 0.1, 1e-4, 1e-8
    p = synth.csr_problem(n=1 << 13, d=d, nnz_per_row=50, M=M, seed=3)
    L = qa.Layout.make(d, M, b)
    nb, NW, gs = L.n_buckets, (d + 31) // 32, d
    A, ip, ix, y = dev(p.vals), dev(p.indptr), dev(p.indices), dev(p.y)
    x, G, z = (torch.zeros(d, dtype=torch.float32, device=DEV) for _ in range(3))
    g = torch.zeros((M, gs), dtype=torch.float32, device=DEV)
    ind = torch.zeros((M, NW), dtype=torch.int32, device=DEV)
    sel = torch.zeros((M, L.code_stride), dtype=torch.int32, device=DEV)
    dense = torch.zeros((M, L.code_stride), dtype=torch.int32, device=DEV)
    cnt = torch.zeros((M, nb), dtype=torch.int32, device=DEV)
    sc = torch.zeros((M, nb), dtype=torch.float32, device=DEV)
    ws_g = workspace(qa.qa_workspace_bytes(L, qa.QA_OP_GRAD_CSR))
    ws_sel = workspace(qa.qa_workspace_bytes(L, qa.QA_OP_SELECT))
    ws_step = workspace(qa.qa_workspace_bytes(L, qa.QA_OP_STEP_SELECTED))
    ox, oG, oz = (np.zeros(d, np.float32) for _ in range(3))
    mth = qa.QA_METHOD_QCMD if method == "qcmd" else qa.QA_METHOD_QRDA
    bits_sparse = bits_dense = 0
    for t in range(1, T + 1):
        rows = synth.minibatch_rows(p.n, M, B, t, 3)
        qa.qa_local_grad_batched(qa.QA_CSR, A, ip, ix, p.n, d, y, dev(rows), B, M, x, g, gs, None, ws_g)
        qa.qa_indicator(L, mth, g, gs, x, G, z, t, eta, lam, delta, ind, NW)
        qa.qa_quantize_pack_selected(L, g, gs, ind, NW, sel, cnt, sc, None, ws_sel)
        qa.qa_decode_selected(L, ind, NW, sel, dense, ws_sel)
        if t % 2:                                # odd steps: dense step on the decoded codes
            if method == "qcmd":
                qa.qa_step_qcmd(L, dense, sc, x, G, z, eta, lam, delta, 0, None)
            else:
                qa.qa_step_qrda(L, dense, sc, x, G, z, t, eta, lam, delta, 0, None)
        else:                                    # even steps: the step reads the sparse messages itself
            if method == "qcmd":
                qa.qa_step_qcmd_selected(L, ind, NW, sel, sc, x, G, z, eta, lam, delta, 0, ws_step)
            else:
                qa.qa_step_qrda_selected(L, ind, NW, sel, sc, x, G, z, t, eta, lam, delta, 0, ws_step)
        # oracle side
        og = np.stack([oracle.local_grad_csr(p.vals, p.indptr, p.indices, d, p.y, rows[m], ox)[0] for m in range(M)])
        oind = np.stack([oracle.indicator(mth, og[m], ox, oG, oz, t, eta, lam, delta) for m in range(M)])
        ocodes = np.zeros((M, L.words), np.uint32)
        oscales = np.zeros((M, nb), np.float32)
        k_total = 0
        for m in range(M):
            s_, c_, sc_, _ = oracle.quantize_selected(og[m], oind[m], bucket=b)
            ocodes[m] = oracle.decode_selected(oind[m], s_, d, bucket=b)
            oscales[m] = sc_
            k_total += int(c_.sum())
        if method == "qcmd":
            oracle.step_qcmd(ocodes, oscales, d, b, ox, oG, oz, eta, lam, delta)
        else:
            oracle.step_qrda(ocodes, oscales, d, b, ox, oG, oz, t, eta, lam, delta)
        torch.cuda.synchronize()
        assert np.array_equal(host(ind).view(np.uint32), oind), f"indicator, step {t}"
        assert int(host(cnt).view(np.uint32).sum()) == k_total
        assert np.array_equal(host(dense).view(np.uint32)[:, :L.words], ocodes), f"codes, step {t}"
        assert np.array_equal(host(x) == 0, ox == 0), f"zero set, step {t}"
        for nm, a_, o_ in (("x", x, ox), ("G", G, oG), ("z", z, oz)):
            assert np.allclose(host(a_), o_, rtol=1e-5, atol=0), f"{nm}, step {t}"
        bits_sparse += M * (32 * nb + d) + 2 * k_total
        bits_dense += M * (32 * nb + 2 * d)
    print(f"{method}: message bits with selection / dense = {bits_sparse / bits_dense:.3f}; "
          f"nnz(x) = {(ox != 0).sum()}")
    assert bits_sparse < 0.6 * bits_dense
