"""Seeded random shapes through the C ABI against the oracle: quantize+pack, the three fused steps
with every second-quantization mode, the server's call, and (where the sparse encoding applies)
the selected quantizer and the step on sparse messages; in a second test tensor lists, the exact
and the stochastic quantizer, the indicator and code selection.  Everything is compared bit for
bit; the shapes mix tiny, ragged and multi-tile vectors, worker counts on both sides of the chunk
sizes, every bucket size, ties, sparse, and scales spread over 80 binades."""
import numpy as np
import pytest
import torch

import oracle

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2208_05631_amd as qa
    from gpu_util import DEV, dev, host, ulp_distance, workspace


def random_indicator(rng, M, d, p):
    bits = rng.random((M, d)) < p
    ind = np.zeros((M, (d + 31) // 32), np.uint32)
    for m in range(M):
        idx = np.nonzero(bits[m])[0]
        np.bitwise_or.at(ind[m], idx // 32, (np.uint32(1) << (idx % 32).astype(np.uint32)))
    return ind


def same_bits(a, b):
    a, b = np.asarray(a), np.asarray(b)
    return a.shape == b.shape and bool(((a.view(np.uint32) == b.view(np.uint32)) | (np.isnan(a) & np.isnan(b))).all())


def random_gradients(rng, kind, M, d):
    if kind == "gauss":
        g = rng.standard_normal((M, d)) * 10.0 ** rng.integers(-6, 2)
    elif kind == "sparse":
        g = rng.laplace(0, 1e-3, (M, d)) * (rng.random((M, d)) < 0.05)
    elif kind == "ties":
        g = rng.integers(-2, 3, (M, d)).astype(np.float64) * 0.25
    else:                                                # scales of the workers far apart: ordered sum
        g = rng.standard_normal((M, d)) * np.exp2(rng.integers(-40, 40, (M, 1)))
    return g.astype(np.float32)


@pytest.mark.parametrize("seed", range(6))
def test_random_shapes_match_oracle_bit_for_bit(seed):
    rng = np.random.default_rng(1000 + seed)
    for case in range(60):
        d = int(rng.choice([rng.integers(1, 70), rng.integers(70, 5000), rng.integers(5000, 40000)]))
        M = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 12, 16, 17, 24, 33, 64]))
        bucket = int(rng.choice([0, 64, 128, 256, 512, 1024, 2048, 4096, 8192, 16384]))
        requant = int(rng.choice([0, 1, 2]))
        if requant == 1 and bucket == 0:
            requant = 2
        kind = str(rng.choice(["gauss", "sparse", "ties", "wide"]))
        what = f"seed {seed} case {case}: d={d} M={M} bucket={bucket} requant={requant} {kind}"
        g = random_gradients(rng, kind, M, d)
        L = qa.Layout.make(d, M, bucket)
        gs = (d + 3) // 4 * 4
        gp = np.zeros((M, gs), np.float32)
        gp[:, :d] = g
        # workers: quantize + pack
        oc, osc, oth = oracle.quantize_pack(g, bucket=bucket)
        codes = torch.full((M, L.code_stride), -1, dtype=torch.int32, device=DEV)
        scales = torch.full((M, L.scale_stride), -7.0, dtype=torch.float32, device=DEV)
        th = torch.full((M, L.scale_stride), -7.0, dtype=torch.float32, device=DEV)
        qa.qa_quantize_pack(L, dev(gp), gs, codes, scales, th, 0,
                            workspace(qa.qa_workspace_bytes(L, qa.QA_OP_QUANTIZE)))
        torch.cuda.synchronize()
        assert np.array_equal(host(codes).view(np.uint32)[:, :L.words], oc), what
        assert same_bits(host(scales)[:, :L.n_buckets], osc) and same_bits(host(th)[:, :L.n_buckets], oth), what
        # fused steps
        x0 = (rng.standard_normal(d) * 1e-2 * (rng.random(d) < 0.5)).astype(np.float32)
        G0 = (rng.random(d) * 1e-4).astype(np.float32)
        z0 = (rng.standard_normal(d) * 1e-3).astype(np.float32)
        ws = workspace(qa.qa_workspace_bytes(L, qa.QA_OP_STEP))
        eta, lam, delta, t = 0.1, float(rng.choice([0.0, 1e-4, 1e-2])), 1e-8, int(rng.integers(1, 9))
        for method in ("qcmd", "qcmd_z", "qrda"):
            ox, oG, oz = x0.copy(), G0.copy(), z0.copy()
            xd, Gd, zd = dev(x0), dev(G0), dev(z0)
            with np.errstate(all="ignore"):
                if method == "qrda":
                    oracle.step_qrda(oc, osc, d, bucket, ox, oG, oz, t, eta, lam, delta, requant)
                    qa.qa_step_qrda(L, codes, scales, xd, Gd, zd, t, eta, lam, delta, requant, ws)
                else:
                    zo, zg = (oz, zd) if method == "qcmd_z" else (None, None)
                    oracle.step_qcmd(oc, osc, d, bucket, ox, oG, zo, eta, lam, delta, requant)
                    qa.qa_step_qcmd(L, codes, scales, xd, Gd, zg, eta, lam, delta, requant, ws)
            torch.cuda.synchronize()
            assert same_bits(host(xd), ox) and same_bits(host(Gd), oG) and same_bits(host(zd), oz), (what, method)
        # the server's call
        if requant:
            bq = bucket if requant == 1 else 0
            L1 = qa.Layout.make(d, 1, bq)
            with np.errstate(all="ignore"):
                qc_ref, qs_ref, _ = oracle.quantize_pack(oracle.aggregate(oc, osc, d, bucket)[None, :], bucket=bq)
            qc = torch.full((1, L1.code_stride), -1, dtype=torch.int32, device=DEV)
            qs = torch.full((1, L1.scale_stride), -7.0, dtype=torch.float32, device=DEV)
            qa.qa_aggregate_quantize(L, codes, scales, requant, qc, qs, None, ws)
            torch.cuda.synchronize()
            assert np.array_equal(host(qc).view(np.uint32)[:, :L1.words], qc_ref), what
            assert same_bits(host(qs)[:, :L1.n_buckets], qs_ref), what
        # sparse messages (every bucket size)
        if True:
            p = float(rng.choice([0.0, 0.05, 0.5, 1.0]))
            shared = bool(rng.random() < 0.3)
            ind = random_indicator(rng, 1 if shared else M, d, p)
            nb, W, NW = L.n_buckets, L.words, (d + 31) // 32
            sel = np.full((M, L.code_stride), 0x5A5A5A5A, np.uint32)
            sc = np.zeros((M, nb), np.float32)
            dense = np.zeros((M, W), np.uint32)
            for m in range(M):
                im = ind[0 if shared else m]
                o_sel, o_cnt, o_sc, _ = oracle.quantize_selected(g[m], im, bucket=bucket)
                for k in range(nb):
                    nwk = (int(o_cnt[k]) + 15) // 16
                    lo = k * (((bucket or d) + 15) // 16)
                    sel[m, lo: lo + nwk] = o_sel[lo: lo + nwk]
                sc[m] = o_sc
                dense[m] = oracle.decode_selected(im, o_sel, d, bucket=bucket)
            ind_rows = ind if not shared else np.repeat(ind, M, 0)
            sel_g = torch.full((M, L.code_stride), 0x5A5A5A5A, dtype=torch.int32, device=DEV)
            cnt_g = torch.zeros((M, nb), dtype=torch.int32, device=DEV)
            sc_g = torch.zeros((M, nb), dtype=torch.float32, device=DEV)
            qa.qa_quantize_pack_selected(L, dev(gp), gs, dev(ind_rows.view(np.int32)), NW, sel_g, cnt_g, sc_g, None,
                                         workspace(qa.qa_workspace_bytes(L, qa.QA_OP_SELECT)))
            torch.cuda.synchronize()
            assert np.array_equal(host(sel_g).view(np.uint32), sel) and same_bits(host(sc_g), sc), what
            ox, oG, oz = x0.copy(), G0.copy(), z0.copy()
            xd, Gd, zd = dev(x0), dev(G0), dev(z0)
            with np.errstate(all="ignore"):
                oracle.step_qrda(dense, sc, d, bucket, ox, oG, oz, t, eta, lam, delta, requant)
            qa.qa_step_qrda_selected(L, dev(ind.view(np.int32)), 0 if shared else NW, dev(sel.view(np.int32)),
                                     dev(sc), xd, Gd, zd, t, eta, lam, delta, requant,
                                     workspace(qa.qa_workspace_bytes(L, qa.QA_OP_STEP_SELECTED)))
            torch.cuda.synchronize()
            assert same_bits(host(xd), ox) and same_bits(host(Gd), oG) and same_bits(host(zd), oz), (what, "sparse")


@pytest.mark.parametrize("seed", range(4))
def test_random_shapes_of_the_other_calls_match_oracle_bit_for_bit(seed):
    rng = np.random.default_rng(2000 + seed)
    for case in range(40):
        M = int(rng.choice([1, 2, 3, 5, 8, 13, 16]))
        # ---- a list of tensors in one flat vector ----
        nseg = int(rng.integers(1, 30))
        lengths = [int(rng.choice([0, rng.integers(1, 20), rng.integers(20, 600), rng.integers(600, 9000)]))
                   for _ in range(nseg)]
        begin, pos = [], int(rng.integers(0, 3)) * 16
        for n in lengths:
            begin.append(pos)
            pos = (pos + n + 15) // 16 * 16 + 16 * int(rng.integers(0, 3))
        d = pos + int(rng.integers(1, 40))
        begin, length = np.array(begin, np.int64), np.array(lengths, np.int64)
        what = f"seed {seed} case {case}: tensors {lengths} d={d} M={M}"
        L = qa.Layout.make(d, M, 0, 0.75, None, nseg)
        table = torch.zeros(qa.qa_segment_plan_bytes(d, nseg), dtype=torch.uint8, device=DEV)
        plan = qa.qa_segment_plan_init(d, begin, length, table)
        g = (rng.standard_normal((M, d)) * 10.0 ** rng.integers(-4, 1) * (rng.random((M, d)) < 0.7)).astype(np.float32)
        gs = (d + 3) // 4 * 4
        gp = np.zeros((M, gs), np.float32)
        gp[:, :d] = g
        c_ref, s_ref, th_ref = oracle.quantize_pack_segments(g, begin, length)
        codes = torch.full((M, L.code_stride), 0x5A5A5A5A, dtype=torch.int32, device=DEV)
        scales = torch.full((M, nseg), -7.0, dtype=torch.float32, device=DEV)
        th = torch.full((M, nseg), -7.0, dtype=torch.float32, device=DEV)
        qa.qa_quantize_pack_segments(L, plan, dev(gp), gs, codes, scales, th,
                                     workspace(qa.qa_segment_workspace_bytes(plan, M, qa.QA_OP_QUANTIZE)))
        torch.cuda.synchronize()
        touched = np.zeros(L.words, bool)
        for b_, n_ in zip(begin, length):
            touched[b_ // 16:(b_ + n_ + 15) // 16] = True
        c = host(codes).view(np.uint32)
        assert np.array_equal(c[:, touched], c_ref[:, touched]) and (c[:, ~touched] == 0x5A5A5A5A).all(), what
        assert same_bits(host(scales), s_ref) and same_bits(host(th), th_ref), what
        x0 = (rng.standard_normal(d) * 0.05).astype(np.float32)
        G0 = (rng.random(d) * 1e-3).astype(np.float32)
        z0 = (rng.standard_normal(d) * 0.01).astype(np.float32)
        requant = bool(rng.random() < 0.5)
        rq = qa.QA_REQUANT_BUCKET if requant else qa.QA_REQUANT_NONE
        ws = workspace(qa.qa_segment_workspace_bytes(plan, M, qa.QA_OP_STEP))
        for method in ("qcmd", "qrda"):
            xr, Gr, zr = x0.copy(), G0.copy(), z0.copy()
            xd, Gd, zd = dev(x0), dev(G0), dev(z0)
            if method == "qrda":
                oracle.step_segments(oracle.QRDA, c_ref, s_ref, d, begin, length, xr, Gr, zr, 3, 0.1, 1e-3, 1e-8, requant)
                qa.qa_step_qrda_segments(L, plan, codes, scales, xd, Gd, zd, 3, 0.1, 1e-3, 1e-8, rq, ws)
            else:
                oracle.step_segments(oracle.QCMD, c_ref, s_ref, d, begin, length, xr, Gr, zr, 3, 0.1, 1e-3, 1e-8, requant)
                qa.qa_step_qcmd_segments(L, plan, codes, scales, xd, Gd, zd, 0.1, 1e-3, 1e-8, rq, ws)
            torch.cuda.synchronize()
            assert same_bits(host(xd), xr) and same_bits(host(Gd), Gr) and same_bits(host(zd), zr), (what, method, requant)
        # ---- exact ranking threshold, stochastic quantizer ----
        d2 = int(rng.choice([rng.integers(1, 300), rng.integers(300, 30000)]))
        bucket = int(rng.choice([64, 128, 256, 512, 1024, 2048, 4096, 0, 8192, 16384]))   # any size
        kind = str(rng.choice(["gauss", "sparse", "ties"]))
        g2 = random_gradients(rng, kind, M, d2)
        what = f"seed {seed} case {case}: d={d2} M={M} bucket={bucket} {kind}"
        L2 = qa.Layout.make(d2, M, bucket)
        gs2 = (d2 + 3) // 4 * 4
        gp2 = np.zeros((M, gs2), np.float32)
        gp2[:, :d2] = g2
        th_ref = np.stack([oracle.exact_thresholds(g2[m], bucket) for m in range(M)])
        c_ref, s_ref, _ = oracle.quantize_pack(g2, bucket, thresholds=th_ref)
        codes = torch.full((M, L2.code_stride), -1, dtype=torch.int32, device=DEV)
        scales = torch.full((M, L2.scale_stride), -7.0, dtype=torch.float32, device=DEV)
        th = torch.full((M, L2.scale_stride), -7.0, dtype=torch.float32, device=DEV)
        nws = qa.qa_workspace_bytes(L2, qa.QA_OP_QUANTIZE_EXACT)      # buckets over several tiles: a sort
        ws2 = torch.empty(nws, dtype=torch.uint8, device=DEV) if nws else None
        qa.qa_quantize_pack(L2, dev(gp2), gs2, codes, scales, th, qa.QA_THRESH_EXACT, ws2)
        torch.cuda.synchronize()
        assert same_bits(host(th)[:, :L2.n_buckets], th_ref), (what, "exact threshold")
        assert np.array_equal(host(codes).view(np.uint32)[:, :L2.words], c_ref), (what, "exact codes")
        assert int(ulp_distance(host(scales)[:, :L2.n_buckets], s_ref).max()) <= (0 if nws == 0 else 1), \
            (what, "exact scales")
        rseed, step = int(rng.integers(0, 2 ** 62)), int(rng.integers(0, 1000))
        bs = int(rng.choice([0, 64, 256, 2048, 4096, 8192]))
        Ls = qa.Layout.make(d2, M, bs)
        oc, osc = oracle.quantize_pack_stochastic(g2, bucket=bs, seed=rseed, step=step)
        codes = torch.full((M, Ls.code_stride), -1, dtype=torch.int32, device=DEV)
        scales = torch.full((M, Ls.scale_stride), -7.0, dtype=torch.float32, device=DEV)
        qa.qa_quantize_pack_stochastic(Ls, dev(gp2), gs2, codes, scales, rseed, step)
        torch.cuda.synchronize()
        assert np.array_equal(host(codes).view(np.uint32)[:, :Ls.words], oc), (what, "stochastic", bs)
        assert same_bits(host(scales)[:, :Ls.n_buckets], osc), (what, "stochastic", bs)
        # ---- indicator, code selection, decode ----
        d3 = int(rng.choice([rng.integers(1, 5000), rng.integers(5000, 40000)]))
        b3 = int(rng.choice([0, 64, 512, 2048, 4096, 8192]))
        method, lam, t = int(rng.integers(0, 2)), float(rng.choice([0.0, 1e-3, 0.05])), int(rng.integers(1, 9))
        x3 = (rng.standard_normal(d3) * 0.1 * (rng.random(d3) < 0.3)).astype(np.float32)
        G3 = (rng.random(d3) * 10.0 ** rng.integers(-6, 1)).astype(np.float32)
        z3 = (rng.standard_normal(d3) * 0.05).astype(np.float32)
        g3 = (rng.standard_normal((M, d3)) * rng.choice([1e-3, 0.05], (M, d3))).astype(np.float32)
        what = f"seed {seed} case {case}: indicator d={d3} M={M} method={method} lam={lam} t={t}"
        L3, NW = qa.Layout.make(d3, M, b3), (d3 + 31) // 32
        stride = d3 + int(rng.integers(0, 5))
        gp3 = np.zeros((M, stride), np.float32)
        gp3[:, :d3] = g3
        ind = torch.full((M, NW), -1, dtype=torch.int32, device=DEV)
        qa.qa_indicator(L3, method, dev(gp3), stride, dev(x3), dev(G3), dev(z3), t, 0.1, lam, 1e-8, ind, NW)
        torch.cuda.synchronize()
        ref = np.stack([oracle.indicator(method, g3[m], x3, G3, z3, t, 0.1, lam, 1e-8) for m in range(M)])
        assert np.array_equal(host(ind).view(np.uint32), ref), what
        dense_ref, _, _ = oracle.quantize_pack(g3, bucket=b3)
        sel = torch.full((M, L3.code_stride), 0x5A5A5A5A, dtype=torch.int32, device=DEV)
        cnt = torch.zeros((M, L3.n_buckets), dtype=torch.int32, device=DEV)
        ws3 = workspace(qa.qa_workspace_bytes(L3, qa.QA_OP_SELECT))
        qa.qa_select_codes(L3, dev(dense_ref.view(np.int32)), ind, NW, sel, cnt, ws3)
        back = torch.full((M, L3.code_stride), -1, dtype=torch.int32, device=DEV)
        qa.qa_decode_selected(L3, ind, NW, sel, back, ws3)
        torch.cuda.synchronize()
        area = ((b3 or d3) + 15) // 16
        for m in range(M):
            o_sel, o_cnt = oracle.select_codes(dense_ref[m], ref[m], d3, b3)
            assert np.array_equal(host(cnt).view(np.uint32)[m], o_cnt), what
            for k in range(L3.n_buckets):
                nwk = (int(o_cnt[k]) + 15) // 16
                assert np.array_equal(host(sel).view(np.uint32)[m, k * area:k * area + nwk],
                                      o_sel[k * area:k * area + nwk]), what
            assert np.array_equal(host(back).view(np.uint32)[m, :L3.words],
                                  oracle.decode_selected(ref[m], o_sel, d3, bucket=b3)), what


@pytest.mark.parametrize("seed", range(2))
def test_random_gradient_shapes_match_oracle(seed):
    """Dense and CSR minibatch gradients: zero pattern exact, values within 1e-6 (binary64 sums in
    another order, exp/log from another library); repeated rows, duplicate and clustered columns."""
    rng = np.random.default_rng(3000 + seed)
    exact = []
    for case in range(80):
        csr = bool(rng.random() < 0.5)
        n, M = int(rng.integers(1, 400)), int(rng.choice([1, 2, 5, 8, 16]))
        B = int(rng.choice([1, 3, 16, 64, 130, 300]))
        d = int(rng.choice([rng.integers(1, 50), rng.integers(50, 3000), 4 * rng.integers(1, 2000)]))
        y = np.where(rng.random(n) < 0.5, -1.0, 1.0).astype(np.float32)
        x = (rng.standard_normal(d) * 10.0 ** rng.integers(-3, 1)).astype(np.float32)
        rows = rng.integers(0, n, (M, B)).astype(np.int32)
        what = f"seed {seed} case {case}: csr={csr} n={n} d={d} B={B} M={M}"
        if csr:
            k = int(rng.integers(1, min(d, 60) + 1))
            idx = rng.integers(0, d, (n, k)).astype(np.int32)
            if rng.random() < 0.5:
                idx = (idx % max(1, d // 50 + 1)).astype(np.int32)
            vals = rng.standard_normal((n, k)).astype(np.float32)
            indptr = (np.arange(n + 1) * k).astype(np.int64)
            ref = [oracle.local_grad_csr(vals.reshape(-1), indptr, idx.reshape(-1), d, y, rows[m], x) for m in range(M)]
            A_d, ip_d, ix_d = dev(vals.reshape(-1)), dev(indptr), dev(idx.reshape(-1))
            fmt, op = qa.QA_CSR, qa.QA_OP_GRAD_CSR
        else:
            A = rng.standard_normal((n, d)).astype(np.float32)
            ref = [oracle.local_grad_dense(A, y, rows[m], x) for m in range(M)]
            A_d, ip_d, ix_d, fmt, op = dev(A), None, None, qa.QA_DENSE, qa.QA_OP_GRAD_DENSE
        gs = (d + 3) // 4 * 4 + 4 * int(rng.integers(0, 3))
        ws = workspace(qa.qa_workspace_bytes(qa.Layout.make(d, M, 0), op))
        g = torch.full((M, gs), 5.0, dtype=torch.float32, device=DEV)
        loss = torch.zeros(M, dtype=torch.float32, device=DEV)
        qa.qa_local_grad_batched(fmt, A_d, ip_d, ix_d, n, d, dev(y), dev(rows), B, M, dev(x), g, gs, loss, ws)
        torch.cuda.synchronize()
        gg, ll = host(g), host(loss)
        R = np.stack([r[0] for r in ref])
        assert np.all(gg[:, d:] == 5.0), what
        assert np.array_equal(gg[:, :d] != 0, R != 0), what
        assert np.allclose(gg[:, :d], R, rtol=1e-6, atol=1e-30), what
        assert np.allclose(ll, [r[1] for r in ref], rtol=1e-6), what
        exact.append((gg[:, :d] == R).mean())
    assert np.mean(exact) > 0.999
