"""Parity at the benchmark's full sizes and launch configuration, on sampled buckets.

With per-bucket scales and no second quantization (or the per-bucket one) every output of the
path depends only on its own 4096-coordinate bucket, so the oracle can recompute sampled
buckets exactly: the generated gradients of those buckets are copied to the host (the values
are consumed, not compared), quantized and stepped by the oracle for every step, and compared
with what the full-size GPU run left in the same places.

Every configuration runs its stated number of steps (T = 50 / 20 / 10).  Thresholds and scales
are compared bit for bit first; where one differs, what the arithmetic guarantees is checked
instead (within one ulp; codes bit-exact for the GPU's own threshold), the oracle continues from
the GPU's message for that bucket, and the count of such buckets is reported and bounded."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2208_05631_amd import synth

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2208_05631_amd as qa
    from gpu_util import DEV, host, quantizer_parity

CASES = {
    # name: d, M, generator, lambda, schedule, requant, T (the configuration's stated step count)
    "opt_qcmd_1e8_M8": (10 ** 8, 8, synth.grad_student_t_sparse, 1e-5, "qcmd", 0, 50),
    "opt_qrda_2.5e8_M32": (250_000_000, 32, synth.grad_gaussian_biased, 1e-5, "qrda", 0, 20),
    "opt_qrda_2.5e8_M32_requant": (250_000_000, 32, synth.grad_gaussian_biased, 1e-5, "qrda", 1, 4),
    "largest_2^30_M64": (1 << 30, 64, synth.grad_laplace_sparse, 1e-6, "alternate", 0, 10),
    # more than 2^32 coordinates: every index and byte offset past 32 bits, ragged last bucket
    "beyond_2^32_M2": ((1 << 32) + 3 * 4096 + 76, 2, synth.grad_laplace_sparse, 1e-6, "alternate", 1, 3),
}


@pytest.mark.parametrize("name", list(CASES))
def test_sampled_buckets_at_full_size(name):
    d, M, gen, lam, schedule, requant, T = CASES[name]
    T = int(os.environ.get("QA_FULLSIZE_STEPS", T))          # shortens the runs while developing
    b, eta, delta = 4096, 0.1, 1e-8
    nb = (d + b - 1) // b
    rng = np.random.default_rng(17)
    sample = np.unique(np.concatenate([[0, 1, nb - 2, nb - 1], rng.integers(0, nb, 60)]))
    W = (d + 15) // 16
    L = qa.Layout.make(d, M, b, code_stride=qa.Layout.spaced_code_stride(d))   # bench.py's stride
    L1 = qa.Layout.make(d, 1, b, code_stride=L.code_stride, scale_stride=L.scale_stride)
    codes = torch.zeros((M, L.code_stride), dtype=torch.int32, device=DEV)
    scales = torch.zeros((M, L.scale_stride), dtype=torch.float32, device=DEV)
    thr = torch.zeros((M, L.scale_stride), dtype=torch.float32, device=DEV)
    x, G, z = (torch.zeros(d, dtype=torch.float32, device=DEV) for _ in range(3))
    gbuf = torch.empty(d, dtype=torch.float32, device=DEV)
    lens = [min(b, d - k * b) for k in sample]
    ox = [np.zeros(n, np.float32) for n in lens]
    oG = [np.zeros(n, np.float32) for n in lens]
    oz = [np.zeros(n, np.float32) for n in lens]
    idx = torch.from_numpy(np.concatenate([np.arange(k * b, k * b + n) for k, n in zip(sample, lens)])).to(DEV)
    offs = np.concatenate([[0], np.cumsum(lens)])
    ks = torch.from_numpy(sample).to(DEV)
    last_bit = 0                                              # buckets whose Delta or s was 1 ulp off

    for t in range(1, T + 1):
        g_s = np.empty((M, int(offs[-1])), np.float32)
        for m in range(M):
            gen(d, m, t, device=DEV, out=gbuf)
            qa.qa_quantize_pack(L1, gbuf, d, codes[m], scales[m], thr[m], 0, None)
            g_s[m] = host(gbuf[idx])
        kind = schedule if schedule != "alternate" else ("qcmd" if t % 2 else "qrda")
        if kind == "qcmd":
            qa.qa_step_qcmd(L, codes, scales, x, G, z if schedule == "alternate" else None, eta, lam,
                            delta, requant, None)
        else:
            qa.qa_step_qrda(L, codes, scales, x, G, z, t, eta, lam, delta, requant, None)
        torch.cuda.synchronize()
        xs, Gs, zs = host(x[idx]), host(G[idx]), host(z[idx])
        sc_s, th_s = host(scales[:, ks]), host(thr[:, ks])
        nonzero_codes = 0
        for j, (k, n) in enumerate(zip(sample, lens)):
            lo, hi = int(offs[j]), int(offs[j + 1])
            oc, osc, oth = oracle.quantize_pack(g_s[:, lo:hi], bucket=b)
            w0, w1 = k * (b // 16), k * (b // 16) + (n + 15) // 16
            gc = host(codes[:, w0:w1]).view(np.uint32)
            if not (np.array_equal(gc, oc) and np.array_equal(sc_s[:, j], osc[:, 0])
                    and np.array_equal(th_s[:, j], oth[:, 0])):
                last_bit += quantizer_parity(g_s[:, lo:hi], b, gc, sc_s[:, j:j + 1], th_s[:, j:j + 1],
                                             what=f"(bucket {k}, step {t})")
                oc, osc = gc, np.ascontiguousarray(sc_s[:, j:j + 1])
            nonzero_codes += int((oracle.unpack(oc[0], n) != 0).sum())
            if kind == "qcmd":
                oracle.step_qcmd(oc, osc, n, b, ox[j], oG[j], oz[j] if schedule == "alternate" else None,
                                 eta, lam, delta, requant)
            else:
                oracle.step_qrda(oc, osc, n, b, ox[j], oG[j], oz[j], t, eta, lam, delta, requant)
            assert np.array_equal(xs[lo:hi] == 0, ox[j] == 0), f"zero set, bucket {k}, step {t}"
            for nm, a, o in (("x", xs, ox[j]), ("G", Gs, oG[j]), ("z", zs, oz[j])):
                if not np.array_equal(a[lo:hi], o):
                    err = np.max(np.abs(a[lo:hi].astype(np.float64) - o) / np.maximum(np.abs(o), 1e-30))
                    assert err <= 1e-5, f"{nm}, bucket {k}, step {t}: rel err {err}"
        assert nonzero_codes > 0
    assert last_bit <= 2, f"{last_bit} sampled buckets with a threshold or scale one ulp off"
    print(f"{name}: T = {T}, {len(sample)} buckets x {M} workers per step, "
          f"{last_bit} with a last-bit difference in threshold or scale")
    # a property that holds at any size: coordinates never touched by any worker keep G == 0
    assert float(G.min().item()) >= 0.0
    # the server's call on the last step's messages, same sampled buckets
    qc = torch.zeros((1, L.code_stride), dtype=torch.int32, device=DEV)
    qs = torch.zeros((1, L.scale_stride), dtype=torch.float32, device=DEV)
    qa.qa_aggregate_quantize(L, codes, scales, qa.QA_REQUANT_BUCKET, qc, qs, None, None)
    torch.cuda.synchronize()
    for j, (k, n) in enumerate(zip(sample, lens)):
        lo, hi = int(offs[j]), int(offs[j + 1])
        oc, osc, _ = oracle.quantize_pack(g_s[:, lo:hi], bucket=b)
        qc_ref, qs_ref, _ = oracle.quantize_pack(oracle.aggregate(oc, osc, n, b)[None, :], bucket=b)
        w0, w1 = k * (b // 16), k * (b // 16) + (n + 15) // 16
        assert np.array_equal(host(qc[0, w0:w1]).view(np.uint32), qc_ref[0]), f"q_t codes, bucket {k}"
        assert host(qs[0, k]) == qs_ref[0, 0], f"q_t scale, bucket {k}"


def test_sparse_encoding_beyond_2_32_coordinates():
    """Indicator, selected quantizer, code selection, decoder and the step on the sparse message
    with every index past 32 bits: all are local to a 4096-bucket, so sampled buckets are checked
    against the oracle."""
    d, M, b = (1 << 32) + 5 * 4096 + 40, 1, 4096
    eta, lam, delta, t = 0.1, 1e-4, 1e-8, 7
    nb, NW = (d + b - 1) // b, (d + 31) // 32
    L = qa.Layout.make(d, M, b)
    gen = torch.Generator(device=DEV); gen.manual_seed(3)
    g = torch.empty(d, dtype=torch.float32, device=DEV)
    synth.grad_laplace_sparse(d, 0, 1, device=DEV, out=g)
    x = torch.zeros(d, dtype=torch.float32, device=DEV)
    G = torch.zeros(d, dtype=torch.float32, device=DEV)
    z = torch.zeros(d, dtype=torch.float32, device=DEV)
    rng = np.random.default_rng(23)
    sample = np.unique(np.concatenate([[0, 1], np.arange(nb - 6, nb), rng.integers(0, nb, 20)]))   # the last six lie past 2^32
    for k in sample:                                       # a state worth marking, in the samples
        n = min(b, d - k * b)
        x[k * b:k * b + n] = torch.from_numpy((rng.standard_normal(n) * 0.1 * (rng.random(n) < 0.1)).astype(np.float32)).to(DEV)
        G[k * b:k * b + n] = torch.from_numpy((rng.random(n) * 1e-6).astype(np.float32)).to(DEV)
        z[k * b:k * b + n] = torch.from_numpy((rng.standard_normal(n) * 7e-4).astype(np.float32)).to(DEV)
    ind = torch.zeros((1, NW), dtype=torch.int32, device=DEV)
    sel = torch.zeros((1, L.code_stride), dtype=torch.int32, device=DEV)
    cnt = torch.zeros((1, nb), dtype=torch.int32, device=DEV)
    sc = torch.zeros((1, nb), dtype=torch.float32, device=DEV)
    dense = torch.zeros((1, L.code_stride), dtype=torch.int32, device=DEV)
    again = torch.zeros((1, L.code_stride), dtype=torch.int32, device=DEV)
    cnt2 = torch.zeros((1, nb), dtype=torch.int32, device=DEV)
    kept = []
    for method in (0, 1):
        qa.qa_indicator(L, method, g, d, x, G, z, t, eta, lam, delta, ind, NW)
        qa.qa_quantize_pack_selected(L, g, d, ind, NW, sel, cnt, sc, None)
        qa.qa_decode_selected(L, ind, NW, sel, dense)
        qa.qa_select_codes(L, dense, ind, NW, again, cnt2)
        torch.cuda.synchronize()
        marked = 0
        for k in sample:
            n = min(b, d - k * b)
            lo = int(k) * b
            gs, xs, Gs, zs = (host(v[lo:lo + n]) for v in (g, x, G, z))
            o_ind = oracle.indicator(method, gs, xs, Gs, zs, t, eta, lam, delta)
            nw = (n + 31) // 32
            assert np.array_equal(host(ind[0, k * 128:k * 128 + nw]).view(np.uint32), o_ind), (method, k)
            o_sel, o_cnt, o_sc, _ = oracle.quantize_selected(gs, o_ind, bucket=0)
            assert int(host(cnt[0, k])) == int(o_cnt[0]) and host(sc[0, k]) == o_sc[0]
            nwk = (int(o_cnt[0]) + 15) // 16
            assert np.array_equal(host(sel[0, k * 256:k * 256 + nwk]).view(np.uint32), o_sel[:nwk])
            o_dense = oracle.decode_selected(o_ind, o_sel, n, bucket=0)
            assert np.array_equal(host(dense[0, k * 256:k * 256 + (n + 15) // 16]).view(np.uint32), o_dense)
            assert np.array_equal(host(again[0, k * 256:k * 256 + nwk]), host(sel[0, k * 256:k * 256 + nwk]))
            assert int(host(cnt2[0, k])) == int(o_cnt[0])
            marked += int(o_cnt[0])
            if method == 1:
                kept.append((int(k), n, o_dense, o_sc, xs.copy(), Gs.copy(), zs.copy()))
        assert marked > 0
    # the step that reads the sparse message directly (in place, last: it changes the state)
    qa.qa_step_qrda_selected(L, ind, NW, sel, sc, x, G, z, t, eta, lam, delta, qa.QA_REQUANT_NONE, None)
    torch.cuda.synchronize()
    for k, n, o_dense, o_sc, xs, Gs, zs in kept:
        oracle.step_qrda(o_dense[None, :], np.asarray(o_sc, np.float32).reshape(1, 1), n, 0, xs, Gs, zs,
                         t, eta, lam, delta)
        lo = k * b
        for got, ref in ((x, xs), (G, Gs), (z, zs)):
            assert np.array_equal(host(got[lo:lo + n]).view(np.uint32), ref.view(np.uint32)), k


def test_tensor_list_beyond_2_32_coordinates():
    """Tensor-list quantizer and step on a flat vector longer than 2^32: one tensor of almost 2^32
    elements (over a million pieces) and two small ones that start past 2^32.  The small tensors
    are compared with the oracle exactly; the large one by its definition on the device in
    binary64 (library reductions) and, given its threshold and scale, exactly on sampled elements."""
    big = (1 << 32) - 1000
    begin = np.array([0, 1 << 32, (1 << 32) + 8192], np.int64)
    length = np.array([big, 5000, 77], np.int64)
    d = int(begin[-1] + length[-1]) + 3
    d += (-d) % 4
    eta, lam, delta = 0.1, 1e-6, 1e-8
    L = qa.Layout.make(d, 1, 0, 0.75, None, 3)
    table = torch.zeros(qa.qa_segment_plan_bytes(d, 3), dtype=torch.uint8, device=DEV)
    plan = qa.qa_segment_plan_init(d, begin, length, table)
    assert plan.n_pieces == (big + 4095) // 4096 + 2 + 1
    g = torch.empty(d, dtype=torch.float32, device=DEV)
    synth.grad_laplace_sparse(d, 0, 1, device=DEV, out=g)
    codes = torch.zeros((1, L.code_stride), dtype=torch.int32, device=DEV)
    scales = torch.zeros((1, 3), dtype=torch.float32, device=DEV)
    th = torch.zeros((1, 3), dtype=torch.float32, device=DEV)
    wq = torch.empty(qa.qa_segment_workspace_bytes(plan, 1, qa.QA_OP_QUANTIZE), dtype=torch.uint8, device=DEV)
    x = torch.zeros(d, dtype=torch.float32, device=DEV)
    G = torch.zeros(d, dtype=torch.float32, device=DEV)
    qa.qa_quantize_pack_segments(L, plan, g, d, codes, scales, th, wq)
    qa.qa_step_qcmd_segments(L, plan, codes, scales, x, G, None, eta, lam, delta, 0, None)
    torch.cuda.synchronize()
    s_h, th_h = host(scales)[0], host(th)[0]
    # small tensors, past 2^32: exact
    for k in (1, 2):
        b0, n = int(begin[k]), int(length[k])
        gs = host(g[b0:b0 + n])[None, :]
        oc, osc, oth = oracle.quantize_pack(gs, bucket=0)
        assert np.array_equal(host(codes[0, b0 // 16:b0 // 16 + (n + 15) // 16]).view(np.uint32), oc[0])
        assert s_h[k] == osc[0, 0] and th_h[k] == oth[0, 0]
        ox, oG = np.zeros(n, np.float32), np.zeros(n, np.float32)
        oracle.step_qcmd(oc, osc, n, 0, ox, oG, None, eta, lam, delta)
        assert np.array_equal(host(x[b0:b0 + n]), ox) and np.array_equal(host(G[b0:b0 + n]), oG)
    # the large tensor: threshold and scale from their definitions, in binary64 on the device
    a = g[:big].abs()
    D = 0.75 * float(a.sum(dtype=torch.float64).item()) / big
    assert abs(th_h[0] - D) <= 1e-6 * D
    kept = a > float(th_h[0])
    s_def = float(torch.where(kept, a, torch.zeros((), device=DEV)).sum(dtype=torch.float64).item()) / \
        int(kept.sum(dtype=torch.int64).item())
    assert abs(s_h[0] - s_def) <= 1e-6 * s_def
    del a, kept
    rng = np.random.default_rng(5)
    idx = np.unique(np.concatenate([[0, 1, big - 2, big - 1], rng.integers(0, big, 4000)]))
    it = torch.from_numpy(idx).to(DEV)
    gv = host(g[it])
    words = host(codes[0][it // 16]).view(np.uint32)
    field = (words >> (2 * (idx % 16)).astype(np.uint32)) & 3
    want = np.where(gv > th_h[0], 1, np.where(gv < -th_h[0], 3, 0))
    assert np.array_equal(field, want)
    q = (np.where(field == 1, 1.0, np.where(field == 3, -1.0, 0.0)) * s_h[0]).astype(np.float32)
    ox, oG = np.zeros(idx.size, np.float32), np.zeros(idx.size, np.float32)
    oracle.update_qcmd(q, ox, oG, None, eta, lam, delta)
    assert np.array_equal(host(x[it]), ox) and np.array_equal(host(G[it]), oG)
    # between and after the tensors nothing is touched
    assert not bool(x[big:1 << 32].any()) and not bool(x[int(begin[2]) + 77:].any())
