"""Parity of the tensor-list entry points (one flat vector holding many tensors, each quantized
on its own) with the CPU oracle, through the C ABI.  Codes, scales, thresholds and zero sets must
be bit-exact; state is asserted within 1e-5 (and is bit-exact in practice)."""
import numpy as np
import pytest
import torch

import oracle

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2208_05631_amd as qa
    from gpu_util import DEV, dev, host, workspace

RTOL = 1e-5


def layout_of(lengths, gaps=(0, 1, 3)):
    begin, pos = [], 0
    for i, n in enumerate(lengths):
        begin.append(pos)
        pos = (pos + n + 15) // 16 * 16 + 16 * gaps[i % len(gaps)]
    return np.array(begin, np.int64), np.array(lengths, np.int64), pos + 7


CASES = {
    "mixed": [150, 6, 2400, 16, 0, 48000, 120, 1, 10, 4097, 33],
    "many_small_in_one_tile": [16] * 40 + [5] * 30 + [100] * 20,
    "conv_net_like": [1 * 5 * 5 * 6, 6, 6 * 5 * 5 * 16, 16, 400 * 120, 120, 120 * 84, 84, 84 * 10, 10],
    "one_large": [3 * 4096 + 77],
    "tile_aligned": [4096, 8192, 4096],
    "all_empty": [0, 0, 0],
}


def close(a, b, what):
    if np.array_equal(a, b):
        return
    err = np.max(np.abs(a.astype(np.float64) - b) / np.maximum(np.abs(b), 1e-30))
    assert err <= RTOL, f"{what}: max rel err {err}"


class Flat:
    def __init__(self, lengths, M, seed):
        self.begin, self.length, self.d = layout_of(lengths)
        self.M, self.nseg = M, len(lengths)
        rng = np.random.default_rng(seed)
        self.rng = rng
        self.tensor_scale = 10.0 ** rng.integers(-4, 2, self.nseg)
        self.covered = np.zeros(self.d, bool)
        for b, n in zip(self.begin, self.length):
            self.covered[b:b + n] = True
        self.L = qa.Layout.make(self.d, M, 0, 0.75, None, self.nseg)
        self.table = torch.zeros(qa.qa_segment_plan_bytes(self.d, self.nseg), dtype=torch.uint8, device=DEV)
        self.plan = qa.qa_segment_plan_init(self.d, self.begin, self.length, self.table)
        self.gs = (self.d + 3) // 4 * 4

    def grads(self):
        g = self.rng.standard_normal((self.M, self.d)) * 0.5            # junk between tensors too
        for k, (b, n) in enumerate(zip(self.begin, self.length)):
            g[:, b:b + n] *= self.tensor_scale[k]
            g[:, b:b + n] *= self.rng.random((self.M, n)) < 0.7          # some exact zeros
        return g.astype(np.float32)

    def gpu_quantize(self, g):
        gp = np.zeros((self.M, self.gs), np.float32)
        gp[:, :self.d] = g
        codes = torch.full((self.M, self.L.code_stride), 0x5A5A5A5A, dtype=torch.int32, device=DEV)
        scales = torch.full((self.M, self.nseg), -7.0, dtype=torch.float32, device=DEV)
        th = torch.full((self.M, self.nseg), -7.0, dtype=torch.float32, device=DEV)
        ws = workspace(qa.qa_segment_workspace_bytes(self.plan, self.M, qa.QA_OP_QUANTIZE))
        qa.qa_quantize_pack_segments(self.L, self.plan, dev(gp), self.gs, codes, scales, th, ws)
        torch.cuda.synchronize()
        return codes, scales, th


@pytest.mark.parametrize("case", sorted(CASES))
@pytest.mark.parametrize("M", [1, 3, 8])
def test_quantize_pack_segments_matches_oracle(case, M):
    f = Flat(CASES[case], M, seed=len(case) + M)
    g = f.grads()
    c_ref, s_ref, th_ref = oracle.quantize_pack_segments(g, f.begin, f.length)
    codes, scales, th = f.gpu_quantize(g)
    c = host(codes).view(np.uint32)
    touched = np.zeros(f.L.words, bool)
    for b, n in zip(f.begin, f.length):
        touched[b // 16:(b + n + 15) // 16] = True
    assert np.array_equal(c[:, touched], c_ref[:, touched])
    assert (c[:, ~touched] == 0x5A5A5A5A).all()                         # left alone
    assert np.array_equal(host(scales).view(np.uint32), s_ref.view(np.uint32))
    assert np.array_equal(host(th).view(np.uint32), th_ref.view(np.uint32))


@pytest.mark.parametrize("case", sorted(CASES))
@pytest.mark.parametrize("M,requant", [(1, False), (4, False), (4, True), (8, True), (6, False)])
def test_steps_over_segments_match_oracle(case, M, requant):
    f = Flat(CASES[case], M, seed=7 * len(case) + M)
    rng = f.rng
    for method in ("qcmd_z", "qcmd", "qrda"):
        x = (rng.standard_normal(f.d) * 0.05).astype(np.float32)
        G = (rng.random(f.d) * 1e-3).astype(np.float32)
        z = (rng.standard_normal(f.d) * 0.01).astype(np.float32)
        xr, Gr, zr = x.copy(), G.copy(), z.copy()
        xd, Gd, zd = dev(x), dev(G), dev(z)
        ws = workspace(qa.qa_segment_workspace_bytes(f.plan, M, qa.QA_OP_STEP))
        rq = qa.QA_REQUANT_BUCKET if requant else qa.QA_REQUANT_NONE
        for t in range(1, 4):
            g = f.grads()
            c_ref, s_ref, _ = oracle.quantize_pack_segments(g, f.begin, f.length)
            codes, scales, _ = f.gpu_quantize(g)
            if method == "qrda":
                oracle.step_segments(oracle.QRDA, c_ref, s_ref, f.d, f.begin, f.length, xr, Gr, zr, t,
                                     0.1, 1e-3, 1e-8, requant)
                qa.qa_step_qrda_segments(f.L, f.plan, codes, scales, xd, Gd, zd, t, 0.1, 1e-3, 1e-8, rq, ws)
            else:
                zz = zr if method == "qcmd_z" else None
                oracle.step_segments(oracle.QCMD, c_ref, s_ref, f.d, f.begin, f.length, xr, Gr, zz, t,
                                     0.1, 1e-3, 1e-8, requant)
                qa.qa_step_qcmd_segments(f.L, f.plan, codes, scales, xd, Gd,
                                         zd if method == "qcmd_z" else None, 0.1, 1e-3, 1e-8, rq, ws)
            torch.cuda.synchronize()
            xg, Gg, zg = host(xd), host(Gd), host(zd)
            what = f"{case} {method} M={M} requant={requant} t={t}"
            assert np.array_equal(xg == 0, xr == 0), what                # zero set: exact
            close(xg, xr, what + " x"); close(Gg, Gr, what + " G"); close(zg, zr, what + " z")
            assert np.array_equal(xg[~f.covered], x[~f.covered])         # between tensors: untouched
            assert np.array_equal(Gg[~f.covered], G[~f.covered])
            assert np.array_equal(zg[~f.covered], z[~f.covered])


def test_segment_calls_reject_what_they_cannot_do():
    f = Flat(CASES["mixed"], 2, seed=1)
    g = f.grads()
    codes, scales, _ = f.gpu_quantize(g)
    x = torch.zeros(f.gs, dtype=torch.float32, device=DEV)
    G = torch.zeros(f.gs, dtype=torch.float32, device=DEV)
    ws = workspace(qa.qa_segment_workspace_bytes(f.plan, 2, qa.QA_OP_STEP))
    with pytest.raises(qa.QaError) as e:
        qa.qa_step_qcmd_segments(f.L, f.plan, codes, scales, x, G, None, 0.1, 0.0, 1e-8,
                                 qa.QA_REQUANT_GLOBAL, ws)
    assert e.value.code == -5
    with pytest.raises(qa.QaError) as e:                                # second quantization needs ws
        qa.qa_step_qcmd_segments(f.L, f.plan, codes, scales, x, G, None, 0.1, 0.0, 1e-8,
                                 qa.QA_REQUANT_BUCKET, None)
    assert e.value.code == -3
    Lb = qa.Layout.make(f.d, 2, 4096, 0.75, None, max(f.nseg, (f.d + 4095) // 4096))
    with pytest.raises(qa.QaError) as e:                                # buckets and tensors do not mix
        qa.qa_step_qcmd_segments(Lb, f.plan, codes, scales, x, G, None, 0.1, 0.0, 1e-8, 0, None)
    assert e.value.code == -1
    Ls = qa.Layout.make(f.d, 2, 0, 0.75, None, f.nseg - 1)
    with pytest.raises(qa.QaError) as e:                                # a scale per tensor is needed
        qa.qa_step_qcmd_segments(Ls, f.plan, codes, scales, x, G, None, 0.1, 0.0, 1e-8, 0, None)
    assert e.value.code == -1
    Ld = qa.Layout.make(f.d + 16, 2, 0, 0.75, None, f.nseg)
    with pytest.raises(qa.QaError) as e:                                # plan of another vector
        qa.qa_step_qcmd_segments(Ld, f.plan, codes, scales, x, G, None, 0.1, 0.0, 1e-8, 0, None)
    assert e.value.code == -1
