"""Parity at the benchmark's full sizes and launch configuration, on sampled buckets.

With per-bucket scales and no second quantization (or the per-bucket one) every output of the
path depends only on its own 4096-coordinate bucket, so the oracle can recompute sampled
buckets exactly: the generated gradients of those buckets are copied to the host (the values
are consumed, not compared), quantized and stepped by the oracle for every step, and compared
with what the full-size GPU run left in the same places."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2208_05631_amd import synth

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2208_05631_amd as qa
    from gpu_util import DEV, host

CASES = {
    # name: d, M, generator, lambda, schedule, requant
    "opt_qcmd_1e8_M8": (10 ** 8, 8, synth.grad_student_t_sparse, 1e-5, "qcmd", 0),
    "opt_qrda_2.5e8_M32": (250_000_000, 32, synth.grad_gaussian_biased, 1e-5, "qrda", 0),
    "opt_qrda_2.5e8_M32_requant": (250_000_000, 32, synth.grad_gaussian_biased, 1e-5, "qrda", 1),
    "largest_2^30_M64": (1 << 30, 64, synth.grad_laplace_sparse, 1e-6, "alternate", 0),
    # more than 2^32 coordinates: every index and byte offset past 32 bits, ragged last bucket
    "beyond_2^32_M2": ((1 << 32) + 3 * 4096 + 76, 2, synth.grad_laplace_sparse, 1e-6, "alternate", 1),
}


@pytest.mark.parametrize("name", list(CASES))
def test_sampled_buckets_at_full_size(name):
    d, M, gen, lam, schedule, requant = CASES[name]
    T = int(os.environ.get("QA_FULLSIZE_STEPS", "3"))
    b, eta, delta = 4096, 0.1, 1e-8
    nb = (d + b - 1) // b
    rng = np.random.default_rng(17)
    sample = np.unique(np.concatenate([[0, 1, nb - 2, nb - 1], rng.integers(0, nb, 60)]))
    W = (d + 15) // 16
    L = qa.Layout.make(d, M, b, code_stride=W + (-W) % 64)      # bench.py's stride: 256-byte rows
    L1 = qa.Layout.make(d, 1, b, code_stride=L.code_stride, scale_stride=L.scale_stride)
    codes = torch.zeros((M, L.code_stride), dtype=torch.int32, device=DEV)
    scales = torch.zeros((M, L.scale_stride), dtype=torch.float32, device=DEV)
    x, G, z = (torch.zeros(d, dtype=torch.float32, device=DEV) for _ in range(3))
    gbuf = torch.empty(d, dtype=torch.float32, device=DEV)
    lens = [min(b, d - k * b) for k in sample]
    ox = [np.zeros(n, np.float32) for n in lens]
    oG = [np.zeros(n, np.float32) for n in lens]
    oz = [np.zeros(n, np.float32) for n in lens]
    idx = torch.from_numpy(np.concatenate([np.arange(k * b, k * b + n) for k, n in zip(sample, lens)])).to(DEV)
    offs = np.concatenate([[0], np.cumsum(lens)])

    for t in range(1, T + 1):
        g_s = np.empty((M, int(offs[-1])), np.float32)
        for m in range(M):
            gen(d, m, t, device=DEV, out=gbuf)
            qa.qa_quantize_pack(L1, gbuf, d, codes[m], scales[m], None, 0, None)
            g_s[m] = host(gbuf[idx])
        kind = schedule if schedule != "alternate" else ("qcmd" if t % 2 else "qrda")
        if kind == "qcmd":
            qa.qa_step_qcmd(L, codes, scales, x, G, z if schedule == "alternate" else None, eta, lam,
                            delta, requant, None)
        else:
            qa.qa_step_qrda(L, codes, scales, x, G, z, t, eta, lam, delta, requant, None)
        torch.cuda.synchronize()
        xs, Gs, zs = host(x[idx]), host(G[idx]), host(z[idx])
        nonzero_codes = 0
        for j, (k, n) in enumerate(zip(sample, lens)):
            lo, hi = int(offs[j]), int(offs[j + 1])
            oc, osc, _ = oracle.quantize_pack(g_s[:, lo:hi], bucket=b)
            w0, w1 = k * (b // 16), k * (b // 16) + (n + 15) // 16
            assert np.array_equal(host(codes[:, w0:w1]).view(np.uint32), oc), f"codes, bucket {k}, step {t}"
            assert np.array_equal(host(scales[:, k]), osc[:, 0]), f"scales, bucket {k}, step {t}"
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
    # a property that holds at any size: coordinates never touched by any worker keep G == 0
    assert float(G.min().item()) >= 0.0
