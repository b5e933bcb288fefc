"""Pins for the CPU oracle: each check ties one part of oracle/qa_oracle.cpp to something the
paper or the mathematics fixes (hand-worked values, closed forms, invariants, brute force,
a library optimiser, Monte Carlo).  No GPU, no product code."""
import math

import numpy as np
import pytest
import torch
from scipy import stats

import oracle
from conftest import golden


def f32(xs):
    return np.array([float(x) for x in xs], np.float32)


# ---------------------------------------------------------------- quantizer, Sections 3.4-3.5

def test_hand_example_quantizer():
    g = golden("quantizer_hand_example.txt")
    v = f32(g["v"])
    Delta, s, cnt = oracle.threshold_scale(v)
    assert Delta == pytest.approx(float(g["Delta"][0]), rel=1e-6)
    assert s == pytest.approx(float(g["s"][0]), rel=1e-6)
    assert cnt == int(g["kept"][0])
    code, sc, th = oracle.quantize(v)
    assert code.tolist() == [int(c) for c in g["codes"]]
    words = oracle.pack(code)
    assert words.size == 1 and int(words[0]) == int(g["word0_hex"][0], 16)
    eps = v.astype(np.float64) - float(sc[0]) * code
    assert float(eps @ eps) == pytest.approx(float(g["err_sq"][0]), rel=1e-6)
    # the expanded objective of Section 3.4 gives the same number
    sum_sq = float(g["sum_sq"][0])
    kept_abs = np.abs(v[code != 0]).astype(np.float64).sum()
    assert cnt * s * s - 2 * s * kept_abs + sum_sq == pytest.approx(float(g["err_sq"][0]), rel=1e-5)


def test_hand_example_exact_threshold_differs_from_approximation():
    g = golden("quantizer_hand_example.txt")
    v = f32(g["v"])
    kept_min, s, obj, k = oracle.exact_threshold(v)
    assert k == int(g["exact_kept"][0])
    assert obj == pytest.approx(float(g["exact_objective"][0]), rel=1e-6)
    assert kept_min == pytest.approx(0.3, rel=1e-6)
    assert s == pytest.approx(1.6 / 3, rel=1e-6)
    # objective reached by the approximate threshold is the printed 0.845 < optimum
    _, s_a, cnt = oracle.threshold_scale(v)
    assert cnt * s_a * s_a == pytest.approx(float(g["approx_objective"][0]), rel=1e-6)
    assert cnt * s_a * s_a < obj


@pytest.mark.parametrize("seed", range(5))
def test_exact_threshold_is_brute_force_optimum(seed):
    rng = np.random.default_rng(seed)
    v = rng.standard_normal(9).astype(np.float32)
    mags = np.sort(np.abs(v.astype(np.float64)))[::-1]
    best = max((mags[:k].sum() ** 2 / k, k) for k in range(1, 10))
    kept_min, s, obj, k = oracle.exact_threshold(v)
    assert obj == pytest.approx(best[0], rel=1e-12) and k == best[1]
    # no other ternary support/scale does better: exhaustive search over all 3^9 sign patterns
    # restricted to "signs follow v" (any other sign only raises the error) and all supports
    vv = v.astype(np.float64)
    best_err = np.inf
    for mask in range(1, 1 << 9):
        sel = np.array([(mask >> i) & 1 for i in range(9)], bool)
        sc = np.abs(vv[sel]).mean()
        err = ((vv - sc * np.sign(vv) * sel) ** 2).sum()
        best_err = min(best_err, err)
    assert (vv @ vv) - obj == pytest.approx(best_err, rel=1e-9)


@pytest.mark.parametrize("seed", range(4))
def test_exact_thresholds_realise_the_optimum_through_the_strict_quantizer(seed):
    rng = np.random.default_rng(200 + seed)
    d, b = 1300, 512
    v = rng.standard_normal(d).astype(np.float32)
    v[rng.random(d) < 0.3] = 0.0
    v[10] = v[11] = v[12]                                    # equal magnitudes cannot be split
    v[600:700] = 0.0
    th = oracle.exact_thresholds(v, bucket=b)
    code, sc, _ = oracle.quantize(v, bucket=b, thresholds=th)
    for k in range(3):
        piece = v[k * b:(k + 1) * b]
        kept_min, s, obj, kk = oracle.exact_threshold(piece)
        c = code[k * b:(k + 1) * b]
        assert (c != 0).sum() == kk and np.array_equal(c != 0, np.abs(piece) >= kept_min)
        assert sc[k] == pytest.approx(s, rel=1e-6)
        _, s_a, cnt_a = oracle.threshold_scale(piece)        # never worse than the approximation
        assert kk * float(sc[k]) ** 2 >= cnt_a * float(s_a) ** 2 * (1 - 1e-6)
    assert oracle.exact_thresholds(np.zeros(5, np.float32))[0] == 0.0
    assert oracle.exact_thresholds(np.array([2.0, -2.0, 2.0], np.float32))[0] == 0.0


@pytest.mark.parametrize("j,bucket", [(10000, 0), (3000, 16384), (2730, 8192)])
def test_exact_threshold_of_a_long_ramp_has_a_closed_form(j, bucket):
    """Section 3.4 over a vector longer than any tile: for the magnitudes 1, 2, ..., n the sum of
    the k largest is k n - k (k - 1) / 2, so the objective is k (n - (k - 1) / 2)^2, a cubic whose
    only maximum over k >= 1 lies at k = (2 n + 1) / 3.  With n = 3 j + 1 that is the integer
    2 j + 1: the kept set is {j + 1, ..., n}, the largest magnitude not kept is j, the scale is
    the mean (n + j + 1) / 2 of the kept ones.  Every quantity is an integer below 2^53.  With
    buckets, every full bucket is a shuffled ramp of its own length."""
    rng = np.random.default_rng(j)
    if bucket == 0:
        n = 3 * j + 1
        v = rng.permutation(np.arange(1, n + 1)).astype(np.float32)
        v *= rng.choice([-1.0, 1.0], n).astype(np.float32)
        kept_min, s, obj, k = oracle.exact_threshold(v)
        assert (k, kept_min) == (2 * j + 1, float(j + 1))
        assert s == (n + j + 1) / 2
        assert obj == k * s * s
        assert oracle.exact_thresholds(v)[0] == float(j)
    else:
        # full buckets hold a ramp 1..bucket (bucket = 3 jb + 1 does not hold for powers of two, so
        # the optimum there is found by evaluating the cubic at the two integers around its peak);
        # the last, short bucket holds a ramp of length 3 j + 1
        nfull = 3
        pieces = [rng.permutation(np.arange(1, bucket + 1)) for _ in range(nfull)]
        pieces.append(rng.permutation(np.arange(1, 3 * j + 2)))
        v = np.concatenate(pieces).astype(np.float32)
        assert 3 * j + 1 < bucket
        th = oracle.exact_thresholds(v, bucket=bucket)
        f = lambda k, n: k * (n - (k - 1) / 2) ** 2
        kf = (2 * bucket + 1) // 3
        kbest = max((kf, kf + 1), key=lambda k: f(k, bucket))
        assert np.array_equal(th, np.array([bucket - kbest] * nfull + [j], np.float32))


@pytest.mark.parametrize("seed", range(4))
def test_approx_threshold_never_beats_exact(seed):
    rng = np.random.default_rng(100 + seed)
    v = (rng.standard_normal(5000) * rng.choice([0.1, 1.0, 5.0], 5000)).astype(np.float32)
    _, s, cnt = oracle.threshold_scale(v)
    _, _, obj, _ = oracle.exact_threshold(v)
    assert cnt * float(s) ** 2 <= obj * (1 + 1e-6)


@pytest.mark.parametrize("seed", range(4))
def test_scale_is_least_squares_optimal(seed):
    """<eps, Q(v)> = 0 and ||v||^2 = ||Q||^2 + ||eps||^2; perturbing s never helps."""
    rng = np.random.default_rng(seed)
    v = rng.laplace(0, 1e-3, 4096).astype(np.float32)
    code, sc, th = oracle.quantize(v)
    s = float(sc[0])
    vv, c = v.astype(np.float64), code.astype(np.float64)
    Q = s * c
    eps = vv - Q
    assert abs(eps @ Q) <= 1e-6 * (vv @ vv)
    assert vv @ vv == pytest.approx(Q @ Q + eps @ eps, rel=1e-6)
    assert eps @ eps <= vv @ vv
    for f in (0.99, 1.01):
        e2 = vv - f * s * c
        assert e2 @ e2 >= eps @ eps
    # signs follow v, support is exactly {|v| > Delta}
    assert np.array_equal(code != 0, np.abs(v) > th[0])
    assert np.all(code[code != 0] == np.sign(v[code != 0]))


def test_gaussian_monte_carlo_matches_closed_forms():
    """Section 3.5: for v ~ N(0, sigma^2), Delta -> 0.75 E|v| = 0.75 sqrt(2/pi) sigma ~ 0.6 sigma."""
    sigma = 3e-3
    rng = np.random.default_rng(7)
    v = (sigma * rng.standard_normal(1_000_000)).astype(np.float32)
    code, sc, th = oracle.quantize(v)
    a = 0.75 * math.sqrt(2 / math.pi)
    assert th[0] / sigma == pytest.approx(a, rel=3e-3)
    assert abs(a - 0.6) < 0.005                       # the paper's "0.6 sigma"
    keep = 2 * stats.norm.sf(a)
    assert (code != 0).mean() == pytest.approx(keep, rel=5e-3)
    s_closed = stats.norm.pdf(a) / stats.norm.sf(a)   # E[|v| ; |v|>a] / P(|v|>a)
    assert sc[0] / sigma == pytest.approx(s_closed, rel=3e-3)
    eps = v.astype(np.float64) - float(sc[0]) * code
    vv = v.astype(np.float64)
    assert (eps @ eps) / (vv @ vv) == pytest.approx(1 - keep * s_closed ** 2, rel=1e-2)


def test_laplace_monte_carlo_matches_closed_forms():
    b = 1e-3
    rng = np.random.default_rng(8)
    v = rng.laplace(0, b, 1_000_000).astype(np.float32)
    code, sc, th = oracle.quantize(v)
    assert th[0] / b == pytest.approx(0.75, rel=3e-3)              # E|v| = b
    assert (code != 0).mean() == pytest.approx(math.exp(-0.75), rel=5e-3)
    assert sc[0] / b == pytest.approx(1.75, rel=3e-3)              # memoryless: Delta + b


def test_threshold_uses_full_length_including_zeros():
    v = np.zeros(1000, np.float32)
    v[:10] = 1.0
    Delta, s, cnt = oracle.threshold_scale(v)
    assert Delta == pytest.approx(0.75 * 10 / 1000, rel=1e-6) and s == 1.0 and cnt == 10


def test_boundary_equal_to_threshold_gives_zero():
    # |v| = (4, 4, 4, 16/3*...): build a vector whose threshold equals one magnitude exactly
    v = f32([1.0, -1.0, 1.0, 1.0])            # Delta = 0.75 exactly; nothing equals it
    code, sc, th = oracle.quantize(v, thresholds=f32([1.0]))
    assert code.tolist() == [0, 0, 0, 0] and sc[0] == 0.0     # strict '>' at equality
    code, sc, th = oracle.quantize(v, thresholds=f32([np.nextafter(np.float32(1), np.float32(0))]))
    assert code.tolist() == [1, -1, 1, 1] and sc[0] == 1.0


def test_all_zero_and_nan_vectors():
    code, sc, th = oracle.quantize(np.zeros(100, np.float32))
    assert not code.any() and sc[0] == 0.0 and th[0] == 0.0
    v = np.ones(64, np.float32)
    v[5] = np.nan
    code, sc, th = oracle.quantize(v)
    assert not code.any() and sc[0] == 0.0 and np.isnan(th[0])


def test_buckets_are_independent_quantizers():
    rng = np.random.default_rng(3)
    d, b = 1000, 256                       # ragged last bucket of 232
    v = rng.standard_normal(d).astype(np.float32) * np.repeat(f32([1, 10, 0.1, 3]), 250)
    code, sc, th = oracle.quantize(v, bucket=b)
    assert sc.size == 4
    for k in range(4):
        piece = v[k * b:(k + 1) * b]
        c1, s1, t1 = oracle.quantize(piece)
        assert np.array_equal(code[k * b:(k + 1) * b], c1) and sc[k] == s1[0] and th[k] == t1[0]
    assert th[3] == pytest.approx(0.75 * np.abs(v[768:]).astype(np.float64).sum() / 232, rel=1e-6)


# ---------------------------------------------------------------- encoding

@pytest.mark.parametrize("d", list(range(1, 70)) + [127, 128, 129, 200])
def test_pack_unpack_roundtrip_and_size(d):
    rng = np.random.default_rng(d)
    code = rng.integers(-1, 2, d).astype(np.int8)
    w = oracle.pack(code)
    assert w.size == (d + 15) // 16                    # 2 bits per component
    assert 32 * w.size >= 2 * d > 32 * (w.size - 1)
    assert np.array_equal(oracle.unpack(w, d), code)
    # independent bit-level decode
    for i in range(d):
        f = (int(w[i // 16]) >> (2 * (i % 16))) & 3
        assert f == {0: 0, 1: 1, -1: 3}[int(code[i])]
    if d % 16:
        assert int(w[-1]) >> (2 * (d % 16)) == 0       # tail bits are zero


def test_reserved_pattern_decodes_to_zero():
    w = np.array([0b10_11_01_00 | (0b10 << 30)], np.uint32)
    assert oracle.unpack(w, 16).tolist() == [0, 1, -1, 0] + [0] * 12


# ---------------------------------------------------------------- aggregation (SynQ_t)

def test_aggregate_is_the_mean_of_decoded_messages():
    rng = np.random.default_rng(11)
    M, d, b = 6, 777, 64                              # M not a power of two
    g = rng.standard_normal((M, d)).astype(np.float32) * 1e-2
    codes, scales, th = oracle.quantize_pack(g, bucket=b)
    gbar = oracle.aggregate(codes, scales, d, bucket=b)
    dec = np.stack([oracle.unpack(codes[m], d).astype(np.float64) *
                    np.repeat(scales[m].astype(np.float64), b)[:d] for m in range(M)])
    assert np.array_equal(gbar, dec.mean(axis=0).astype(np.float32)) or \
        np.allclose(gbar, dec.mean(axis=0), rtol=1e-7, atol=0)
    assert np.all(np.abs(gbar) <= np.repeat(scales.max(axis=0), b)[:d] * (1 + 1e-7))


def test_aggregate_special_cases():
    rng = np.random.default_rng(12)
    d = 300
    g1 = rng.standard_normal((1, d)).astype(np.float32)
    codes, scales, _ = oracle.quantize_pack(g1)
    code, sc, _ = oracle.quantize(g1[0])
    assert np.array_equal(oracle.aggregate(codes, scales, d), sc[0] * code.astype(np.float32))
    g8 = np.repeat(g1, 8, axis=0)                      # identical workers, M a power of two
    codes8, scales8, _ = oracle.quantize_pack(g8)
    assert np.array_equal(oracle.aggregate(codes8, scales8, d), sc[0] * code.astype(np.float32))


def test_requantize_is_quantizer_applied_to_average():
    rng = np.random.default_rng(13)
    gbar = rng.standard_normal(500).astype(np.float32)
    q = oracle.requantize(gbar, bucket=128)
    code, sc, _ = oracle.quantize(gbar, bucket=128)
    assert np.array_equal(q, np.repeat(sc, 128)[:500] * code)
    qg = oracle.requantize(gbar, bucket=0)
    code, sc, _ = oracle.quantize(gbar)
    assert np.array_equal(qg, sc[0] * code)


# ---------------------------------------------------------------- updates, Section 3.2

def test_hand_example_qcmd():
    g = golden("qcmd_hand_example.txt")
    x, G = f32(g["x"]), f32(g["G_prev"])
    oracle.update_qcmd(f32(g["q"]), x, G, None, float(g["eta"][0]), float(g["lambda"][0]),
                       float(g["delta"][0]))
    assert np.allclose(G, f32(g["G"]), rtol=1e-6)
    assert np.allclose(x, f32(g["x_next"]), rtol=1e-6, atol=0)
    assert x[1] == 0.0 and not np.signbit(x[1])


def test_hand_example_qrda():
    g = golden("qrda_hand_example.txt")
    x = np.full(3, 7.0, np.float32)                   # must be overwritten
    G, z = f32(g["G_prev"]), f32(g["z_prev"])
    oracle.update_qrda(f32(g["q"]), x, G, z, int(g["t"][0]), float(g["eta"][0]),
                       float(g["lambda"][0]), float(g["delta"][0]))
    assert np.allclose(z, f32(g["z"]), rtol=1e-6)
    assert np.allclose(np.float32(float(g["delta"][0])) + np.sqrt(G), f32(g["H"]), rtol=1e-6)
    assert np.allclose(x, f32(g["x_next"]), rtol=1e-6, atol=0)
    assert x[0] == 0.0 and not np.signbit(x[0]) and not np.signbit(x[1])


def _argmin_1d(h, lo, hi):
    """Brute force: dense grid, then golden-section refinement around the best grid point."""
    xs = np.linspace(lo, hi, 200001)
    i = int(np.argmin(h(xs)))
    a, b = xs[max(i - 1, 0)], xs[min(i + 1, xs.size - 1)]
    phi = (math.sqrt(5) - 1) / 2
    for _ in range(200):
        c, d = b - phi * (b - a), a + phi * (b - a)
        if h(c) < h(d):
            b = d
        else:
            a = c
    return 0.5 * (a + b)


@pytest.mark.parametrize("seed", range(3))
def test_qcmd_update_minimises_its_subproblem(seed):
    """Equation CMD2: argmin eta*q*x + eta*lambda*|x| + (H/2)(x - x_t)^2 per coordinate."""
    rng = np.random.default_rng(seed)
    d, eta, lam, delta = 8, 0.3, 0.4, 0.05
    x0 = rng.standard_normal(d).astype(np.float32)
    G0 = (rng.random(d) * 2).astype(np.float32)
    q = rng.standard_normal(d).astype(np.float32)
    x, G = x0.copy(), G0.copy()
    oracle.update_qcmd(q, x, G, None, eta, lam, delta)
    H = delta + np.sqrt(G0.astype(np.float64) + q.astype(np.float64) ** 2)
    for i in range(d):
        h = lambda t: eta * q[i] * t + eta * lam * np.abs(t) + 0.5 * H[i] * (t - x0[i]) ** 2
        assert x[i] == pytest.approx(_argmin_1d(h, -6, 6), abs=2e-6)
        # KKT (proof of Proposition 1): H (x_t - x+) - eta q in eta*lambda*d|x+|
        r = H[i] * (float(x0[i]) - float(x[i])) - eta * float(q[i])
        if x[i] != 0:
            assert r == pytest.approx(eta * lam * np.sign(x[i]), abs=1e-5)
        else:
            assert abs(r) <= eta * lam + 1e-6


@pytest.mark.parametrize("seed", range(3))
def test_qrda_update_minimises_its_subproblem(seed):
    """Equation RDA2: argmin eta*<z/t, x> + eta*lambda*|x| + (1/t)(H/2) x^2 per coordinate."""
    rng = np.random.default_rng(10 + seed)
    d, eta, lam, delta, t = 8, 0.3, 0.2, 0.05, 5
    G0 = (rng.random(d) * 2).astype(np.float32)
    z0 = (rng.standard_normal(d) * 2).astype(np.float32)
    q = rng.standard_normal(d).astype(np.float32)
    x, G, z = np.zeros(d, np.float32), G0.copy(), z0.copy()
    oracle.update_qrda(q, x, G, z, t, eta, lam, delta)
    zz = z0.astype(np.float64) + q.astype(np.float64)
    assert np.allclose(z, zz, rtol=1e-6, atol=1e-7)
    H = delta + np.sqrt(G0.astype(np.float64) + q.astype(np.float64) ** 2)
    for i in range(d):
        h = lambda u: eta * (zz[i] / t) * u + eta * lam * np.abs(u) + 0.5 * H[i] / t * u ** 2
        assert x[i] == pytest.approx(_argmin_1d(h, -30, 30), abs=1e-5)
        # optimality condition used in the proof of Proposition 2:
        #   -z - (1/eta) H x+ in t*lambda*d|x+|
        r = -zz[i] - H[i] * float(x[i]) / eta
        if x[i] != 0:
            assert r == pytest.approx(t * lam * np.sign(x[i]), abs=1e-4)
        else:
            assert abs(r) <= t * lam + 1e-6
    # the formula exactly as printed (divide by t, multiply by t) agrees
    lit = oracle.qrda_literal_f64(zz, H, t, eta, lam)
    assert np.allclose(x, lit, rtol=1e-6, atol=1e-9)


def _duchi_cmd_f64(gs, eta, lam, delta):
    """Independent few-line binary64 CMD adagrad with l1 (Duchi et al.; equation CMD1)."""
    x = np.zeros(gs.shape[1]); G = np.zeros_like(x)
    for g in gs:
        G += g * g
        H = delta + np.sqrt(G)
        u = x - eta * g / H
        x = np.sign(u) * np.maximum(np.abs(u) - lam * eta / H, 0.0)
    return x, G


def _duchi_rda_f64(gs, eta, lam, delta):
    """Independent few-line binary64 RDA adagrad with l1 (equation RDA1)."""
    z = np.zeros(gs.shape[1]); G = np.zeros_like(z)
    for t, g in enumerate(gs, 1):
        G += g * g; z += g
        H = delta + np.sqrt(G)
        x = -np.sign(z) * (eta * t / H) * np.maximum(np.abs(z) / t - lam, 0.0)
    return x, G, z


def test_identity_quantizer_recovers_cmd_and_rda_adagrad():
    rng = np.random.default_rng(21)
    T, d, eta, lam, delta = 40, 50, 0.1, 0.02, 1e-3
    gs = (rng.standard_normal((T, d)) * rng.random(d)).astype(np.float32)
    x, G = np.zeros(d, np.float32), np.zeros(d, np.float32)
    for g in gs:
        oracle.update_qcmd(g, x, G, None, eta, lam, delta)
    xr, Gr = _duchi_cmd_f64(gs.astype(np.float64), eta, lam, delta)
    assert np.allclose(G, Gr, rtol=1e-5) and np.allclose(x, xr, rtol=2e-4, atol=1e-6)
    x, G, z = (np.zeros(d, np.float32) for _ in range(3))
    for t, g in enumerate(gs, 1):
        oracle.update_qrda(g, x, G, z, t, eta, lam, delta)
    xr, Gr, zr = _duchi_rda_f64(gs.astype(np.float64), eta, lam, delta)
    assert np.allclose(z, zr, rtol=1e-4, atol=1e-5) and np.allclose(x, xr, rtol=2e-3, atol=1e-5)
    assert (x == 0).sum() == (xr == 0).sum()


def test_lambda_zero_identity_quantizer_is_torch_adagrad():
    rng = np.random.default_rng(22)
    T, d, eta, delta = 30, 64, 0.05, 1e-6
    gs = rng.standard_normal((T, d)).astype(np.float32)
    x0 = rng.standard_normal(d).astype(np.float32)
    x, G = x0.copy(), np.zeros(d, np.float32)
    p = torch.nn.Parameter(torch.from_numpy(x0.copy()))
    opt = torch.optim.Adagrad([p], lr=eta, eps=delta, lr_decay=0, initial_accumulator_value=0)
    for g in gs:
        oracle.update_qcmd(g, x, G, None, eta, 0.0, delta)
        p.grad = torch.from_numpy(g.copy())
        opt.step()
    assert np.allclose(x, p.detach().numpy(), rtol=1e-5, atol=1e-6)


def test_prox_gd_special_case():
    """H == 1 (G = 0 before and q = 0 ... not reachable); instead: delta large, G tiny ->
    the update is ISTA soft-thresholding with step eta/delta."""
    x = f32([0.5, -0.2, 0.01])
    G = np.zeros(3, np.float32)
    q = f32([1e-20, -1e-20, 0])
    oracle.update_qcmd(q, x, G, None, 0.1, 1.0, 1.0)
    assert np.allclose(x, [0.4, -0.1, 0.0], rtol=1e-6)


def test_lemma_1_adagrad_inequality():
    """(1/2) sum_t sum_i q_ti^2 / H_ti <= sum_i ||q_{1:T,i}||_2  (Lemma 1, Section 4)."""
    rng = np.random.default_rng(23)
    T, d = 60, 40
    qs = rng.standard_normal((T, d)).astype(np.float32)
    for delta in (1e-8, 0.5):
        x, G = np.zeros(d, np.float32), np.zeros(d, np.float32)
        lhs = 0.0
        for q in qs:
            oracle.update_qcmd(q, x, G, None, 0.1, 0.0, delta)
            lhs += 0.5 * float((q.astype(np.float64) ** 2 / (delta + np.sqrt(G.astype(np.float64)))).sum())
        assert lhs <= float(np.sqrt(G.astype(np.float64)).sum()) * (1 + 1e-6)


def test_qcmd_can_track_z():
    rng = np.random.default_rng(24)
    q = rng.standard_normal(33).astype(np.float32)
    x, G, z = (rng.standard_normal(33).astype(np.float32) for _ in range(3))
    G = np.abs(G)
    x2, G2, z0 = x.copy(), G.copy(), z.copy()
    oracle.update_qcmd(q, x, G, z, 0.1, 0.01, 1e-3)
    oracle.update_qcmd(q, x2, G2, None, 0.1, 0.01, 1e-3)
    assert np.array_equal(x, x2) and np.array_equal(G, G2) and np.array_equal(z, z0 + q)


# ---------------------------------------------------------------- whole step from packed codes

@pytest.mark.parametrize("requant", [0, 1, 2])
def test_step_equals_composition_of_its_parts(requant):
    rng = np.random.default_rng(30 + requant)
    M, d, b = 4, 1000, 256
    g = rng.standard_normal((M, d)).astype(np.float32) * 1e-2
    codes, scales, _ = oracle.quantize_pack(g, bucket=b)
    gbar = oracle.aggregate(codes, scales, d, bucket=b)
    q = gbar if requant == 0 else oracle.requantize(gbar, bucket=b if requant == 1 else 0)
    st = [rng.standard_normal(d).astype(np.float32) * 0.01 for _ in range(3)]
    st[1] = np.abs(st[1])
    xa, Ga, za = (s.copy() for s in st)
    xb, Gb, zb = (s.copy() for s in st)
    oracle.step_qcmd(codes, scales, d, b, xa, Ga, za, 0.1, 1e-3, 1e-8, requant)
    oracle.update_qcmd(q, xb, Gb, zb, 0.1, 1e-3, 1e-8)
    assert np.array_equal(xa, xb) and np.array_equal(Ga, Gb) and np.array_equal(za, zb)
    oracle.step_qrda(codes, scales, d, b, xa, Ga, za, 3, 0.1, 1e-3, 1e-8, requant)
    oracle.update_qrda(q, xb, Gb, zb, 3, 0.1, 1e-3, 1e-8)
    assert np.array_equal(xa, xb) and np.array_equal(Ga, Gb) and np.array_equal(za, zb)


def test_double_quantized_q_takes_three_values_per_piece():
    rng = np.random.default_rng(40)
    M, d, b = 3, 512, 128
    g = rng.standard_normal((M, d)).astype(np.float32)
    codes, scales, _ = oracle.quantize_pack(g, bucket=b)
    x, G, z = (np.zeros(d, np.float32) for _ in range(3))
    oracle.step_qrda(codes, scales, d, b, x, G, z, 1, 0.1, 0.0, 1e-8, 1)   # z = q after one step
    for k in range(4):
        vals = np.unique(np.abs(z[k * b:(k + 1) * b]))
        assert vals.size <= 2 and vals[0] == 0.0


# ---------------------------------------------------------------- local gradient

def _loss_f64(A, y, rows, x):
    m = y[rows].astype(np.float64) * (A[rows].astype(np.float64) @ x.astype(np.float64))
    return np.logaddexp(0.0, -m).mean()


def test_logistic_gradient_finite_differences():
    rng = np.random.default_rng(50)
    n, d, B = 40, 12, 9
    A = rng.standard_normal((n, d)).astype(np.float32)
    y = np.where(rng.random(n) < 0.5, -1.0, 1.0).astype(np.float32)
    rows = rng.integers(0, n, B).astype(np.int32)
    rows[3] = rows[0]                                    # a repeated row counts twice
    x = (rng.standard_normal(d) * 0.5).astype(np.float32)
    g, loss = oracle.local_grad_dense(A, y, rows, x)
    assert loss == pytest.approx(_loss_f64(A, y, rows, x), rel=1e-6)
    h = 1e-3
    for j in range(d):
        e = np.zeros(d, np.float32); e[j] = h
        fd = (_loss_f64(A, y, rows, x + e) - _loss_f64(A, y, rows, x - e)) / (2.0 * float(e[j]))
        assert g[j] == pytest.approx(fd, rel=2e-4, abs=2e-6)


def test_logistic_extreme_margins_are_finite():
    A = f32([200.0, -200.0]).reshape(2, 1)
    y = f32([1.0, 1.0])
    g, loss = oracle.local_grad_dense(A, y, np.array([0, 1], np.int32), f32([1.0]))
    assert np.isfinite(g).all() and loss == pytest.approx(100.0, rel=1e-6)
    # row 0: margin +200 -> no loss, no gradient; row 1: margin -200 -> loss 200, sigma = 1,
    # gradient -(y/B) * a = -(1/2)(-200) = 100
    assert g[0] == pytest.approx(100.0, rel=1e-6)


def test_dense_and_csr_gradients_agree_bit_for_bit():
    rng = np.random.default_rng(51)
    n, d, B = 64, 200, 16
    A = rng.standard_normal((n, d)).astype(np.float32) * (rng.random((n, d)) < 0.05)
    y = np.where(rng.random(n) < 0.5, -1.0, 1.0).astype(np.float32)
    indptr = np.zeros(n + 1, np.int64); idx = []; vals = []
    for i in range(n):
        nz = np.nonzero(A[i])[0]
        idx.append(nz); vals.append(A[i, nz]); indptr[i + 1] = indptr[i] + nz.size
    idx = np.concatenate(idx).astype(np.int32); vals = np.concatenate(vals).astype(np.float32)
    rows = rng.integers(0, n, B).astype(np.int32)
    x = rng.standard_normal(d).astype(np.float32)
    gd, ld = oracle.local_grad_dense(A, y, rows, x)
    gc, lc = oracle.local_grad_csr(vals, indptr, idx, d, y, rows, x)
    assert np.array_equal(gd, gc) and ld == lc
    touched = np.zeros(d, bool); touched[np.concatenate([np.nonzero(A[r])[0] for r in rows])] = True
    assert not gc[~touched].any()
