"""Pins for the oracle's stochastic ternary quantizer (TernGrad with Philox4x32-10): published
known-answer vectors of the generator, unbiasedness E[Q(v)] = v by Monte Carlo, and the
properties that follow from keep-probability |v|/max|v|.  No GPU, no product code."""
import numpy as np
import pytest
from scipy import stats

import oracle
from conftest import golden


def test_philox_known_answers():
    for k, words in golden("philox4x32_10_kat.txt").items():
        w = [int(x, 16) for x in words]
        assert oracle.philox4x32_10(w[:4], w[4:6]).tolist() == w[6:], k


def test_uniform_numbers_are_uniform_and_keyed():
    u = np.array([oracle.uniform(7, 3, 2, i) for i in range(20000)])
    assert 0.0 <= u.min() and u.max() < 1.0
    assert stats.kstest(u, "uniform").pvalue > 1e-3
    assert np.all(u * 2 ** 24 == np.floor(u * 2 ** 24))             # 24-bit grid
    base = [oracle.uniform(7, 3, 2, i) for i in range(16)]
    for other in ((8, 3, 2), (7, 4, 2), (7, 3, 1), (7 + (1 << 32), 3, 2)):
        assert [oracle.uniform(*other, i) for i in range(16)] != base
    assert [oracle.uniform(7, 3, 2, i) for i in range(16)] == base    # reproducible
    # components 4j..4j+3 are the four output words of counter j
    r = oracle.philox4x32_10([5, 0, 2, 3], [7, 0])
    assert [oracle.uniform(7, 3, 2, 20 + e) for e in range(4)] == [float(np.float32(int(w) >> 8) * np.float32(2.0 ** -24)) for w in r]
    assert oracle.uniform(7, 3, 2, 4 * (1 << 32)) == float(np.float32(int(oracle.philox4x32_10([0, 1, 2, 3], [7, 0])[0]) >> 8) * np.float32(2.0 ** -24))


def test_stochastic_quantizer_is_unbiased_and_respects_its_probabilities():
    rng = np.random.default_rng(0)
    d, reps = 64, 4000
    v = rng.standard_normal(d).astype(np.float32)
    v[3] = 0.0
    imax = int(np.argmax(np.abs(v)))
    acc = np.zeros(d)
    kept = np.zeros(d)
    for seed in range(reps):
        code, sc = oracle.quantize_stochastic(v, seed=seed, step=1, m=0)
        assert sc[0] == np.abs(v).max()
        assert code[imax] == np.sign(v[imax]) and code[3] == 0        # p = 1 always, p = 0 never
        assert np.all((code == 0) | (code == np.sign(v)))
        acc += float(sc[0]) * code
        kept += code != 0
    p = np.abs(v) / np.abs(v).max()
    sigma = float(np.abs(v).max()) * np.sqrt(p * (1 - p) / reps)
    assert np.all(np.abs(acc / reps - v) <= 4.5 * sigma + 1e-7)       # E[s*code] = v
    assert np.all(np.abs(kept / reps - p) <= 4.5 * np.sqrt(p * (1 - p) / reps) + 1e-7)


def test_stochastic_quantizer_buckets_zero_and_nan():
    v = np.zeros(300, np.float32)
    v[200:] = np.linspace(-1, 1, 100, dtype=np.float32)
    v[250] = np.nan
    code, sc = oracle.quantize_stochastic(v, bucket=100, seed=1)
    assert sc.tolist() == [0.0, 0.0, 1.0]
    assert not code[:200].any() and code[250] == 0 and code[200] == -1 and code[299] == 1
    c2, _ = oracle.quantize_stochastic(v, bucket=100, seed=1, m=1)    # another worker, other draws
    assert not np.array_equal(code, c2)


@pytest.mark.parametrize("bucket", [64, 256, 0])
def test_bucketed_stochastic_quantizer_follows_its_definition_elementwise(bucket):
    """Per bucket s = max|v|; component i (index in the whole vector, which is also what the
    generator's counter takes) is kept iff u_i < |v_i| / s in binary32, and coded as its sign."""
    rng = np.random.default_rng(bucket)
    d, seed, step, m = 700, 99, 5, 3
    v = (rng.standard_normal(d) * 10.0 ** rng.integers(-3, 2, d)).astype(np.float32)
    code, sc = oracle.quantize_stochastic(v, bucket=bucket, seed=seed, step=step, m=m)
    b = bucket or d
    for k in range((d + b - 1) // b):
        lo, hi = k * b, min((k + 1) * b, d)
        s = np.abs(v[lo:hi]).max()
        assert sc[k] == s
        for i in range(lo, hi):
            u = np.float32(oracle.uniform(seed, step, m, i))
            keep = u < np.float32(np.abs(v[i])) / np.float32(s)
            assert code[i] == (int(np.sign(v[i])) if keep else 0), (k, i)
