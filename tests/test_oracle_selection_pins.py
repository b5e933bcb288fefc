"""Pins for the oracle's indicator / selection / sparse-encoding functions (Section 3.2 and the
Encode paragraph): hand example, definition through the already pinned update and quantizer
functions, round trips, special cases.  No GPU, no product code."""
import numpy as np
import pytest

import oracle
from conftest import golden


def f32(xs):
    return np.array([float(x) for x in xs], np.float32)


def bits_of(ind, d):
    return np.array([(int(ind[i // 32]) >> (i % 32)) & 1 for i in range(d)], bool)


def test_hand_example_indicator_selection_and_message_size():
    g = golden("indicator_hand_example.txt")
    x, G, gr = f32(g["x"]), f32(g["G"]), f32(g["g"])
    ind = oracle.indicator(oracle.QCMD, gr, x, G, None, 1, float(g["eta"][0]), float(g["lambda"][0]),
                           float(g["delta"][0]))
    assert bits_of(ind, 3).astype(int).tolist() == [int(b) for b in g["indicator_bits"]]
    sel, cnt, sc, th = oracle.quantize_selected(gr, ind)
    assert cnt[0] == int(g["selected_count"][0])
    assert th[0] == pytest.approx(float(g["selected_Delta"][0]), rel=1e-6)
    assert sc[0] == pytest.approx(float(g["selected_s"][0]), rel=1e-6)
    assert oracle.unpack(sel, int(cnt[0])).tolist() == [int(c) for c in g["selected_codes"]]
    dense = oracle.decode_selected(ind, sel, 3)
    assert oracle.unpack(dense, 3).tolist() == [int(c) for c in g["decoded"]]
    assert 32 + 3 + 2 * int(cnt[0]) == int(g["message_bits"][0])


@pytest.mark.parametrize("method", [oracle.QCMD, oracle.QRDA])
def test_indicator_follows_its_definition_through_the_pinned_updates(method):
    rng = np.random.default_rng(method)
    d, eta, lam, delta, t = 300, 0.1, 0.3, 1e-3, 7
    x = (rng.standard_normal(d) * (rng.random(d) < 0.3)).astype(np.float32)
    G = (rng.random(d) * 2).astype(np.float32)
    z = (rng.standard_normal(d) * 2).astype(np.float32)
    g = (rng.standard_normal(d) * rng.choice([0.01, 1.0], d)).astype(np.float32)
    ind = oracle.indicator(method, g, x, G, z, t, eta, lam, delta)
    xh, Gh, zh = x.copy(), G.copy(), z.copy()
    if method == oracle.QCMD:
        oracle.update_qcmd(g, xh, Gh, None, eta, lam, delta)      # the worker's own update, q := g
    else:
        oracle.update_qrda(g, xh, Gh, zh, t, eta, lam, delta)
    expect = (x != 0) | (xh != 0)
    assert np.array_equal(bits_of(ind, d), expect)
    assert 0 < expect.sum() < d                                   # both outcomes occur
    assert int(ind[-1]) >> (d % 32) == 0                          # unused bits stay zero


@pytest.mark.parametrize("d,bucket", [(1000, 0), (1000, 256), (9000, 4096), (4096, 4096),
                                      # one scale for a message of many tiles; buckets below and
                                      # above a 4096-tile on a ragged length
                                      (70001, 0), (70001, 64), (70001, 2048), (70001, 16384)])
def test_quantize_selected_is_the_quantizer_on_the_compacted_vector(d, bucket):
    rng = np.random.default_rng(d + bucket)
    g = rng.standard_normal(d).astype(np.float32)
    mask = rng.random(d) < 0.2
    mask[:5] = False
    if bucket:
        mask[bucket:2 * bucket] = False                           # an empty bucket
    ind = np.zeros(oracle.n_ind_words(d), np.uint32)
    for i in np.nonzero(mask)[0]:
        ind[i // 32] |= np.uint32(1 << (i % 32))
    sel, cnt, sc, th = oracle.quantize_selected(g, ind, bucket=bucket)
    b = bucket or d
    area = (b + 15) // 16
    dense = oracle.unpack(oracle.decode_selected(ind, sel, d, bucket=bucket), d)
    for k in range(oracle.n_buckets(d, bucket)):
        lo, hi = k * b, min((k + 1) * b, d)
        v = g[lo:hi][mask[lo:hi]]
        assert cnt[k] == v.size
        if v.size == 0:
            assert sc[k] == 0 and th[k] == 0
            continue
        c, s1, t1 = oracle.quantize(v)                            # pinned quantizer, length k
        assert sc[k] == s1[0] and th[k] == t1[0]
        assert np.array_equal(oracle.unpack(sel[k * area:], v.size), c)
        assert np.array_equal(dense[lo:hi][mask[lo:hi]], c)
    assert not dense[~mask].any()


def test_all_ones_indicator_equals_dense_path():
    rng = np.random.default_rng(5)
    d, b = 5000, 1024
    g = rng.standard_normal(d).astype(np.float32)
    ind = np.full(oracle.n_ind_words(d), 0xFFFFFFFF, np.uint32)
    ind[-1] = np.uint32((1 << (d % 32)) - 1)
    sel, cnt, sc, th = oracle.quantize_selected(g, ind, bucket=b)
    codes, scales, thr = oracle.quantize_pack(g[None, :], bucket=b)
    assert np.array_equal(sc, scales[0]) and np.array_equal(th, thr[0])
    assert np.array_equal(oracle.decode_selected(ind, sel, d, bucket=b), codes[0])
    assert cnt.sum() == d


def test_indicator_or():
    rng = np.random.default_rng(6)
    ind = rng.integers(0, 2 ** 32, (5, 10), dtype=np.uint64).astype(np.uint32)
    assert np.array_equal(oracle.indicator_or(ind, 320), np.bitwise_or.reduce(ind, axis=0))


@pytest.mark.parametrize("d,bucket", [(37, 0), (1000, 256), (9000, 4096), (70001, 0), (70001, 512),
                                      (70001, 8192)])
def test_select_codes_is_numpy_compaction_and_inverts_under_decode(d, bucket):
    """S(q, I) on a coded message: the marked components' codes in index order (numpy boolean
    indexing is the definition), per bucket; decode puts them back, zeros elsewhere."""
    rng = np.random.default_rng(d)
    code = rng.integers(-1, 2, d).astype(np.int8)
    dense = oracle.pack(code)
    mask = rng.random(d) < 0.3
    if bucket:
        mask[:bucket] = False                                      # an empty bucket
    ind = np.zeros(oracle.n_ind_words(d), np.uint32)
    for i in np.nonzero(mask)[0]:
        ind[i // 32] |= np.uint32(1 << (i % 32))
    sel, cnt = oracle.select_codes(dense, ind, d, bucket=bucket)
    b = bucket or d
    area = (b + 15) // 16
    for k in range(oracle.n_buckets(d, bucket)):
        lo, hi = k * b, min((k + 1) * b, d)
        want = code[lo:hi][mask[lo:hi]]
        assert cnt[k] == want.size
        assert np.array_equal(oracle.unpack(sel[k * area:], want.size), want)
        nw = (want.size + 15) // 16
        assert np.array_equal(sel[k * area:k * area + nw], oracle.pack(want))   # unused bits zero
    back = oracle.unpack(oracle.decode_selected(ind, sel, d, bucket=bucket), d)
    assert np.array_equal(back, np.where(mask, code, 0))
    # the reserved pattern 10 is read as 0
    dense2 = dense.copy()
    dense2[0] = (dense2[0] & ~np.uint32(3)) | np.uint32(2)
    ind2 = ind.copy()
    ind2[0] |= np.uint32(1)
    sel2, _ = oracle.select_codes(dense2, ind2, d, bucket=bucket)
    assert oracle.unpack(sel2, 1)[0] == 0


def test_one_scale_message_of_a_long_vector_has_32_plus_d_plus_2k_bits():
    """Encode paragraph of Section 3.5 for a sparse model: one float, d indicator bits and two
    bits for each of the k selected components, for a vector much longer than any tile.  The
    selected codes form ONE stream of 2k bits from bit 0 of the message's code area; nothing
    beyond it is written; the threshold's length is k."""
    rng = np.random.default_rng(12)
    d = 50000
    g = (rng.standard_normal(d) * 1e-2).astype(np.float32)
    mask = rng.random(d) < 0.07
    ind = np.zeros(oracle.n_ind_words(d), np.uint32)
    for i in np.nonzero(mask)[0]:
        ind[i // 32] |= np.uint32(1 << (i % 32))
    k = int(mask.sum())
    sel, cnt, sc, th = oracle.quantize_selected(g, ind, bucket=0)
    assert cnt.shape == (1,) and sc.shape == (1,) and int(cnt[0]) == k
    nw = (k + 15) // 16
    assert not sel[nw:].any()                                     # 2k bits and nothing else
    assert (int(sel[nw - 1]) >> (2 * (k % 16))) == 0 or k % 16 == 0   # unused bits of the last word
    v = g[mask]
    assert th[0] == np.float32(0.75 * np.abs(v.astype(np.float64)).sum() / k)
    kept = np.abs(v) > th[0]
    assert sc[0] == np.float32(np.abs(v[kept].astype(np.float64)).sum() / kept.sum())
    want = np.where(v > th[0], 1, np.where(v < -th[0], -1, 0)).astype(np.int8)
    assert np.array_equal(oracle.unpack(sel, k), want)
    bits = 32 + d + 2 * k
    assert bits == 32 * sc.size + 32 * ind.size - (32 * ind.size - d) + 2 * int(cnt.sum())
    # the dense message of the same vector costs 32 + 2d bits: the sparse one is smaller iff k < d/2
    assert bits < 32 + 2 * d
