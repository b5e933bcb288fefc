"""Pins for the oracle's tensor-list functions: a list of tensors in one flat vector is quantized
and stepped tensor by tensor.  The pins tie these functions to the single-vector ones (which
have their own pins against the paper's worked examples and closed forms):
  * tensors of one common length laid end to end ARE the bucketed quantizer;
  * scaling a tensor by a power of two keeps its codes and scales its scale exactly;
  * every tensor's result equals the single-vector result on a private copy of that tensor;
  * coordinates between tensors keep code 0 and their state."""
import numpy as np
import pytest

import oracle


def tensors(rng, lengths, gap_words=(0, 1, 3)):
    """Begin offsets (multiples of 16) for the given lengths with varying gaps; returns begin, d."""
    begin, pos = [], 0
    for i, n in enumerate(lengths):
        begin.append(pos)
        pos = (pos + n + 15) // 16 * 16 + 16 * gap_words[i % len(gap_words)]
    return np.array(begin, np.int64), pos + 5


LENGTHS = [150, 6, 2400, 16, 0, 48000, 120, 1, 10, 4097, 33]


def test_equal_lengths_end_to_end_are_the_bucketed_quantizer():
    rng = np.random.default_rng(1)
    b, nseg, M = 192, 7, 3
    d = b * nseg
    g = (rng.standard_normal((M, d)) * np.logspace(-3, 1, nseg).repeat(b)).astype(np.float32)
    begin = np.arange(nseg, dtype=np.int64) * b
    length = np.full(nseg, b, np.int64)
    c, s, th = oracle.quantize_pack_segments(g, begin, length)
    c0, s0, th0 = oracle.quantize_pack(g, b)
    assert np.array_equal(c, c0) and np.array_equal(s, s0) and np.array_equal(th, th0)
    for method in (oracle.QCMD, oracle.QRDA):
        for requant in (False, True):
            st = [rng.standard_normal(d).astype(np.float32) * 0.1,
                  rng.random(d).astype(np.float32), rng.standard_normal(d).astype(np.float32)]
            a = [v.copy() for v in st]
            r = [v.copy() for v in st]
            oracle.step_segments(method, c, s, d, begin, length, *a, 3, 0.1, 0.01, 1e-8, requant)
            rq = oracle.REQUANT_BUCKET if requant else oracle.REQUANT_NONE
            if method == oracle.QCMD:
                oracle.step_qcmd(c0, s0, d, b, *r, 0.1, 0.01, 1e-8, rq)
            else:
                oracle.step_qrda(c0, s0, d, b, *r, 3, 0.1, 0.01, 1e-8, rq)
            for u, v in zip(a, r):
                assert np.array_equal(u, v)


def test_power_of_two_scaling_of_one_tensor_changes_only_its_scale():
    rng = np.random.default_rng(2)
    lengths = [100, 37, 512]
    begin, d = tensors(rng, lengths)
    length = np.array(lengths, np.int64)
    g = np.zeros((1, d), np.float32)
    for b, n in zip(begin, lengths):
        g[0, b:b + n] = rng.standard_normal(n)
    c, s, th = oracle.quantize_pack_segments(g, begin, length)
    g2 = g.copy()
    g2[0, begin[1]:begin[1] + 37] *= 8.0
    c2, s2, th2 = oracle.quantize_pack_segments(g2, begin, length)
    assert np.array_equal(c, c2)
    assert s2[0, 1] == 8 * s[0, 1] and th2[0, 1] == 8 * th[0, 1]
    assert s2[0, 0] == s[0, 0] and s2[0, 2] == s[0, 2]


def test_each_tensor_equals_the_single_vector_functions_on_a_private_copy():
    rng = np.random.default_rng(3)
    M = 4
    begin, d = tensors(rng, LENGTHS)
    length = np.array(LENGTHS, np.int64)
    g = (rng.standard_normal((M, d)) * 0.01).astype(np.float32)       # gaps hold non-zero junk
    c, s, th = oracle.quantize_pack_segments(g, begin, length)
    covered = np.zeros(d, bool)
    for k, (b, n) in enumerate(zip(begin, LENGTHS)):
        covered[b:b + n] = True
        if n == 0:
            assert not s[:, k].any() and not th[:, k].any()
            continue
        ck, sk, tk = oracle.quantize_pack(g[:, b:b + n].copy(), 0)
        W = (n + 15) // 16
        assert np.array_equal(c[:, b // 16:b // 16 + W], ck)
        assert np.array_equal(s[:, k], sk[:, 0]) and np.array_equal(th[:, k], tk[:, 0])
    for m in range(M):
        code = oracle.unpack(c[m], d)
        assert not code[~covered].any()                                # no tensor: field 0
    for method in (oracle.QCMD, oracle.QRDA):
        for requant in (False, True):
            x = (rng.standard_normal(d) * 0.1).astype(np.float32)
            G = rng.random(d).astype(np.float32)
            z = rng.standard_normal(d).astype(np.float32)
            x1, G1, z1 = x.copy(), G.copy(), z.copy()
            oracle.step_segments(method, c, s, d, begin, length, x1, G1, z1, 5, 0.1, 0.02, 1e-8,
                                 requant)
            assert np.array_equal(x1[~covered], x[~covered])           # state between tensors
            assert np.array_equal(G1[~covered], G[~covered])
            assert np.array_equal(z1[~covered], z[~covered])
            for k, (b, n) in enumerate(zip(begin, LENGTHS)):
                if n == 0:
                    continue
                W = (n + 15) // 16
                xs, Gs, zs = x[b:b + n].copy(), G[b:b + n].copy(), z[b:b + n].copy()
                ck = np.ascontiguousarray(c[:, b // 16:b // 16 + W])
                sk = np.ascontiguousarray(s[:, k:k + 1])
                rq = oracle.REQUANT_GLOBAL if requant else oracle.REQUANT_NONE
                if method == oracle.QCMD:
                    oracle.step_qcmd(ck, sk, n, 0, xs, Gs, zs, 0.1, 0.02, 1e-8, rq)
                else:
                    oracle.step_qrda(ck, sk, n, 0, xs, Gs, zs, 5, 0.1, 0.02, 1e-8, rq)
                assert np.array_equal(x1[b:b + n], xs), (method, requant, k)
                assert np.array_equal(G1[b:b + n], Gs)
                assert np.array_equal(z1[b:b + n], zs)


def test_qcmd_without_z_and_tensor_shorter_than_a_word():
    begin = np.array([0, 16], np.int64)
    length = np.array([3, 5], np.int64)
    g = np.zeros((1, 32), np.float32)
    g[0, :3] = [4.0, -1.0, 1.0]          # mean|v| = 2, Delta = 1.5: keeps 4 -> s = 4, codes + 0 0
    g[0, 16:21] = [-2.0, -2.0, 2.0, 0.0, 0.0]   # mean 1.2, Delta 0.9: keeps three 2s -> s = 2
    g[0, 3:16] = 100.0                   # junk between the tensors
    c, s, th = oracle.quantize_pack_segments(g, begin, length)
    assert list(s[0]) == [4.0, 2.0] and list(th[0]) == [1.5, np.float32(0.75 * 1.2)]
    assert c[0, 0] == 0b01 and c[0, 1] == (0b11 | 0b11 << 2 | 0b01 << 4)
    x = np.zeros(32, np.float32)
    G = np.zeros(32, np.float32)
    oracle.step_segments(oracle.QCMD, c, s, 32, begin, length, x, G, None, 1, 1.0, 0.0, 1e-8)
    # H = 1e-8 + |q| = |q| in binary32, so x = -eta q / |q| = -sign(q) on the kept coordinates, 0 elsewhere
    expect = np.zeros(32, np.float32)
    expect[0] = -1.0
    expect[16:19] = [1.0, 1.0, -1.0]
    assert np.array_equal(x, expect)
    assert G[0] == 16.0 and list(G[16:19]) == [4.0, 4.0, 4.0] and G.sum() == 28.0
