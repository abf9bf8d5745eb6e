"""Pins of the oracle's intra-node stage of hierarchical C_LP_S (Section 3.5, "Hierarchical Communications")."""
import numpy as np
import pytest


def vals(n, seed):
    return (np.random.default_rng(seed).standard_normal(n) * 1e-3).astype(np.float32)


@pytest.mark.parametrize("n,C", [(1, 256), (300, 256), (2 * 4096 + 9, 4096)])
def test_single_local_worker_is_plain_compression(oracle, n, C):
    x = vals(n, n)
    d1, d2 = vals(n, 1) * np.float32(0.1), None
    d2 = d1.copy()
    c1, m1 = oracle.reduce_compress_minmax_u8([x], d1, C)
    c2, m2 = oracle.compress_minmax_u8(x, d2, C)
    assert np.array_equal(c1, c2) and np.array_equal(m1, m2) and np.array_equal(d1, d2)


@pytest.mark.parametrize("k", [2, 3, 4, 8])
def test_aggregate_is_left_to_right_average_then_Q(oracle, k):
    """The leader compresses exactly the ascending-order fp32 average: statistics, round-trip bound and
    error-feedback identity hold with respect to it, and the order is visible through 2^24 + 1 + 1 - 2^24."""
    n, C = 3 * 256 + 40, 256
    xs = [vals(n, 10 * k + j) for j in range(k)]
    s = xs[0].copy()
    for j in range(1, k):
        s = (s + xs[j]).astype(np.float32)
    a = (s * (np.float32(1.0) / np.float32(k))).astype(np.float32)
    d0 = vals(n, 99) * np.float32(0.05)
    d = d0.copy()
    codes, mm = oracle.reduce_compress_minmax_u8(xs, d, C)
    v = (a + d0).astype(np.float32)
    deq = oracle.decompress_minmax_u8(codes, mm, C)
    for c, lo in enumerate(range(0, n, C)):
        hi = min(n, lo + C)
        assert mm[2 * c] == v[lo:hi].min() and mm[2 * c + 1] == v[lo:hi].max()
        r = float(mm[2 * c + 1]) - float(mm[2 * c])
        assert np.all(np.abs(v[lo:hi].astype(np.float64) - deq[lo:hi]) <= r / 255 / 2 * (1 + 1e-4) + 1e-9)
    assert np.array_equal(d, (v - deq).astype(np.float32))
    exact = np.mean(np.stack(xs).astype(np.float64), 0)
    assert np.max(np.abs(a - exact)) <= 1e-6 * np.max(np.abs(exact)) + 1e-9
    if k == 4:
        big = np.float32(2.0 ** 24)
        ys = [np.full(256, t, np.float32) for t in (big, 1.0, 1.0, -big)]
        codes, mm = oracle.reduce_compress_minmax_u8(ys, None, 256)
        assert mm.tolist() == [0.0, 0.0]        # ((2^24 + 1) + 1) - 2^24 = 0 in fp32, any other order gives 2/4


def test_two_level_pipeline_error_bounds(oracle):
    """2 nodes x 3 local workers: leaders' codes decode to within half a level of the node average, and the
    inter-node server step decodes to within half a level of the mean of what the leaders sent."""
    C, n = 256, 3 * 256 + 17
    nodes = [[vals(n, 100 + 10 * a + b) for b in range(3)] for a in range(2)]
    enc = [oracle.reduce_compress_minmax_u8(xs, None, C) for xs in nodes]
    sent = []
    for (codes, mm), xs in zip(enc, nodes):
        deq = oracle.decompress_minmax_u8(codes, mm, C)
        avg = np.mean(np.stack(xs).astype(np.float64), 0)
        rng_ = np.repeat((mm[1::2] - mm[0::2]).astype(np.float64), C)[:n]
        assert np.all(np.abs(deq - avg) <= rng_ / 255 / 2 * (1 + 1e-4) + 1e-9)
        sent.append(deq.astype(np.float64))
    c, m, out = oracle.drr_minmax_u8([e[0] for e in enc], [e[1] for e in enc], None, C)
    rng_ = np.repeat((m[1::2] - m[0::2]).astype(np.float64), C)[:n]
    assert np.all(np.abs(out - np.mean(sent, 0)) <= rng_ / 255 / 2 * (1 + 1e-4) + 1e-9)


@pytest.mark.parametrize("k", [1, 2, 5, 8])
def test_centralized_full_precision_average(oracle, k):
    """C_FP_S: the textbook mean (fp64) within fp32 rounding, the left-to-right order made visible, k = 1 the identity,
    and equal to the server step of C_LP_S on a lossless grid (Q = identity)."""
    n = 1000
    xs = [vals(n, 50 * k + j) for j in range(k)]
    out = oracle.centralized_avg_fp(xs)
    exact = np.mean(np.stack(xs).astype(np.float64), 0)
    assert np.max(np.abs(out - exact)) <= 1e-6 * np.max(np.abs(exact)) + 1e-10
    if k == 1:
        assert out.tobytes() == xs[0].tobytes()
    big = np.float32(2.0 ** 24)
    ys = [np.full(8, t, np.float32) for t in (big, 1.0, 1.0, -big)]
    assert oracle.centralized_avg_fp(ys)[0] == 0.0                       # ((2^24 + 1) + 1) - 2^24 = 0 in fp32
    assert oracle.centralized_avg_fp(ys[1:3] + ys[0:1] + ys[3:])[0] == 0.5
    # lossless grid: MinMax-u8 is the identity, so the C_LP_S server step must decode to the same average
    C, p = 256, -9
    rng = np.random.default_rng(k)
    gs = []
    for j in range(k):
        jj = rng.integers(0, 256, 2 * C); jj[::C] = 0; jj[1::C] = 255
        gs.append((jj * 2.0 ** p).astype(np.float32))
    enc = [oracle.compress_minmax_u8(g, None, C) for g in gs]
    avg = oracle.centralized_avg_fp(gs)
    codes, mm, outq = oracle.drr_minmax_u8([e[0] for e in enc], [e[1] for e in enc], None, C)
    rng_ = np.repeat((mm[1::2] - mm[0::2]).astype(np.float64), C)
    assert np.all(np.abs(outq - avg) <= rng_ / 255 / 2 * (1 + 1e-4) + 1e-9)
    for c in range(2):
        assert mm[2 * c] == avg[c * C:(c + 1) * C].min() and mm[2 * c + 1] == avg[c * C:(c + 1) * C].max()


# ----------------------------------------------------------------------------- intra-node stage, sign codec
@pytest.mark.parametrize("n,C", [(1, 256), (300, 256), (2 * 2048 + 9, 2048)])
def test_sign_single_local_worker_is_plain_sign_compression(oracle, n, C):
    x = vals(n, n + 5)
    d1 = vals(n, 2) * np.float32(0.1)
    d2 = d1.copy()
    b1, s1 = oracle.reduce_compress_sign([x], d1, C)
    b2, s2 = oracle.sign_compress_ef(x, d2, C)
    assert np.array_equal(b1, b2) and np.array_equal(s1, s2) and np.array_equal(d1, d2)


@pytest.mark.parametrize("k", [2, 3, 8])
def test_sign_aggregate_is_left_to_right_average_then_sign(oracle, k):
    """Bits are the signs of (ascending-order fp32 average + error state), the scale is the chunk mean of its
    magnitude (fp64 check), the new error state closes the identity v = decode + delta', and the summation order is
    visible through 2^24 + 1 + 1 - 2^24."""
    n, C = 3 * 256 + 40, 256
    xs = [vals(n, 20 * k + j) for j in range(k)]
    s = xs[0].copy()
    for j in range(1, k):
        s = (s + xs[j]).astype(np.float32)
    a = (s * (np.float32(1.0) / np.float32(k))).astype(np.float32)
    d0 = vals(n, 98) * np.float32(0.05)
    d = d0.copy()
    bits, scale = oracle.reduce_compress_sign(xs, d, C)
    v = (a + d0).astype(np.float32)
    want_bits = np.packbits((v >= 0).astype(np.uint8), bitorder="little")
    got_bits = bits.view(np.uint8)[:want_bits.size]
    assert np.array_equal(got_bits, want_bits)
    for c, lo in enumerate(range(0, n, C)):
        hi = min(n, lo + C)
        assert abs(float(scale[c]) - np.mean(np.abs(v[lo:hi].astype(np.float64)))) <= 1e-6 * float(scale[c]) + 1e-12
    deq = oracle.decompress_sign(bits, scale, n, C)
    assert np.array_equal(d, (v - deq).astype(np.float32))
    if k == 3:
        big = np.float32(2.0 ** 24)
        ys = [np.full(256, t, np.float32) for t in (big, 1.0, -big)]
        b, sc = oracle.reduce_compress_sign(ys, None, 256)
        assert sc.tolist() == [0.0] and not np.any(b != 0xFFFFFFFF)   # (2^24 + 1) - 2^24 = 0 in fp32: +0 everywhere
