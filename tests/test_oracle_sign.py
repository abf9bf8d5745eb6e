"""Pins of the CPU oracle for the 1-bit sign codec (the Q of "1-bit Adam", Section 4.1, inside C_LP_S, Section 3.2)."""
import numpy as np
import pytest

SIZES = [1, 2, 3, 5, 31, 32, 33, 255, 256, 257, 2047, 2048, 2049, 2 * 2048 + 7]


def lap(n, seed):
    r = np.random.default_rng(seed)
    return r.laplace(0.0, 1e-3, n).astype(np.float32)


def tree_sum_numpy(a, C):
    """Independent emulation of the ordered |v| sum: rows of 64 groups of four, sequential row adds, 6 butterfly levels."""
    a = np.abs(a.astype(np.float32))
    pad = (-a.size) % 256
    a = np.concatenate([a, np.zeros(pad, np.float32)]).reshape(-1, 64, 4)
    g = ((a[:, :, 0] + a[:, :, 1]).astype(np.float32) + (a[:, :, 2] + a[:, :, 3]).astype(np.float32)).astype(np.float32)
    acc = np.zeros(64, np.float32)
    for row in g:
        acc = (acc + row).astype(np.float32)
    for s in (1, 2, 4, 8, 16, 32):
        acc = (acc + acc[np.arange(64) ^ s]).astype(np.float32)
    assert np.all(acc == acc[0])
    return acc[0]


@pytest.mark.parametrize("n", SIZES)
@pytest.mark.parametrize("C", [256, 2048, 768])
def test_bits_scale_and_identities(oracle, n, C):
    """P9/P10/A12: bit = (v >= 0) LSB-first over the bucket, tail bits 0, scale = mean|v| in the fixed order,
    sum_i deq_i*sign(v_i) = L*scale, residual = v - (+-scale)."""
    x = lap(n, n + C)
    res0 = lap(n, n + C + 1) * np.float32(0.1)
    res = res0.copy()
    bits, scale = oracle.sign_compress_ef(x, res, C)
    v = (x + res0).astype(np.float32)
    want_bits = np.packbits((v >= 0).astype(np.uint8), bitorder="little")
    want_bits = np.concatenate([want_bits, np.zeros((-want_bits.size) % 4, np.uint8)]).view(np.uint32)
    np.testing.assert_array_equal(bits, want_bits)
    deq = oracle.decompress_sign(bits, scale, n, C)
    for c, lo in enumerate(range(0, n, C)):
        hi = min(n, lo + C)
        L = hi - lo
        s_tree = tree_sum_numpy(v[lo:hi], C)
        pow2 = C & (C - 1) == 0
        want = np.float32(s_tree * (np.float32(1.0) / np.float32(C))) if (L == C and pow2) else np.float32(s_tree / np.float32(L))
        assert scale[c] == want
        assert scale[c] >= 0
        exact = np.mean(np.abs(v[lo:hi].astype(np.float64)))
        assert abs(scale[c] - exact) <= 1e-6 * exact + 1e-45
        sgn = np.where(v[lo:hi] >= 0, 1.0, -1.0)
        assert np.all(deq[lo:hi] == sgn * scale[c])
        assert abs(np.sum(deq[lo:hi].astype(np.float64) * sgn) - L * float(scale[c])) <= 1e-9
        np.testing.assert_array_equal(res[lo:hi], (v[lo:hi] - deq[lo:hi]).astype(np.float32))
        # the residual of |v| about its mean sums to ~0
        assert abs(np.sum(np.abs(v[lo:hi].astype(np.float64)) - float(scale[c]))) <= 2e-6 * L * exact + 1e-40


def test_sign_flip_symmetry(oracle):
    """Negating every (non-zero) input flips every bit and leaves the scales bit-identical."""
    n, C = 3 * 2048 + 100, 2048
    x = lap(n, 3)
    x[x == 0] = 1e-3
    b1, s1 = oracle.sign_compress_ef(x, None, C)
    b2, s2 = oracle.sign_compress_ef(-x, None, C)
    np.testing.assert_array_equal(s1, s2)
    full = np.unpackbits(b1.view(np.uint8), bitorder="little")[:n] ^ np.unpackbits(b2.view(np.uint8), bitorder="little")[:n]
    assert full.all()
    # tail bits stay zero in both
    tail = np.unpackbits(b1.view(np.uint8), bitorder="little")[n:]
    assert not tail.any()


def test_zero_and_negative_zero_are_positive(oracle):
    x = np.array([0.0, -0.0, 1.0, -1.0] * 64, np.float32)
    bits, scale = oracle.sign_compress_ef(x, None, 256)
    assert np.unpackbits(bits.view(np.uint8), bitorder="little")[:8].tolist() == [1, 1, 1, 0, 1, 1, 1, 0]
    assert scale[0] == 0.5


def test_ordered_sum_differs_from_naive_order(oracle):
    """The reduction order is part of the definition: on data where fp32 addition is visibly
    non-associative the oracle's scale equals the tree value and not the sequential sum."""
    C = 2048
    r = np.random.default_rng(8)
    x = (r.standard_normal(C) * np.exp(r.standard_normal(C) * 4)).astype(np.float32)
    _, scale = oracle.sign_compress_ef(x, None, C)
    seq = np.float32(0)
    for a in np.abs(x):
        seq = np.float32(seq + a)
    tree = tree_sum_numpy(x, C)
    assert scale[0] == np.float32(tree * np.float32(1.0 / C))
    assert tree != seq       # the test data does discriminate


@pytest.mark.parametrize("k", [1, 2, 3, 8])
def test_server_step_sign_brute_force(oracle, k):
    """Server side with the sign codec against a direct per-element evaluation (ascending-j sum of +-scale_j,
    times fl(1/k), plus epsilon, then Q again)."""
    n, C = 2 * 256 + 77, 256
    bits_in, scale_in = [], []
    for j in range(k):
        b, s = oracle.sign_compress_ef(lap(n, 60 + j), None, C)
        bits_in.append(b); scale_in.append(s)
    eps0 = lap(n, 1) * np.float32(0.05)
    eps = eps0.copy()
    bits, scale, out = oracle.drr_sign(bits_in, scale_in, eps, n, C)
    a = np.empty(n, np.float32)
    invk = np.float32(1.0) / np.float32(k)
    for i in range(n):
        s = None
        for j in range(k):
            bit = (int(bits_in[j][i >> 5]) >> (i & 31)) & 1
            d = scale_in[j][i // C] if bit else -scale_in[j][i // C]
            s = np.float32(d) if s is None else np.float32(s + d)
        a[i] = np.float32(s * invk)
    w = (a + eps0).astype(np.float32)
    b2, s2 = oracle.sign_compress_ef(a, eps0.copy(), C)     # Q on (a + eps) is the worker-side Q
    np.testing.assert_array_equal(bits, b2)
    np.testing.assert_array_equal(scale, s2)
    want_bits = np.packbits((w >= 0).astype(np.uint8), bitorder="little")
    np.testing.assert_array_equal(bits.view(np.uint8)[:want_bits.size], want_bits)
    np.testing.assert_array_equal(out, oracle.decompress_sign(bits, scale, n, C))
    np.testing.assert_array_equal(eps, (w - out).astype(np.float32))
    if k == 1:
        # a single worker without server error: decoded input goes through unchanged in sign
        bb, ss, oo = oracle.drr_sign(bits_in, scale_in, None, n, C)
        np.testing.assert_array_equal(bb, bits_in[0])
        np.testing.assert_array_equal(ss, scale_in[0])
