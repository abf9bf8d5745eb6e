"""Pins of the CPU oracle for decentralised averaging (D_FP_S / D_LP_S, Section 3.2; ring peers, Section 3.4)."""
import numpy as np
import pytest


def replicas(k, n, seed):
    r = np.random.default_rng(seed)
    base = (r.standard_normal(n) * 0.02).astype(np.float32)
    return base, [(base + (r.standard_normal(n) * 1e-3).astype(np.float32)).astype(np.float32) for _ in range(k)]


@pytest.mark.parametrize("k", [1, 2, 3, 5, 8])
def test_fp_closed_form_circulant_power(oracle, k):
    """P7: r rounds of ring averaging equal W^r x with W = circulant(1/3 on the diagonal and both neighbours)."""
    n, rounds = 1000, 5
    _, xs = replicas(k, n, k)
    W = np.zeros((k, k))
    for i in range(k):
        for j in (i - 1, i, i + 1):
            W[i, j % k] += 1.0 / 3.0
    X0 = np.stack(xs).astype(np.float64)
    cur = xs
    for _ in range(rounds):
        cur = oracle.ring_avg_fp(cur)
    want = np.linalg.matrix_power(W, rounds) @ X0
    got = np.stack(cur).astype(np.float64)
    assert np.max(np.abs(got - want)) <= 1e-6 * np.max(np.abs(want))
    if k == 8:
        # contraction of the disagreement by the second-largest eigenvalue modulus (1+2cos(2pi/8))/3
        lam = (1 + 2 * np.cos(2 * np.pi / 8)) / 3
        d0 = np.linalg.norm(X0 - X0.mean(0))
        d1 = np.linalg.norm(np.stack(oracle.ring_avg_fp(xs)).astype(np.float64) - X0.mean(0))
        assert d1 <= lam * d0 * (1 + 1e-5)


@pytest.mark.parametrize("k", [1, 2, 3, 8])
def test_fp_literal_neighbours_and_order(oracle, k):
    """R7: x_i' = ((x_{i-1} + x_i) + x_{i+1}) * fl(1/3) with literal modular indices, one rounding per operation."""
    n = 777
    _, xs = replicas(k, n, 50 + k)
    xs[0][:5] = [2.0 ** 24, 1.0, -1.0, 3.0, 2.0 ** -30]   # make the association visible
    got = oracle.ring_avg_fp(xs)
    third = np.float32(1.0) / np.float32(3.0)
    for i in range(k):
        l, m, r = xs[(i - 1) % k], xs[i], xs[(i + 1) % k]
        want = (((l + m).astype(np.float32) + r).astype(np.float32) * third).astype(np.float32)
        np.testing.assert_array_equal(got[i], want)


@pytest.mark.parametrize("k", [2, 3, 8])
def test_mean_preservation(oracle, k):
    """P6: the replica mean is preserved by FP and by LP averaging (symmetric ring weights)."""
    n, C = 4 * 256 + 19, 256
    base, xs = replicas(k, n, 90 + k)
    m0 = np.mean(np.stack(xs).astype(np.float64), axis=0)
    fp = oracle.ring_avg_fp(xs)
    assert np.max(np.abs(np.mean(np.stack(fp).astype(np.float64), 0) - m0)) <= 1e-6 * np.max(np.abs(m0))
    xhat = [base.copy() for _ in range(k)]
    cur = xs
    for _ in range(5):
        cur, _, _ = oracle.ring_avg_lp(cur, xhat, C)
        m = np.mean(np.stack(cur).astype(np.float64), axis=0)
        assert np.max(np.abs(m - m0)) <= 1e-6 * np.max(np.abs(m0))


def test_lp_consensus_and_tracking(oracle):
    """LP rounds contract the disagreement between replicas, and the public copies xhat track x
    to within half a quantisation level of the difference that was sent."""
    k, n, C = 8, 8 * 256, 256
    base, xs = replicas(k, n, 5)
    xhat = [base.copy() for _ in range(k)]
    X0 = np.stack(xs).astype(np.float64)
    d_prev = np.linalg.norm(X0 - X0.mean(0))
    cur = xs
    for _ in range(5):
        before = [h.copy() for h in xhat]
        nxt, codes, mm = oracle.ring_avg_lp(cur, xhat, C)
        for i in range(k):
            d = (cur[i] - before[i]).astype(np.float64)
            rng_ = np.repeat((mm[i][1::2] - mm[i][0::2]).astype(np.float64), C)[:n]
            assert np.all(np.abs(xhat[i] - before[i] - d) <= rng_ / 255 / 2 * (1 + 1e-4) + 1e-8)
        X = np.stack(nxt).astype(np.float64)
        dn = np.linalg.norm(X - X.mean(0))
        assert dn < d_prev
        d_prev = dn
        cur = nxt


def test_lp_lossless_equals_fp(oracle):
    """P4: if every difference x_i - xhat_i lies on a lossless grid, Q is the identity, xhat' = x and D_LP_S = D_FP_S."""
    k, C, nch, p = 4, 256, 3, -12
    rng = np.random.default_rng(3)
    n = C * nch
    base = (rng.integers(-500, 500, n) * 2.0 ** p).astype(np.float32)
    xs = []
    for i in range(k):
        j = rng.integers(0, 256, n)
        for c in range(nch):
            j[c * C] = 0
            j[c * C + 1] = 255
        xs.append((base + (j * 2.0 ** p).astype(np.float32)).astype(np.float32))
    xhat = [base.copy() for _ in range(k)]
    lp, codes, mm = oracle.ring_avg_lp(xs, xhat, C)
    for i in range(k):
        np.testing.assert_array_equal(xhat[i], xs[i])
    fp = oracle.ring_avg_fp(xs)
    for i in range(k):
        np.testing.assert_array_equal(lp[i], fp[i])   # own-term x - xhat' is exactly 0


def test_lp_wire_is_compressed_difference(oracle):
    """R8: what is sent is Q(x_i - xhat_i) (no error state), and xhat_i' = xhat_i + decode of it."""
    k, n, C = 3, 2 * 256 + 50, 256
    base, xs = replicas(k, n, 11)
    xhat0 = [base.copy() for _ in range(k)]
    xhat = [h.copy() for h in xhat0]
    outs, codes, mm = oracle.ring_avg_lp(xs, xhat, C)
    third = np.float32(1.0) / np.float32(3.0)
    for i in range(k):
        d = (xs[i] - xhat0[i]).astype(np.float32)
        c2, m2 = oracle.compress_minmax_u8(d, None, C)
        np.testing.assert_array_equal(codes[i], c2)
        np.testing.assert_array_equal(mm[i], m2)
        q = oracle.decompress_minmax_u8(c2, m2, C)
        np.testing.assert_array_equal(xhat[i], (xhat0[i] + q).astype(np.float32))
    for i in range(k):
        l, m, r = xhat[(i - 1) % k], xhat[i], xhat[(i + 1) % k]
        avg = (((l + m).astype(np.float32) + r).astype(np.float32) * third).astype(np.float32)
        want = (avg + (xs[i] - m).astype(np.float32)).astype(np.float32)
        np.testing.assert_array_equal(outs[i], want)
