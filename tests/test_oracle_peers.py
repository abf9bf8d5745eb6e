"""Pins of the oracle's decentralised averaging with the random peer strategy (Section 3.4)."""
import numpy as np
import pytest


def reps(k, n, seed):
    r = np.random.default_rng(seed)
    return [r.standard_normal(n).astype(np.float32) for _ in range(k)]


def test_hypercube_rounds_reach_the_global_mean(oracle):
    """Closed form: for k = 2^d, rounds with peers i^1, i^2, ..., i^(k/2) are a butterfly all-reduce:
    afterwards every replica equals the mean of all k (the C_FP_S result divided by k)."""
    k, n = 8, 5000
    xs = reps(k, n, 1)
    mean = np.mean(np.stack(xs).astype(np.float64), axis=0)
    cur = xs
    for bit in (1, 2, 4):
        cur = oracle.peer_avg_fp(cur, [i ^ bit for i in range(k)])
    for i in range(k):
        assert np.max(np.abs(cur[i] - mean)) <= 4e-7 * max(1.0, np.max(np.abs(mean)))
    for i in range(1, k):
        assert np.array_equal(cur[i], cur[0])        # fp addition is commutative: partners always hold equal bits


def test_matching_is_symmetric_and_preserves_the_mean(oracle):
    k, n = 6, 1234
    xs = reps(k, n, 2)
    peer = [3, 4, 5, 0, 1, 2]
    out = oracle.peer_avg_fp(xs, peer)
    for i in range(k):
        assert np.array_equal(out[i], out[peer[i]])
        want = ((xs[i] + xs[peer[i]]).astype(np.float32) * np.float32(0.5)).astype(np.float32)
        assert np.array_equal(out[i], want)
    m0 = np.mean(np.stack(xs).astype(np.float64), 0)
    m1 = np.mean(np.stack(out).astype(np.float64), 0)
    assert np.max(np.abs(m0 - m1)) <= 1e-7


def test_self_peer_is_identity_and_general_maps(oracle):
    k, n = 4, 777
    xs = reps(k, n, 3)
    out = oracle.peer_avg_fp(xs, [0, 1, 2, 3])
    for i in range(k):
        assert out[i].tobytes() == xs[i].tobytes()
    # a non-symmetric choice (everyone probes worker 0): each output is the midpoint with replica 0
    out = oracle.peer_avg_fp(xs, [0, 0, 0, 0])
    for i in range(k):
        mid = (xs[i].astype(np.float64) + xs[0]) / 2
        assert np.max(np.abs(out[i] - mid)) <= 2e-7 * max(1.0, np.max(np.abs(mid)))
    with pytest.raises(ValueError):
        oracle.peer_avg_fp(xs, [0, 1, 2, 4])


def base_and_reps(k, n, seed):
    r = np.random.default_rng(seed)
    base = (r.standard_normal(n) * 0.02).astype(np.float32)
    return base, [(base + (r.standard_normal(n) * 1e-3).astype(np.float32)).astype(np.float32) for _ in range(k)]


def test_lp_peers_mean_preservation_and_wire(oracle):
    """Low precision with chosen peers: for a matching the replica mean is preserved exactly in real arithmetic
    whatever Q does; the wire is Q(x - xhat) and xhat advances by its decode."""
    k, n, C = 6, 3 * 256 + 31, 256
    base, xs = base_and_reps(k, n, 7)
    peer = [1, 0, 3, 2, 5, 4]
    hat0 = [base.copy() for _ in range(k)]
    hat = [h.copy() for h in hat0]
    outs, codes, mm = oracle.peer_avg_lp(xs, hat, peer, C)
    m0 = np.mean(np.stack(xs).astype(np.float64), 0)
    m1 = np.mean(np.stack(outs).astype(np.float64), 0)
    assert np.max(np.abs(m0 - m1)) <= 1e-6 * np.max(np.abs(m0))
    for i in range(k):
        d = (xs[i] - hat0[i]).astype(np.float32)
        c2, m2 = oracle.compress_minmax_u8(d, None, C)
        assert np.array_equal(codes[i], c2) and np.array_equal(mm[i], m2)
        assert np.array_equal(hat[i], (hat0[i] + oracle.decompress_minmax_u8(c2, m2, C)).astype(np.float32))
    for i in range(k):
        a, b = hat[i], hat[peer[i]]
        want = (((a + b).astype(np.float32) * np.float32(0.5)).astype(np.float32) + (xs[i] - a).astype(np.float32)).astype(np.float32)
        assert np.array_equal(outs[i], want)


def test_lp_peers_lossless_equals_fp(oracle):
    """If every difference lies on a lossless grid, Q is the identity, xhat' = x, and the LP result is the FP one."""
    k, C, nch, p = 4, 256, 2, -12
    rng = np.random.default_rng(3)
    n = C * nch
    base = (rng.integers(-500, 500, n) * 2.0 ** p).astype(np.float32)
    xs = []
    for i in range(k):
        j = rng.integers(0, 256, n)
        j[::C] = 0; j[1::C] = 255
        xs.append((base + (j * 2.0 ** p).astype(np.float32)).astype(np.float32))
    hat = [base.copy() for _ in range(k)]
    peer = [2, 3, 0, 1]
    lp, _, _ = oracle.peer_avg_lp(xs, hat, peer, C)
    fp = oracle.peer_avg_fp(xs, peer)
    for i in range(k):
        assert np.array_equal(hat[i], xs[i]) and np.array_equal(lp[i], fp[i])
