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
