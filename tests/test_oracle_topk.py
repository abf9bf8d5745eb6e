"""Pins of the oracle's per-chunk top-K codec (the aggressive compression the paper names for C_LP_S, Section 3.2)."""
import numpy as np
import pytest

SIZES = [1, 5, 255, 256, 257, 1000, 4095, 4096, 4097, 2 * 4096 + 7]


def t3(n, seed):
    return (np.random.default_rng(seed).standard_t(3, n) * 1e-3).astype(np.float32)


def brute_force_topk(v, keep):
    """Indices of the `keep` largest |v|, lower index first among equals (stable sort on the negated magnitude)."""
    order = np.argsort(-np.abs(v).astype(np.float64), kind="stable")
    return np.sort(order[:min(keep, v.size)])


@pytest.mark.parametrize("n", SIZES)
@pytest.mark.parametrize("C,keep", [(256, 1), (256, 8), (256, 256), (4096, 128), (4096, 1000)])
def test_selection_brute_force_and_error_state(oracle, n, C, keep):
    x = t3(n, n + keep)
    x[::7] = np.round(x[::7] * 1e3) / 1e3          # plenty of exact ties (and zeros)
    d0 = t3(n, n + 1) * np.float32(0.1)
    d = d0.copy()
    idx, val = oracle.compress_topk(x, d, C, keep)
    v = (x + d0).astype(np.float32)
    dec = oracle.decompress_topk(idx, val, n, C, keep)
    for c, lo in enumerate(range(0, n, C)):
        hi = min(n, lo + C)
        want = brute_force_topk(v[lo:hi], keep)
        got = idx[c * keep:(c + 1) * keep]
        nk = want.size
        assert np.array_equal(got[:nk], want.astype(np.uint16))
        assert np.all(got[nk:] == 0xFFFF) and not val[c * keep + nk:(c + 1) * keep].any()
        assert val[c * keep:c * keep + nk].tobytes() == (v[lo:hi][want] + np.float32(0)).tobytes()   # -0 stored as +0
        assert np.all(np.diff(got[:nk].astype(np.int64)) > 0)                      # ascending, unique
        kept = np.zeros(hi - lo, bool); kept[want] = True
        if (~kept).any():
            assert np.abs(v[lo:hi][~kept]).max() <= np.abs(v[lo:hi][kept]).min()      # nothing larger was dropped
    # error-feedback identity is exact for this codec: decoded + residual == v bit for bit (up to the sign of zero)
    assert np.array_equal(dec + d, v)
    assert np.all((dec == 0) | (d == 0))
    e2 = float(np.sum(v.astype(np.float64) ** 2))
    assert abs(float(np.sum(d.astype(np.float64) ** 2)) + float(np.sum(dec.astype(np.float64) ** 2)) - e2) <= 1e-9 * max(e2, 1e-30)


def test_keep_everything_is_lossless_and_ties_take_lowest_indices(oracle):
    C = 256
    x = t3(3 * C, 1)
    idx, val = oracle.compress_topk(x, None, C, C)
    assert np.array_equal(oracle.decompress_topk(idx, val, x.size, C, C), x)
    flat = np.full(C, 0.25, np.float32); flat[100] = -0.25
    idx, val = oracle.compress_topk(flat, None, C, 10)
    assert idx.tolist() == list(range(10))
    z = np.zeros(C, np.float32); z[5] = -0.0
    idx, val = oracle.compress_topk(z, None, C, 7)
    assert idx.tolist() == list(range(7)) and not np.signbit(val).any()


def test_telescoping_with_error_state(oracle):
    """With the error state, everything dropped is sent later: sum_t decode_t = sum_t x_t - delta_T."""
    n, C, keep, T = 1000, 256, 16, 30
    d = np.zeros(n, np.float32)
    sx = np.zeros(n, np.float64); sq = np.zeros(n, np.float64)
    for t in range(T):
        x = t3(n, 700 + t)
        sx += x
        idx, val = oracle.compress_topk(x, d, C, keep)
        sq += oracle.decompress_topk(idx, val, n, C, keep)
    assert np.max(np.abs(sq - (sx - d))) <= T * 2e-9


@pytest.mark.parametrize("k", [1, 2, 3, 8])
def test_server_step_is_dense_average_then_topk(oracle, k):
    n, C, keep = 3 * 256 + 50, 256, 24
    enc = [oracle.compress_topk(t3(n, 900 + j), None, C, keep) for j in range(k)]
    eps0 = t3(n, 3) * np.float32(0.05)
    eps = eps0.copy()
    idx, val, out = oracle.drr_topk([e[0] for e in enc], [e[1] for e in enc], eps, n, C, keep)
    dense = [oracle.decompress_topk(e[0], e[1], n, C, keep) for e in enc]
    s = dense[0].copy()
    for j in range(1, k):
        s = (s + dense[j]).astype(np.float32)
    w = ((s * (np.float32(1.0) / np.float32(k))).astype(np.float32) + eps0).astype(np.float32)
    for c, lo in enumerate(range(0, n, C)):
        hi = min(n, lo + C)
        want = brute_force_topk(w[lo:hi], keep)
        assert np.array_equal(idx[c * keep:c * keep + want.size], want.astype(np.uint16))
        assert val[c * keep:c * keep + want.size].tobytes() == (w[lo:hi][want] + np.float32(0)).tobytes()
    assert np.array_equal(out + eps, w)
    assert np.array_equal(out, oracle.decompress_topk(idx, val, n, C, keep))
    exact = np.mean(np.stack(dense).astype(np.float64), 0) + eps0
    assert np.max(np.abs(w - exact)) <= 1e-6 * np.max(np.abs(exact)) + 1e-9


def test_invalid(oracle):
    x = np.zeros(300, np.float32)
    for keep in (0, 257):
        with pytest.raises(ValueError):
            oracle.compress_topk(x, None, 256, keep)
    with pytest.raises(ValueError):
        oracle.decompress_topk(np.array([300] + [0xFFFF] * 3, np.uint16), np.zeros(4, np.float32), 300, 256, 2)
