"""Pins of the oracle's decode + bucket-level SGD step (Section 3.5: the optimizer runs on the flattened bucket)."""
import numpy as np
import pytest


def lossless_codes(oracle, rng, n, C, p=-10):
    """A gradient on a grid where MinMax-u8 is exact, so decode(codes) is known in closed form."""
    j = rng.integers(0, 256, n)
    for lo in range(0, n, C):
        hi = min(n, lo + C)
        j[lo] = 0
        j[hi - 1] = 255 if hi - lo > 1 else 0
    g = ((j - 128) * 2.0 ** p).astype(np.float32)
    if n % C == 1:
        g[-1] = g[-1]      # a one-element last chunk is flat: still exact
    codes, mm = oracle.compress_minmax_u8(g, None, C)
    assert np.array_equal(oracle.decompress_minmax_u8(codes, mm, C), g)
    return g, codes, mm


@pytest.mark.parametrize("n,C", [(1, 256), (300, 256), (3 * 4096 + 17, 4096)])
def test_plain_sgd_closed_form(oracle, n, C):
    """No momentum, no decay: p_T = p_0 - T*lr*g (exactly representable values -> exact)."""
    rng = np.random.default_rng(n)
    g, codes, mm = lossless_codes(oracle, rng, n, C)
    p0 = (rng.integers(-1000, 1000, n) * 2.0 ** -8).astype(np.float32)
    p = p0.copy()
    lr = np.float32(0.5)
    for _ in range(3):
        oracle.decompress_sgd_step(0, codes, mm, n, C, p, None, lr)
    assert np.array_equal(p, (p0.astype(np.float64) - 3 * 0.5 * g.astype(np.float64)).astype(np.float32))
    # lr = 0 leaves the parameters bit-identical
    q = p.copy()
    oracle.decompress_sgd_step(0, codes, mm, n, C, q, None, np.float32(0.0))
    assert q.tobytes() == p.tobytes()


def test_momentum_closed_form(oracle):
    """Constant gradient: m_T = g*(1-mu^T)/(1-mu), p_T = p_0 - lr*sum_t m_t; a zero buffer gives m_1 = g."""
    n, C, T = 2000, 256, 12
    rng = np.random.default_rng(1)
    g, codes, mm = lossless_codes(oracle, rng, n, C)
    p0 = rng.standard_normal(n).astype(np.float32)
    p, m = p0.copy(), np.zeros(n, np.float32)
    lr, mu = 0.1, 0.9
    oracle.decompress_sgd_step(0, codes, mm, n, C, p, m, lr, mu)
    assert np.array_equal(m, g)                                    # first step: buffer = gradient
    for _ in range(T - 1):
        oracle.decompress_sgd_step(0, codes, mm, n, C, p, m, lr, mu)
    g64 = g.astype(np.float64)
    mT = g64 * (1 - mu ** T) / (1 - mu)
    sum_m = g64 * (T - mu * (1 - mu ** T) / (1 - mu)) / (1 - mu)
    assert np.max(np.abs(m - mT)) <= 1e-6 * np.max(np.abs(mT))
    assert np.max(np.abs(p - (p0 - lr * sum_m))) <= 2e-6 * max(1.0, np.max(np.abs(p0)))


def test_weight_decay_and_order_of_operations(oracle):
    """g + wd*p enters both the momentum and the update; each operation rounds once (independent NumPy emulation)."""
    n, C = 1000, 256
    rng = np.random.default_rng(2)
    x = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    codes, mm = oracle.compress_minmax_u8(x, None, C)
    g = oracle.decompress_minmax_u8(codes, mm, C)
    p0 = rng.standard_normal(n).astype(np.float32)
    m0 = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    lr, mu, wd = np.float32(0.03), np.float32(0.9), np.float32(1e-2)
    p, m = p0.copy(), m0.copy()
    oracle.decompress_sgd_step(0, codes, mm, n, C, p, m, lr, mu, wd)
    gg = (g + (wd * p0).astype(np.float32)).astype(np.float32)
    mm_ = ((mu * m0).astype(np.float32) + gg).astype(np.float32)
    pp = (p0 - (lr * mm_).astype(np.float32)).astype(np.float32)
    assert np.array_equal(m, mm_) and np.array_equal(p, pp)
    # fp64 model: p' = p - lr*(mu*m + g + wd*p)
    ref = p0 - 0.03 * (0.9 * m0.astype(np.float64) + g + 1e-2 * p0)
    assert np.max(np.abs(p - ref)) <= 1e-6 * np.max(np.abs(ref))


def test_sign_codec_decode_feeds_the_step(oracle):
    n, C = 3 * 256 + 9, 256
    rng = np.random.default_rng(3)
    x = rng.laplace(0, 1e-3, n).astype(np.float32)
    bits, scale = oracle.sign_compress_ef(x, None, C)
    p0 = rng.standard_normal(n).astype(np.float32)
    p = p0.copy()
    oracle.decompress_sgd_step(1, bits, scale, n, C, p, None, np.float32(1.0))
    step = p0.astype(np.float64) - p
    want = np.where(x >= 0, 1.0, -1.0) * np.repeat(scale.astype(np.float64), C)[:n]
    assert np.max(np.abs(step - want)) <= 1e-7          # |p0| ~ 1: the subtraction rounds at 6e-8
    assert np.all(np.sign(step) == np.where(x >= 0, 1.0, -1.0))


# ----------------------------------------------------------------------------- the step after a top-K round
def _topk_inputs(n, C, keep, seed):
    r = np.random.default_rng(seed)
    x = (r.standard_normal(n) * 1e-2).astype(np.float32)
    return x


def test_topk_plain_sgd_moves_only_the_kept_entries(oracle):
    """Without momentum and weight decay the kept entries move by fl(lr * value) and every other parameter keeps its
    bits (g = +0 there): checked against the sparse entries themselves, not against a dense decode."""
    n, C, keep = 3 * 256 + 40, 256, 8
    x = _topk_inputs(n, C, keep, 1)
    idx, val = oracle.compress_topk(x, None, C, keep)
    p0 = (np.random.default_rng(2).standard_normal(n)).astype(np.float32)
    p0[5] = -0.0
    p = p0.copy()
    lr = np.float32(0.1)
    oracle.decompress_sgd_step_topk(idx, val, n, C, keep, p, None, float(lr))
    want = p0.copy()
    for c in range((n + C - 1) // C):
        for s_ in range(keep):
            q = int(idx[c * keep + s_])
            if q != 0xFFFF:
                want[c * C + q] = p0[c * C + q] - lr * val[c * keep + s_]
    assert p.tobytes() == want.tobytes()
    assert np.count_nonzero(p != p0) <= ((n + C - 1) // C) * keep


def test_topk_sgd_with_everything_kept_is_the_dense_step(oracle):
    """keep = C makes the codec lossless: the step must equal the fp64 formula of SGD with weight decay and momentum on
    the exact gradient, over three steps (state carried)."""
    n, C = 2 * 256, 256
    p = (np.random.default_rng(3).standard_normal(n)).astype(np.float32)
    m = np.zeros(n, np.float32)
    p64, m64 = p.astype(np.float64), m.astype(np.float64)
    lr, mu, wd = 0.05, 0.9, 1e-2
    for step in range(3):
        g = _topk_inputs(n, C, C, 10 + step)
        idx, val = oracle.compress_topk(g, None, C, C)
        oracle.decompress_sgd_step_topk(idx, val, n, C, C, p, m, lr, mu, wd)
        g64 = g.astype(np.float64) + wd * p64
        m64 = mu * m64 + g64
        p64 = p64 - lr * m64
    assert np.max(np.abs(p - p64)) <= 1e-5 * np.max(np.abs(p64))
    assert np.max(np.abs(m - m64)) <= 1e-5 * np.max(np.abs(m64)) + 1e-9


def test_topk_sgd_momentum_decays_where_nothing_is_kept(oracle):
    """Entries that are never selected see g = 0: their momentum decays geometrically and the parameter follows the
    closed form p_T = p_0 - lr * m_0 * (mu + mu^2 + ... + mu^T)."""
    n, C, keep = 256, 256, 4
    g = np.zeros(n, np.float32)
    g[:4] = [5.0, -6.0, 7.0, -8.0]                       # always the four kept entries
    idx, val = oracle.compress_topk(g, None, C, keep)
    p = np.ones(n, np.float32)
    m = np.full(n, 0.5, np.float32)
    lr, mu, T = 0.1, 0.5, 6
    for _ in range(T):
        oracle.decompress_sgd_step_topk(idx, val, n, C, keep, p, m, lr, mu, 0.0)
    geo = sum(mu ** t for t in range(1, T + 1))
    assert np.allclose(p[4:], 1.0 - lr * 0.5 * geo, rtol=1e-6)
    assert np.allclose(m[4:], 0.5 * mu ** T, rtol=1e-6)
    assert np.all(p[:4] != p[4])                          # the kept entries did move differently
