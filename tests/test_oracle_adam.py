"""Pins of the oracle's Adam-type bucket step and of the momentum compression of 1-bit Adam (reading R20)."""
import numpy as np
import pytest
import torch


def lossless_codes(oracle, vals, C):
    """MinMax codes whose decode is exactly vals (every chunk spans a 255-step power-of-two grid)."""
    codes, mm = oracle.compress_minmax_u8(vals, None, C)
    assert np.array_equal(oracle.decompress_minmax_u8(codes, mm, C), vals)
    return codes, mm


def grid_values(rng, n, C, p=-10):
    j = rng.integers(0, 256, n)
    j[::C] = 0
    j[1::C] = 255
    return ((j - 128) * 2.0 ** p).astype(np.float32)


def test_adam_matches_torch_adam_state_and_fp64_update(oracle):
    """Five steps: m and v follow torch.optim.Adam's exp_avg / exp_avg_sq (same recurrences; torch's bias
    correction only enters its parameter update), and p follows p - lr*m/(sqrt(v)+eps) evaluated in fp64."""
    rng = np.random.default_rng(0)
    n, C = 4 * 256, 256
    p0 = rng.standard_normal(n).astype(np.float32)
    p, m, v = p0.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32)
    tp = torch.nn.Parameter(torch.from_numpy(p0.copy()).double())
    # the betas torch sees are the fp32 values the oracle receives, so 1 - beta is the same number on both sides
    opt = torch.optim.Adam([tp], lr=1e-3, betas=(float(np.float32(0.9)), float(np.float32(0.999))), eps=1e-8)
    p64 = p0.astype(np.float64)
    for it in range(5):
        g = grid_values(rng, n, C)
        codes, mm = lossless_codes(oracle, g, C)
        oracle.decompress_adam_step(0, codes, mm, n, C, p, m, v, 1e-3, 0.9, 0.999, 1e-8)
        tp.grad = torch.from_numpy(g).double()
        opt.step()
        st = opt.state[tp]
        em, ev = st["exp_avg"].numpy(), st["exp_avg_sq"].numpy()
        assert np.max(np.abs(m - em)) <= 4e-7 * np.max(np.abs(em))
        assert np.max(np.abs(v - ev)) <= 4e-7 * np.max(np.abs(ev))
        p64 = p64 - 1e-3 * em / (np.sqrt(ev) + 1e-8)
        assert np.max(np.abs(p - p64)) <= 1e-6 * (it + 1)


def test_adam_first_step_is_sign_descent(oracle):
    """From m = v = 0 with eps = 0: u = (1-b1) g / (sqrt(1-b2) |g|), a constant-magnitude step along sign(g)."""
    rng = np.random.default_rng(1)
    n, C = 2 * 256, 256
    g = grid_values(rng, n, C)
    g[g == 0] = np.float32(2.0 ** -10)
    g[0], g[1] = np.float32(-128 * 2.0 ** -10), np.float32(127 * 2.0 ** -10)
    codes, mm = lossless_codes(oracle, g, C)
    p0 = rng.standard_normal(n).astype(np.float32)
    p, m, v = p0.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32)
    lr, b1, b2 = 0.01, 0.9, 0.999
    oracle.decompress_adam_step(0, codes, mm, n, C, p, m, v, lr, b1, b2, 0.0)
    want = p0.astype(np.float64) - lr * (1 - np.float32(b1)) / np.sqrt(1 - np.float64(np.float32(b2))) * np.sign(g)
    assert np.max(np.abs(p - want)) <= 1e-6


def test_adam_identities(oracle):
    rng = np.random.default_rng(2)
    n, C = 3 * 256 + 17, 256
    x = (rng.standard_normal(n) * 1e-2).astype(np.float32)
    codes, mm = oracle.compress_minmax_u8(x, None, C)
    d = oracle.decompress_minmax_u8(codes, mm, C)
    p0 = rng.standard_normal(n).astype(np.float32)
    m0 = (rng.standard_normal(n) * 1e-2).astype(np.float32)
    v0 = (rng.random(n) * 1e-4 + 1e-6).astype(np.float32)
    # lr = 0: parameters untouched, state still advances
    p, m, v = p0.copy(), m0.copy(), v0.copy()
    oracle.decompress_adam_step(0, codes, mm, n, C, p, m, v, 0.0, 0.9, 0.999, 1e-8)
    assert np.array_equal(p, p0) and not np.array_equal(m, m0) and not np.array_equal(v, v0)
    # beta1 = beta2 = 0: m = d, v = d*d exactly
    p, m, v = p0.copy(), m0.copy(), v0.copy()
    oracle.decompress_adam_step(0, codes, mm, n, C, p, m, v, 1e-3, 0.0, 0.0, 1e-8)
    assert np.array_equal(m, d + np.float32(0)) and np.array_equal(v, (d * d).astype(np.float32))
    # frozen variance: m becomes the decoded tensor bit for bit, v untouched, update uses the old v
    p, m, v = p0.copy(), m0.copy(), v0.copy()
    oracle.decompress_adam_step(0, codes, mm, n, C, p, m, v, 1e-3, 0.9, 0.999, 1e-8, variance_frozen=True)
    assert np.array_equal(m.view(np.uint32), d.view(np.uint32)) and np.array_equal(v, v0)
    want = p0.astype(np.float64) - 1e-3 * d.astype(np.float64) / (np.sqrt(v0.astype(np.float64)) + 1e-8)
    assert np.max(np.abs(p - want)) <= 2e-7 * np.max(np.abs(want))
    # huge eps: u -> m/eps
    p, m, v = p0.copy(), m0.copy(), v0.copy()
    oracle.decompress_adam_step(0, codes, mm, n, C, p, m, v, 1.0, 0.9, 0.999, 1e6, variance_frozen=True)
    assert np.max(np.abs((p0 - p) - d / 1e6)) <= 1e-7
    # weight decay enters the update after the division, scaled by lr (decoupled from the variance)
    p, m, v = p0.copy(), m0.copy(), v0.copy()
    oracle.decompress_adam_step(0, codes, mm, n, C, p, m, v, 1e-3, 0.9, 0.999, 1e-8, weight_decay=0.1, variance_frozen=True)
    want_wd = want - 1e-3 * 0.1 * p0.astype(np.float64)
    assert np.max(np.abs(p - want_wd)) <= 2e-7 * np.max(np.abs(want_wd))


def test_adam_sign_codec_frozen(oracle):
    """Sign codec: the decoded momentum is +-scale, so with frozen variance p moves by lr*scale/(sqrt(v)+eps)."""
    rng = np.random.default_rng(3)
    n, C = 2 * 256, 256
    x = (rng.standard_normal(n) * 1e-2).astype(np.float32)
    bits, scale = oracle.sign_compress_ef(x, None, C)
    p0 = rng.standard_normal(n).astype(np.float32)
    p, m = p0.copy(), np.zeros(n, np.float32)
    v = np.full(n, 4e-6, np.float32)
    oracle.decompress_adam_step(1, bits, scale, n, C, p, m, v, 1e-3, 0.9, 0.999, 0.0, variance_frozen=True)
    sc = np.repeat(scale, C)[:n].astype(np.float64)
    want = p0 - 1e-3 * np.where(x >= 0, sc, -sc) / np.sqrt(np.float64(np.float32(4e-6)))
    assert np.max(np.abs(p - want)) <= 2e-7 * np.max(np.abs(want))
    assert np.array_equal(np.abs(m), np.repeat(scale, C)[:n])


def test_momentum_compress_special_cases(oracle):
    rng = np.random.default_rng(4)
    n, C = 5 * 256 + 100, 512
    g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    m = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    r0 = (rng.standard_normal(n) * 1e-4).astype(np.float32)
    # beta1 = 0 compresses g, beta1 = 1 compresses m
    for beta, src in ((0.0, g), (1.0, m)):
        ra, rb = r0.copy(), r0.copy()
        ba, sa = oracle.momentum_sign_compress_ef(g, m, beta, ra, C)
        bb, sb = oracle.sign_compress_ef(src, rb, C)
        assert np.array_equal(ba, bb) and np.array_equal(sa, sb) and np.array_equal(ra, rb)
    g0, m0 = g.copy(), m.copy()
    # general beta: error-feedback identity  decode + residual' == (beta*m + (1-beta)*g) + residual  (to rounding),
    # and the scale is the chunk mean of |u + residual|
    ra = r0.copy()
    bits, scale = oracle.momentum_sign_compress_ef(g, m, 0.9, ra, C)
    u = np.float64(np.float32(0.9)) * m + (1 - np.float64(np.float32(0.9))) * g + r0
    dec = oracle.decompress_sign(bits, scale, n, C)
    assert np.max(np.abs(dec.astype(np.float64) + ra - u)) <= 3e-7 * np.max(np.abs(u))
    for c in range((n + C - 1) // C):
        seg = u[c * C:(c + 1) * C]
        assert abs(scale[c] - np.mean(np.abs(seg))) <= 1e-6 * np.mean(np.abs(seg))
    assert np.array_equal(g, g0) and np.array_equal(m, m0)   # inputs are not modified


def test_one_bit_adam_compression_stage_tracks_uncompressed_momentum(oracle):
    """k workers, 40 steps of the compression stage: with both error states, the time-sum of the decoded momenta
    stays within a bounded distance of the time-sum of the exact average momenta (error compensation telescopes)."""
    rng = np.random.default_rng(5)
    k, n, C, T, beta = 4, 2 * 256, 256, 40, 0.9
    m = np.zeros(n, np.float32)
    delta = [np.zeros(n, np.float32) for _ in range(k)]
    eps = np.zeros(n, np.float32)
    acc_dec, acc_exact = np.zeros(n), np.zeros(n)
    mean_abs = 0.0
    for t in range(T):
        gs = [(rng.standard_normal(n) * 1e-2 + 5e-3).astype(np.float32) for _ in range(k)]
        packed = [oracle.momentum_sign_compress_ef(gs[j], m, beta, delta[j], C) for j in range(k)]
        exact = np.mean([np.float64(np.float32(beta)) * m + (1 - np.float64(np.float32(beta))) * gs[j] for j in range(k)], 0)
        bits_out, scale_out, _ = oracle.drr_sign([b for b, _ in packed], [s for _, s in packed], eps, n, C)
        dec = oracle.decompress_sign(bits_out, scale_out, n, C)
        acc_dec += dec
        acc_exact += exact
        mean_abs = max(mean_abs, float(np.mean(np.abs(exact))))
        m = dec
    resid = np.abs(acc_dec - acc_exact)
    # what is missing from the decoded sum sits in the error states; the error states stay bounded
    # (a few times the typical magnitude), while both sums grow linearly with T
    assert np.max(resid) <= 12 * mean_abs
    assert np.max(np.abs(acc_exact)) >= 0.5 * T * 5e-3 * (1 - beta)


def test_adam_after_topk_keep_everything_is_torch_adam(oracle):
    """keep = C makes the top-K round lossless, so three steps must follow torch.optim.Adam's state and the fp64
    parameter formula exactly as the dense step does."""
    rng = np.random.default_rng(20)
    n, C = 3 * 256 + 100, 256
    p0 = rng.standard_normal(n).astype(np.float32)
    p, m, v = p0.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32)
    tp = torch.nn.Parameter(torch.from_numpy(p0.copy()).double())
    opt = torch.optim.Adam([tp], lr=1e-3, betas=(float(np.float32(0.9)), float(np.float32(0.999))), eps=1e-8)
    p64 = p0.astype(np.float64)
    for it in range(3):
        g = (rng.standard_normal(n) * 1e-2).astype(np.float32)
        idx, val = oracle.compress_topk(g, None, C, C)
        oracle.decompress_adam_step_topk(idx, val, n, C, C, p, m, v, 1e-3, 0.9, 0.999, 1e-8)
        tp.grad = torch.from_numpy(g).double()
        opt.step()
        st = opt.state[tp]
        em, ev = st["exp_avg"].numpy(), st["exp_avg_sq"].numpy()
        assert np.max(np.abs(m - em)) <= 4e-7 * np.max(np.abs(em))
        assert np.max(np.abs(v - ev)) <= 4e-7 * np.max(np.abs(ev))
        p64 = p64 - 1e-3 * em / (np.sqrt(ev) + 1e-8)
        assert np.max(np.abs(p - p64)) <= 1e-6 * (it + 1)


def test_adam_after_topk_where_nothing_is_kept(oracle):
    """Dropped positions see a zero gradient: m decays by beta1 and v by beta2 exactly (one multiplication each), the
    parameter moves by the decayed momentum; kept positions follow the dense recurrences; with the variance frozen the
    momentum is REPLACED by the decoded tensor (0 where nothing was kept) and v stays."""
    rng = np.random.default_rng(21)
    n, C, keep = 4 * 256, 256, 8
    g = (rng.standard_normal(n) * 1e-2).astype(np.float32)
    idx, val = oracle.compress_topk(g, None, C, keep)
    kept = np.zeros(n, bool)
    for c in range(n // C):
        kept[c * C + idx[c * keep:(c + 1) * keep].astype(np.int64)] = True
    assert kept.sum() == keep * (n // C)
    p0 = rng.standard_normal(n).astype(np.float32)
    m0 = (rng.standard_normal(n) * 1e-2).astype(np.float32)
    v0 = (np.abs(rng.standard_normal(n)) * 1e-4 + 1e-6).astype(np.float32)
    b1, b2, lr, eps = np.float32(0.9), np.float32(0.999), np.float32(1e-2), np.float32(1e-8)
    p, m, v = p0.copy(), m0.copy(), v0.copy()
    oracle.decompress_adam_step_topk(idx, val, n, C, keep, p, m, v, float(lr), float(b1), float(b2), float(eps))
    d = ~kept
    assert np.array_equal(m[d], b1 * m0[d]) and np.array_equal(v[d], b2 * v0[d])
    want = p0[d].astype(np.float64) - float(lr) * m[d].astype(np.float64) / (np.sqrt(v[d].astype(np.float64)) + float(eps))
    assert np.max(np.abs(p[d] - want)) <= 1e-6
    mk = float(b1) * m0[kept].astype(np.float64) + (1 - float(b1)) * g[kept].astype(np.float64)
    vk = float(b2) * v0[kept].astype(np.float64) + (1 - float(b2)) * g[kept].astype(np.float64) ** 2
    assert np.max(np.abs(m[kept] - mk)) <= 1e-7 and np.max(np.abs(v[kept] - vk)) <= 1e-9
    # frozen variance
    p, m, v = p0.copy(), m0.copy(), v0.copy()
    oracle.decompress_adam_step_topk(idx, val, n, C, keep, p, m, v, float(lr), float(b1), float(b2), float(eps), 0.0, True)
    assert np.array_equal(v, v0)
    assert not m[d].any() and np.array_equal(m[kept], g[kept])
    assert np.array_equal(p[d], p0[d])                      # a zero momentum moves nothing
    want = p0[kept].astype(np.float64) - float(lr) * g[kept].astype(np.float64) / (np.sqrt(v0[kept].astype(np.float64)) + float(eps))
    assert np.max(np.abs(p[kept] - want)) <= 1e-6


def test_adam_after_topk_equals_the_dense_step_on_the_decoded_tensor(oracle):
    """The composition itself: the same bits as the pinned dense step fed with a lossless MinMax coding of the decoded
    top-K tensor (values on a 255-step grid so that the MinMax round trip is exact)."""
    rng = np.random.default_rng(22)
    n, C, keep = 2 * 256, 256, 16
    g = grid_values(rng, n, C)
    idx, val = oracle.compress_topk(g, None, C, keep)
    dec = oracle.decompress_topk(idx, val, n, C, keep)
    dec[0::C], dec[1::C] = np.float32(-128 * 2.0 ** -10), np.float32(127 * 2.0 ** -10)   # span the grid in every chunk
    idx2, val2 = oracle.compress_topk(dec, None, C, C)                                   # lossless top-K of it
    codes, mm = lossless_codes(oracle, dec, C)
    for frozen in (False, True):
        for wd in (0.0, 0.01):
            a = [rng.standard_normal(n).astype(np.float32), (rng.standard_normal(n) * 1e-2).astype(np.float32),
                 (np.abs(rng.standard_normal(n)) * 1e-4).astype(np.float32)]
            b = [t.copy() for t in a]
            oracle.decompress_adam_step_topk(idx2, val2, n, C, C, a[0], a[1], a[2], 1e-3, 0.9, 0.999, 1e-8, wd, frozen)
            oracle.decompress_adam_step(0, codes, mm, n, C, b[0], b[1], b[2], 1e-3, 0.9, 0.999, 1e-8, wd, frozen)
            for x, y in zip(a, b):
                assert np.array_equal(x.view(np.uint32), y.view(np.uint32))
