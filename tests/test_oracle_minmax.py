"""Pins of the CPU oracle for the MinMax-u8 codec and the C_LP_S arithmetic (Section 3.2 of the paper).

Nothing here compares the oracle with itself or with the GPU path: every check is an invariant,
a closed form, a special case that reduces to a textbook computation, or an exact (fp64 / integer)
brute force on small inputs.
"""
import numpy as np
import pytest

SIZES = [1, 2, 3, 5, 31, 32, 33, 255, 256, 257, 511, 512 + 7, 4095, 4096, 4097, 2 * 4096 + 7]


def ulp(a):
    return np.spacing(np.abs(a).astype(np.float32)).astype(np.float64)


def chunks(n, C):
    return [(lo, min(n, lo + C)) for lo in range(0, n, C)]


def rand(n, seed, dist="normal"):
    r = np.random.default_rng(seed)
    if dist == "normal":
        return (r.standard_normal(n) * 1e-3).astype(np.float32)
    if dist == "t3":
        return (r.standard_t(3, n) * 1e-3).astype(np.float32)
    raise ValueError(dist)


@pytest.mark.parametrize("n", SIZES)
@pytest.mark.parametrize("C", [256, 4096])
@pytest.mark.parametrize("dist", ["normal", "t3"])
def test_roundtrip_bound_and_nearest_level(oracle, n, C, dist):
    """P1: |v - deq| <= (max-min)/255/2 (the bound the method promises), codes are the nearest of
    256 uniform levels computed exactly in fp64, min -> 0, max -> 255, codes monotone in v."""
    x = rand(n, 100 + n, dist)
    codes, mm = oracle.compress_minmax_u8(x, None, C)
    deq = oracle.decompress_minmax_u8(codes, mm, C)
    for c, (lo, hi) in enumerate(chunks(n, C)):
        v = x[lo:hi].astype(np.float64)
        mn, mx = float(mm[2 * c]), float(mm[2 * c + 1])
        assert mn == v.min() and mx == v.max()
        r = mx - mn
        if r == 0:
            assert (codes[lo:hi] == 0).all() and (deq[lo:hi] == np.float32(mn)).all()
            continue
        t = (v - mn) / r * 255.0                       # exact position on the level grid
        assert np.all(np.abs(codes[lo:hi] - t) <= 0.5 + 1e-3)
        assert codes[lo:hi][np.argmin(v)] == 0 and codes[lo:hi][np.argmax(v)] == 255
        order = np.argsort(v, kind="stable")
        assert np.all(np.diff(codes[lo:hi][order].astype(np.int32)) >= 0)
        bound = r / 255.0 / 2.0 * (1 + 1e-4) + 2 * ulp(np.float32(max(abs(mn), abs(mx))))
        assert np.all(np.abs(v - deq[lo:hi]) <= bound)
        # dequantised values sit on the grid mn + code*step
        grid = mn + codes[lo:hi].astype(np.float64) * (r / 255.0)
        assert np.all(np.abs(deq[lo:hi] - grid) <= 3 * ulp(np.float32(max(abs(mn), abs(mx)))))


@pytest.mark.parametrize("n", SIZES)
def test_error_feedback_identity(oracle, n):
    """P2: residual' + dequantised = x + residual (C_LP_S delta update)."""
    C = 256
    x = rand(n, 7 + n)
    d0 = rand(n, 9 + n) * np.float32(0.1)
    d = d0.copy()
    codes, mm = oracle.compress_minmax_u8(x, d, C)
    deq = oracle.decompress_minmax_u8(codes, mm, C)
    v = x.astype(np.float64) + d0.astype(np.float64)
    v32 = (x + d0).astype(np.float64)                 # the carry-in is one fp32 addition
    assert np.all(np.abs(d.astype(np.float64) + deq - v32) <= 2 * np.maximum(ulp(v32), ulp(deq)))
    assert np.all(np.abs(v32 - v) <= ulp(v32))
    # statistics are taken over x + delta, not over x
    for c, (lo, hi) in enumerate(chunks(n, C)):
        assert mm[2 * c] == (x + d0)[lo:hi].min() and mm[2 * c + 1] == (x + d0)[lo:hi].max()


def test_telescoping_sum_pins_carry_sign(oracle):
    """P3: with v_t = x_t + delta_{t-1}, sum_t deq_t = sum_t x_t + delta_0 - delta_T.  The literal
    reading 'x - delta' of the printed C_LP_S equations would break this."""
    n, C, T = 3000, 256, 40
    d = np.zeros(n, np.float32)
    sx = np.zeros(n, np.float64)
    sq = np.zeros(n, np.float64)
    for t in range(T):
        x = rand(n, 500 + t)
        sx += x
        codes, mm = oracle.compress_minmax_u8(x, d, C)
        sq += oracle.decompress_minmax_u8(codes, mm, C)
    lhs, rhs = sq, sx - d.astype(np.float64)
    assert np.max(np.abs(lhs - rhs)) <= T * 4e-10      # T roundings near 1e-3 magnitudes
    # constant input: the running mean of the decoded stream converges to x at rate step/T
    x = rand(n, 999)
    d[:] = 0
    acc = np.zeros(n, np.float64)
    for t in range(T):
        codes, mm = oracle.compress_minmax_u8(x, d, C)
        acc += oracle.decompress_minmax_u8(codes, mm, C)
    step = np.repeat((mm[1::2] - mm[0::2]).astype(np.float64) / 255.0, C)[:n]
    assert np.all(np.abs(acc / T - x) <= 1.01 * step / T + 1e-9)


def lossless_chunks(rng, nchunks, C, p):
    """Chunks whose values are exactly mn + j*2^p with all of j=0 and j=255 present."""
    out = np.empty(nchunks * C, np.float32)
    js = np.empty(nchunks * C, np.int64)
    for c in range(nchunks):
        j = rng.integers(0, 256, C)
        j[rng.integers(0, C // 2)] = 0
        j[C // 2 + rng.integers(0, C // 2)] = 255
        base = float(rng.integers(-1000, 1000)) * 2.0 ** p
        out[c * C:(c + 1) * C] = (base + j * 2.0 ** p).astype(np.float32)
        js[c * C:(c + 1) * C] = j
    return out, js


@pytest.mark.parametrize("k", [1, 2, 3, 4, 8, 16])
def test_lossless_special_case_is_plain_average(oracle, k):
    """P4: on a grid where MinMax-u8 is lossless, C_LP_S reduces to C_FP_S (times 1/k):
    worker compression returns the input, and the server average is the plain left-to-right
    fp32 sum of the inputs times fl(1/k)."""
    C, nch, p = 256, 5, -10
    rng = np.random.default_rng(k)
    xs, codes_in, mm_in = [], [], []
    for j in range(k):
        x, js = lossless_chunks(rng, nch, C, p)
        res = np.zeros_like(x)
        codes, mm = oracle.compress_minmax_u8(x, res, C)
        assert np.array_equal(codes, js.astype(np.uint8))
        assert np.array_equal(oracle.decompress_minmax_u8(codes, mm, C), x)
        assert not res.any()
        xs.append(x); codes_in.append(codes); mm_in.append(mm)
    s = xs[0].copy()
    for j in range(1, k):
        s = (s + xs[j]).astype(np.float32)
    avg = (s * (np.float32(1.0) / np.float32(k))).astype(np.float32)
    eps = np.zeros(nch * C, np.float32)
    codes, mm, out = oracle.drr_minmax_u8(codes_in, mm_in, eps, C)
    # the recompression of avg is lossy in general; what it compresses must be avg exactly, so the
    # stored statistics are the min/max of avg and decoded + residual returns avg:
    assert np.all(np.abs(out.astype(np.float64) + eps.astype(np.float64) - avg)
                  <= 2 * ulp(np.maximum(np.abs(avg), np.abs(out))))
    for c in range(nch):
        assert mm[2 * c] == avg[c * C:(c + 1) * C].min() and mm[2 * c + 1] == avg[c * C:(c + 1) * C].max()
    if k == 1:
        np.testing.assert_array_equal(out, xs[0])
        np.testing.assert_array_equal(codes, codes_in[0])


def test_sum_order_is_ascending_worker_index(oracle):
    """R2/A6: the k-way sum is taken left to right.  Inputs chosen so that any other order rounds differently."""
    C = 256
    big, small = np.float32(2.0 ** 24), np.float32(1.0)
    # worker values per element: [big, small, small, -big] -> ((big+1)+1)-big = 0 in fp32 left-to-right,
    # while e.g. (small+small)+big-big = 2.
    vals = [big, small, small, -big]
    codes_in, mm_in = [], []
    for v in vals:
        x = np.full(C, v, np.float32)      # flat chunk: decoded exactly
        c, m = oracle.compress_minmax_u8(x, None, C)
        codes_in.append(c); mm_in.append(m)
    codes, mm, out = oracle.drr_minmax_u8(codes_in, mm_in, None, C)
    s = np.float32(np.float32(np.float32(big + small) + small) + (-big))
    assert out[0] == np.float32(s * np.float32(0.25))
    assert out[0] == 0.0


def test_no_error_state_equals_zero_state_on_first_call(oracle):
    """P5: Section 3.2, C_LP_S(x, None, None) = Q(sum_j Q(x_j)); equal to zero-initialised states at t=0."""
    n, C, k = 5 * 256 + 77, 256, 4
    ca, ma, cb, mb = [], [], [], []
    for j in range(k):
        x = rand(n, 40 + j)
        c1, m1 = oracle.compress_minmax_u8(x, None, C)
        z = np.zeros(n, np.float32)
        c2, m2 = oracle.compress_minmax_u8(x, z, C)
        np.testing.assert_array_equal(c1, c2); np.testing.assert_array_equal(m1, m2)
        ca.append(c1); ma.append(m1)
    r1 = oracle.drr_minmax_u8(ca, ma, None, C)
    r2 = oracle.drr_minmax_u8(ca, ma, np.zeros(n, np.float32), C)
    for a, b in zip(r1, r2):
        np.testing.assert_array_equal(a, b)


def test_flat_chunk_and_signed_zero(oracle):
    """A4/A5: max == min gives codes 0, exact decode, zero residual; -0 and +0 are the same minimum."""
    C = 256
    x = np.full(2 * C, 0.375, np.float32)
    x[C:] = np.float32(-0.0)
    x[C + 3] = np.float32(0.0)
    res = np.zeros_like(x)
    codes, mm = oracle.compress_minmax_u8(x, res, C)
    assert not codes.any() and not res.any()
    assert mm.tolist() == [0.375, 0.375, 0.0, 0.0]
    assert not np.signbit(mm).any()
    np.testing.assert_array_equal(oracle.decompress_minmax_u8(codes, mm, C), np.abs(x))
    # without an error state nothing else would turn -0 into +0: the stored statistics still are +0
    codes, mm = oracle.compress_minmax_u8(x, None, C)
    assert not np.signbit(mm).any() and not codes.any()
    y = np.full(C, -0.0, np.float32)
    y[7] = -1.0                                  # max is -0 -> stored as +0
    codes, mm = oracle.compress_minmax_u8(y, None, C)
    assert mm.tolist() == [-1.0, 0.0] and not np.signbit(mm[1])


def test_half_to_even_rounding(oracle):
    """A3: a value exactly between two levels goes to the even code."""
    C = 256
    x = np.zeros(C, np.float32)
    x[1] = 255.0                       # step = 1, inv = 1 exactly
    x[2:12] = np.arange(10, dtype=np.float32) + 0.5   # ties 0.5,1.5,...,9.5
    codes, mm = oracle.compress_minmax_u8(x, None, C)
    assert codes[2:12].tolist() == [0, 2, 2, 4, 4, 6, 6, 8, 8, 10]


def test_partition_equivalence(oracle):
    """P11: the server step on the whole padded bucket equals the k ScatterReduce partitions
    (Section 3.4) processed separately, because chunks never straddle a partition."""
    C, k = 256, 4
    n = k * C * 3
    codes_in, mm_in = [], []
    for j in range(k):
        c, m = oracle.compress_minmax_u8(rand(n, 70 + j, "t3"), None, C)
        codes_in.append(c); mm_in.append(m)
    eps = rand(n, 5) * np.float32(1e-2)
    e_all = eps.copy()
    whole = oracle.drr_minmax_u8(codes_in, mm_in, e_all, C)
    part = n // k
    for p in range(k):
        sl = slice(p * part, (p + 1) * part)
        msl = slice(2 * p * part // C, 2 * (p + 1) * part // C)
        e = eps[sl].copy()
        got = oracle.drr_minmax_u8([np.ascontiguousarray(c[sl]) for c in codes_in],
                                   [np.ascontiguousarray(m[msl]) for m in mm_in], e, C)
        np.testing.assert_array_equal(got[0], whole[0][sl])
        np.testing.assert_array_equal(got[1], whole[1][msl])
        np.testing.assert_array_equal(got[2], whole[2][sl])
        np.testing.assert_array_equal(e, e_all[sl])


def test_server_step_brute_force_fp64(oracle):
    """The server step against an exact-arithmetic model: the average of the decoded worker
    values (fp64) plus epsilon must lie within half a level (+ fp32 slack) of what is decoded
    from the recompressed codes, and epsilon' must be the difference."""
    C, k, n = 256, 8, 3 * 256 + 100
    codes_in, mm_in, deqs = [], [], []
    for j in range(k):
        c, m = oracle.compress_minmax_u8(rand(n, 300 + j), None, C)
        codes_in.append(c); mm_in.append(m)
        mn = np.repeat(m[0::2].astype(np.float64), C)[:n]; mx = np.repeat(m[1::2].astype(np.float64), C)[:n]
        deqs.append(mn + c * (mx - mn) / 255.0)
    eps0 = rand(n, 17) * np.float32(0.01)
    eps = eps0.copy()
    codes, mm, out = oracle.drr_minmax_u8(codes_in, mm_in, eps, C)
    w = np.mean(deqs, axis=0) + eps0
    for c, (lo, hi) in enumerate(chunks(n, C)):
        r = float(mm[2 * c + 1]) - float(mm[2 * c])
        assert abs(mm[2 * c] - w[lo:hi].min()) <= 1e-9 and abs(mm[2 * c + 1] - w[lo:hi].max()) <= 1e-9
        assert np.all(np.abs(out[lo:hi] - w[lo:hi]) <= r / 255 / 2 * (1 + 1e-4) + 2e-9)
        assert np.all(np.abs(eps[lo:hi] - (w[lo:hi] - out[lo:hi])) <= 2e-9)


def test_tiny_range_chunk_does_not_misbehave(oracle):
    """A chunk whose range is so small that 255/range overflows still yields valid codes
    (0 for the minimum, 255 for everything above it) and satisfies the round-trip bound."""
    C = 256
    x = np.zeros(C, np.float32)
    x[5] = np.float32(1e-40)
    codes, mm = oracle.compress_minmax_u8(x, None, C)
    assert codes[5] == 255 and codes.sum() == 255
    deq = oracle.decompress_minmax_u8(codes, mm, C)
    assert np.all(np.abs(deq.astype(np.float64) - x) <= 1e-40)


def test_invalid_arguments(oracle):
    x = np.zeros(256, np.float32)
    for C in (0, 100, 255, 16384 + 256, 300):
        with pytest.raises(ValueError):
            oracle.compress_minmax_u8(x, None, C)
    with pytest.raises(ValueError):
        oracle.compress_minmax_u8(np.zeros(0, np.float32), None, 256)


@pytest.mark.parametrize("n", SIZES + [4096 - 1, 4096 + 1])
@pytest.mark.parametrize("C", [256, 4096])
@pytest.mark.parametrize("ef", [False, True])
def test_independent_numpy_fp32_emulation(oracle, n, C, ef):
    """P8: a second implementation in NumPy float32 (every operation rounds once, written from the definition of
    the codec, not from the oracle's source) agrees bit for bit on codes, statistics and residuals."""
    f = np.float32
    x = rand(n, 4000 + n + C, "t3")
    d0 = (rand(n, 4001 + n) * f(0.1)) if ef else None
    d = None if d0 is None else d0.copy()
    codes, mm = oracle.compress_minmax_u8(x, d, C)
    for c, (lo, hi) in enumerate(chunks(n, C)):
        v = (x[lo:hi] + d0[lo:hi]).astype(f) if ef else x[lo:hi]
        mn, mx = f(v.min() + f(0)), f(v.max() + f(0))
        r = f(mx - mn)
        if r == 0:
            want_codes = np.zeros(hi - lo, np.uint8); step = f(0)
        else:
            inv, step = f(f(255) / r), f(r / f(255))
            t = ((v - mn).astype(f) * inv).astype(f)
            want_codes = np.clip(np.rint(t), 0, 255).astype(np.uint8)
        assert np.array_equal(codes[lo:hi], want_codes)
        assert mm[2 * c].tobytes() == mn.tobytes() and mm[2 * c + 1].tobytes() == mx.tobytes()
        if ef:
            deq = (mn + (want_codes.astype(f) * step).astype(f)).astype(f)
            assert np.array_equal(d[lo:hi], (v - deq).astype(f))
