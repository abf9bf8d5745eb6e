"""GPU parity: every entry point of libbagua_hip.so against the CPU oracle on the same seeded inputs.

Bar: bit-exact codes, sign words, (min,max), scales; fp32 outputs (residuals, averages, replicas) within
1e-6 relative / 1e-7 absolute -- and the count of fp32 words that are not bit-identical is asserted to be 0,
since both sides are specified with one rounding per operation in a fixed order.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

SIZES = [1, 3, 255, 256, 257, 4095, 4096, 4097, 2 * 4096 + 7, 70001]


@pytest.fixture(scope="module")
def bg():
    import paper_2107_01499_amd as b
    assert torch.cuda.is_available()
    return b


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.cpu().numpy()


def vals(n, seed, dist="normal"):
    r = np.random.default_rng(seed)
    if dist == "normal":
        return (r.standard_normal(n) * 1e-3).astype(np.float32)
    if dist == "t3":
        return (r.standard_t(3, n) * 1e-3).astype(np.float32)
    if dist == "laplace":
        return r.laplace(0, 1e-3, n).astype(np.float32)
    raise ValueError(dist)


def assert_fp32_close_and_exact(got, want, what):
    got, want = np.asarray(got), np.asarray(want)
    assert got.shape == want.shape, what
    err = np.abs(got.astype(np.float64) - want.astype(np.float64))
    assert np.all(err <= 1e-6 * np.abs(want.astype(np.float64)) + 1e-7), what
    nbad = int(np.count_nonzero(got.view(np.uint32) != want.view(np.uint32)))
    assert nbad == 0, "%s: %d fp32 words not bit-identical" % (what, nbad)


# ----------------------------------------------------------------------------- MinMax-u8 worker side
def gpu_compress(bg, x, res, C):
    n = x.size
    xg = dev(x)
    rg = None if res is None else dev(res)
    codes = torch.full((n,), 0xAB, dtype=torch.uint8, device="cuda")
    mm = torch.full((2 * bg.num_chunks(n, C),), float("nan"), device="cuda")
    bg.bagua_compress_minmax_u8(xg, rg, C, codes, mm)
    torch.cuda.synchronize()
    assert np.array_equal(host(xg), x)            # input untouched
    return host(codes), host(mm), None if rg is None else host(rg)


@pytest.mark.parametrize("n", SIZES)
@pytest.mark.parametrize("C", [256, 768, 2048, 4096, 8192, 16384])
@pytest.mark.parametrize("ef", [False, True])
def test_compress_minmax(bg, oracle, n, C, ef):
    print("compress_minmax n=%d C=%d ef=%s" % (n, C, ef), flush=True)
    x = vals(n, n + C, "t3" if (n % 2) else "normal")
    res = vals(n, n + C + 1) * np.float32(0.1) if ef else None
    res_o = None if res is None else res.copy()
    co, mo = oracle.compress_minmax_u8(x, res_o, C)
    cg, mg, rg = gpu_compress(bg, x, res, C)
    assert np.array_equal(cg, co)
    assert np.array_equal(mg.view(np.uint32), mo.view(np.uint32))
    if ef:
        assert_fp32_close_and_exact(rg, res_o, "residual")


def test_compress_edge_cases(bg, oracle):
    C = 256
    x = np.zeros(6 * C, np.float32)
    x[0:C] = 0.375                                  # flat chunk
    x[C:2 * C] = np.float32(-0.0); x[C + 3] = 0.0   # signed zeros
    x[2 * C + 5] = np.float32(1e-40)                # denormal range: 255/range overflows
    x[3 * C:4 * C] = np.linspace(-1e38, 1e38, C).astype(np.float32)   # huge range
    x[4 * C:5 * C] = np.arange(C, dtype=np.float32); x[4 * C + 2:4 * C + 12] = np.arange(10, dtype=np.float32) + 0.5
    x[4 * C + 1] = 255.0                            # ties -> even
    x[5 * C:] = np.float32(1e-42) * np.arange(C, dtype=np.float32)   # all denormal
    for ef in (False, True):
        res = np.zeros_like(x) if ef else None
        res_o = None if res is None else res.copy()
        co, mo = oracle.compress_minmax_u8(x, res_o, C)
        cg, mg, rg = gpu_compress(bg, x, res, C)
        assert np.array_equal(cg, co)
        assert np.array_equal(mg.view(np.uint32), mo.view(np.uint32))
        if ef:
            assert_fp32_close_and_exact(rg, res_o, "residual")


def test_decompress_both_codecs(bg, oracle):
    for n, C in [(1, 256), (257, 256), (3 * 4096 + 5, 4096), (70001, 2048)]:
        x = vals(n, n, "t3")
        co, mo = oracle.compress_minmax_u8(x, None, C)
        out = torch.empty(n, device="cuda")
        bg.bagua_decompress(bg.CODEC_MINMAX_U8, dev(co), dev(mo), n, C, out)
        assert_fp32_close_and_exact(host(out), oracle.decompress_minmax_u8(co, mo, C), "decompress minmax")
        bo, so = oracle.sign_compress_ef(x, None, C)
        bg.bagua_decompress(bg.CODEC_SIGN1, dev(bo.view(np.int32)), dev(so), n, C, out)
        assert_fp32_close_and_exact(host(out), oracle.decompress_sign(bo, so, n, C), "decompress sign")


# ----------------------------------------------------------------------------- MinMax-u8 server side
@pytest.mark.parametrize("k", [1, 2, 3, 4, 8, 16, 32])
@pytest.mark.parametrize("n,C", [(1, 256), (257, 256), (3 * 4096 + 77, 4096), (5 * 8192 + 1, 8192), (40000, 16384), (9000, 768)])
@pytest.mark.parametrize("ef,want_out", [(True, True), (False, False), (True, False), (False, True)])
def test_drr_minmax(bg, oracle, k, n, C, ef, want_out):
    print("drr_minmax k=%d n=%d C=%d ef=%s out=%s" % (k, n, C, ef, want_out), flush=True)
    codes_in, mm_in = [], []
    for j in range(k):
        c, m = oracle.compress_minmax_u8(vals(n, 1000 * k + j, "t3" if j % 2 else "normal"), None, C)
        codes_in.append(c); mm_in.append(m)
    eps = vals(n, 5) * np.float32(0.05) if ef else None
    eps_o = None if eps is None else eps.copy()
    co, mo, oo = oracle.drr_minmax_u8(codes_in, mm_in, eps_o, C, want_fp32=want_out)
    eg = None if eps is None else dev(eps)
    cg = torch.full((n,), 0xAB, dtype=torch.uint8, device="cuda")
    mg = torch.full((2 * bg.num_chunks(n, C),), float("nan"), device="cuda")
    og = torch.full((n,), float("nan"), device="cuda") if want_out else None
    bg.bagua_decompress_reduce_recompress(bg.CODEC_MINMAX_U8, [dev(c) for c in codes_in], [dev(m) for m in mm_in],
                                          eg, n, C, cg, mg, og)
    torch.cuda.synchronize()
    assert np.array_equal(host(cg), co)
    assert np.array_equal(host(mg).view(np.uint32), mo.view(np.uint32))
    if ef:
        assert_fp32_close_and_exact(host(eg), eps_o, "server residual")
    if want_out:
        assert_fp32_close_and_exact(host(og), oo, "out_fp32")


def test_c_lp_s_three_iterations_state_carried(bg, oracle):
    """Configuration-1-like loop: k workers compress with delta, the server averages with epsilon, three
    iterations with fresh gradients; all state lives on the GPU between iterations."""
    n, C, k = 5 * 4096 + 300, 4096, 4
    nc = bg.num_chunks(n, C)
    d_o = [np.zeros(n, np.float32) for _ in range(k)]
    e_o = np.zeros(n, np.float32)
    d_g = [torch.zeros(n, device="cuda") for _ in range(k)]
    e_g = torch.zeros(n, device="cuda")
    for it in range(3):
        cs_o, ms_o, cs_g, ms_g = [], [], [], []
        for j in range(k):
            x = vals(n, 100 * it + j)
            c, m = oracle.compress_minmax_u8(x, d_o[j], C)
            cs_o.append(c); ms_o.append(m)
            cg = torch.empty(n, dtype=torch.uint8, device="cuda"); mg = torch.empty(2 * nc, device="cuda")
            bg.bagua_compress_minmax_u8(dev(x), d_g[j], C, cg, mg)
            cs_g.append(cg); ms_g.append(mg)
        co, mo, oo = oracle.drr_minmax_u8(cs_o, ms_o, e_o, C)
        cg = torch.empty(n, dtype=torch.uint8, device="cuda"); mg = torch.empty(2 * nc, device="cuda")
        og = torch.empty(n, device="cuda")
        bg.bagua_decompress_reduce_recompress(bg.CODEC_MINMAX_U8, cs_g, ms_g, e_g, n, C, cg, mg, og)
        assert np.array_equal(host(cg), co) and np.array_equal(host(mg).view(np.uint32), mo.view(np.uint32))
        assert_fp32_close_and_exact(host(og), oo, "out iteration %d" % it)
        assert_fp32_close_and_exact(host(e_g), e_o, "epsilon iteration %d" % it)
        for j in range(k):
            assert_fp32_close_and_exact(host(d_g[j]), d_o[j], "delta iteration %d" % it)


# ----------------------------------------------------------------------------- sign codec
@pytest.mark.parametrize("n", SIZES)
@pytest.mark.parametrize("C", [256, 768, 2048, 4096, 16384])
@pytest.mark.parametrize("ef", [False, True])
def test_sign_compress(bg, oracle, n, C, ef):
    print("sign_compress n=%d C=%d ef=%s" % (n, C, ef), flush=True)
    x = vals(n, 3 * n + C, "laplace")
    x[::97] = 0.0
    x[1::97] = -0.0
    res = vals(n, n + 1, "laplace") * np.float32(0.1) if ef else None
    res_o = None if res is None else res.copy()
    bo, so = oracle.sign_compress_ef(x, res_o, C)
    rg = None if res is None else dev(res)
    bits = torch.full(((n + 31) // 32,), -1, dtype=torch.int32, device="cuda")
    scale = torch.full((bg.num_chunks(n, C),), float("nan"), device="cuda")
    bg.bagua_sign_compress_ef(dev(x), rg, C, bits, scale)
    torch.cuda.synchronize()
    assert np.array_equal(host(bits).view(np.uint32), bo)
    assert np.array_equal(host(scale).view(np.uint32), so.view(np.uint32))
    if ef:
        assert_fp32_close_and_exact(host(rg), res_o, "sign residual")


@pytest.mark.parametrize("k", [1, 2, 3, 8, 32])
@pytest.mark.parametrize("n,C", [(1, 256), (257, 256), (5 * 2048 + 77, 2048), (3 * 4096 + 31, 4096), (40000, 16384), (9000, 768)])
@pytest.mark.parametrize("ef,want_out", [(True, True), (False, False)])
def test_drr_sign(bg, oracle, k, n, C, ef, want_out):
    print("drr_sign k=%d n=%d C=%d ef=%s" % (k, n, C, ef), flush=True)
    bits_in, scale_in = [], []
    for j in range(k):
        b, s = oracle.sign_compress_ef(vals(n, 77 * k + j, "laplace"), None, C)
        bits_in.append(b); scale_in.append(s)
    eps = vals(n, 6, "laplace") * np.float32(0.05) if ef else None
    eps_o = None if eps is None else eps.copy()
    bo, so, oo = oracle.drr_sign(bits_in, scale_in, eps_o, n, C, want_fp32=want_out)
    eg = None if eps is None else dev(eps)
    bg_ = torch.full(((n + 31) // 32,), -1, dtype=torch.int32, device="cuda")
    sg = torch.full((bg.num_chunks(n, C),), float("nan"), device="cuda")
    og = torch.full((n,), float("nan"), device="cuda") if want_out else None
    bg.bagua_decompress_reduce_recompress(bg.CODEC_SIGN1, [dev(b.view(np.int32)) for b in bits_in],
                                          [dev(s) for s in scale_in], eg, n, C, bg_, sg, og)
    torch.cuda.synchronize()
    assert np.array_equal(host(bg_).view(np.uint32), bo)
    assert np.array_equal(host(sg).view(np.uint32), so.view(np.uint32))
    if ef:
        assert_fp32_close_and_exact(host(eg), eps_o, "sign server residual")
    if want_out:
        assert_fp32_close_and_exact(host(og), oo, "sign out_fp32")


# ----------------------------------------------------------------------------- decentralised averaging
def make_replicas(k, n, seed):
    r = np.random.default_rng(seed)
    base = (r.standard_normal(n) * 0.02).astype(np.float32)
    return base, [(base + (r.standard_normal(n) * 1e-3).astype(np.float32)).astype(np.float32) for _ in range(k)]


@pytest.mark.parametrize("k", [1, 2, 3, 8, 16, 17, 32])
@pytest.mark.parametrize("n", [1, 255, 1027, 70001])
def test_ring_avg_fp(bg, oracle, k, n):
    print("ring_fp k=%d n=%d" % (k, n), flush=True)
    _, xs = make_replicas(k, n, k * 7 + n)
    cur_o = xs
    cur_g = [dev(x) for x in xs]
    for rnd in range(3):
        cur_o = oracle.ring_avg_fp(cur_o)
        nxt = [torch.full((n,), float("nan"), device="cuda") for _ in range(k)]
        bg.bagua_decentralized_avg(bg.AVG_FP, cur_g, nxt)
        cur_g = nxt
        for i in range(k):
            assert_fp32_close_and_exact(host(cur_g[i]), cur_o[i], "ring fp round %d peer %d" % (rnd, i))


@pytest.mark.parametrize("k,C", [(1, 256), (2, 4096), (3, 768), (8, 4096), (8, 256), (5, 2048), (9, 4096), (4, 8192), (16, 16384)])
@pytest.mark.parametrize("n", [1, 257, 3 * 4096 + 77, 70001])
def test_ring_avg_lp(bg, oracle, k, C, n):
    print("ring_lp k=%d C=%d n=%d" % (k, C, n), flush=True)
    base, xs = make_replicas(k, n, k * 13 + n + C)
    nc = bg.num_chunks(n, C)
    hat_o = [base.copy() for _ in range(k)]
    hat_g = [dev(base) for _ in range(k)]
    cur_o = xs
    cur_g = [dev(x) for x in xs]
    for rnd in range(3):
        cur_o, codes_o, mm_o = oracle.ring_avg_lp(cur_o, hat_o, C)
        nxt = [torch.full((n,), float("nan"), device="cuda") for _ in range(k)]
        codes = [torch.full((n,), 0xAB, dtype=torch.uint8, device="cuda") for _ in range(k)]
        mm = [torch.full((2 * nc,), float("nan"), device="cuda") for _ in range(k)]
        bg.bagua_decentralized_avg(bg.AVG_LP_MINMAX_U8, cur_g, nxt, hat_g, codes, mm, C)
        cur_g = nxt
        for i in range(k):
            assert np.array_equal(host(codes[i]), codes_o[i]), "codes round %d peer %d" % (rnd, i)
            assert np.array_equal(host(mm[i]).view(np.uint32), mm_o[i].view(np.uint32))
            assert_fp32_close_and_exact(host(hat_g[i]), hat_o[i], "xhat round %d peer %d" % (rnd, i))
            assert_fp32_close_and_exact(host(cur_g[i]), cur_o[i], "x round %d peer %d" % (rnd, i))


# ----------------------------------------------------------------------------- flatten
def test_flatten_gaps_misaligned_and_tiny(bg, oracle):
    r = np.random.default_rng(0)
    sizes = [1, 7, 64, 1000, 3, 4096, 0, 129, 30522, 5, 5, 5, 8191, 2]
    srcs = [r.standard_normal(s).astype(np.float32) for s in sizes]
    offs, pos = [], 0
    for i, s in enumerate(sizes):
        pos += (i % 3)
        offs.append(pos)
        pos += s
    total = pos + 50
    want = oracle.bucket_flatten(srcs, offs, total)
    # sources at deliberately odd (4-byte aligned only) device addresses
    arena = torch.zeros(sum(sizes) + 4 * len(sizes) + 8, device="cuda")
    gs, p = [], 1
    for s in srcs:
        t = arena[p:p + s.size]
        t.copy_(torch.from_numpy(s))
        gs.append(t)
        p += s.size + 1
    bucket = torch.full((total,), float("nan"), device="cuda")
    ws = torch.empty(bg.bagua_flatten_workspace_bytes(len(srcs), total), dtype=torch.uint8, device="cuda")
    bg.bagua_bucket_flatten(gs, offs, bucket, ws)
    torch.cuda.synchronize()
    assert host(bucket).tobytes() == want.tobytes()
    # planned run again into a fresh bucket
    bucket2 = torch.full((total,), float("nan"), device="cuda")
    bg.bagua_bucket_flatten_run(ws, len(srcs), bucket2)
    assert host(bucket2).tobytes() == want.tobytes()


@pytest.mark.parametrize("src_shift", [0, 1, 2, 3])
@pytest.mark.parametrize("dst_shift", [0, 1, 2, 3])
def test_flatten_every_source_and_destination_alignment(bg, oracle, src_shift, dst_shift):
    """Whole tiles inside one tensor whose source is src_shift elements past a 16-byte boundary and whose bucket
    offset is dst_shift elements past one: the realigning 128-bit path and the element path, also fused into the
    compression."""
    r = np.random.default_rng(10 * src_shift + dst_shift)
    sizes = [5000, 1024 * 3 + 5, 9000]
    srcs = [(r.standard_normal(s) * 1e-3).astype(np.float32) for s in sizes]
    offs, pos = [], dst_shift
    for s in sizes:
        offs.append(pos)
        pos += s + 4 - (s % 4) + 0          # next tensor keeps the same destination shift
    total = pos + 7
    arena = torch.zeros(sum(sizes) + 64, device="cuda")
    gs, p_ = [], src_shift
    for s in srcs:
        t = arena[p_:p_ + s.size]
        t.copy_(torch.from_numpy(s))
        gs.append(t)
        p_ += (s.size + 3) // 4 * 4 + 4
        p_ = p_ - (p_ % 4) + src_shift
    want = oracle.bucket_flatten(srcs, offs, total)
    bucket = torch.full((total,), float("nan"), device="cuda")
    ws = torch.empty(bg.bagua_flatten_workspace_bytes(len(gs), total), dtype=torch.uint8, device="cuda")
    bg.bagua_bucket_flatten(gs, offs, bucket, ws)
    assert host(bucket).tobytes() == want.tobytes()
    C = 1024
    codes = torch.empty(total, dtype=torch.uint8, device="cuda")
    mm = torch.empty(2 * bg.num_chunks(total, C), device="cuda")
    bg.bagua_flatten_compress_minmax_u8(ws, len(gs), None, total, C, codes, mm)
    co, mo = oracle.compress_minmax_u8(want, None, C)
    assert np.array_equal(host(codes), co) and np.array_equal(host(mm), mo)


def test_flatten_empty_table_zero_fills(bg):
    bucket = torch.full((5000,), float("nan"), device="cuda")
    ws = torch.empty(bg.bagua_flatten_workspace_bytes(0, 5000), dtype=torch.uint8, device="cuda")
    bg.bagua_bucket_flatten([], [], bucket, ws)
    assert not host(bucket).view(np.uint32).any()


def test_flatten_resnet50_bucket(bg, oracle):
    from bagua_workloads import resnet50_shapes, pack_buckets
    from bagua_workloads.shapes import numel
    shapes = resnet50_shapes()
    b = pack_buckets(shapes, 8, 4096)[0]
    r = np.random.default_rng(2)
    srcs = [r.standard_normal(numel(shapes[t][1])).astype(np.float32) for t in b.tensors]
    want = oracle.bucket_flatten(srcs, b.offsets, b.n_pad)
    gs = [dev(s) for s in srcs]
    bucket = torch.full((b.n_pad,), float("nan"), device="cuda")
    ws = torch.empty(bg.bagua_flatten_workspace_bytes(len(gs), b.n_pad), dtype=torch.uint8, device="cuda")
    bg.bagua_bucket_flatten(gs, b.offsets, bucket, ws)
    assert host(bucket).tobytes() == want.tobytes()


def test_non_default_stream(bg, oracle):
    n, C = 3 * 4096 + 1, 4096
    x = vals(n, 1)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        xg = dev(x)
        codes = torch.empty(n, dtype=torch.uint8, device="cuda")
        mm = torch.empty(2 * bg.num_chunks(n, C), device="cuda")
        bg.bagua_compress_minmax_u8(xg, None, C, codes, mm)
    s.synchronize()
    co, mo = oracle.compress_minmax_u8(x, None, C)
    assert np.array_equal(host(codes), co) and np.array_equal(host(mm), mo)


# ----------------------------------------------------------------------------- flatten fused into compress
@pytest.mark.parametrize("ef", [False, True])
@pytest.mark.parametrize("C", [256, 4096, 16384])
@pytest.mark.parametrize("want_bucket", [False, True])
def test_flatten_compress_fused(bg, oracle, ef, C, want_bucket):
    """bagua_flatten_compress_minmax_u8 == flatten then compress (oracle composition): gaps, tiny and empty
    tensors, sources at odd 4-byte addresses, a ragged last chunk."""
    print("flatten_compress C=%d ef=%s bucket=%s" % (C, ef, want_bucket), flush=True)
    r = np.random.default_rng(C + ef)
    sizes = [1, 7, 64, 1000, 3, 4096, 0, 129, 30522, 5, 5, 5, 8191, 2, 70000, 256, 1024]
    srcs = [(r.standard_normal(s) * 1e-3).astype(np.float32) for s in sizes]
    offs, pos = [], 0
    for i, s in enumerate(sizes):
        pos += (i % 3)
        offs.append(pos)
        pos += s
    total = pos + 50
    flat = oracle.bucket_flatten(srcs, offs, total)
    res = (r.standard_normal(total) * 1e-4).astype(np.float32) if ef else None
    res_o = None if res is None else res.copy()
    co, mo = oracle.compress_minmax_u8(flat, res_o, C)
    for aligned in (False, True):
        arena = torch.zeros(sum(sizes) + 8 * len(sizes) + 8, device="cuda")
        gs, p = [], (0 if aligned else 1)
        for s in srcs:
            t = arena[p:p + s.size]
            t.copy_(torch.from_numpy(s))
            gs.append(t)
            p += s.size + (((-s.size) % 4) if aligned else 1)
        ws = torch.empty(bg.bagua_flatten_workspace_bytes(len(gs), total), dtype=torch.uint8, device="cuda")
        bg.bagua_flatten_plan(gs, offs, total, ws)
        rg = None if res is None else dev(res)
        codes = torch.full((total,), 0xAB, dtype=torch.uint8, device="cuda")
        mm = torch.full((2 * bg.num_chunks(total, C),), float("nan"), device="cuda")
        bucket = torch.full((total,), float("nan"), device="cuda") if want_bucket else None
        bg.bagua_flatten_compress_minmax_u8(ws, len(gs), rg, total, C, codes, mm, bucket)
        torch.cuda.synchronize()
        assert np.array_equal(host(codes), co)
        assert np.array_equal(host(mm).view(np.uint32), mo.view(np.uint32))
        if ef:
            assert_fp32_close_and_exact(host(rg), res_o, "fused residual")
        if want_bucket:
            assert host(bucket).tobytes() == flat.tobytes()


def test_flatten_compress_fused_resnet50(bg, oracle):
    from bagua_workloads import resnet50_shapes, pack_buckets
    from bagua_workloads.shapes import numel
    shapes = resnet50_shapes()
    C = 4096
    b = pack_buckets(shapes, 8, C)[0]
    r = np.random.default_rng(2)
    srcs = [(r.standard_normal(numel(shapes[t][1])) * 1e-3).astype(np.float32) for t in b.tensors]
    flat = oracle.bucket_flatten(srcs, b.offsets, b.n_pad)
    res_o = np.zeros(b.n_pad, np.float32)
    co, mo = oracle.compress_minmax_u8(flat, res_o, C)
    gs = [dev(s) for s in srcs]
    ws = torch.empty(bg.bagua_flatten_workspace_bytes(len(gs), b.n_pad), dtype=torch.uint8, device="cuda")
    bg.bagua_flatten_plan(gs, b.offsets, b.n_pad, ws)
    rg = torch.zeros(b.n_pad, device="cuda")
    codes = torch.empty(b.n_pad, dtype=torch.uint8, device="cuda")
    mm = torch.empty(2 * b.n_pad // C, device="cuda")
    bg.bagua_flatten_compress_minmax_u8(ws, len(gs), rg, b.n_pad, C, codes, mm)
    assert np.array_equal(host(codes), co) and np.array_equal(host(mm).view(np.uint32), mo.view(np.uint32))
    assert_fp32_close_and_exact(host(rg), res_o, "fused residual resnet50")


# ----------------------------------------------------------------------------- state round trip, graph replay
def test_error_state_checkpoint_round_trip(bg):
    """The only persistent state of the path are the caller-owned residual buffers: three iterations straight
    equal two iterations + copying the residuals out and back in (as a checkpoint would) + one iteration."""
    n, C, k = 6 * 4096 + 100, 4096, 3
    nc = bg.num_chunks(n, C)
    xs = [[dev(vals(n, 10 * it + j)) for j in range(k)] for it in range(3)]

    def run(iters, delta, eps):
        out = None
        for it in iters:
            codes = [torch.empty(n, dtype=torch.uint8, device="cuda") for _ in range(k)]
            mm = [torch.empty(2 * nc, device="cuda") for _ in range(k)]
            for j in range(k):
                bg.bagua_compress_minmax_u8(xs[it][j], delta[j], C, codes[j], mm[j])
            c2 = torch.empty(n, dtype=torch.uint8, device="cuda"); m2 = torch.empty(2 * nc, device="cuda")
            out = torch.empty(n, device="cuda")
            bg.bagua_decompress_reduce_recompress(bg.CODEC_MINMAX_U8, codes, mm, eps, n, C, c2, m2, out)
        return out

    d1 = [torch.zeros(n, device="cuda") for _ in range(k)]; e1 = torch.zeros(n, device="cuda")
    straight = run(range(3), d1, e1)
    d2 = [torch.zeros(n, device="cuda") for _ in range(k)]; e2 = torch.zeros(n, device="cuda")
    run(range(2), d2, e2)
    saved = [host(d).copy() for d in d2], host(e2).copy()
    d3 = [dev(s) for s in saved[0]]; e3 = dev(saved[1])
    resumed = run([2], d3, e3)
    assert torch.equal(straight.view(torch.int32), resumed.view(torch.int32))
    assert torch.equal(e1.view(torch.int32), e3.view(torch.int32))
    for a, b in zip(d1, d3):
        assert torch.equal(a.view(torch.int32), b.view(torch.int32))


@pytest.mark.parametrize("codec", [0, 1])
def test_server_step_on_partition_slices(bg, oracle, codec):
    """ScatterReduce view: server p processes partition p only.  Running the server step on the k partition slices
    (three chunks each, so the metadata slices are only 8- or 4-byte aligned) equals one pass over the whole bucket."""
    k, C, per = 4, 256, 3
    n = k * per * C
    nc = n // C
    xs = [vals(n, 70 + j) for j in range(k)]
    if codec == 0:
        enc = [oracle.compress_minmax_u8(x, None, C) for x in xs]
        codes_g = [torch.from_numpy(e[0]).cuda() for e in enc]
        want = oracle.drr_minmax_u8([e[0] for e in enc], [e[1] for e in enc], np.zeros(n, np.float32), C)
        cw, mw = 1, 2          # code units and metadata floats per element / per chunk
        codes_out = torch.empty(n, dtype=torch.uint8, device="cuda")
    else:
        enc = [oracle.sign_compress_ef(x, None, C) for x in xs]
        codes_g = [torch.from_numpy(e[0].view(np.int32)).cuda() for e in enc]
        want = oracle.drr_sign([e[0] for e in enc], [e[1] for e in enc], np.zeros(n, np.float32), n, C)
        cw, mw = 1.0 / 32, 1
        codes_out = torch.empty(n // 32, dtype=torch.int32, device="cuda")
    meta_g = [torch.from_numpy(e[1]).cuda() for e in enc]
    meta_out = torch.empty(mw * nc, device="cuda")
    eps, out = torch.zeros(n, device="cuda"), torch.empty(n, device="cuda")
    odd_slices = 0
    for p in range(k):
        lo, hi = p * per * C, (p + 1) * per * C
        cl, ch = int(lo * cw), int(hi * cw)
        ml, mh = mw * p * per, mw * (p + 1) * per
        odd_slices += meta_g[0][ml:mh].data_ptr() % 16 != 0
        bg.bagua_decompress_reduce_recompress(codec, [c[cl:ch] for c in codes_g], [m[ml:mh] for m in meta_g], eps[lo:hi],
                                              hi - lo, C, codes_out[cl:ch], meta_out[ml:mh], out[lo:hi])
    torch.cuda.synchronize()
    assert odd_slices > 0      # the case this test is about did occur
    assert np.array_equal(host(codes_out).view(want[0].dtype), want[0])
    assert np.array_equal(host(meta_out).view(np.uint32), want[1].view(np.uint32))
    assert np.array_equal(host(out).view(np.uint32), want[2].view(np.uint32))


def test_hip_graph_replay_matches_eager(bg, oracle):
    """The entry points allocate nothing and only enqueue kernels, so a step can be captured into a HIP graph.
    Replayed several times with eager work and synchronisation in between, every replay must equal the oracle."""
    n, C, k = 5 * 4096 + 300, 4096, 4
    nc = bg.num_chunks(n, C)
    x = [torch.zeros(n, device="cuda") for _ in range(k)]
    delta = [torch.zeros(n, device="cuda") for _ in range(k)]
    eps = torch.zeros(n, device="cuda")
    codes = [torch.empty(n, dtype=torch.uint8, device="cuda") for _ in range(k)]
    mm = [torch.empty(2 * nc, device="cuda") for _ in range(k)]
    c2 = torch.empty(n, dtype=torch.uint8, device="cuda"); m2 = torch.empty(2 * nc, device="cuda"); out = torch.empty(n, device="cuda")
    bits = torch.empty((n + 31) // 32, dtype=torch.int32, device="cuda"); scale = torch.empty(bg.num_chunks(n, 2048), device="cuda")

    def step():
        for j in range(k):
            bg.bagua_compress_minmax_u8(x[j], delta[j], C, codes[j], mm[j])
        bg.bagua_decompress_reduce_recompress(bg.CODEC_MINMAX_U8, codes, mm, eps, n, C, c2, m2, out)
        bg.bagua_sign_compress_ef(out, None, 2048, bits, scale)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                  # warm-up outside capture
    torch.cuda.current_stream().wait_stream(side)
    for d in delta:
        d.zero_()
    eps.zero_()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for d in delta:
        d.zero_()
    eps.zero_()
    d_o = [np.zeros(n, np.float32) for _ in range(k)]
    e_o = np.zeros(n, np.float32)
    for it in range(3):
        xs = [vals(n, 500 + 10 * it + j) for j in range(k)]
        for j in range(k):
            x[j].copy_(torch.from_numpy(xs[j]))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        enc = [oracle.compress_minmax_u8(xs[j], d_o[j], C) for j in range(k)]
        co, mo, oo = oracle.drr_minmax_u8([e[0] for e in enc], [e[1] for e in enc], e_o, C)
        bo, so = oracle.sign_compress_ef(oo, None, 2048)
        assert np.array_equal(host(c2), co), "replay %d" % it
        assert np.array_equal(host(out).view(np.uint32), oo.view(np.uint32)), "replay %d" % it
        assert np.array_equal(host(eps).view(np.uint32), e_o.view(np.uint32)), "replay %d" % it
        assert np.array_equal(host(bits).view(np.uint32), bo) and np.array_equal(host(scale).view(np.uint32), so.view(np.uint32))
        for j in range(k):
            assert np.array_equal(host(delta[j]).view(np.uint32), d_o[j].view(np.uint32))


def test_hip_graph_replay_of_the_widened_rows(bg, oracle):
    """One compression-stage iteration of 1-bit Adam, a top-K round and a low-precision peer round captured in one
    HIP graph; three replays with fresh inputs, each equal to the oracle's chain with the state carried along."""
    n, C, k, keep = 3 * 2048 + 77, 2048, 4, 64
    nc, nw = bg.num_chunks(n, C), (n + 31) // 32
    f = lambda *shape: torch.zeros(*shape, device="cuda")
    g_in = [f(n) for _ in range(k)]
    m_g, v_g, p_g = f(n), f(n), f(n)
    delta, eps = [f(n) for _ in range(k)], f(n)
    bits = [torch.zeros(nw, dtype=torch.int32, device="cuda") for _ in range(k)]
    scale = [f(nc) for _ in range(k)]
    b2, s2 = torch.zeros(nw, dtype=torch.int32, device="cuda"), f(nc)
    tdelta = [f(n) for _ in range(k)]
    tidx = [torch.zeros(nc * keep, dtype=torch.int16, device="cuda") for _ in range(k)]
    tval = [f(nc * keep) for _ in range(k)]
    teps, ti2, tv2, tout = f(n), torch.zeros(nc * keep, dtype=torch.int16, device="cuda"), f(nc * keep), f(n)
    hat = [f(n) for _ in range(k)]
    lp_out = [f(n) for _ in range(k)]
    lp_codes = [torch.zeros(n, dtype=torch.uint8, device="cuda") for _ in range(k)]
    lp_mm = [f(2 * nc) for _ in range(k)]
    peer = [1, 0, 3, 2]

    def step():
        for j in range(k):
            bg.bagua_momentum_sign_compress_ef(g_in[j], m_g, 0.9, delta[j], C, bits[j], scale[j])
        bg.bagua_decompress_reduce_recompress(bg.CODEC_SIGN1, bits, scale, eps, n, C, b2, s2, None)
        bg.bagua_decompress_adam_step(bg.CODEC_SIGN1, b2, s2, n, C, p_g, m_g, v_g, 1e-3, 0.9, 0.999, 1e-8, 0.0, True)
        for j in range(k):
            bg.bagua_compress_topk_ef(g_in[j], tdelta[j], C, keep, tidx[j], tval[j])
        bg.bagua_decompress_reduce_recompress_topk(tidx, tval, keep, teps, n, C, ti2, tv2, tout)
        bg.bagua_decentralized_avg_peers_lp(g_in, lp_out, hat, lp_codes, lp_mm, peer, C)

    state = [m_g, v_g, p_g, eps, teps] + delta + tdelta + hat
    v0, p0 = np.abs(vals(n, 1)).astype(np.float32) * np.float32(1e-3) + np.float32(1e-8), vals(n, 2)

    def reset():
        for t in state:
            t.zero_()
        v_g.copy_(torch.from_numpy(v0)); p_g.copy_(torch.from_numpy(p0))

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    reset()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    reset()
    torch.cuda.synchronize()
    z = lambda: np.zeros(n, np.float32)
    m_o, v_o, p_o, eps_o, teps_o = z(), v0.copy(), p0.copy(), z(), z()
    d_o, td_o, hat_o = [z() for _ in range(k)], [z() for _ in range(k)], [z() for _ in range(k)]
    for it in range(3):
        gs = [vals(n, 900 + 10 * it + j) for j in range(k)]
        for j in range(k):
            g_in[j].copy_(torch.from_numpy(gs[j]))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        enc = [oracle.momentum_sign_compress_ef(gs[j], m_o, 0.9, d_o[j], C) for j in range(k)]
        bo, so, _ = oracle.drr_sign([e[0] for e in enc], [e[1] for e in enc], eps_o, n, C, want_fp32=False)
        oracle.decompress_adam_step(1, bo, so, n, C, p_o, m_o, v_o, 1e-3, 0.9, 0.999, 1e-8, 0.0, True)
        tenc = [oracle.compress_topk(gs[j], td_o[j], C, keep) for j in range(k)]
        io2, vo2, oo = oracle.drr_topk([e[0] for e in tenc], [e[1] for e in tenc], teps_o, n, C, keep)
        want, wc, wm = oracle.peer_avg_lp(gs, hat_o, peer, C)
        tag = "replay %d" % it
        assert np.array_equal(host(b2).view(np.uint32), bo), tag
        for got, ref in ((p_g, p_o), (m_g, m_o), (v_g, v_o), (eps, eps_o), (tout, oo), (teps, teps_o), (tv2, vo2)):
            assert np.array_equal(host(got).view(np.uint32), ref.view(np.uint32)), tag
        assert np.array_equal(host(ti2).view(np.uint16), io2), tag
        for j in range(k):
            assert np.array_equal(host(delta[j]).view(np.uint32), d_o[j].view(np.uint32)), tag
            assert np.array_equal(host(tdelta[j]).view(np.uint32), td_o[j].view(np.uint32)), tag
            assert np.array_equal(host(lp_out[j]).view(np.uint32), want[j].view(np.uint32)), tag
            assert np.array_equal(host(hat[j]).view(np.uint32), hat_o[j].view(np.uint32)), tag
            assert np.array_equal(host(lp_codes[j]), wc[j]), tag


def test_flatten_thousands_of_tiny_tensors(bg, oracle):
    """Many tensors of 0-5 elements with random gaps: every tile holds hundreds of tensors, so the per-lane
    binary search and the element-wise walk of both the flatten kernel and the fused gather are exercised."""
    r = np.random.default_rng(11)
    sizes = r.integers(0, 6, 3000).tolist() + [5000] + r.integers(0, 6, 500).tolist()
    srcs = [r.standard_normal(s).astype(np.float32) for s in sizes]
    offs, pos = [], 0
    for s in sizes:
        pos += int(r.integers(0, 3))
        offs.append(pos)
        pos += s
    total = pos + 7
    flat = oracle.bucket_flatten(srcs, offs, total)
    arena = torch.zeros(sum(sizes) + len(sizes) + 8, device="cuda")
    gs, p = [], 3
    for s in srcs:
        t = arena[p:p + s.size]
        if s.size:
            t.copy_(torch.from_numpy(s))
        gs.append(t)
        p += s.size
    ws = torch.empty(bg.bagua_flatten_workspace_bytes(len(gs), total), dtype=torch.uint8, device="cuda")
    bucket = torch.full((total,), float("nan"), device="cuda")
    bg.bagua_bucket_flatten(gs, offs, bucket, ws)
    assert host(bucket).tobytes() == flat.tobytes()
    C = 256
    res_o = (r.standard_normal(total) * 0.1).astype(np.float32)
    rg = dev(res_o)
    co, mo = oracle.compress_minmax_u8(flat, res_o, C)
    codes = torch.empty(total, dtype=torch.uint8, device="cuda"); mm = torch.empty(2 * bg.num_chunks(total, C), device="cuda")
    b2 = torch.full((total,), float("nan"), device="cuda")
    bg.bagua_flatten_compress_minmax_u8(ws, len(gs), rg, total, C, codes, mm, b2)
    assert np.array_equal(host(codes), co) and np.array_equal(host(mm).view(np.uint32), mo.view(np.uint32))
    assert_fp32_close_and_exact(host(rg), res_o, "residual")
    assert host(b2).tobytes() == flat.tobytes()


@pytest.mark.parametrize("aligned", [False, True])
def test_unflatten_inverts_flatten(bg, oracle, aligned):
    """bagua_bucket_unflatten_run scatters the bucket back into the planned tensors: equal to the oracle's inverse,
    gaps of the bucket ignored, memory outside the tensors untouched."""
    r = np.random.default_rng(21 + aligned)
    sizes = [1, 7, 64, 1000, 3, 4096, 0, 129, 30522, 5, 5, 5, 8191, 2, 70000] + r.integers(0, 6, 400).tolist()
    offs, pos = [], 0
    for i, s in enumerate(sizes):
        pos += (i % 3)
        offs.append(pos)
        pos += s
    total = pos + 50
    bucket = r.standard_normal(total).astype(np.float32)
    want = [np.empty(s, np.float32) for s in sizes]
    oracle.bucket_unflatten(bucket, want, offs)
    arena = torch.full((sum(sizes) + 8 * len(sizes) + 8,), 777.0, device="cuda")
    gs, p = [], (0 if aligned else 1)
    for s in sizes:
        gs.append(arena[p:p + s])
        p += s + (((-s) % 4) if aligned else 1)
    ws = torch.empty(bg.bagua_flatten_workspace_bytes(len(gs), total), dtype=torch.uint8, device="cuda")
    bg.bagua_flatten_plan(gs, offs, total, ws)
    bg.bagua_bucket_unflatten_run(ws, len(gs), dev(bucket))
    torch.cuda.synchronize()
    covered = 0
    for t, w in zip(gs, want):
        assert host(t).tobytes() == w.tobytes()
        covered += w.size
    assert int((arena != 777.0).sum().item()) <= covered          # nothing outside the tensors was written
    assert int((arena == 777.0).sum().item()) >= arena.numel() - covered


def test_binding_refuses_undersized_buffers(bg):
    """The C entry points see only pointers; the binding refuses tensors smaller than what the call reads or writes."""
    n, C = 3 * 4096 + 5, 4096
    x = torch.zeros(n, device="cuda")
    ok_codes, ok_mm = torch.empty(n, dtype=torch.uint8, device="cuda"), torch.empty(2 * 4, device="cuda")
    bg.bagua_compress_minmax_u8(x, None, C, ok_codes, ok_mm)
    with pytest.raises(ValueError):
        bg.bagua_compress_minmax_u8(x, None, C, ok_codes[:-1].clone(), ok_mm)
    with pytest.raises(ValueError):
        bg.bagua_compress_minmax_u8(x, None, C, ok_codes, ok_mm[:-1].clone())
    with pytest.raises(ValueError):
        bg.bagua_compress_minmax_u8(x, torch.zeros(n - 1, device="cuda"), C, ok_codes, ok_mm)
    with pytest.raises(ValueError):
        bg.bagua_sign_compress_ef(x, None, C, torch.empty((n + 31) // 32 - 1, dtype=torch.int32, device="cuda"),
                                  torch.empty(4, device="cuda"))
    with pytest.raises(ValueError):
        bg.bagua_decompress(bg.CODEC_MINMAX_U8, ok_codes, ok_mm, n, C, torch.empty(n - 1, device="cuda"))
    with pytest.raises(ValueError):
        bg.bagua_decentralized_avg(bg.AVG_FP, [x, x.clone()], [torch.empty(n, device="cuda"), torch.empty(n - 1, device="cuda")])
    with pytest.raises(ValueError):
        bg.bagua_decentralized_avg_peers([x, x.clone()], [torch.empty_like(x), torch.empty_like(x)], [1])
    torch.cuda.synchronize()
