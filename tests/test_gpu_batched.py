"""Batched entry points (B non-contiguous buckets, one launch) against the per-bucket CPU oracle: each bucket must
come out exactly as the oracle computes it on its own (own chunk grid, own ragged last chunk)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

NS = [1, 4096, 4097, 3 * 4096 + 77, 256, 70001, 8192, 5]          # ragged, tiny and multi-chunk buckets


@pytest.fixture(scope="module")
def bg():
    import paper_2107_01499_amd as b
    assert torch.cuda.is_available()
    return b


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.cpu().numpy()


def same(got, want, what):
    got, want = np.ascontiguousarray(got), np.ascontiguousarray(want)
    assert got.shape == want.shape, what
    assert got.tobytes() == want.tobytes(), what


def vals(n, seed):
    r = np.random.default_rng(seed)
    v = (r.standard_normal(n) * 1e-3).astype(np.float32)
    v[r.integers(0, n, max(1, n // 50))] = 0.0
    return v


def ws_for(bg, B, k=0):
    return torch.empty(bg.bagua_batch_workspace_bytes(B, k), dtype=torch.uint8, device="cuda")


@pytest.mark.parametrize("C", [256, 4096])
@pytest.mark.parametrize("ef", [False, True])
def test_compress_minmax_batched(bg, oracle, C, ef):
    print("compress_minmax_batched C=%d ef=%s" % (C, ef), flush=True)
    B = len(NS)
    xs = [vals(n, 10 + b) for b, n in enumerate(NS)]
    res = [vals(n, 50 + b) * 0.1 for b, n in enumerate(NS)]
    xg = [dev(x) for x in xs]
    rg = [dev(r) for r in res] if ef else None
    codes = [torch.full((n,), 0xAB, dtype=torch.uint8, device="cuda") for n in NS]
    mms = [torch.full((2 * bg.num_chunks(n, C),), float("nan"), device="cuda") for n in NS]
    bg.bagua_compress_minmax_u8_batched(xg, rg, C, codes, mms, ws_for(bg, B))
    torch.cuda.synchronize()
    for b in range(B):
        ro = res[b].copy() if ef else None
        co, mo = oracle.compress_minmax_u8(xs[b], ro, C)
        same(host(codes[b]), co, "codes %d" % b)
        same(host(mms[b]), mo, "minmax %d" % b)
        if ef:
            same(host(rg[b]), ro, "residual %d" % b)


@pytest.mark.parametrize("C", [256, 2048])
@pytest.mark.parametrize("ef", [False, True])
def test_sign_compress_batched(bg, oracle, C, ef):
    print("sign_compress_batched C=%d ef=%s" % (C, ef), flush=True)
    B = len(NS)
    xs = [vals(n, 20 + b) for b, n in enumerate(NS)]
    res = [vals(n, 60 + b) * 0.1 for b, n in enumerate(NS)]
    xg = [dev(x) for x in xs]
    rg = [dev(r) for r in res] if ef else None
    bits = [torch.full(((n + 31) // 32,), -1, dtype=torch.int32, device="cuda") for n in NS]
    scales = [torch.full((bg.num_chunks(n, C),), float("nan"), device="cuda") for n in NS]
    bg.bagua_sign_compress_ef_batched(xg, rg, C, bits, scales, ws_for(bg, B))
    torch.cuda.synchronize()
    for b in range(B):
        ro = res[b].copy() if ef else None
        bo, so = oracle.sign_compress_ef(xs[b], ro, C)
        same(host(bits[b]).view(np.uint32), bo, "bits %d" % b)
        same(host(scales[b]), so, "scale %d" % b)
        if ef:
            same(host(rg[b]), ro, "residual %d" % b)


@pytest.mark.parametrize("k", [1, 3, 8, 17])
@pytest.mark.parametrize("ef,want_out", [(False, False), (True, True), (True, False)])
def test_drr_minmax_batched(bg, oracle, k, ef, want_out):
    print("drr_minmax_batched k=%d ef=%s out=%s" % (k, ef, want_out), flush=True)
    C, B = 4096, len(NS)
    enc = [[oracle.compress_minmax_u8(vals(n, 100 * b + j), None, C) for j in range(k)] for b, n in enumerate(NS)]
    eps = [vals(n, 70 + b) * 0.1 for b, n in enumerate(NS)]
    ci = [[dev(enc[b][j][0]) for j in range(k)] for b in range(B)]
    mi = [[dev(enc[b][j][1]) for j in range(k)] for b in range(B)]
    eg = [dev(e) for e in eps] if ef else None
    co = [torch.full((n,), 0xAB, dtype=torch.uint8, device="cuda") for n in NS]
    mo = [torch.full((2 * bg.num_chunks(n, C),), float("nan"), device="cuda") for n in NS]
    og = [torch.full((n,), float("nan"), device="cuda") for n in NS] if want_out else None
    bg.bagua_decompress_reduce_recompress_batched(bg.CODEC_MINMAX_U8, ci, mi, eg, NS, C, co, mo, og, ws_for(bg, B, k))
    torch.cuda.synchronize()
    for b in range(B):
        eo = eps[b].copy() if ef else None
        c2, m2, o2 = oracle.drr_minmax_u8([e[0] for e in enc[b]], [e[1] for e in enc[b]], eo, C)
        same(host(co[b]), c2, "codes %d" % b)
        same(host(mo[b]), m2, "minmax %d" % b)
        if want_out:
            same(host(og[b]), o2, "out %d" % b)
        if ef:
            same(host(eg[b]), eo, "eps %d" % b)


@pytest.mark.parametrize("k", [1, 8, 9])
@pytest.mark.parametrize("ef,want_out", [(False, True), (True, True)])
def test_drr_sign_batched(bg, oracle, k, ef, want_out):
    print("drr_sign_batched k=%d ef=%s out=%s" % (k, ef, want_out), flush=True)
    C, B = 2048, len(NS)
    enc = [[oracle.sign_compress_ef(vals(n, 100 * b + j), None, C) for j in range(k)] for b, n in enumerate(NS)]
    eps = [vals(n, 80 + b) * 0.1 for b, n in enumerate(NS)]
    ci = [[dev(enc[b][j][0].view(np.int32)) for j in range(k)] for b in range(B)]
    mi = [[dev(enc[b][j][1]) for j in range(k)] for b in range(B)]
    eg = [dev(e) for e in eps] if ef else None
    co = [torch.full(((n + 31) // 32,), -1, dtype=torch.int32, device="cuda") for n in NS]
    mo = [torch.full((bg.num_chunks(n, C),), float("nan"), device="cuda") for n in NS]
    og = [torch.full((n,), float("nan"), device="cuda") for n in NS] if want_out else None
    bg.bagua_decompress_reduce_recompress_batched(bg.CODEC_SIGN1, ci, mi, eg, NS, C, co, mo, og, ws_for(bg, B, k))
    torch.cuda.synchronize()
    for b in range(B):
        eo = eps[b].copy() if ef else None
        b2, s2, o2 = oracle.drr_sign([e[0] for e in enc[b]], [e[1] for e in enc[b]], eo, NS[b], C)
        same(host(co[b]).view(np.uint32), b2, "bits %d" % b)
        same(host(mo[b]), s2, "scale %d" % b)
        if want_out:
            same(host(og[b]), o2, "out %d" % b)
        if ef:
            same(host(eg[b]), eo, "eps %d" % b)


def test_flatten_batched(bg, oracle):
    print("flatten_batched", flush=True)
    r = np.random.default_rng(5)
    layouts = [[1, 7, 64, 1000, 3, 4096, 0, 129], [30522, 5, 5], [2048], [5, 8191, 2, 70000, 256]]
    plans, Ts, buckets, wants = [], [], [], []
    keep = []
    for li, sizes in enumerate(layouts):
        srcs = [r.standard_normal(s).astype(np.float32) for s in sizes]
        offs, pos = [], 0
        for i, s in enumerate(sizes):
            pos += (i + li) % 3
            offs.append(pos)
            pos += s
        total = pos + 13 * li
        wants.append(oracle.bucket_flatten(srcs, offs, total))
        gs = [dev(s) for s in srcs]
        ws = torch.empty(bg.bagua_flatten_workspace_bytes(len(gs), total), dtype=torch.uint8, device="cuda")
        bg.bagua_flatten_plan(gs, offs, total, ws)
        keep.append(gs)
        plans.append(ws)
        Ts.append(len(gs))
        buckets.append(torch.full((total,), float("nan"), device="cuda"))
    bg.bagua_bucket_flatten_batched_run(plans, Ts, buckets, ws_for(bg, len(layouts)))
    torch.cuda.synchronize()
    for b in range(len(layouts)):
        assert host(buckets[b]).tobytes() == wants[b].tobytes(), b
    # the same as a prepared call, twice, after the buckets were overwritten
    call = bg.bagua_bucket_flatten_batched_run(plans, Ts, buckets, ws_for(bg, len(layouts)), prepare=True)
    for rep in range(2):
        for bkt in buckets:
            bkt.fill_(float("nan"))
        call()
        torch.cuda.synchronize()
        for b in range(len(layouts)):
            assert host(buckets[b]).tobytes() == wants[b].tobytes(), (rep, b)


def test_batched_many_buckets_and_reuse(bg, oracle):
    """More buckets than one table-upload launch carries, run twice with the same workspace (second call smaller)."""
    print("batched many buckets", flush=True)
    C = 256
    for B in (300, 7):
        ns = [256 * (1 + (b % 5)) + (b % 3) for b in range(B)]
        xs = [vals(n, b) for b, n in enumerate(ns)]
        xg = [dev(x) for x in xs]
        codes = [torch.empty(n, dtype=torch.uint8, device="cuda") for n in ns]
        mms = [torch.empty(2 * bg.num_chunks(n, C), device="cuda") for n in ns]
        ws = ws_for(bg, 300)
        bg.bagua_compress_minmax_u8_batched(xg, None, C, codes, mms, ws)
        torch.cuda.synchronize()
        for b in range(B):
            co, mo = oracle.compress_minmax_u8(xs[b], None, C)
            same(host(codes[b]), co, "codes %d" % b)
            same(host(mms[b]), mo, "minmax %d" % b)


def test_prepared_calls(bg, oracle):
    """prepare=True marshals once and launches nothing; every later call of the object is the whole batched step on the
    buffers as they are then (error feedback carries over from call to call)."""
    print("prepared batched calls", flush=True)
    C, B, k = 256, len(NS), 3
    xs = [vals(n, 300 + b) for b, n in enumerate(NS)]
    res = [np.zeros(n, np.float32) for n in NS]
    xg, rg = [dev(x) for x in xs], [dev(r) for r in res]
    bits = [torch.zeros((n + 31) // 32, dtype=torch.int32, device="cuda") for n in NS]
    sc = [torch.full((bg.num_chunks(n, C),), float("nan"), device="cuda") for n in NS]
    ws = ws_for(bg, B, k)
    call = bg.bagua_sign_compress_ef_batched(xg, rg, C, bits, sc, ws, prepare=True)
    torch.cuda.synchronize()
    assert all(torch.isnan(s).all() for s in sc) and all(int(r.count_nonzero()) == 0 for r in rg)   # nothing ran yet
    for rep in range(2):
        call()
        torch.cuda.synchronize()
        for b in range(B):
            bo, so = oracle.sign_compress_ef(xs[b], res[b], C)            # updates res[b] in place
            same(host(bits[b]).view(np.uint32), bo, "bits %d rep %d" % (b, rep))
            same(host(sc[b]), so, "scale %d rep %d" % (b, rep))
            same(host(rg[b]), res[b], "residual %d rep %d" % (b, rep))
    # MinMax compression, prepared, with error feedback carried over two calls
    mres = [np.zeros(n, np.float32) for n in NS]
    mrg = [dev(r) for r in mres]
    codes = [torch.empty(n, dtype=torch.uint8, device="cuda") for n in NS]
    mms = [torch.empty(2 * bg.num_chunks(n, C), device="cuda") for n in NS]
    mcall = bg.bagua_compress_minmax_u8_batched(xg, mrg, C, codes, mms, ws_for(bg, B), prepare=True)
    for rep in range(2):
        mcall()
        torch.cuda.synchronize()
        for b in range(B):
            co, mo = oracle.compress_minmax_u8(xs[b], mres[b], C)
            same(host(codes[b]), co, "codes %d rep %d" % (b, rep))
            same(host(mms[b]), mo, "minmax %d rep %d" % (b, rep))
            same(host(mrg[b]), mres[b], "minmax residual %d rep %d" % (b, rep))
    # the server step over what k workers sent (the same bits k times), prepared, after the inputs changed once more
    eps = [np.zeros(n, np.float32) for n in NS]
    eg = [dev(e) for e in eps]
    bo_g = [torch.zeros_like(b_) for b_ in bits]
    so_g = [torch.zeros_like(s_) for s_ in sc]
    out = [torch.empty(n, device="cuda") for n in NS]
    drr = bg.bagua_decompress_reduce_recompress_batched(bg.CODEC_SIGN1, [[bits[b]] * k for b in range(B)],
                                                        [[sc[b]] * k for b in range(B)], eg, NS, C, bo_g, so_g, out, ws,
                                                        prepare=True)
    call()                                                                # third compression: new bits, new scales
    drr()
    torch.cuda.synchronize()
    for b in range(B):
        bo, so = oracle.sign_compress_ef(xs[b], res[b], C)
        b2, s2, o2 = oracle.drr_sign([bo] * k, [so] * k, eps[b], NS[b], C)
        same(host(bo_g[b]).view(np.uint32), b2, "server bits %d" % b)
        same(host(so_g[b]), s2, "server scale %d" % b)
        same(host(out[b]), o2, "server out %d" % b)
        same(host(eg[b]), eps[b], "server residual %d" % b)


def test_batched_validation(bg):
    lib = bg.binding.raw()
    import ctypes
    INVALID, ALIGN = 1, 2
    A, Bp, Cc, D, W = 0x100000, 0x200000, 0x300000, 0x400000, 0x500000
    one = lambda v: (ctypes.c_void_p * 1)(v)
    n1 = (ctypes.c_size_t * 1)(64)
    wsb = bg.bagua_batch_workspace_bytes(1, 0)
    assert lib.bagua_compress_minmax_u8_batched(one(A), None, n1, 1, 256, one(Bp), one(Cc), W, wsb - 1, None) == INVALID
    assert lib.bagua_compress_minmax_u8_batched(one(A), None, n1, 0, 256, one(Bp), one(Cc), W, wsb, None) == INVALID
    assert lib.bagua_compress_minmax_u8_batched(one(A + 4), None, n1, 1, 256, one(Bp), one(Cc), W, wsb, None) == ALIGN
    assert lib.bagua_compress_minmax_u8_batched(one(A), None, n1, 1, 256, one(A), one(Cc), W, wsb, None) == INVALID   # codes alias x
    assert lib.bagua_compress_minmax_u8_batched(one(A), None, n1, 1, 256, one(Bp), one(Cc), A, wsb, None) == INVALID  # table over x
    n0 = (ctypes.c_size_t * 1)(0)
    assert lib.bagua_sign_compress_ef_batched(one(A), None, n0, 1, 256, one(Bp), one(Cc), W, wsb, None) == INVALID
    assert lib.bagua_decompress_reduce_recompress_batched(7, one(A), one(Bp), 1, None, n1, 1, 256, one(Cc), one(D), None, W,
                                                          bg.bagua_batch_workspace_bytes(1, 1), None) == INVALID
