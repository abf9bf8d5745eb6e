"""Seeded random differential test: every entry point against the oracle on shapes, worker counts, chunk sizes,
option combinations and value mixes drawn at random (fixed seeds, so every run checks the same cases)."""
import os

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

# BAGUA_RANDOM_CASES multiplies the number of seeds of every test below (default 1: the committed cases).
MULT = max(1, int(os.environ.get("BAGUA_RANDOM_CASES", "1")))

CHUNKS = [256, 512, 768, 1024, 1280, 2048, 2816, 4096, 4352, 8192, 12544, 16384]


@pytest.fixture(scope="module")
def bg():
    import paper_2107_01499_amd as b
    assert torch.cuda.is_available()
    return b


def dev(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(a).cuda()


def same(t, ref, what):
    got = t.cpu().numpy()
    assert got.size == ref.size, what
    assert np.array_equal(got.view(np.uint8).reshape(-1), np.ascontiguousarray(ref).view(np.uint8).reshape(-1)), what


def values(r, n):
    """Gradient-like values with the awkward cases mixed in: exact zeros and -0, ties, a flat stretch, denormals,
    a few huge entries."""
    scale = 10.0 ** r.uniform(-6, 1)
    x = (r.standard_normal(n) * scale).astype(np.float32)
    style = r.integers(0, 6)
    if style == 1:
        x[r.random(n) < 0.3] = 0.0
        x[r.random(n) < 0.05] = -0.0
    elif style == 2:
        x = np.round(x / np.float32(scale) * 4).astype(np.float32) * np.float32(scale / 4)   # many ties
    elif style == 3 and n > 10:
        a = int(r.integers(0, n - 1)); b = int(r.integers(a + 1, n))
        x[a:b] = x[a]                                                                       # flat stretch
    elif style == 4:
        x[r.random(n) < 0.1] = np.float32(1e-41)
        x[r.random(n) < 0.1] = np.float32(-3e-42)
    elif style == 5:
        x[r.random(n) < 0.01] = np.float32(1e34)
        x[r.random(n) < 0.01] = np.float32(-7e33)
    return x


def shape(r):
    C = int(r.choice(CHUNKS))
    n = int(r.choice([r.integers(1, 300), r.integers(1, 4 * C + 2), r.integers(1, 200000)]))
    return n, C


@pytest.mark.parametrize("seed", range(24 * MULT))
def test_random_c_lp_s_minmax(bg, oracle, seed):
    r = np.random.default_rng(1000 + seed)
    n, C = shape(r)
    k = int(r.integers(1, 33)) if n < 50000 else int(r.integers(1, 9))
    ef_w, ef_s, want_out = bool(r.integers(0, 2)), bool(r.integers(0, 2)), bool(r.integers(0, 2))
    print("minmax seed=%d n=%d C=%d k=%d ef=%s/%s out=%s" % (seed, n, C, k, ef_w, ef_s, want_out), flush=True)
    nc = (n + C - 1) // C
    enc_o, codes_g, mm_g = [], [], []
    for j in range(k):
        x = values(r, n)
        res = values(r, n) * np.float32(0.01) if ef_w else None
        res_o = None if res is None else res.copy()
        co, mo = oracle.compress_minmax_u8(x, res_o, C)
        cg, mg = torch.full((n,), 9, dtype=torch.uint8, device="cuda"), torch.full((2 * nc,), float("nan"), device="cuda")
        rg = None if res is None else dev(res)
        bg.bagua_compress_minmax_u8(dev(x), rg, C, cg, mg)
        same(cg, co, "codes %d" % j); same(mg, mo, "minmax %d" % j)
        if ef_w:
            same(rg, res_o, "delta %d" % j)
        enc_o.append((co, mo)); codes_g.append(cg); mm_g.append(mg)
    eps = values(r, n) * np.float32(0.01) if ef_s else None
    eps_o = None if eps is None else eps.copy()
    c2, m2, o2 = oracle.drr_minmax_u8([e[0] for e in enc_o], [e[1] for e in enc_o], eps_o, C, want_fp32=want_out)
    eg = None if eps is None else dev(eps)
    cg2, mg2 = torch.empty(n, dtype=torch.uint8, device="cuda"), torch.empty(2 * nc, device="cuda")
    og = torch.full((n,), float("nan"), device="cuda") if want_out else None
    bg.bagua_decompress_reduce_recompress(bg.CODEC_MINMAX_U8, codes_g, mm_g, eg, n, C, cg2, mg2, og)
    same(cg2, c2, "codes'"); same(mg2, m2, "minmax'")
    if ef_s:
        same(eg, eps_o, "eps")
    if want_out:
        same(og, o2, "out")
    dec = torch.empty(n, device="cuda")
    bg.bagua_decompress(bg.CODEC_MINMAX_U8, cg2, mg2, n, C, dec)
    same(dec, oracle.decompress_minmax_u8(c2, m2, C), "decode")


@pytest.mark.parametrize("seed", range(24 * MULT))
def test_random_c_lp_s_sign(bg, oracle, seed):
    r = np.random.default_rng(2000 + seed)
    n, C = shape(r)
    k = int(r.integers(1, 33)) if n < 50000 else int(r.integers(1, 9))
    ef_w, ef_s, want_out, mom = (bool(r.integers(0, 2)) for _ in range(4))
    print("sign seed=%d n=%d C=%d k=%d ef=%s/%s out=%s mom=%s" % (seed, n, C, k, ef_w, ef_s, want_out, mom), flush=True)
    nc, nw = (n + C - 1) // C, (n + 31) // 32
    m = values(r, n)
    enc_o, bits_g, sc_g = [], [], []
    for j in range(k):
        x = values(r, n)
        res = values(r, n) * np.float32(0.01) if ef_w else None
        res_o = None if res is None else res.copy()
        rg = None if res is None else dev(res)
        bgpu, sgpu = torch.full((nw,), 0x55aa55aa, dtype=torch.int32, device="cuda"), torch.full((nc,), float("nan"), device="cuda")
        if mom:
            bo, so = oracle.momentum_sign_compress_ef(x, m, 0.9, res_o, C)
            bg.bagua_momentum_sign_compress_ef(dev(x), dev(m), 0.9, rg, C, bgpu, sgpu)
        else:
            bo, so = oracle.sign_compress_ef(x, res_o, C)
            bg.bagua_sign_compress_ef(dev(x), rg, C, bgpu, sgpu)
        same(bgpu, bo, "bits %d" % j); same(sgpu, so, "scale %d" % j)
        if ef_w:
            same(rg, res_o, "delta %d" % j)
        enc_o.append((bo, so)); bits_g.append(bgpu); sc_g.append(sgpu)
    eps = values(r, n) * np.float32(0.01) if ef_s else None
    eps_o = None if eps is None else eps.copy()
    b2, s2, o2 = oracle.drr_sign([e[0] for e in enc_o], [e[1] for e in enc_o], eps_o, n, C, want_fp32=want_out)
    eg = None if eps is None else dev(eps)
    bg2, sg2 = torch.empty(nw, dtype=torch.int32, device="cuda"), torch.empty(nc, device="cuda")
    og = torch.full((n,), float("nan"), device="cuda") if want_out else None
    bg.bagua_decompress_reduce_recompress(bg.CODEC_SIGN1, bits_g, sc_g, eg, n, C, bg2, sg2, og)
    same(bg2, b2, "bits'"); same(sg2, s2, "scale'")
    if ef_s:
        same(eg, eps_o, "eps")
    if want_out:
        same(og, o2, "out")


@pytest.mark.parametrize("seed", range(16 * MULT))
def test_random_decentralised(bg, oracle, seed):
    r = np.random.default_rng(3000 + seed)
    n, C = shape(r)
    k = int(r.integers(1, 33)) if n < 50000 else int(r.integers(1, 9))
    print("decentralised seed=%d n=%d C=%d k=%d" % (seed, n, C, k), flush=True)
    nc = (n + C - 1) // C
    base = values(r, n)
    xs = [(base + values(r, n) * np.float32(0.05)).astype(np.float32) for _ in range(k)]
    xg = [dev(x) for x in xs]
    out = [torch.full((n,), float("nan"), device="cuda") for _ in range(k)]
    bg.bagua_decentralized_avg(bg.AVG_FP, xg, out)
    for a, b in zip(out, oracle.ring_avg_fp(xs)):
        same(a, b, "ring fp")
    peer = [int(p) for p in r.integers(0, k, k)] if seed % 2 else None
    if peer is None:
        perm = r.permutation(k)
        peer = list(range(k))
        for a, b in zip(perm[0::2], perm[1::2]):
            peer[a], peer[b] = int(b), int(a)
    bg.bagua_decentralized_avg_peers(xg, out, peer)
    for a, b in zip(out, oracle.peer_avg_fp(xs, peer)):
        same(a, b, "peer fp")
    cen = torch.empty(n, device="cuda")
    bg.bagua_centralized_avg_fp(xg, cen)
    same(cen, oracle.centralized_avg_fp(xs), "centralised")
    for which in ("ring", "peers"):
        hat_o = [base.copy() for _ in range(k)]
        hat_g = [dev(base) for _ in range(k)]
        cg = [torch.empty(n, dtype=torch.uint8, device="cuda") for _ in range(k)]
        mg = [torch.empty(2 * nc, device="cuda") for _ in range(k)]
        if which == "ring":
            want, wc, wm = oracle.ring_avg_lp(xs, hat_o, C)
            bg.bagua_decentralized_avg(bg.AVG_LP_MINMAX_U8, xg, out, hat_g, cg, mg, C)
        else:
            want, wc, wm = oracle.peer_avg_lp(xs, hat_o, peer, C)
            bg.bagua_decentralized_avg_peers_lp(xg, out, hat_g, cg, mg, peer, C)
        for i in range(k):
            same(out[i], want[i], "%s lp out %d" % (which, i)); same(hat_g[i], hat_o[i], "%s lp xhat %d" % (which, i))
            same(cg[i], wc[i], "%s lp codes %d" % (which, i)); same(mg[i], wm[i], "%s lp minmax %d" % (which, i))


@pytest.mark.parametrize("seed", range(16 * MULT))
def test_random_topk_and_optimizer_steps(bg, oracle, seed):
    r = np.random.default_rng(4000 + seed)
    n, C = shape(r)
    k = int(r.integers(1, 9))
    keep = int(r.choice([1, max(1, C // 32), int(r.integers(1, C + 1))]))
    ef = bool(r.integers(0, 2))
    print("topk/opt seed=%d n=%d C=%d k=%d keep=%d ef=%s" % (seed, n, C, k, keep, ef), flush=True)
    nc = (n + C - 1) // C
    enc_o, ig, vg = [], [], []
    for j in range(k):
        x = values(r, n)
        res = values(r, n) * np.float32(0.01) if ef else None
        res_o = None if res is None else res.copy()
        io, vo = oracle.compress_topk(x, res_o, C, keep)
        i_g, v_g = torch.full((nc * keep,), 7, dtype=torch.int16, device="cuda"), torch.full((nc * keep,), float("nan"), device="cuda")
        rg = None if res is None else dev(res)
        bg.bagua_compress_topk_ef(dev(x), rg, C, keep, i_g, v_g)
        same(i_g, io, "idx %d" % j); same(v_g, vo, "val %d" % j)
        if ef:
            same(rg, res_o, "delta %d" % j)
        enc_o.append((io, vo)); ig.append(i_g); vg.append(v_g)
    eps = values(r, n) * np.float32(0.01) if ef else None
    eps_o = None if eps is None else eps.copy()
    io2, vo2, oo = oracle.drr_topk([e[0] for e in enc_o], [e[1] for e in enc_o], eps_o, n, C, keep, want_fp32=True)
    eg = None if eps is None else dev(eps)
    i2, v2, o2 = torch.empty(nc * keep, dtype=torch.int16, device="cuda"), torch.empty(nc * keep, device="cuda"), torch.empty(n, device="cuda")
    bg.bagua_decompress_reduce_recompress_topk(ig, vg, keep, eg, n, C, i2, v2, o2)
    same(i2, io2, "idx'"); same(v2, vo2, "val'"); same(o2, oo, "out")
    if ef:
        same(eg, eps_o, "eps")
    # optimizer steps fed by a MinMax- or sign-coded tensor
    codec = int(r.integers(0, 2))
    g = (values(r, n) * np.float32(1e-2)).astype(np.float32)
    codes, meta = oracle.compress_minmax_u8(g, None, C) if codec == 0 else oracle.sign_compress_ef(g, None, C)
    cg, mg = dev(codes), dev(meta)
    p_o, m_o = values(r, n), values(r, n) * np.float32(0.1)
    v_o = np.abs(values(r, n)).astype(np.float32) * np.float32(1e-3)
    p_g, m_g, v_g2 = dev(p_o), dev(m_o), dev(v_o)
    wd = float(r.choice([0.0, 1e-2]))
    frozen = bool(r.integers(0, 2))
    oracle.decompress_adam_step(codec, codes, meta, n, C, p_o, m_o, v_o, 1e-3, 0.9, 0.999, 1e-8, wd, frozen)
    bg.bagua_decompress_adam_step(codec, cg, mg, n, C, p_g, m_g, v_g2, 1e-3, 0.9, 0.999, 1e-8, wd, frozen)
    same(p_g, p_o, "adam p"); same(m_g, m_o, "adam m"); same(v_g2, v_o, "adam v")
    use_mom = bool(r.integers(0, 2))
    mo_o = m_o.copy() if use_mom else None
    mo_g = dev(mo_o) if use_mom else None
    oracle.decompress_sgd_step(codec, codes, meta, n, C, p_o, mo_o, 0.05, 0.9, wd)
    bg.bagua_decompress_sgd_step(codec, cg, mg, n, C, p_g, mo_g, 0.05, 0.9, wd)
    same(p_g, p_o, "sgd p")
    if use_mom:
        same(mo_g, mo_o, "sgd m")


def random_layout(r):
    """Tensors of random sizes (some empty) with random gaps between their bucket ranges, every tensor at a device
    address that is only 4-byte aligned by a random amount."""
    T = int(r.integers(1, 12))
    sizes = [int(r.choice([0, r.integers(1, 9), r.integers(1, 700), r.integers(1, 40000)])) for _ in range(T)]
    srcs = [values(r, s) if s else np.zeros(0, np.float32) for s in sizes]
    offs, pos = [], 0
    for s in sizes:
        pos += int(r.choice([0, 0, r.integers(0, 5), r.integers(0, 300)]))
        offs.append(pos)
        pos += s
    total = max(1, pos + int(r.integers(0, 50)))
    arena = torch.zeros(sum(sizes) + 8 * T + 8, device="cuda")
    gs, p0 = [], 0
    for x in srcs:
        p0 += int(r.integers(0, 4))
        t = arena[p0:p0 + x.size]
        t.copy_(torch.from_numpy(x))
        gs.append(t)
        p0 += x.size
    return srcs, gs, offs, total


@pytest.mark.parametrize("seed", range(24 * MULT))
def test_random_flatten_and_its_fusions(bg, oracle, seed):
    r = np.random.default_rng(5000 + seed)
    C = int(r.choice(CHUNKS))
    srcs, gs, offs, total = random_layout(r)
    ef, want_bucket = bool(r.integers(0, 2)), bool(r.integers(0, 2))
    print("flatten/fusions seed=%d T=%d total=%d C=%d ef=%s bucket=%s" % (seed, len(gs), total, C, ef, want_bucket), flush=True)
    flat = oracle.bucket_flatten(srcs, offs, total)
    ws = torch.empty(bg.bagua_flatten_workspace_bytes(len(gs), total), dtype=torch.uint8, device="cuda")
    bucket = torch.full((total,), float("nan"), device="cuda")
    bg.bagua_bucket_flatten(gs, offs, bucket, ws)
    same(bucket, flat, "flatten")
    bucket2 = torch.full((total,), float("nan"), device="cuda")
    bg.bagua_bucket_flatten_static(gs, offs, bucket2)
    same(bucket2, flat, "flatten_static")
    nc = (total + C - 1) // C
    res = values(r, total) * np.float32(0.01)
    # gather fused into the MinMax compression
    ro, rg = (res.copy(), dev(res)) if ef else (None, None)
    co, mo = oracle.compress_minmax_u8(flat, ro, C)
    cg, mg = torch.full((total,), 0xAB, dtype=torch.uint8, device="cuda"), torch.full((2 * nc,), float("nan"), device="cuda")
    bo = torch.full((total,), float("nan"), device="cuda") if want_bucket else None
    bg.bagua_flatten_compress_minmax_u8(ws, len(gs), rg, total, C, cg, mg, bo)
    same(cg, co, "fused minmax codes"); same(mg, mo, "fused minmax meta")
    if ef:
        same(rg, ro, "fused minmax residual")
    if want_bucket:
        same(bo, flat, "fused minmax bucket")
    # gather fused into the sign compression
    ro, rg = (res.copy(), dev(res)) if ef else (None, None)
    bo_, so = oracle.sign_compress_ef(flat, ro, C)
    bits, sc = torch.full(((total + 31) // 32,), -1, dtype=torch.int32, device="cuda"), torch.full((nc,), float("nan"), device="cuda")
    bo = torch.full((total,), float("nan"), device="cuda") if want_bucket else None
    bg.bagua_flatten_sign_compress_ef(ws, len(gs), rg, total, C, bits, sc, bo)
    same(bits, bo_, "fused sign bits"); same(sc, so, "fused sign scale")
    if ef:
        same(rg, ro, "fused sign residual")
    if want_bucket:
        same(bo, flat, "fused sign bucket")
    # decode fused into the inverse scatter, then the plain inverse scatter
    for codec, (codes, meta) in ((bg.CODEC_MINMAX_U8, (co, mo)), (bg.CODEC_SIGN1, (bo_, so))):
        dec = oracle.decompress_minmax_u8(codes, meta, C) if codec == bg.CODEC_MINMAX_U8 else oracle.decompress_sign(codes, meta, total, C)
        want = [np.full(x.size, np.float32(7.0)) for x in srcs]
        oracle.bucket_unflatten(dec, want, offs)
        for t in gs:
            t.fill_(7.0)
        bg.bagua_decompress_unflatten(codec, dev(codes), dev(meta), total, C, ws, len(gs))
        for i, (t, w) in enumerate(zip(gs, want)):
            same(t, w, "decode+scatter codec %d tensor %d" % (codec, i))
        for t in gs:
            t.fill_(-3.0)
        bg.bagua_bucket_unflatten_run(ws, len(gs), dev(dec))
        for i, (t, w) in enumerate(zip(gs, want)):
            if w.size:
                same(t, w, "scatter codec %d tensor %d" % (codec, i))


@pytest.mark.parametrize("seed", range(16 * MULT))
def test_random_batched_and_intra_node(bg, oracle, seed):
    r = np.random.default_rng(6000 + seed)
    C = int(r.choice(CHUNKS))
    B = int(r.integers(1, 9))
    ns = [shape(r)[0] for _ in range(B)]
    k = int(r.integers(1, 10))
    ef, want_out = bool(r.integers(0, 2)), bool(r.integers(0, 2))
    print("batched seed=%d B=%d ns=%s C=%d k=%d ef=%s out=%s" % (seed, B, ns, C, k, ef, want_out), flush=True)
    ws = torch.empty(bg.bagua_batch_workspace_bytes(B, k), dtype=torch.uint8, device="cuda")
    ncs = [(n + C - 1) // C for n in ns]
    for sign in (False, True):
        xs = [[values(r, n) for n in ns] for _ in range(k)]                 # xs[j][b]
        res = [values(r, n) * np.float32(0.01) for n in ns]
        enc = [[None] * B for _ in range(k)]
        # worker 0 goes through the batched compression (with its error state), the others are encoded by the oracle
        rg = [dev(x) for x in res] if ef else None
        if sign:
            cg = [torch.full(((n + 31) // 32,), -1, dtype=torch.int32, device="cuda") for n in ns]
            mg = [torch.full((c,), float("nan"), device="cuda") for c in ncs]
            bg.bagua_sign_compress_ef_batched([dev(x) for x in xs[0]], rg, C, cg, mg, ws)
        else:
            cg = [torch.full((n,), 0xAB, dtype=torch.uint8, device="cuda") for n in ns]
            mg = [torch.full((2 * c,), float("nan"), device="cuda") for c in ncs]
            bg.bagua_compress_minmax_u8_batched([dev(x) for x in xs[0]], rg, C, cg, mg, ws)
        comp = oracle.sign_compress_ef if sign else oracle.compress_minmax_u8
        for b in range(B):
            ro = res[b].copy() if ef else None
            enc[0][b] = comp(xs[0][b], ro, C)
            same(cg[b], enc[0][b][0], "batched codes %d" % b); same(mg[b], enc[0][b][1], "batched meta %d" % b)
            if ef:
                same(rg[b], ro, "batched residual %d" % b)
            for j in range(1, k):
                enc[j][b] = comp(xs[j][b], None, C)
        eps = [values(r, n) * np.float32(0.01) for n in ns]
        eg = [dev(e) for e in eps] if ef else None
        ci = [[dev(enc[j][b][0]) for j in range(k)] for b in range(B)]
        mi = [[dev(enc[j][b][1]) for j in range(k)] for b in range(B)]
        if sign:
            co = [torch.full(((n + 31) // 32,), -1, dtype=torch.int32, device="cuda") for n in ns]
            mo = [torch.full((c,), float("nan"), device="cuda") for c in ncs]
        else:
            co = [torch.full((n,), 0xAB, dtype=torch.uint8, device="cuda") for n in ns]
            mo = [torch.full((2 * c,), float("nan"), device="cuda") for c in ncs]
        og = [torch.full((n,), float("nan"), device="cuda") for n in ns] if want_out else None
        bg.bagua_decompress_reduce_recompress_batched(bg.CODEC_SIGN1 if sign else bg.CODEC_MINMAX_U8, ci, mi, eg, ns, C,
                                                      co, mo, og, ws)
        for b in range(B):
            eo = eps[b].copy() if ef else None
            cs, ms = [enc[j][b][0] for j in range(k)], [enc[j][b][1] for j in range(k)]
            c2, m2, o2 = oracle.drr_sign(cs, ms, eo, ns[b], C) if sign else oracle.drr_minmax_u8(cs, ms, eo, C)
            same(co[b], c2, "server codes %d" % b); same(mo[b], m2, "server meta %d" % b)
            if want_out:
                same(og[b], o2, "server out %d" % b)
            if ef:
                same(eg[b], eo, "server eps %d" % b)
    # intra-node stage of the hierarchical variant, both codecs, on the first bucket's size
    n, nc = ns[0], ncs[0]
    xs = [values(r, n) for _ in range(k)]
    res = values(r, n) * np.float32(0.01)
    xg = [dev(x) for x in xs]
    ro, rg = (res.copy(), dev(res)) if ef else (None, None)
    c1, m1 = oracle.reduce_compress_minmax_u8(xs, ro, C)
    cg, mg = torch.empty(n, dtype=torch.uint8, device="cuda"), torch.empty(2 * nc, device="cuda")
    bg.bagua_reduce_compress_minmax_u8(xg, rg, C, cg, mg)
    same(cg, c1, "intra-node minmax codes"); same(mg, m1, "intra-node minmax meta")
    if ef:
        same(rg, ro, "intra-node minmax residual")
    ro, rg = (res.copy(), dev(res)) if ef else (None, None)
    b1, s1 = oracle.reduce_compress_sign(xs, ro, C)
    bgd, sg = torch.full(((n + 31) // 32,), -1, dtype=torch.int32, device="cuda"), torch.empty(nc, device="cuda")
    bg.bagua_reduce_compress_sign_ef(xg, rg, C, bgd, sg)
    same(bgd, b1, "intra-node sign bits"); same(sg, s1, "intra-node sign scale")
    if ef:
        same(rg, ro, "intra-node sign residual")
    # SGD step fed by a top-K round
    keep = int(r.choice([1, max(1, C // 32), int(r.integers(1, C + 1))]))
    io, vo = oracle.compress_topk(values(r, n), None, C, keep)
    p_o, m_o = values(r, n), values(r, n) * np.float32(0.1)
    use_mom, wd = bool(r.integers(0, 2)), float(r.choice([0.0, 1e-2]))
    p_g = dev(p_o)
    mo_o = m_o.copy() if use_mom else None
    mo_g = dev(mo_o) if use_mom else None
    oracle.decompress_sgd_step_topk(io, vo, n, C, keep, p_o, mo_o, 0.05, 0.9 if use_mom else 0.0, wd)
    bg.bagua_decompress_sgd_step_topk(dev(io), dev(vo), n, C, keep, p_g, mo_g, 0.05, 0.9 if use_mom else 0.0, wd)
    same(p_g, p_o, "topk sgd p")
    if use_mom:
        same(mo_g, mo_o, "topk sgd m")
    # Adam-type step fed by the same top-K round
    v_o = np.abs(values(r, n)).astype(np.float32) * np.float32(1e-3)
    a_o = [p_o.copy(), m_o.copy(), v_o]
    a_g = [dev(t) for t in a_o]
    frozen = bool(r.integers(0, 2))
    oracle.decompress_adam_step_topk(io, vo, n, C, keep, a_o[0], a_o[1], a_o[2], 1e-3, 0.9, 0.999, 1e-8, wd, frozen)
    bg.bagua_decompress_adam_step_topk(dev(io), dev(vo), n, C, keep, a_g[0], a_g[1], a_g[2], 1e-3, 0.9, 0.999, 1e-8, wd, frozen)
    same(a_g[0], a_o[0], "topk adam p"); same(a_g[1], a_o[1], "topk adam m"); same(a_g[2], a_o[2], "topk adam v")
