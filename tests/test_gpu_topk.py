"""GPU parity of the per-chunk top-K codec (worker side, server side, decode) against the oracle."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def bg():
    import paper_2107_01499_amd as b
    assert torch.cuda.is_available()
    return b


def dev(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(a).cuda()


def host_u16(t):
    return t.cpu().numpy().view(np.uint16)


def t3(n, seed, ties=True):
    x = (np.random.default_rng(seed).standard_t(3, n) * 1e-3).astype(np.float32)
    if ties:
        x[::7] = np.round(x[::7] * 1e3) / 1e3      # exact ties, zeros and negative zeros
    return x


@pytest.mark.parametrize("n", [1, 5, 255, 256, 257, 4095, 4096, 4097, 2 * 4096 + 7, 70001])
@pytest.mark.parametrize("C,keep", [(256, 1), (256, 8), (256, 256), (768, 100), (4096, 128), (4096, 1000), (16384, 512)])
@pytest.mark.parametrize("ef", [False, True])
def test_compress_topk(bg, oracle, n, C, keep, ef):
    print("compress_topk n=%d C=%d keep=%d ef=%s" % (n, C, keep, ef), flush=True)
    x = t3(n, n + keep)
    res = t3(n, n + 1) * np.float32(0.1) if ef else None
    res_o = None if res is None else res.copy()
    io, vo = oracle.compress_topk(x, res_o, C, keep)
    nc = bg.num_chunks(n, C)
    rg = None if res is None else dev(res)
    ig = torch.full((nc * keep,), 0x1234, dtype=torch.int16, device="cuda")
    vg = torch.full((nc * keep,), float("nan"), device="cuda")
    bg.bagua_compress_topk_ef(dev(x), rg, C, keep, ig, vg)
    torch.cuda.synchronize()
    assert np.array_equal(host_u16(ig), io)
    assert np.array_equal(vg.cpu().numpy().view(np.uint32), vo.view(np.uint32))
    if ef:
        assert np.array_equal(rg.cpu().numpy().view(np.uint32), res_o.view(np.uint32))
    out = torch.full((n,), float("nan"), device="cuda")
    bg.bagua_decompress_topk(ig, vg, n, C, keep, out)
    assert np.array_equal(out.cpu().numpy().view(np.uint32), oracle.decompress_topk(io, vo, n, C, keep).view(np.uint32))


def test_topk_degenerate_chunks(bg, oracle):
    C, keep = 256, 10
    x = np.zeros(4 * C, np.float32)
    x[0:C] = 0.25; x[100] = -0.25                 # all magnitudes equal: lowest indices win
    x[C:2 * C] = 0.0; x[C + 5] = -0.0             # all zero
    x[2 * C:3 * C] = np.arange(C, dtype=np.float32) * np.float32(1e-45)   # denormals, increasing
    x[3 * C:] = np.float32(3e38) * np.where(np.arange(C) % 2, 1, -1)       # huge, alternating sign
    io, vo = oracle.compress_topk(x, None, C, keep)
    ig = torch.empty(4 * keep, dtype=torch.int16, device="cuda"); vg = torch.empty(4 * keep, device="cuda")
    bg.bagua_compress_topk_ef(dev(x), None, C, keep, ig, vg)
    assert np.array_equal(host_u16(ig), io) and np.array_equal(vg.cpu().numpy().view(np.uint32), vo.view(np.uint32))


@pytest.mark.parametrize("k", [1, 2, 3, 8, 32])
@pytest.mark.parametrize("n,C,keep", [(1, 256, 4), (257, 256, 16), (3 * 4096 + 77, 4096, 128), (40000, 16384, 300), (9000, 768, 768)])
@pytest.mark.parametrize("ef,want_out", [(True, True), (False, False)])
def test_drr_topk(bg, oracle, k, n, C, keep, ef, want_out):
    print("drr_topk k=%d n=%d C=%d keep=%d ef=%s" % (k, n, C, keep, ef), flush=True)
    enc = [oracle.compress_topk(t3(n, 17 * k + j), None, C, keep) for j in range(k)]
    eps = t3(n, 3, ties=False) * np.float32(0.05) if ef else None
    eps_o = None if eps is None else eps.copy()
    io, vo, oo = oracle.drr_topk([e[0] for e in enc], [e[1] for e in enc], eps_o, n, C, keep, want_fp32=want_out)
    nc = bg.num_chunks(n, C)
    eg = None if eps is None else dev(eps)
    ig = torch.full((nc * keep,), 0x1234, dtype=torch.int16, device="cuda")
    vg = torch.full((nc * keep,), float("nan"), device="cuda")
    og = torch.full((n,), float("nan"), device="cuda") if want_out else None
    bg.bagua_decompress_reduce_recompress_topk([dev(e[0]) for e in enc], [dev(e[1]) for e in enc], keep, eg, n, C, ig, vg, og)
    torch.cuda.synchronize()
    assert np.array_equal(host_u16(ig), io)
    assert np.array_equal(vg.cpu().numpy().view(np.uint32), vo.view(np.uint32))
    if ef:
        assert np.array_equal(eg.cpu().numpy().view(np.uint32), eps_o.view(np.uint32))
    if want_out:
        assert np.array_equal(og.cpu().numpy().view(np.uint32), oo.view(np.uint32))


def test_topk_c_lp_s_iterations(bg, oracle):
    """Three C_LP_S iterations with the top-K codec, worker and server error states carried on the GPU."""
    n, C, keep, k = 5 * 4096 + 300, 4096, 64, 4
    nc = bg.num_chunks(n, C)
    d_o = [np.zeros(n, np.float32) for _ in range(k)]; e_o = np.zeros(n, np.float32)
    d_g = [torch.zeros(n, device="cuda") for _ in range(k)]; e_g = torch.zeros(n, device="cuda")
    for it in range(3):
        enc_o, ig, vg = [], [], []
        for j in range(k):
            x = t3(n, 100 * it + j)
            enc_o.append(oracle.compress_topk(x, d_o[j], C, keep))
            i_ = torch.empty(nc * keep, dtype=torch.int16, device="cuda"); v_ = torch.empty(nc * keep, device="cuda")
            bg.bagua_compress_topk_ef(dev(x), d_g[j], C, keep, i_, v_)
            ig.append(i_); vg.append(v_)
        io, vo, oo = oracle.drr_topk([e[0] for e in enc_o], [e[1] for e in enc_o], e_o, n, C, keep)
        i2 = torch.empty(nc * keep, dtype=torch.int16, device="cuda"); v2 = torch.empty(nc * keep, device="cuda")
        og = torch.empty(n, device="cuda")
        bg.bagua_decompress_reduce_recompress_topk(ig, vg, keep, e_g, n, C, i2, v2, og)
        assert np.array_equal(host_u16(i2), io) and np.array_equal(v2.cpu().numpy().view(np.uint32), vo.view(np.uint32))
        assert np.array_equal(og.cpu().numpy().view(np.uint32), oo.view(np.uint32))
        assert np.array_equal(e_g.cpu().numpy().view(np.uint32), e_o.view(np.uint32))
        for j in range(k):
            assert np.array_equal(d_g[j].cpu().numpy().view(np.uint32), d_o[j].view(np.uint32))
