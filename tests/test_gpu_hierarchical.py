"""GPU parity of the intra-node stage of hierarchical C_LP_S, and the two-level pipeline, against the oracle."""
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
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def vals(n, seed):
    return (np.random.default_rng(seed).standard_t(3, n) * 1e-3).astype(np.float32)


@pytest.mark.parametrize("k", [1, 2, 3, 8, 32])
@pytest.mark.parametrize("n,C", [(1, 256), (257, 256), (3 * 4096 + 77, 4096), (70001, 8192), (40000, 16384)])
@pytest.mark.parametrize("ef", [False, True])
def test_reduce_compress(bg, oracle, k, n, C, ef):
    print("reduce_compress k=%d n=%d C=%d ef=%s" % (k, n, C, ef), flush=True)
    xs = [vals(n, 31 * k + j) for j in range(k)]
    res = vals(n, 7) * np.float32(0.05) if ef else None
    res_o = None if res is None else res.copy()
    co, mo = oracle.reduce_compress_minmax_u8(xs, res_o, C)
    rg = None if res is None else dev(res)
    codes = torch.full((n,), 0xAB, dtype=torch.uint8, device="cuda")
    mm = torch.full((2 * bg.num_chunks(n, C),), float("nan"), device="cuda")
    bg.bagua_reduce_compress_minmax_u8([dev(x) for x in xs], rg, C, codes, mm)
    torch.cuda.synchronize()
    assert np.array_equal(codes.cpu().numpy(), co)
    assert np.array_equal(mm.cpu().numpy().view(np.uint32), mo.view(np.uint32))
    if ef:
        assert np.array_equal(rg.cpu().numpy().view(np.uint32), res_o.view(np.uint32))


@pytest.mark.parametrize("k", [1, 2, 4, 32])
@pytest.mark.parametrize("n,C", [(1, 256), (257, 256), (3 * 2048 + 77, 2048), (70001, 8192), (40000, 16384)])
@pytest.mark.parametrize("ef", [False, True])
def test_reduce_compress_sign(bg, oracle, k, n, C, ef):
    print("reduce_compress_sign k=%d n=%d C=%d ef=%s" % (k, n, C, ef), flush=True)
    xs = [vals(n, 37 * k + j) for j in range(k)]
    xs[0][::17] = 0.0
    res = vals(n, 8) * np.float32(0.05) if ef else None
    res_o = None if res is None else res.copy()
    bo, so = oracle.reduce_compress_sign(xs, res_o, C)
    rg = None if res is None else dev(res)
    bits = torch.full(((n + 31) // 32,), -1, dtype=torch.int32, device="cuda")
    scale = torch.full((bg.num_chunks(n, C),), float("nan"), device="cuda")
    bg.bagua_reduce_compress_sign_ef([dev(x) for x in xs], rg, C, bits, scale)
    torch.cuda.synchronize()
    assert np.array_equal(bits.cpu().numpy().view(np.uint32), bo)
    assert np.array_equal(scale.cpu().numpy().view(np.uint32), so.view(np.uint32))
    if ef:
        assert np.array_equal(rg.cpu().numpy().view(np.uint32), res_o.view(np.uint32))


def test_two_level_pipeline(bg, oracle):
    """4 nodes x 2 local workers, two iterations with all error states carried: intra-node reduce+compress at the
    leaders, inter-node server step, decode on every worker."""
    nodes, kl, n, C = 4, 2, 5 * 4096 + 300, 4096
    nc = bg.num_chunks(n, C)
    d_o = [np.zeros(n, np.float32) for _ in range(nodes)]
    e_o = np.zeros(n, np.float32)
    d_g = [torch.zeros(n, device="cuda") for _ in range(nodes)]
    e_g = torch.zeros(n, device="cuda")
    for it in range(2):
        enc_o, cg, mg = [], [], []
        for a in range(nodes):
            xs = [vals(n, 1000 * it + 10 * a + b) for b in range(kl)]
            enc_o.append(oracle.reduce_compress_minmax_u8(xs, d_o[a], C))
            c = torch.empty(n, dtype=torch.uint8, device="cuda"); m = torch.empty(2 * nc, device="cuda")
            bg.bagua_reduce_compress_minmax_u8([dev(x) for x in xs], d_g[a], C, c, m)
            cg.append(c); mg.append(m)
        co, mo, oo = oracle.drr_minmax_u8([e[0] for e in enc_o], [e[1] for e in enc_o], e_o, C)
        c2 = torch.empty(n, dtype=torch.uint8, device="cuda"); m2 = torch.empty(2 * nc, device="cuda")
        bg.bagua_decompress_reduce_recompress(bg.CODEC_MINMAX_U8, cg, mg, e_g, n, C, c2, m2, None)
        out = torch.empty(n, device="cuda")
        bg.bagua_decompress(bg.CODEC_MINMAX_U8, c2, m2, n, C, out)
        assert np.array_equal(c2.cpu().numpy(), co) and np.array_equal(m2.cpu().numpy().view(np.uint32), mo.view(np.uint32))
        assert np.array_equal(out.cpu().numpy().view(np.uint32), oo.view(np.uint32))
        assert np.array_equal(e_g.cpu().numpy().view(np.uint32), e_o.view(np.uint32))
        for a in range(nodes):
            assert np.array_equal(d_g[a].cpu().numpy().view(np.uint32), d_o[a].view(np.uint32))
