"""GPU parity of the decode + bucket-level SGD step against the oracle."""
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


def bit_equal(t, a, what):
    got = t.cpu().numpy()
    err = np.abs(got.astype(np.float64) - a.astype(np.float64))
    assert np.all(err <= 1e-6 * np.abs(a.astype(np.float64)) + 1e-7), what
    assert np.array_equal(got.view(np.uint32), a.view(np.uint32)), what


@pytest.mark.parametrize("codec", [0, 1])
@pytest.mark.parametrize("n,C", [(1, 256), (257, 256), (3 * 4096 + 77, 4096), (70001, 2048), (40000, 16384)])
@pytest.mark.parametrize("mom,wd", [(False, 0.0), (True, 0.0), (False, 1e-2), (True, 1e-2)])
def test_decompress_sgd_step(bg, oracle, codec, n, C, mom, wd):
    print("sgd codec=%d n=%d C=%d mom=%s wd=%g" % (codec, n, C, mom, wd), flush=True)
    r = np.random.default_rng(n + C + codec)
    x = (r.standard_t(3, n) * 1e-3).astype(np.float32)
    if codec == 0:
        codes, meta = oracle.compress_minmax_u8(x, None, C)
        cg = dev(codes)
    else:
        codes, meta = oracle.sign_compress_ef(x, None, C)
        cg = dev(codes.view(np.int32))
    p_o = r.standard_normal(n).astype(np.float32)
    m_o = (r.standard_normal(n) * 1e-3).astype(np.float32) if mom else None
    p_g, m_g, meta_g = dev(p_o), (dev(m_o) if mom else None), dev(meta)
    lr, mu = 0.05, 0.9
    for _ in range(3):            # state carried across steps on both sides
        oracle.decompress_sgd_step(codec, codes, meta, n, C, p_o, m_o, lr, mu, wd)
        bg.bagua_decompress_sgd_step(codec, cg, meta_g, n, C, p_g, m_g, lr, mu, wd)
    torch.cuda.synchronize()
    bit_equal(p_g, p_o, "param")
    if mom:
        bit_equal(m_g, m_o, "momentum")


@pytest.mark.parametrize("n,C,keep", [(1, 256, 1), (257, 256, 8), (3 * 4096 + 77, 4096, 128), (70001, 2048, 2048), (40000, 16384, 7)])
@pytest.mark.parametrize("mom,wd,lr", [(False, 0.0, 0.1), (False, 0.0, -0.1), (True, 0.0, 0.1), (False, 1e-2, 0.1), (True, 1e-2, 0.05)])
def test_decompress_sgd_step_topk(bg, oracle, n, C, keep, mom, wd, lr):
    """Two steps with state carried; lr < 0 without momentum / weight decay takes the dense form (-0 parameters)."""
    print("sgd topk n=%d C=%d keep=%d mom=%s wd=%g lr=%g" % (n, C, keep, mom, wd, lr), flush=True)
    r = np.random.default_rng(n + C + keep)
    p_o = r.standard_normal(n).astype(np.float32)
    p_o[::13] = -0.0
    m_o = (r.standard_normal(n) * 0.1).astype(np.float32) if mom else None
    pg, mg = dev(p_o), (dev(m_o) if mom else None)
    for step in range(2):
        x = (r.standard_t(3, n) * 1e-3).astype(np.float32)
        idx, val = oracle.compress_topk(x, None, C, keep)
        oracle.decompress_sgd_step_topk(idx, val, n, C, keep, p_o, m_o, lr, 0.9, wd)
        bg.bagua_decompress_sgd_step_topk(dev(idx.view(np.int16)), dev(val), n, C, keep, pg, mg, lr, 0.9, wd)
        torch.cuda.synchronize()
        bit_equal(pg, p_o, "param step %d" % step)
        if mom:
            bit_equal(mg, m_o, "momentum step %d" % step)
