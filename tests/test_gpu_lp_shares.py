"""GPU parity of one peer's share of D_LP_S (encode; apply + mix): k peers, each with its own copies of its
neighbours' public replicas as on k separate GPUs, must reproduce the oracle's ring round bit for bit."""
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


def same(t, ref, what):
    assert np.array_equal(t.cpu().numpy().view(np.uint8).reshape(-1), np.ascontiguousarray(ref).view(np.uint8).reshape(-1)), what


@pytest.mark.parametrize("n,C", [(1, 256), (255, 256), (3 * 4096 + 1027, 4096), (70001, 2048), (5000, 768), (16384 + 5, 16384)])
def test_lp_encode_against_oracle_steps(bg, oracle, n, C):
    r = np.random.default_rng(n + C)
    x = (r.standard_normal(n) * 0.02).astype(np.float32)
    hat = (x + (r.standard_normal(n) * 1e-3).astype(np.float32)).astype(np.float32)
    d = (x - hat).astype(np.float32)
    codes, mm = oracle.compress_minmax_u8(d, None, C)
    hat_new = (hat + oracle.decompress_minmax_u8(codes, mm, C)).astype(np.float32)
    nc = (n + C - 1) // C
    hg, cg, mg = dev(hat), torch.full((n,), 3, dtype=torch.uint8, device="cuda"), torch.full((2 * nc,), float("nan"), device="cuda")
    xg = dev(x)
    bg.bagua_lp_encode(xg, hg, C, cg, mg)
    torch.cuda.synchronize()
    same(cg, codes, "codes"); same(mg, mm, "minmax"); same(hg, hat_new, "xhat"); same(xg, x, "x untouched")


@pytest.mark.parametrize("k", [1, 2, 3, 5, 8])
@pytest.mark.parametrize("n,C", [(300, 256), (3 * 4096 + 1027, 4096), (40001, 1024)])
def test_sharded_ring_equals_oracle_round(bg, oracle, k, n, C):
    print("lp shares k=%d n=%d C=%d" % (k, n, C), flush=True)
    r = np.random.default_rng(17 * k + n)
    nc = (n + C - 1) // C
    base = (r.standard_normal(n) * 0.02).astype(np.float32)
    xs = [(base + (r.standard_normal(n) * 1e-3).astype(np.float32)).astype(np.float32) for _ in range(k)]
    hat_o = [base.copy() for _ in range(k)]
    # "GPU" i holds its own public copy and one copy of each distinct neighbour's
    held = [sorted({(i - 1) % k, i, (i + 1) % k}) for i in range(k)]
    hat_g = [{j: dev(base) for j in held[i]} for i in range(k)]
    codes = [torch.empty(n, dtype=torch.uint8, device="cuda") for _ in range(k)]
    mm = [torch.empty(2 * nc, device="cuda") for _ in range(k)]
    for rnd in range(3):
        want, wc, wm = oracle.ring_avg_lp(xs, hat_o, C)
        xg = [dev(x) for x in xs]
        out = [torch.full((n,), float("nan"), device="cuda") for _ in range(k)]
        for i in range(k):                                  # every peer publishes
            bg.bagua_lp_encode(xg[i], hat_g[i][i], C, codes[i], mm[i])
        for i in range(k):                                  # codes have "arrived": every peer applies and mixes
            le, ri = (i - 1) % k, (i + 1) % k
            if k == 1:
                bg.bagua_lp_apply_mix(xg[i], hat_g[i][i], hat_g[i][i], hat_g[i][i], None, None, None, None, C, out[i])
            elif le == ri:
                bg.bagua_lp_apply_mix(xg[i], hat_g[i][i], hat_g[i][le], hat_g[i][le], codes[le], mm[le], None, None, C, out[i])
            else:
                bg.bagua_lp_apply_mix(xg[i], hat_g[i][i], hat_g[i][le], hat_g[i][ri], codes[le], mm[le], codes[ri], mm[ri],
                                      C, out[i])
        torch.cuda.synchronize()
        for i in range(k):
            tag = "round %d peer %d" % (rnd, i)
            same(out[i], want[i], tag + " out"); same(codes[i], wc[i], tag + " codes"); same(mm[i], wm[i], tag + " minmax")
            for j in held[i]:
                same(hat_g[i][j], hat_o[j], tag + " copy of %d" % j)
        xs = [(w + (r.standard_normal(n) * 1e-4).astype(np.float32)).astype(np.float32) for w in want]


def test_apply_mix_without_codes_is_a_pure_mix(bg):
    """No codes: the copies are only read, and the result is the three-way mix of current copies."""
    n, C = 1000, 256
    r = np.random.default_rng(5)
    x, ho, hl, hr = [dev((r.standard_normal(n) * 0.02).astype(np.float32)) for _ in range(4)]
    hl0, hr0 = hl.clone(), hr.clone()
    out = torch.empty(n, device="cuda")
    bg.bagua_lp_apply_mix(x, ho, hl, hr, None, None, None, None, C, out)
    want = ((hl + ho) + hr) * torch.tensor(1.0 / 3.0, dtype=torch.float32, device="cuda") + (x - ho)
    torch.cuda.synchronize()
    assert torch.equal(out, want) and torch.equal(hl, hl0) and torch.equal(hr, hr0)
