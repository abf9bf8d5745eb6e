"""GPU parity of decentralised averaging with chosen peers (random peer strategy) against the oracle."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def bg():
    import paper_2107_01499_amd as b
    assert torch.cuda.is_available()
    return b


@pytest.mark.parametrize("n", [1, 255, 1027, 70001])
@pytest.mark.parametrize("k,peer", [(1, [0]), (2, [1, 0]), (6, [3, 4, 5, 0, 1, 2]), (8, [1, 0, 3, 2, 5, 4, 7, 6]),
                                    (4, [0, 0, 0, 0]), (5, [1, 2, 3, 4, 0]), (7, [1, 0, 2, 4, 3, 6, 5]), (32, None)])
def test_peer_avg(bg, oracle, n, k, peer):
    r = np.random.default_rng(n + k)
    if peer is None:
        perm = r.permutation(k)
        peer = [0] * k
        for a, b in zip(perm[0::2], perm[1::2]):
            peer[a], peer[b] = int(b), int(a)
    print("peer_avg n=%d k=%d peer=%s" % (n, k, peer), flush=True)
    xs = [r.standard_normal(n).astype(np.float32) for _ in range(k)]
    want = oracle.peer_avg_fp(xs, peer)
    xg = [torch.from_numpy(x).cuda() for x in xs]
    og = [torch.full((n,), float("nan"), device="cuda") for _ in range(k)]
    bg.bagua_decentralized_avg_peers(xg, og, peer)
    torch.cuda.synchronize()
    for i in range(k):
        assert np.array_equal(og[i].cpu().numpy().view(np.uint32), want[i].view(np.uint32)), "peer %d" % i
        assert np.array_equal(xg[i].cpu().numpy(), xs[i])


def test_hypercube_rounds_on_gpu_equal_global_mean(bg):
    k, n = 8, 100000
    r = np.random.default_rng(0)
    xs = [r.standard_normal(n).astype(np.float32) for _ in range(k)]
    mean = np.mean(np.stack(xs).astype(np.float64), 0)
    cur = [torch.from_numpy(x).cuda() for x in xs]
    nxt = [torch.empty(n, device="cuda") for _ in range(k)]
    for bit in (1, 2, 4):
        bg.bagua_decentralized_avg_peers(cur, nxt, [i ^ bit for i in range(k)])
        cur, nxt = nxt, cur
    for i in range(k):
        assert np.max(np.abs(cur[i].cpu().numpy() - mean)) <= 4e-7 * max(1.0, np.max(np.abs(mean)))


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5, 8, 9, 32])
@pytest.mark.parametrize("n", [1, 255, 1027, 70001])
def test_centralized_avg_fp(bg, oracle, k, n):
    """C_FP_S average against the oracle, bit for bit (values chosen so that the summation order matters)."""
    r = np.random.default_rng(n + k)
    xs = [(r.standard_normal(n) * 10.0 ** r.integers(-3, 4)).astype(np.float32) for _ in range(k)]
    want = oracle.centralized_avg_fp(xs)
    out = torch.full((n,), float("nan"), device="cuda")
    bg.bagua_centralized_avg_fp([torch.from_numpy(x).cuda() for x in xs], out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy().view(np.uint32), want.view(np.uint32))


def _matching(r, k):
    perm = r.permutation(k)
    peer = [0] * k
    for a, b in zip(perm[0::2], perm[1::2]):
        peer[a], peer[b] = int(b), int(a)
    return peer


@pytest.mark.parametrize("n,chunk", [(1, 256), (255, 256), (4096 * 3 + 1027, 4096), (70001, 1024), (70001, 2048),
                                     (5000, 768), (2816 * 3 + 2000, 2816), (8192 * 2 + 300, 8192), (16384 + 5, 16384)])
@pytest.mark.parametrize("k,peer", [(2, [1, 0]), (6, [3, 4, 5, 0, 1, 2]), (8, "matching"), (32, "matching"),
                                    (1, [0]), (4, [0, 0, 0, 0]), (5, [1, 2, 3, 4, 0]), (7, [1, 0, 2, 4, 3, 6, 5])])
def test_peer_avg_lp(bg, oracle, n, chunk, k, peer):
    """D_LP_S with chosen peers: codes, (min,max), the advanced xhat and the outputs equal the oracle's, bit for
    bit, over two rounds (the second starts from the first's xhat).  Matchings with chunk <= 4096 run the fused
    pair kernel; every other case the two-pass path."""
    r = np.random.default_rng(n + 7 * k + chunk)
    if peer == "matching":
        peer = _matching(r, k)
    print("peer_avg_lp n=%d chunk=%d k=%d peer=%s" % (n, chunk, k, peer), flush=True)
    base = (r.standard_normal(n) * 0.02).astype(np.float32)
    xs = [(base + (r.standard_normal(n) * 1e-3).astype(np.float32)).astype(np.float32) for _ in range(k)]
    hat = [base.copy() for _ in range(k)]
    hat_g = [torch.from_numpy(base).cuda() for _ in range(k)]
    nc = (n + chunk - 1) // chunk
    for rnd in range(2):
        want, wcodes, wmm = oracle.peer_avg_lp(xs, hat, peer, chunk)
        xg = [torch.from_numpy(x).cuda() for x in xs]
        og = [torch.full((n,), float("nan"), device="cuda") for _ in range(k)]
        cg = [torch.full((n,), 77, dtype=torch.uint8, device="cuda") for _ in range(k)]
        mg = [torch.full((2 * nc,), float("nan"), device="cuda") for _ in range(k)]
        bg.bagua_decentralized_avg_peers_lp(xg, og, hat_g, cg, mg, peer, chunk)
        torch.cuda.synchronize()
        for i in range(k):
            tag = "round %d peer %d" % (rnd, i)
            assert np.array_equal(cg[i].cpu().numpy(), wcodes[i]), tag
            assert np.array_equal(mg[i].cpu().numpy().view(np.uint32), wmm[i].view(np.uint32)), tag
            assert np.array_equal(hat_g[i].cpu().numpy().view(np.uint32), hat[i].view(np.uint32)), tag
            assert np.array_equal(og[i].cpu().numpy().view(np.uint32), want[i].view(np.uint32)), tag
            assert np.array_equal(xg[i].cpu().numpy(), xs[i]), tag
        xs = [(w - np.float32(0.01) * (r.standard_normal(n) * 1e-2).astype(np.float32)).astype(np.float32) for w in want]
