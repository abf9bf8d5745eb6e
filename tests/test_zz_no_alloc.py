"""bagua_bucket_flatten_static (no workspace, tensor table in the library's fixed device array) against
bagua_bucket_flatten on the same inputs: byte-identical buckets, on two calls in a row, the second with a
smaller layout (so the second must not see anything the first left in the shared table)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def bg():
    import paper_2107_01499_amd as b
    assert torch.cuda.is_available()
    return b


def layout(sizes, seed, tail):
    """Tensors at odd (4-byte aligned only) device addresses with small gaps between their bucket ranges."""
    r = np.random.default_rng(seed)
    offs, pos = [], 0
    for i, s in enumerate(sizes):
        pos += i % 3
        offs.append(pos)
        pos += s
    total = pos + tail
    arena = torch.zeros(sum(sizes) + 2 * len(sizes) + 8, device="cuda")
    gs, p = [], 1
    for s in sizes:
        t = arena[p:p + s]
        t.copy_(torch.from_numpy(r.standard_normal(s).astype(np.float32)))
        gs.append(t)
        p += s + 1
    return gs, offs, total


def both(bg, gs, offs, total):
    want = torch.full((total,), float("nan"), device="cuda")
    ws = torch.empty(bg.bagua_flatten_workspace_bytes(len(gs), total), dtype=torch.uint8, device="cuda")
    bg.bagua_bucket_flatten(gs, offs, want, ws)
    got = torch.full((total,), float("nan"), device="cuda")
    bg.bagua_bucket_flatten_static(gs, offs, got)
    torch.cuda.synchronize()
    return got.cpu().numpy().tobytes(), want.cpu().numpy().tobytes()


def test_static_flatten_equals_workspace_flatten_twice(bg):
    print("static flatten: 150 tensors, then 5 tensors", flush=True)
    big = [1, 7, 64, 1000, 3, 4096, 0, 129, 30522, 5] * 15            # 150 tensors: three descriptor launches
    got, want = both(bg, *layout(big, 1, 50))
    assert got == want
    small = [300, 0, 1025, 2, 77]                                      # fewer tensors, fewer tiles than before
    got, want = both(bg, *layout(small, 2, 3))
    assert got == want
    # an empty table zero-fills
    bucket = torch.full((5000,), float("nan"), device="cuda")
    bg.bagua_bucket_flatten_static([], [], bucket)
    assert not bucket.cpu().numpy().view(np.uint32).any()


def test_static_flatten_limits(bg):
    lib = bg.binding.raw()
    UNSUPPORTED = 4
    A = 0x100000
    assert lib.bagua_bucket_flatten_static(None, None, None, 0, A, 67108864 + 1, None) == UNSUPPORTED
    import ctypes
    T = 4097
    arr = (ctypes.c_void_p * T)()
    num = (ctypes.c_size_t * T)()
    off = (ctypes.c_size_t * T)()
    assert lib.bagua_bucket_flatten_static(arr, num, off, T, A, 1 << 20, None) == UNSUPPORTED


def test_static_flatten_and_batched_calls_under_graph_capture(bg, oracle):
    """What the no-allocation entry point is for: a flatten recorded into a HIP graph, followed by the batched
    compression and the batched server step of the same buckets (their bucket tables travel as kernel arguments, so
    they can be recorded too).  Three replays with fresh gradients and eager work in between; every replay must
    equal the oracle's chain with the error states carried along."""
    print("graph capture: static flatten + batched compress + batched server step", flush=True)
    C, k = 1024, 3
    sizes = [700, 0, 1025, 2, 3000, 77]
    r = np.random.default_rng(11)
    offs, pos = [], 0
    for i, s in enumerate(sizes):
        pos += i % 2
        offs.append(pos)
        pos += s
    total = pos + 9
    nc = bg.num_chunks(total, C)
    # k workers, each with its own layer tensors (sources only 4-byte aligned) and bucket
    arenas = [torch.zeros(sum(sizes) + 2 * len(sizes) + 8, device="cuda") for _ in range(k)]
    layers = []
    for j in range(k):
        gs, p = [], 1
        for s in sizes:
            gs.append(arenas[j][p:p + s])
            p += s + 1
        layers.append(gs)
    bucket = [torch.full((total,), float("nan"), device="cuda") for _ in range(k)]
    delta = [torch.zeros(total, device="cuda") for _ in range(k)]
    codes = [torch.empty(total, dtype=torch.uint8, device="cuda") for _ in range(k)]
    mm = [torch.empty(2 * nc, device="cuda") for _ in range(k)]
    eps, out = torch.zeros(total, device="cuda"), torch.empty(total, device="cuda")
    c2, m2 = torch.empty(total, dtype=torch.uint8, device="cuda"), torch.empty(2 * nc, device="cuda")
    ws1 = torch.empty(bg.bagua_batch_workspace_bytes(k, 0), dtype=torch.uint8, device="cuda")
    ws2 = torch.empty(bg.bagua_batch_workspace_bytes(1, k), dtype=torch.uint8, device="cuda")

    def step():
        for j in range(k):      # the shared table is rewritten by every call; calls on one stream are ordered
            bg.bagua_bucket_flatten_static(layers[j], offs, bucket[j])
        bg.bagua_compress_minmax_u8_batched(bucket, delta, C, codes, mm, ws1)
        bg.bagua_decompress_reduce_recompress_batched(bg.CODEC_MINMAX_U8, [codes], [mm], [eps], [total], C, [c2], [m2], [out], ws2)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                  # outside capture: the scratch address is looked up here
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for d in delta:
        d.zero_()
    eps.zero_()
    d_o = [np.zeros(total, np.float32) for _ in range(k)]
    e_o = np.zeros(total, np.float32)
    for it in range(3):
        srcs = [[(r.standard_normal(s) * 1e-3).astype(np.float32) for s in sizes] for _ in range(k)]
        for j in range(k):
            for t, a in zip(layers[j], srcs[j]):
                t.copy_(torch.from_numpy(a))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        flat = [oracle.bucket_flatten(srcs[j], offs, total) for j in range(k)]
        enc = [oracle.compress_minmax_u8(flat[j], d_o[j], C) for j in range(k)]
        co, mo, oo = oracle.drr_minmax_u8([e[0] for e in enc], [e[1] for e in enc], e_o, C)
        for j in range(k):
            assert bucket[j].cpu().numpy().tobytes() == flat[j].tobytes(), "replay %d bucket %d" % (it, j)
            assert delta[j].cpu().numpy().tobytes() == d_o[j].tobytes(), "replay %d delta %d" % (it, j)
        assert c2.cpu().numpy().tobytes() == co.tobytes(), "replay %d" % it
        assert m2.cpu().numpy().tobytes() == mo.tobytes(), "replay %d" % it
        assert out.cpu().numpy().tobytes() == oo.tobytes(), "replay %d" % it
        assert eps.cpu().numpy().tobytes() == e_o.tobytes(), "replay %d" % it
