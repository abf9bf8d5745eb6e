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
