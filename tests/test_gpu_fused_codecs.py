"""The remaining fusions around the flatten (Section 3.5): gather fused into the sign compression, and the final decode
fused into the inverse scatter.  Both against the oracle's composition of the unfused steps, bit for bit."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def bg():
    import paper_2107_01499_amd as b
    assert torch.cuda.is_available()
    return b


def host(t):
    return t.cpu().numpy()


def layout(seed, tail):
    """Tensors of awkward sizes at odd (4-byte aligned only) device addresses with gaps between their bucket ranges."""
    r = np.random.default_rng(seed)
    sizes = [1, 7, 64, 1000, 3, 4096, 0, 129, 30522, 5, 5, 5, 8191, 2, 70000, 256, 1024]
    srcs = [(r.standard_normal(s) * 1e-3).astype(np.float32) for s in sizes]
    offs, pos = [], 0
    for i, s in enumerate(sizes):
        pos += i % 3
        offs.append(pos)
        pos += s
    total = pos + tail
    arena = torch.zeros(sum(sizes) + 2 * len(sizes) + 8, device="cuda")
    gs, p = [], 1
    for s in srcs:
        t = arena[p:p + s.size]
        t.copy_(torch.from_numpy(s))
        gs.append(t)
        p += s.size + 1
    return srcs, gs, offs, total


@pytest.mark.parametrize("ef", [False, True])
@pytest.mark.parametrize("C", [256, 2048, 4096])
@pytest.mark.parametrize("want_bucket", [False, True])
def test_flatten_sign_compress_fused(bg, oracle, ef, C, want_bucket):
    print("flatten_sign_compress C=%d ef=%s bucket=%s" % (C, ef, want_bucket), flush=True)
    srcs, gs, offs, total = layout(C + ef, 77)
    ws = torch.empty(bg.bagua_flatten_workspace_bytes(len(gs), total), dtype=torch.uint8, device="cuda")
    bg.bagua_flatten_plan(gs, offs, total, ws)
    res = (np.random.default_rng(9).standard_normal(total) * 1e-4).astype(np.float32)
    rg = torch.from_numpy(res.copy()).cuda() if ef else None
    bits = torch.full(((total + 31) // 32,), -1, dtype=torch.int32, device="cuda")
    scale = torch.full((bg.num_chunks(total, C),), float("nan"), device="cuda")
    bucket = torch.full((total,), float("nan"), device="cuda") if want_bucket else None
    bg.bagua_flatten_sign_compress_ef(ws, len(gs), rg, total, C, bits, scale, bucket)
    torch.cuda.synchronize()
    flat = oracle.bucket_flatten(srcs, offs, total)
    ro = res.copy() if ef else None
    bo, so = oracle.sign_compress_ef(flat, ro, C)
    assert host(bits).view(np.uint32).tobytes() == bo.tobytes()
    assert host(scale).tobytes() == so.tobytes()
    if ef:
        assert host(rg).tobytes() == ro.tobytes()
    if want_bucket:
        assert host(bucket).tobytes() == flat.tobytes()


@pytest.mark.parametrize("codec", ["minmax", "sign"])
@pytest.mark.parametrize("C", [256, 768, 4096])
def test_decompress_unflatten_fused(bg, oracle, codec, C):
    print("decompress_unflatten %s C=%d" % (codec, C), flush=True)
    srcs, gs, offs, total = layout(3 * C, 41)
    x = (np.random.default_rng(C).standard_normal(total) * 1e-3).astype(np.float32)
    if codec == "minmax":
        codes, meta = oracle.compress_minmax_u8(x, None, C)
        dec = oracle.decompress_minmax_u8(codes, meta, C)
        cg, cid = torch.from_numpy(codes).cuda(), bg.CODEC_MINMAX_U8
    else:
        codes, meta = oracle.sign_compress_ef(x, None, C)
        dec = oracle.decompress_sign(codes, meta, total, C)
        cg, cid = torch.from_numpy(codes.view(np.int32)).cuda(), bg.CODEC_SIGN1
    want = [np.full(s.size, np.float32(7.0)) for s in srcs]
    oracle.bucket_unflatten(dec, want, offs)
    for t in gs:
        t.fill_(7.0)
    ws = torch.empty(bg.bagua_flatten_workspace_bytes(len(gs), total), dtype=torch.uint8, device="cuda")
    bg.bagua_flatten_plan(gs, offs, total, ws)
    bg.bagua_decompress_unflatten(cid, cg, torch.from_numpy(meta).cuda(), total, C, ws, len(gs))
    torch.cuda.synchronize()
    for i, (t, w) in enumerate(zip(gs, want)):
        assert host(t).tobytes() == w.tobytes(), "tensor %d" % i
    # the same through the unfused calls
    out = torch.empty(total, device="cuda")
    bg.bagua_decompress(cid, cg, torch.from_numpy(meta).cuda(), total, C, out)
    assert host(out).tobytes() == dec.tobytes()
