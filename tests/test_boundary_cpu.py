"""The C-ABI library: loads, exports every symbol the header declares, and rejects invalid arguments
before touching the GPU (these calls return from host-side validation; no kernel is launched)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def bg():
    import paper_2107_01499_amd as b
    return b


def declared_functions():
    text = open(os.path.join(ROOT, "include", "bagua_hip.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bagua_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(bg):
    names = declared_functions()
    assert len(names) >= 10
    lib = ctypes.CDLL(bg.binding.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(bg.binding.EXPORTS)


def test_status_strings(bg):
    assert bg.status_string(0) == "BAGUA_OK"
    assert bg.status_string(1) == "BAGUA_ERR_INVALID_ARG"
    assert bg.status_string(2) == "BAGUA_ERR_ALIGNMENT"
    assert bg.status_string(3) == "BAGUA_ERR_LAUNCH"
    assert bg.status_string(4) == "BAGUA_ERR_UNSUPPORTED"
    assert bg.status_string(77) == "BAGUA_ERR_UNKNOWN"


def test_validation_errors_without_gpu(bg):
    lib = bg.binding.raw()
    # fake, 16-byte aligned "device pointers", far enough apart not to overlap; validation fails before any is used
    A, B, Cc, D, E = 0x100000, 0x200000, 0x300000, 0x400000, 0x500000
    INVALID, ALIGN = 1, 2
    # compress: NULL, n == 0, bad chunk sizes, misalignment, aliasing
    assert lib.bagua_compress_minmax_u8(None, None, 10, 256, B, Cc, None) == INVALID
    assert lib.bagua_compress_minmax_u8(A, None, 0, 256, B, Cc, None) == INVALID
    for chunk in (0, 100, 255, 300, 16384 + 256):
        assert lib.bagua_compress_minmax_u8(A, None, 10, chunk, B, Cc, None) == INVALID
    assert lib.bagua_compress_minmax_u8(A + 4, None, 10, 256, B, Cc, None) == ALIGN
    assert lib.bagua_compress_minmax_u8(A, D + 8, 10, 256, B, Cc, None) == ALIGN
    assert lib.bagua_compress_minmax_u8(A, A, 10, 256, B, Cc, None) == INVALID           # residual aliases x
    assert lib.bagua_compress_minmax_u8(A, D, 64, 256, A + 32, Cc, None) == INVALID      # codes inside x
    assert lib.bagua_compress_minmax_u8(A, D, 64, 256, B, D + 16, None) == INVALID       # minmax inside residual
    assert lib.bagua_sign_compress_ef(A, None, 10, 128, B, Cc, None) == INVALID
    assert lib.bagua_sign_compress_ef(A, None, 10, 256, B + 1, Cc, None) == ALIGN
    assert lib.bagua_sign_compress_ef(A, None, 64, 256, A, Cc, None) == INVALID          # bits alias x
    # d-r-r: k range, codec enum, NULL entries, outputs overlapping inputs
    arr = (ctypes.c_void_p * 33)(*[A + 0x1000 * i for i in range(33)])
    marr = (ctypes.c_void_p * 33)(*[B + 0x1000 * i for i in range(33)])
    assert lib.bagua_decompress_reduce_recompress(0, arr, marr, 0, None, 10, 256, Cc, D, None, None) == INVALID
    assert lib.bagua_decompress_reduce_recompress(0, arr, marr, 33, None, 10, 256, Cc, D, None, None) == INVALID
    assert lib.bagua_decompress_reduce_recompress(2, arr, marr, 2, None, 10, 256, Cc, D, None, None) == INVALID
    assert lib.bagua_decompress_reduce_recompress(0, arr, marr, 2, None, 10, 256, A + 0x1000, D, None, None) == INVALID  # out aliases in
    assert lib.bagua_decompress_reduce_recompress(0, arr, marr, 2, E, 10, 256, Cc, D, E + 16, None) == INVALID  # out overlaps eps
    arr2 = (ctypes.c_void_p * 2)(A, None)
    assert lib.bagua_decompress_reduce_recompress(0, arr2, marr, 2, None, 10, 256, Cc, D, None, None) == INVALID
    assert lib.bagua_decompress(0, A, B, 64, 256, A + 16, None) == INVALID                # out overlaps codes
    # decentralised: aliasing and mode
    xin = (ctypes.c_void_p * 2)(0x10000, 0x20000)
    xout = (ctypes.c_void_p * 2)(0x30000, 0x40000)
    assert lib.bagua_decentralized_avg(5, xin, xout, None, None, None, 2, 16, 0, None) == INVALID
    assert lib.bagua_decentralized_avg(0, xin, xin, None, None, None, 2, 16, 0, None) == INVALID
    assert lib.bagua_decentralized_avg(1, xin, xout, None, None, None, 2, 16, 256, None) == INVALID  # LP needs xhat
    assert lib.bagua_decentralized_avg(0, xin, xout, None, None, None, 0, 16, 0, None) == INVALID
    # LP mode: codes of one peer inside another peer's replica
    hat = (ctypes.c_void_p * 2)(0x50000, 0x60000)
    mm = (ctypes.c_void_p * 2)(0x90000, 0xa0000)
    assert lib.bagua_decentralized_avg(1, xin, xout, hat, (ctypes.c_void_p * 2)(0x70000, 0x10010), mm, 2, 16, 256, None) == INVALID
    # flatten: overlap, overflow, workspace too small
    src = (ctypes.c_void_p * 2)(A, A)
    numel = (ctypes.c_size_t * 2)(10, 10)
    assert lib.bagua_flatten_plan(src, numel, (ctypes.c_size_t * 2)(0, 5), 2, 100, A, 1 << 20, None) == INVALID
    assert lib.bagua_flatten_plan(src, numel, (ctypes.c_size_t * 2)(0, 95), 2, 100, A, 1 << 20, None) == INVALID
    assert lib.bagua_flatten_plan(src, numel, (ctypes.c_size_t * 2)(0, 10), 2, 100, A, 8, None) == INVALID
    assert lib.bagua_decompress(0, None, A, 10, 256, A, None) == INVALID
    assert bg.bagua_flatten_workspace_bytes(3, 10000) >= 3 * 24 + 4 * 4


def test_missing_library_fails_loudly(bg, monkeypatch):
    monkeypatch.setattr(bg.binding, "LIB_PATH", "/nonexistent/libbagua_hip.so")
    with pytest.raises(ImportError):
        bg.binding._load()


def test_peer_validation_without_gpu(bg):
    lib = bg.binding.raw()
    xin = (ctypes.c_void_p * 2)(0x10000, 0x20000)
    xout = (ctypes.c_void_p * 2)(0x30000, 0x40000)
    assert lib.bagua_decentralized_avg_peers(xin, xout, (ctypes.c_int * 2)(1, 2), 2, 16, None) == 1    # peer out of range
    assert lib.bagua_decentralized_avg_peers(xin, xin, (ctypes.c_int * 2)(1, 0), 2, 16, None) == 1     # aliasing
    assert lib.bagua_decentralized_avg_peers(xin, xout, None, 2, 16, None) == 1
    hat = (ctypes.c_void_p * 2)(0x50000, 0x60000)
    cd = (ctypes.c_void_p * 2)(0x70000, 0x80000)
    mm = (ctypes.c_void_p * 2)(0x90000, 0xa0000)
    ok_peer = (ctypes.c_int * 2)(1, 0)
    lp = lib.bagua_decentralized_avg_peers_lp
    assert lp(xin, xout, hat, cd, mm, (ctypes.c_int * 2)(1, -1), 2, 16, 256, None) == 1   # peer out of range
    assert lp(xin, xout, xin, cd, mm, ok_peer, 2, 16, 256, None) == 1                      # xhat aliases x_in
    assert lp(xin, xout, xout, cd, mm, ok_peer, 2, 16, 256, None) == 1                     # xhat aliases x_out
    assert lp(xin, xout, hat, cd, mm, ok_peer, 2, 16, 100, None) == 1                      # bad chunk
    assert lp(xin, xout, None, cd, mm, ok_peer, 2, 16, 256, None) == 1
    assert lp(xin, xout, hat, (ctypes.c_void_p * 2)(0x70004, 0x80000), mm, ok_peer, 2, 16, 256, None) == 2
    assert lib.bagua_decompress_sgd_step(0, 0x1000, 0x1000, 16, 256, 0x2000, 0x2000, 0.1, 0.9, 0.0, None) == 1  # param aliases momentum
    assert lib.bagua_decompress_sgd_step(3, 0x1000, 0x1000, 16, 256, 0x2000, None, 0.1, 0.9, 0.0, None) == 1
    assert lib.bagua_flatten_compress_minmax_u8(None, 1, None, 16, 256, 0x1000, 0x1000, None, None) == 1
    adam = lib.bagua_decompress_adam_step
    assert adam(0, 0x1000, 0x1000, 16, 256, 0x2000, 0x2000, 0x4000, 0.1, 0.9, 0.999, 1e-8, 0.0, 0, None) == 1  # m aliases param
    assert adam(0, 0x1000, 0x1000, 16, 256, 0x2000, 0x3000, 0x3020, 0.1, 0.9, 0.999, 1e-8, 0.0, 0, None) == 1  # v overlaps m
    assert adam(0, 0x1000, 0x1000, 16, 256, 0x2000, 0x3000, None, 0.1, 0.9, 0.999, 1e-8, 0.0, 1, None) == 1
    assert adam(2, 0x1000, 0x1000, 16, 256, 0x2000, 0x3000, 0x4000, 0.1, 0.9, 0.999, 1e-8, 0.0, 0, None) == 1
    assert adam(0, 0x1000, 0x1000, 16, 256, 0x2004, 0x3000, 0x4000, 0.1, 0.9, 0.999, 1e-8, 0.0, 0, None) == 2
    enc, mix = lib.bagua_lp_encode, lib.bagua_lp_apply_mix
    X, H, HL, HR, CL, ML, CR, MR, O = (0x100000 * i for i in range(1, 10))
    assert enc(X, X, 64, 256, CL, ML, None) == 1                                  # xhat aliases x
    assert enc(X, H, 64, 100, CL, ML, None) == 1
    assert enc(X, H + 4, 64, 256, CL, ML, None) == 2
    assert mix(X, H, HL, HR, CL, None, CR, MR, 64, 256, O, None) == 1             # codes without statistics
    assert mix(X, H, HL, HL, CL, ML, CR, MR, 64, 256, O, None) == 1               # one copy, two code streams
    assert mix(X, H, HL, HR, CL, ML, CR, MR, 64, 256, HL, None) == 1              # output aliases a copy
    assert mix(X, H, H, HR, CL, ML, CR, MR, 64, 256, O, None) == 1                # own copy would be advanced twice
    assert mix(X, H, HL, HR, CL, ML + 2, CR, MR, 64, 256, O, None) == 2
    ms = lib.bagua_momentum_sign_compress_ef
    assert ms(0x1000, None, 0.9, None, 16, 256, 0x5000, 0x6000, None) == 1
    assert ms(0x1000, 0x2000, 0.9, 0x1000, 16, 256, 0x5000, 0x6000, None) == 1      # residual aliases g
    assert ms(0x1000, 0x2000, 0.9, 0x3000, 16, 100, 0x5000, 0x6000, None) == 1
    assert ms(0x1000, 0x2008, 0.9, 0x3000, 16, 256, 0x5000, 0x6000, None) == 2


def test_header_is_valid_c_and_cpp(tmp_path):
    """include/bagua_hip.h is a plain C header: it must compile as C99 and as C++ without any HIP or torch include."""
    import subprocess
    src_c = tmp_path / "use_header.c"
    src_c.write_text('#include "bagua_hip.h"\nint main(void) { return BAGUA_MAX_WORKERS != 32; }\n')
    inc = os.path.join(ROOT, "include")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only", "-I", inc, str(src_c)], check=True)
    src_cpp = tmp_path / "use_header.cpp"
    src_cpp.write_text('#include "bagua_hip.h"\nint main() { return BAGUA_OK; }\n')
    subprocess.run(["g++", "-std=c++17", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-I", inc, str(src_cpp)], check=True)


def test_binding_refuses_per_worker_lists_of_unequal_length(bg):
    """The C side reads k pointers from every per-worker array, so the binding must refuse a shorter list before it
    builds the pointer arrays (the tensors here are never dereferenced: the length check comes first)."""
    import torch
    t = [torch.zeros(256) for _ in range(3)]
    u8 = [torch.zeros(256, dtype=torch.uint8) for _ in range(3)]
    with pytest.raises(ValueError, match="meta_in names 2"):
        bg.bagua_decompress_reduce_recompress(bg.CODEC_MINMAX_U8, u8, t[:2], None, 256, 256, u8[0], t[0])
    with pytest.raises(ValueError, match="x_out names 2"):
        bg.bagua_decentralized_avg(bg.AVG_FP, t, t[:2])
    with pytest.raises(ValueError, match="minmax names 1"):
        bg.bagua_decentralized_avg(bg.AVG_LP_MINMAX_U8, t, t, t, u8, t[:1], 256)
    with pytest.raises(ValueError, match="x_out names 4"):
        bg.bagua_decentralized_avg_peers(t, t + t[:1], [0, 1, 2])
    with pytest.raises(ValueError, match="codes names 2"):
        bg.bagua_decentralized_avg_peers_lp(t, t, t, u8[:2], t, [0, 1, 2], 256)
    i16 = [torch.zeros(8, dtype=torch.int16) for _ in range(3)]
    with pytest.raises(ValueError, match="val_in names 2"):
        bg.bagua_decompress_reduce_recompress_topk(i16, t[:2], 8, None, 256, 256, i16[0], t[0])


def test_validation_of_the_batched_and_fused_entry_points_without_gpu(bg):
    """Host-side checks of the entry points added after the first set: every call returns before anything is enqueued."""
    lib = bg.binding.raw()
    INVALID, ALIGN, UNSUPPORTED = 1, 2, 4
    A, B, Cc, D, W = 0x100000, 0x200000, 0x300000, 0x400000, 0x500000
    one = lambda v: (ctypes.c_void_p * 1)(v)
    n1, n0 = (ctypes.c_size_t * 1)(64), (ctypes.c_size_t * 1)(0)
    wsb = bg.bagua_batch_workspace_bytes(1, 0)
    assert wsb > 0 and bg.bagua_batch_workspace_bytes(3, 8) > bg.bagua_batch_workspace_bytes(3, 0)
    assert bg.bagua_batch_workspace_bytes(1, 33) == 0                                  # k out of range
    f = lib.bagua_compress_minmax_u8_batched
    assert f(one(A), None, n1, 1, 256, one(B), one(Cc), W, wsb - 1, None) == INVALID       # workspace too small
    assert f(one(A), None, n1, 0, 256, one(B), one(Cc), W, wsb, None) == INVALID           # no buckets
    assert f(one(A), None, n0, 1, 256, one(B), one(Cc), W, wsb, None) == INVALID           # empty bucket
    assert f(one(A), None, n1, 1, 100, one(B), one(Cc), W, wsb, None) == INVALID           # bad chunk
    assert f(one(A + 4), None, n1, 1, 256, one(B), one(Cc), W, wsb, None) == ALIGN
    assert f(one(A), None, n1, 1, 256, one(A), one(Cc), W, wsb, None) == INVALID           # codes alias x
    assert f(one(A), None, n1, 1, 256, one(B), one(Cc), A, wsb, None) == INVALID           # table over x
    g = lib.bagua_sign_compress_ef_batched
    assert g(one(A), one(None), n1, 1, 256, one(B), one(Cc), W, wsb, None) == INVALID      # residual array with a NULL entry
    assert g(one(A), None, n1, 1, 256, one(B + 2), one(Cc), W, wsb, None) == ALIGN
    h = lib.bagua_decompress_reduce_recompress_batched
    wk = bg.bagua_batch_workspace_bytes(1, 1)
    assert h(7, one(A), one(B), 1, None, n1, 1, 256, one(Cc), one(D), None, W, wk, None) == INVALID    # codec
    assert h(0, one(A), one(B), 0, None, n1, 1, 256, one(Cc), one(D), None, W, wk, None) == INVALID    # k
    assert h(0, one(A), one(B), 1, None, n1, 1, 256, one(A), one(D), None, W, wk, None) == INVALID     # output over input
    assert lib.bagua_bucket_flatten_batched_run(one(A), n1, one(B), n0, 1, W, wsb, None) == INVALID     # empty bucket
    # no-allocation flatten: limits
    assert lib.bagua_bucket_flatten_static(None, None, None, 0, A, 67108864 + 1, None) == UNSUPPORTED
    T = 4097
    arr, num, off = (ctypes.c_void_p * T)(), (ctypes.c_size_t * T)(), (ctypes.c_size_t * T)()
    assert lib.bagua_bucket_flatten_static(arr, num, off, T, A, 1 << 20, None) == UNSUPPORTED
    assert lib.bagua_bucket_flatten_static(None, None, None, 0, A + 4, 1024, None) == ALIGN
    # fused forms
    assert lib.bagua_flatten_sign_compress_ef(W, 1, None, 0, 256, B, Cc, None, None) == INVALID
    assert lib.bagua_flatten_sign_compress_ef(W, 1, None, 64, 256, B + 4, Cc, None, None) == ALIGN
    assert lib.bagua_decompress_unflatten(5, A, B, 64, 256, W, 1, None) == INVALID
    assert lib.bagua_decompress_unflatten(0, A, B, 64, 256, W + 8, 1, None) == ALIGN
    assert lib.bagua_reduce_compress_sign_ef(one(A), 0, None, 64, 256, B, Cc, None) == INVALID
    assert lib.bagua_reduce_compress_sign_ef(one(A), 1, None, 64, 256, A, Cc, None) == INVALID         # bits alias x
    assert lib.bagua_decompress_sgd_step_topk(A, B, 64, 256, 0, Cc, None, 0.1, 0.0, 0.0, None) == INVALID   # keep = 0
    assert lib.bagua_decompress_sgd_step_topk(A, B, 64, 256, 300, Cc, None, 0.1, 0.0, 0.0, None) == INVALID  # keep > chunk
    assert lib.bagua_decompress_sgd_step_topk(A, B, 64, 256, 8, Cc + 4, None, 0.1, 0.0, 0.0, None) == ALIGN
    at = lib.bagua_decompress_adam_step_topk
    assert at(A, B, 64, 256, 0, Cc, D, W, 0.1, 0.9, 0.999, 1e-8, 0.0, 0, None) == INVALID          # keep = 0
    assert at(A, B, 64, 256, 8, Cc, None, W, 0.1, 0.9, 0.999, 1e-8, 0.0, 0, None) == INVALID       # no momentum buffer
    assert at(A, B, 64, 256, 8, Cc, D, D, 0.1, 0.9, 0.999, 1e-8, 0.0, 0, None) == INVALID          # m aliases v
    assert at(A, B, 64, 256, 8, Cc, D + 4, W, 0.1, 0.9, 0.999, 1e-8, 0.0, 0, None) == ALIGN
    # probes
    assert lib.bagua_probe_read(None, 10, B, None) == INVALID
    assert lib.bagua_probe_streams(one(A), one(B), None, 1, 1, 0, 1, 100, None) == INVALID             # n not a multiple of 256
    three = (ctypes.c_void_p * 3)(A, Cc, D)
    assert lib.bagua_probe_streams(three, one(B), None, 3, 1, 0, 1, 256, None) == UNSUPPORTED            # combination not offered
