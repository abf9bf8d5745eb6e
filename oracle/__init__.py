"""ctypes front end of the CPU oracle (oracle/bagua_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
cpu_baseline leg.  The GPU package never imports this module.  All arrays are numpy,
C-contiguous, float32 / uint8 / uint32; in-out residuals and replicas are updated in place.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_lib = None

_c_sz = ctypes.c_size_t
_c_p = ctypes.c_void_p


def lib():
    """Load (building if necessary) the oracle shared library."""
    global _lib
    if _lib is None:
        # BAGUA_ORACLE_LIB: a test may point this module at another build of the oracle's source
        # (tests/test_oracle_mutants.py checks that the pins reject deliberately wrong builds).
        path = os.environ.get("BAGUA_ORACLE_LIB") or _build.LIB
        if not os.path.exists(path):
            if path != _build.LIB:
                raise FileNotFoundError(path)
            _build.build()
        _lib = ctypes.CDLL(path)
        for name in ("oracle_compress_minmax_u8", "oracle_decompress_minmax_u8", "oracle_drr_minmax_u8",
                     "oracle_ring_avg_fp", "oracle_ring_avg_lp", "oracle_sign_compress_ef",
                     "oracle_decompress_sign", "oracle_drr_sign", "oracle_bucket_flatten"):
            getattr(_lib, name).restype = ctypes.c_int
        _lib.oracle_compress_minmax_u8.argtypes = [_c_p, _c_p, _c_sz, _c_sz, _c_p, _c_p]
        _lib.oracle_decompress_minmax_u8.argtypes = [_c_p, _c_p, _c_sz, _c_sz, _c_p]
        _lib.oracle_drr_minmax_u8.argtypes = [_c_p, _c_p, ctypes.c_int, _c_p, _c_sz, _c_sz, _c_p, _c_p, _c_p]
        _lib.oracle_ring_avg_fp.argtypes = [_c_p, _c_p, ctypes.c_int, _c_sz]
        _lib.oracle_ring_avg_lp.argtypes = [_c_p, _c_p, _c_p, _c_p, _c_p, ctypes.c_int, _c_sz, _c_sz]
        _lib.oracle_sign_compress_ef.argtypes = [_c_p, _c_p, _c_sz, _c_sz, _c_p, _c_p]
        _lib.oracle_decompress_sign.argtypes = [_c_p, _c_p, _c_sz, _c_sz, _c_p]
        _lib.oracle_drr_sign.argtypes = [_c_p, _c_p, ctypes.c_int, _c_p, _c_sz, _c_sz, _c_p, _c_p, _c_p]
        _lib.oracle_bucket_flatten.argtypes = [_c_p, _c_p, _c_p, _c_sz, _c_p, _c_sz]
        _lib.oracle_set_threads.argtypes = [ctypes.c_int]
        _lib.oracle_get_threads.restype = ctypes.c_int
        _lib.oracle_max_threads.restype = ctypes.c_int
    return _lib


def set_threads(t):
    lib().oracle_set_threads(int(t))


def get_threads():
    return lib().oracle_get_threads()


def max_threads():
    return lib().oracle_max_threads()


def num_chunks(n, chunk):
    return (n + chunk - 1) // chunk if chunk > 0 else 0


def _chk(a, dtype):
    assert isinstance(a, np.ndarray) and a.dtype == dtype and a.flags["C_CONTIGUOUS"], (type(a), getattr(a, "dtype", None))
    return a.ctypes.data


def _ptr_array(arrays, dtype):
    ptrs = (ctypes.c_void_p * len(arrays))()
    for i, a in enumerate(arrays):
        ptrs[i] = _chk(a, dtype)
    return ptrs


def _ok(rc, what):
    if rc != 0:
        raise ValueError("%s: oracle status %d" % (what, rc))


def compress_minmax_u8(x, residual, chunk):
    """Worker side of C_LP_S with Q = MinMax-u8. Returns (codes, minmax); residual updated in place (or None)."""
    n = x.size
    codes = np.empty(n, np.uint8)
    minmax = np.empty(2 * num_chunks(n, chunk), np.float32)
    _ok(lib().oracle_compress_minmax_u8(_chk(x, np.float32), None if residual is None else _chk(residual, np.float32),
                                         n, chunk, _chk(codes, np.uint8), _chk(minmax, np.float32)), "compress_minmax_u8")
    return codes, minmax


def decompress_minmax_u8(codes, minmax, chunk):
    n = codes.size
    out = np.empty(n, np.float32)
    _ok(lib().oracle_decompress_minmax_u8(_chk(codes, np.uint8), _chk(minmax, np.float32), n, chunk,
                                           _chk(out, np.float32)), "decompress_minmax_u8")
    return out


def drr_minmax_u8(codes_in, minmax_in, server_residual, chunk, want_fp32=True):
    """Server side of C_LP_S with Q = MinMax-u8. Returns (codes', minmax', out_fp32 or None)."""
    k = len(codes_in)
    n = codes_in[0].size
    codes = np.empty(n, np.uint8)
    minmax = np.empty(2 * num_chunks(n, chunk), np.float32)
    out = np.empty(n, np.float32) if want_fp32 else None
    _ok(lib().oracle_drr_minmax_u8(_ptr_array(codes_in, np.uint8), _ptr_array(minmax_in, np.float32), k,
                                    None if server_residual is None else _chk(server_residual, np.float32),
                                    n, chunk, _chk(codes, np.uint8), _chk(minmax, np.float32),
                                    None if out is None else _chk(out, np.float32)), "drr_minmax_u8")
    return codes, minmax, out


def ring_avg_fp(x_in):
    """D_FP_S on a ring, averaged. Returns the list of new replicas."""
    k = len(x_in)
    n = x_in[0].size
    outs = [np.empty(n, np.float32) for _ in range(k)]
    _ok(lib().oracle_ring_avg_fp(_ptr_array(x_in, np.float32), _ptr_array(outs, np.float32), k, n), "ring_avg_fp")
    return outs


def ring_avg_lp(x_in, xhat, chunk):
    """D_LP_S on a ring, one round. xhat (list) is updated in place. Returns (x_out, codes, minmax) lists."""
    k = len(x_in)
    n = x_in[0].size
    nc = num_chunks(n, chunk)
    outs = [np.empty(n, np.float32) for _ in range(k)]
    codes = [np.empty(n, np.uint8) for _ in range(k)]
    minmax = [np.empty(2 * nc, np.float32) for _ in range(k)]
    _ok(lib().oracle_ring_avg_lp(_ptr_array(x_in, np.float32), _ptr_array(outs, np.float32),
                                  _ptr_array(xhat, np.float32), _ptr_array(codes, np.uint8),
                                  _ptr_array(minmax, np.float32), k, n, chunk), "ring_avg_lp")
    return outs, codes, minmax


def sign_compress_ef(x, residual, chunk):
    """Worker side of C_LP_S with Q = Sign-1bit. Returns (bits u32[ceil(n/32)], scale f32[nc])."""
    n = x.size
    bits = np.empty((n + 31) // 32, np.uint32)
    scale = np.empty(num_chunks(n, chunk), np.float32)
    _ok(lib().oracle_sign_compress_ef(_chk(x, np.float32), None if residual is None else _chk(residual, np.float32),
                                       n, chunk, _chk(bits, np.uint32), _chk(scale, np.float32)), "sign_compress_ef")
    return bits, scale


def decompress_sign(bits, scale, n, chunk):
    out = np.empty(n, np.float32)
    _ok(lib().oracle_decompress_sign(_chk(bits, np.uint32), _chk(scale, np.float32), n, chunk,
                                      _chk(out, np.float32)), "decompress_sign")
    return out


def drr_sign(bits_in, scale_in, server_residual, n, chunk, want_fp32=True):
    """Server side of C_LP_S with Q = Sign-1bit. Returns (bits', scale', out_fp32 or None)."""
    k = len(bits_in)
    bits = np.empty((n + 31) // 32, np.uint32)
    scale = np.empty(num_chunks(n, chunk), np.float32)
    out = np.empty(n, np.float32) if want_fp32 else None
    _ok(lib().oracle_drr_sign(_ptr_array(bits_in, np.uint32), _ptr_array(scale_in, np.float32), k,
                               None if server_residual is None else _chk(server_residual, np.float32),
                               n, chunk, _chk(bits, np.uint32), _chk(scale, np.float32),
                               None if out is None else _chk(out, np.float32)), "drr_sign")
    return bits, scale, out


def bucket_flatten(srcs, dst_offset, bucket_numel):
    """Flatten: copy every tensor to its element offset in a zero-filled bucket."""
    T = len(srcs)
    numel = (ctypes.c_size_t * max(T, 1))(*[s.size for s in srcs])
    offs = (ctypes.c_size_t * max(T, 1))(*[int(o) for o in dst_offset])
    bucket = np.empty(bucket_numel, np.float32)
    ptrs = (ctypes.c_void_p * max(T, 1))()
    for i, s in enumerate(srcs):
        ptrs[i] = _chk(s, np.float32) if s.size else None
    _ok(lib().oracle_bucket_flatten(ptrs, numel, offs, T, _chk(bucket, np.float32), bucket_numel), "bucket_flatten")
    return bucket


def decompress_sgd_step(codec, codes, meta, n, chunk, param, momentum_buf, lr, momentum=0.0, weight_decay=0.0):
    """Decode a compressed bucket and apply SGD (optional weight decay and momentum) in place on param / momentum_buf."""
    f = lib().oracle_decompress_sgd_step
    f.restype = ctypes.c_int
    f.argtypes = [ctypes.c_int, _c_p, _c_p, _c_sz, _c_sz, _c_p, _c_p, ctypes.c_float, ctypes.c_float, ctypes.c_float]
    cp = _chk(codes, np.uint8) if codec == 0 else _chk(codes, np.uint32)
    _ok(f(codec, cp, _chk(meta, np.float32), n, chunk, _chk(param, np.float32),
          None if momentum_buf is None else _chk(momentum_buf, np.float32), lr, momentum, weight_decay), "decompress_sgd_step")


def decompress_sgd_step_topk(idx, val, n, chunk, keep, param, momentum_buf, lr, momentum=0.0, weight_decay=0.0):
    """Decode of a top-K bucket fused with the SGD step on the flat bucket; param / momentum_buf updated in place."""
    f = lib().oracle_decompress_sgd_step_topk
    f.restype = ctypes.c_int
    f.argtypes = [_c_p, _c_p, _c_sz, _c_sz, _c_sz, _c_p, _c_p, ctypes.c_float, ctypes.c_float, ctypes.c_float]
    _ok(f(_chk(idx, np.uint16), _chk(val, np.float32), n, chunk, keep, _chk(param, np.float32),
          None if momentum_buf is None else _chk(momentum_buf, np.float32), lr, momentum, weight_decay),
        "decompress_sgd_step_topk")


def peer_avg_fp(x_in, peer):
    """D_FP_S with one chosen peer per worker: x_i' = (x_i + x_peer[i]) / 2. Returns the list of new replicas."""
    k = len(x_in)
    n = x_in[0].size
    outs = [np.empty(n, np.float32) for _ in range(k)]
    f = lib().oracle_peer_avg_fp
    f.restype = ctypes.c_int
    f.argtypes = [_c_p, _c_p, _c_p, ctypes.c_int, _c_sz]
    pa = (ctypes.c_int * k)(*[int(p) for p in peer])
    _ok(f(_ptr_array(x_in, np.float32), _ptr_array(outs, np.float32), pa, k, n), "peer_avg_fp")
    return outs


def reduce_compress_minmax_u8(xs, residual, chunk):
    """Intra-node stage of hierarchical C_LP_S: average k_local uncompressed buckets, then the leader compresses."""
    k, n = len(xs), xs[0].size
    codes = np.empty(n, np.uint8)
    minmax = np.empty(2 * num_chunks(n, chunk), np.float32)
    f = lib().oracle_reduce_compress_minmax_u8
    f.restype = ctypes.c_int
    f.argtypes = [_c_p, ctypes.c_int, _c_p, _c_sz, _c_sz, _c_p, _c_p]
    _ok(f(_ptr_array(xs, np.float32), k, None if residual is None else _chk(residual, np.float32), n, chunk,
          _chk(codes, np.uint8), _chk(minmax, np.float32)), "reduce_compress_minmax_u8")
    return codes, minmax


def reduce_compress_sign(xs, residual, chunk):
    """Intra-node stage of hierarchical C_LP_S with the 1-bit sign codec (Section 3.5 "Hierarchical Communications";
    Q of Section 4.1's 1-bit Adam): the k_local uncompressed buckets are averaged as in reduce_compress_minmax_u8
    (ascending order, one multiply by fl(1/k_local)), then the leader sign-compresses the average with its error
    state.  Written as that composition: centralized_avg_fp, then sign_compress_ef.  Returns (bits, scale)."""
    return sign_compress_ef(centralized_avg_fp(xs), residual, chunk)


def bucket_unflatten(bucket, dsts, src_offset):
    """Inverse of bucket_flatten: writes every tensor's range of the bucket into the given arrays (in place)."""
    T = len(dsts)
    numel = (ctypes.c_size_t * max(T, 1))(*[d.size for d in dsts])
    offs = (ctypes.c_size_t * max(T, 1))(*[int(o) for o in src_offset])
    ptrs = (ctypes.c_void_p * max(T, 1))()
    for i, d in enumerate(dsts):
        ptrs[i] = _chk(d, np.float32) if d.size else None
    f = lib().oracle_bucket_unflatten
    f.restype = ctypes.c_int
    f.argtypes = [_c_p, _c_sz, _c_p, _c_p, _c_p, _c_sz]
    _ok(f(_chk(bucket, np.float32), bucket.size, ptrs, numel, offs, T), "bucket_unflatten")


def compress_topk(x, residual, chunk, keep):
    """Worker side of C_LP_S with Q = per-chunk top-K. Returns (idx u16[nc*keep], val f32[nc*keep])."""
    n = x.size
    nc = num_chunks(n, chunk)
    idx = np.empty(nc * keep, np.uint16)
    val = np.empty(nc * keep, np.float32)
    f = lib().oracle_compress_topk
    f.restype = ctypes.c_int
    f.argtypes = [_c_p, _c_p, _c_sz, _c_sz, _c_sz, _c_p, _c_p]
    _ok(f(_chk(x, np.float32), None if residual is None else _chk(residual, np.float32), n, chunk, keep,
          _chk(idx, np.uint16), _chk(val, np.float32)), "compress_topk")
    return idx, val


def decompress_topk(idx, val, n, chunk, keep):
    out = np.empty(n, np.float32)
    f = lib().oracle_decompress_topk
    f.restype = ctypes.c_int
    f.argtypes = [_c_p, _c_p, _c_sz, _c_sz, _c_sz, _c_p]
    _ok(f(_chk(idx, np.uint16), _chk(val, np.float32), n, chunk, keep, _chk(out, np.float32)), "decompress_topk")
    return out


def drr_topk(idx_in, val_in, server_residual, n, chunk, keep, want_fp32=True):
    """Server side of C_LP_S with Q = top-K. Returns (idx', val', out_fp32 or None)."""
    k = len(idx_in)
    nc = num_chunks(n, chunk)
    idx = np.empty(nc * keep, np.uint16)
    val = np.empty(nc * keep, np.float32)
    out = np.empty(n, np.float32) if want_fp32 else None
    f = lib().oracle_drr_topk
    f.restype = ctypes.c_int
    f.argtypes = [_c_p, _c_p, ctypes.c_int, _c_p, _c_sz, _c_sz, _c_sz, _c_p, _c_p, _c_p]
    _ok(f(_ptr_array(idx_in, np.uint16), _ptr_array(val_in, np.float32), k,
          None if server_residual is None else _chk(server_residual, np.float32), n, chunk, keep,
          _chk(idx, np.uint16), _chk(val, np.float32), None if out is None else _chk(out, np.float32)), "drr_topk")
    return idx, val, out


def centralized_avg_fp(xs):
    """C_FP_S, averaged: (x_0 + x_1 + ...) * fl(1/k) in ascending order."""
    k, n = len(xs), xs[0].size
    out = np.empty(n, np.float32)
    f = lib().oracle_centralized_avg_fp
    f.restype = ctypes.c_int
    f.argtypes = [_c_p, ctypes.c_int, _c_sz, _c_p]
    _ok(f(_ptr_array(xs, np.float32), k, n, _chk(out, np.float32)), "centralized_avg_fp")
    return out


def peer_avg_lp(x_in, xhat, peer, chunk):
    """D_LP_S with one chosen peer per worker. xhat (list) is updated in place. Returns (x_out, codes, minmax) lists."""
    k, n = len(x_in), x_in[0].size
    nc = num_chunks(n, chunk)
    outs = [np.empty(n, np.float32) for _ in range(k)]
    codes = [np.empty(n, np.uint8) for _ in range(k)]
    minmax = [np.empty(2 * nc, np.float32) for _ in range(k)]
    f = lib().oracle_peer_avg_lp
    f.restype = ctypes.c_int
    f.argtypes = [_c_p, _c_p, _c_p, _c_p, _c_p, _c_p, ctypes.c_int, _c_sz, _c_sz]
    pa = (ctypes.c_int * k)(*[int(p) for p in peer])
    _ok(f(_ptr_array(x_in, np.float32), _ptr_array(outs, np.float32), _ptr_array(xhat, np.float32),
          _ptr_array(codes, np.uint8), _ptr_array(minmax, np.float32), pa, k, n, chunk), "peer_avg_lp")
    return outs, codes, minmax


def decompress_adam_step(codec, codes, meta, n, chunk, param, m, v, lr, beta1=0.9, beta2=0.999, eps=1e-8,
                         weight_decay=0.0, variance_frozen=False):
    """Decode a compressed bucket and apply the Adam-type update in place on param, m (and v unless frozen)."""
    f = lib().oracle_decompress_adam_step
    f.restype = ctypes.c_int
    cf = ctypes.c_float
    f.argtypes = [ctypes.c_int, _c_p, _c_p, _c_sz, _c_sz, _c_p, _c_p, _c_p, cf, cf, cf, cf, cf, ctypes.c_int]
    cp = _chk(codes, np.uint8) if codec == 0 else _chk(codes, np.uint32)
    _ok(f(codec, cp, _chk(meta, np.float32), n, chunk, _chk(param, np.float32), _chk(m, np.float32),
          _chk(v, np.float32), lr, beta1, beta2, eps, weight_decay, int(bool(variance_frozen))), "decompress_adam_step")


def decompress_adam_step_topk(idx, val, n, chunk, keep, param, m, v, lr, beta1=0.9, beta2=0.999, eps=1e-8,
                              weight_decay=0.0, variance_frozen=False):
    """Decode of a top-K bucket fused with the Adam-type update, in place on param, m (and v unless frozen)."""
    f = lib().oracle_decompress_adam_step_topk
    f.restype = ctypes.c_int
    cf = ctypes.c_float
    f.argtypes = [_c_p, _c_p, _c_sz, _c_sz, _c_sz, _c_p, _c_p, _c_p, cf, cf, cf, cf, cf, ctypes.c_int]
    _ok(f(_chk(idx, np.uint16), _chk(val, np.float32), n, chunk, keep, _chk(param, np.float32), _chk(m, np.float32),
          _chk(v, np.float32), lr, beta1, beta2, eps, weight_decay, int(bool(variance_frozen))), "decompress_adam_step_topk")


def momentum_sign_compress_ef(g, m, beta1, residual, chunk):
    """Sign-compress beta1*m + (1-beta1)*g with error feedback (residual updated in place). Returns (bits, scale)."""
    n = g.size
    bits = np.empty((n + 31) // 32, np.uint32)
    scale = np.empty(num_chunks(n, chunk), np.float32)
    f = lib().oracle_momentum_sign_compress_ef
    f.restype = ctypes.c_int
    f.argtypes = [_c_p, _c_p, ctypes.c_float, _c_p, _c_sz, _c_sz, _c_p, _c_p]
    _ok(f(_chk(g, np.float32), _chk(m, np.float32), beta1, None if residual is None else _chk(residual, np.float32),
          n, chunk, _chk(bits, np.uint32), _chk(scale, np.float32)), "momentum_sign_compress_ef")
    return bits, scale
