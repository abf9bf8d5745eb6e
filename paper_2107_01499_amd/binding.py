"""Thin ctypes binding of libbagua_hip.so (include/bagua_hip.h).

Argument marshalling only: every function takes torch tensors that already live on the GPU,
passes their device pointers and the current HIP stream to the C entry point of the same name,
and raises BaguaError on a non-zero status.  PyTorch is used for device memory and streams;
no arithmetic of the method happens in Python and there is no CPU fallback: if the shared
library is missing, importing this module fails.
"""
import ctypes
import os

import torch  # noqa: F401  (must be imported before the library so that both share one HIP runtime)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "lib", "libbagua_hip.so")

CODEC_MINMAX_U8 = 0
CODEC_SIGN1 = 1
AVG_FP = 0
AVG_LP_MINMAX_U8 = 1
MAX_WORKERS = 32

EXPORTS = (
    "bagua_status_string", "bagua_flatten_workspace_bytes", "bagua_flatten_plan", "bagua_bucket_flatten_run",
    "bagua_bucket_flatten", "bagua_compress_minmax_u8", "bagua_decompress_reduce_recompress",
    "bagua_decentralized_avg", "bagua_sign_compress_ef", "bagua_decompress", "bagua_flatten_compress_minmax_u8",
    "bagua_decompress_sgd_step", "bagua_decentralized_avg_peers", "bagua_reduce_compress_minmax_u8",
    "bagua_bucket_unflatten_run", "bagua_compress_topk_ef", "bagua_decompress_reduce_recompress_topk",
    "bagua_decompress_topk", "bagua_centralized_avg_fp", "bagua_decentralized_avg_peers_lp",
    "bagua_decompress_adam_step", "bagua_momentum_sign_compress_ef", "bagua_lp_encode", "bagua_lp_apply_mix", "bagua_bucket_flatten_static",
    "bagua_batch_workspace_bytes", "bagua_compress_minmax_u8_batched", "bagua_sign_compress_ef_batched",
    "bagua_decompress_reduce_recompress_batched", "bagua_bucket_flatten_batched_run", "bagua_probe_read",
    "bagua_probe_streams", "bagua_flatten_sign_compress_ef", "bagua_decompress_unflatten", "bagua_reduce_compress_sign_ef", "bagua_decompress_sgd_step_topk", "bagua_decompress_adam_step_topk",
)


class BaguaError(RuntimeError):
    def __init__(self, fn, status):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (fn, status_string(status), status))


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError("libbagua_hip.so is not built (%s missing); run __graft_entry__.build() or "
                          "python paper_2107_01499_amd/build.py" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    sz, vp, i32 = ctypes.c_size_t, ctypes.c_void_p, ctypes.c_int
    lib.bagua_status_string.restype = ctypes.c_char_p
    lib.bagua_status_string.argtypes = [i32]
    lib.bagua_flatten_workspace_bytes.restype = sz
    lib.bagua_flatten_workspace_bytes.argtypes = [sz, sz]
    lib.bagua_flatten_plan.argtypes = [vp, vp, vp, sz, sz, vp, sz, vp]
    lib.bagua_bucket_flatten_run.argtypes = [vp, sz, vp, sz, vp]
    lib.bagua_compress_topk_ef.argtypes = [vp, vp, sz, sz, sz, vp, vp, vp]
    lib.bagua_decompress_reduce_recompress_topk.argtypes = [vp, vp, i32, sz, vp, sz, sz, vp, vp, vp, vp]
    lib.bagua_decompress_topk.argtypes = [vp, vp, sz, sz, sz, vp, vp]
    lib.bagua_bucket_unflatten_run.argtypes = [vp, sz, vp, sz, vp]
    lib.bagua_bucket_flatten.argtypes = [vp, vp, vp, sz, vp, sz, vp, sz, vp]
    lib.bagua_bucket_flatten_static.argtypes = [vp, vp, vp, sz, vp, sz, vp]
    lib.bagua_compress_minmax_u8.argtypes = [vp, vp, sz, sz, vp, vp, vp]
    lib.bagua_decompress_reduce_recompress.argtypes = [i32, vp, vp, i32, vp, sz, sz, vp, vp, vp, vp]
    lib.bagua_decentralized_avg.argtypes = [i32, vp, vp, vp, vp, vp, i32, sz, sz, vp]
    lib.bagua_sign_compress_ef.argtypes = [vp, vp, sz, sz, vp, vp, vp]
    lib.bagua_decompress.argtypes = [i32, vp, vp, sz, sz, vp, vp]
    lib.bagua_flatten_compress_minmax_u8.argtypes = [vp, sz, vp, sz, sz, vp, vp, vp, vp]
    lib.bagua_reduce_compress_minmax_u8.argtypes = [vp, i32, vp, sz, sz, vp, vp, vp]
    lib.bagua_centralized_avg_fp.argtypes = [vp, i32, sz, vp, vp]
    lib.bagua_decentralized_avg_peers.argtypes = [vp, vp, vp, i32, sz, vp]
    lib.bagua_decentralized_avg_peers_lp.argtypes = [vp, vp, vp, vp, vp, vp, i32, sz, sz, vp]
    lib.bagua_decompress_sgd_step.argtypes = [i32, vp, vp, sz, sz, vp, vp, ctypes.c_float, ctypes.c_float,
                                              ctypes.c_float, vp]
    cf = ctypes.c_float
    lib.bagua_decompress_adam_step.argtypes = [i32, vp, vp, sz, sz, vp, vp, vp, cf, cf, cf, cf, cf, i32, vp]
    lib.bagua_momentum_sign_compress_ef.argtypes = [vp, vp, cf, vp, sz, sz, vp, vp, vp]
    lib.bagua_lp_encode.argtypes = [vp, vp, sz, sz, vp, vp, vp]
    lib.bagua_lp_apply_mix.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, sz, sz, vp, vp]
    lib.bagua_flatten_sign_compress_ef.argtypes = [vp, sz, vp, sz, sz, vp, vp, vp, vp]
    lib.bagua_decompress_unflatten.argtypes = [i32, vp, vp, sz, sz, vp, sz, vp]
    lib.bagua_reduce_compress_sign_ef.argtypes = [vp, i32, vp, sz, sz, vp, vp, vp]
    lib.bagua_decompress_sgd_step_topk.argtypes = [vp, vp, sz, sz, sz, vp, vp, ctypes.c_float, ctypes.c_float,
                                                   ctypes.c_float, vp]
    lib.bagua_decompress_adam_step_topk.argtypes = [vp, vp, sz, sz, sz, vp, vp, vp, cf, cf, cf, cf, cf, i32, vp]
    lib.bagua_probe_read.argtypes = [vp, sz, vp, vp]
    lib.bagua_probe_streams.argtypes = [vp, vp, vp, i32, i32, i32, i32, sz, vp]
    lib.bagua_batch_workspace_bytes.argtypes = [sz, i32]
    lib.bagua_compress_minmax_u8_batched.argtypes = [vp, vp, vp, sz, sz, vp, vp, vp, sz, vp]
    lib.bagua_sign_compress_ef_batched.argtypes = [vp, vp, vp, sz, sz, vp, vp, vp, sz, vp]
    lib.bagua_decompress_reduce_recompress_batched.argtypes = [i32, vp, vp, i32, vp, vp, sz, sz, vp, vp, vp, vp, sz, vp]
    lib.bagua_bucket_flatten_batched_run.argtypes = [vp, vp, vp, vp, sz, vp, sz, vp]
    for name in EXPORTS[2:]:
        if name != "bagua_batch_workspace_bytes":
            getattr(lib, name).restype = i32
    lib.bagua_batch_workspace_bytes.restype = sz
    return lib


_lib = _load()


def status_string(status):
    return _lib.bagua_status_string(int(status)).decode()


def _check(fn, rc):
    if rc != 0:
        raise BaguaError(fn, rc)


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _ptr(t, dtype=None, nbytes=None):
    """Device pointer of a tensor (None passes through).  nbytes: the number of bytes the entry point will read or
    write through this pointer; a smaller tensor is refused here, because the C side sees only the pointer."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous GPU tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError("expected dtype %s, got %s" % (dtype, t.dtype))
    if nbytes is not None and t.numel() * t.element_size() < nbytes:
        raise ValueError("tensor of %d bytes is too small: the call needs %d bytes" % (t.numel() * t.element_size(), nbytes))
    return ctypes.c_void_p(t.data_ptr())


def _ptr_array(tensors, dtype=None, nbytes=None):
    arr = (ctypes.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i] = None if t is None else _ptr(t, dtype, nbytes).value
    return arr


def _same_len(k, **lists):
    """Every per-worker list of a call must name exactly k tensors: the C side reads k pointers from each array."""
    for name, lst in lists.items():
        if lst is not None and len(lst) != k:
            raise ValueError("%s names %d tensors, expected %d (one per worker)" % (name, len(lst), k))


def num_chunks(n, chunk):
    return (n + chunk - 1) // chunk if chunk > 0 else 0


def _code_bytes(codec, n):
    """Bytes of the code stream of n elements: one byte each (MinMax-u8) or one bit each in 32-bit words (sign)."""
    return n if codec == CODEC_MINMAX_U8 else 4 * ((n + 31) // 32)


def _meta_bytes(codec, n, chunk):
    """Bytes of the per-chunk metadata: (min, max) pairs (MinMax-u8) or one scale (sign)."""
    return 4 * num_chunks(n, chunk) * (2 if codec == CODEC_MINMAX_U8 else 1)


def bagua_flatten_workspace_bytes(T, bucket_numel):
    return int(_lib.bagua_flatten_workspace_bytes(T, bucket_numel))


def _flatten_args(srcs, dst_offset):
    T = len(srcs)
    ptrs = (ctypes.c_void_p * max(T, 1))()
    numel = (ctypes.c_size_t * max(T, 1))()
    offs = (ctypes.c_size_t * max(T, 1))()
    for i, s in enumerate(srcs):
        if s.dtype != torch.float32 or not s.is_cuda or not s.is_contiguous():
            raise ValueError("flatten sources must be contiguous fp32 GPU tensors")
        ptrs[i] = s.data_ptr() if s.numel() else None
        numel[i] = s.numel()
        offs[i] = int(dst_offset[i])
    return T, ptrs, numel, offs


def bagua_flatten_plan(srcs, dst_offset, bucket_numel, workspace, stream=None):
    """Upload the tensor table of one bucket into `workspace` (uint8 GPU tensor). Synchronises the stream."""
    T, ptrs, numel, offs = _flatten_args(srcs, dst_offset)
    _check("bagua_flatten_plan", _lib.bagua_flatten_plan(ptrs, numel, offs, T, bucket_numel, _ptr(workspace),
                                                         workspace.numel() * workspace.element_size(), _stream(stream)))


def bagua_bucket_flatten_run(workspace, T, bucket, stream=None):
    _check("bagua_bucket_flatten_run", _lib.bagua_bucket_flatten_run(_ptr(workspace), T, _ptr(bucket, torch.float32),
                                                                     bucket.numel(), _stream(stream)))


def bagua_bucket_unflatten_run(workspace, T, bucket, stream=None):
    """Inverse of the flatten: scatter the bucket back into the tensors the workspace was planned with."""
    _check("bagua_bucket_unflatten_run", _lib.bagua_bucket_unflatten_run(_ptr(workspace), T, _ptr(bucket, torch.float32),
                                                                         bucket.numel(), _stream(stream)))


def bagua_bucket_flatten(srcs, dst_offset, bucket, workspace, stream=None):
    T, ptrs, numel, offs = _flatten_args(srcs, dst_offset)
    _check("bagua_bucket_flatten", _lib.bagua_bucket_flatten(ptrs, numel, offs, T, _ptr(bucket, torch.float32),
                                                             bucket.numel(), _ptr(workspace),
                                                             workspace.numel() * workspace.element_size(),
                                                             _stream(stream)))


def bagua_bucket_flatten_static(srcs, dst_offset, bucket, stream=None):
    """bagua_bucket_flatten with the tensor table in the library's own fixed device array (no workspace)."""
    T, ptrs, numel, offs = _flatten_args(srcs, dst_offset)
    _check("bagua_bucket_flatten_static", _lib.bagua_bucket_flatten_static(
        ptrs, numel, offs, T, _ptr(bucket, torch.float32), bucket.numel(), _stream(stream)))


def bagua_compress_minmax_u8(x, residual, chunk, codes, minmax, stream=None):
    _check("bagua_compress_minmax_u8", _lib.bagua_compress_minmax_u8(
        _ptr(x, torch.float32), _ptr(residual, torch.float32, 4 * x.numel()), x.numel(), chunk,
        _ptr(codes, torch.uint8, x.numel()), _ptr(minmax, torch.float32, 8 * num_chunks(x.numel(), chunk)),
        _stream(stream)))


def bagua_flatten_compress_minmax_u8(workspace, T, residual, n, chunk, codes, minmax, bucket_out=None, stream=None):
    _check("bagua_flatten_compress_minmax_u8", _lib.bagua_flatten_compress_minmax_u8(
        _ptr(workspace), T, _ptr(residual, torch.float32, 4 * n), n, chunk, _ptr(codes, torch.uint8, n),
        _ptr(minmax, torch.float32, 8 * num_chunks(n, chunk)), _ptr(bucket_out, torch.float32, 4 * n), _stream(stream)))


def bagua_flatten_sign_compress_ef(workspace, T, residual, n, chunk, bits, scale, bucket_out=None, stream=None):
    _check("bagua_flatten_sign_compress_ef", _lib.bagua_flatten_sign_compress_ef(
        _ptr(workspace), T, _ptr(residual, torch.float32, 4 * n), n, chunk, _ptr(bits, torch.int32, _code_bytes(CODEC_SIGN1, n)),
        _ptr(scale, torch.float32, _meta_bytes(CODEC_SIGN1, n, chunk)), _ptr(bucket_out, torch.float32, 4 * n), _stream(stream)))


def bagua_decompress_unflatten(codec, codes, meta, n, chunk, workspace, T, stream=None):
    """Decode a compressed bucket straight into the tensors the workspace was planned with."""
    _check("bagua_decompress_unflatten", _lib.bagua_decompress_unflatten(
        codec, _ptr(codes, None, _code_bytes(codec, n)), _ptr(meta, torch.float32, _meta_bytes(codec, n, chunk)), n, chunk,
        _ptr(workspace), T, _stream(stream)))


def bagua_decompress_reduce_recompress(codec, codes_in, meta_in, server_residual, n, chunk, codes_out, meta_out,
                                       out_fp32=None, stream=None):
    k = len(codes_in)
    _same_len(k, meta_in=meta_in)
    _check("bagua_decompress_reduce_recompress", _lib.bagua_decompress_reduce_recompress(
        codec, _ptr_array(codes_in, None, _code_bytes(codec, n)),
        _ptr_array(meta_in, torch.float32, _meta_bytes(codec, n, chunk)), k, _ptr(server_residual, torch.float32, 4 * n),
        n, chunk, _ptr(codes_out, None, _code_bytes(codec, n)), _ptr(meta_out, torch.float32, _meta_bytes(codec, n, chunk)),
        _ptr(out_fp32, torch.float32, 4 * n), _stream(stream)))


def bagua_decentralized_avg(mode, x_in, x_out, xhat=None, codes=None, minmax=None, chunk=0, stream=None):
    k = len(x_in)
    n = x_in[0].numel()
    _same_len(k, x_out=x_out, xhat=xhat, codes=codes, minmax=minmax)
    _check("bagua_decentralized_avg", _lib.bagua_decentralized_avg(
        mode, _ptr_array(x_in, torch.float32, 4 * n), _ptr_array(x_out, torch.float32, 4 * n),
        None if xhat is None else _ptr_array(xhat, torch.float32, 4 * n),
        None if codes is None else _ptr_array(codes, torch.uint8, n),
        None if minmax is None else _ptr_array(minmax, torch.float32, 8 * num_chunks(n, chunk)), k, n, chunk,
        _stream(stream)))


def bagua_lp_encode(x, xhat, chunk, codes, minmax, stream=None):
    n = x.numel()
    _check("bagua_lp_encode", _lib.bagua_lp_encode(
        _ptr(x, torch.float32), _ptr(xhat, torch.float32, 4 * n), n, chunk, _ptr(codes, torch.uint8, n),
        _ptr(minmax, torch.float32, 8 * num_chunks(n, chunk)), _stream(stream)))


def bagua_lp_apply_mix(x, xhat_own, xhat_left, xhat_right, codes_left, minmax_left, codes_right, minmax_right, chunk,
                       x_out, stream=None):
    n = x.numel()
    mb = 8 * num_chunks(n, chunk)
    _check("bagua_lp_apply_mix", _lib.bagua_lp_apply_mix(
        _ptr(x, torch.float32), _ptr(xhat_own, torch.float32, 4 * n), _ptr(xhat_left, torch.float32, 4 * n),
        _ptr(xhat_right, torch.float32, 4 * n), _ptr(codes_left, torch.uint8, n), _ptr(minmax_left, torch.float32, mb),
        _ptr(codes_right, torch.uint8, n), _ptr(minmax_right, torch.float32, mb), n, chunk,
        _ptr(x_out, torch.float32, 4 * n), _stream(stream)))


def bagua_reduce_compress_minmax_u8(xs, residual, chunk, codes, minmax, stream=None):
    n = xs[0].numel()
    _check("bagua_reduce_compress_minmax_u8", _lib.bagua_reduce_compress_minmax_u8(
        _ptr_array(xs, torch.float32, 4 * n), len(xs), _ptr(residual, torch.float32, 4 * n), n, chunk,
        _ptr(codes, torch.uint8, n), _ptr(minmax, torch.float32, 8 * num_chunks(n, chunk)), _stream(stream)))


def bagua_reduce_compress_sign_ef(xs, residual, chunk, bits, scale, stream=None):
    n = xs[0].numel()
    _check("bagua_reduce_compress_sign_ef", _lib.bagua_reduce_compress_sign_ef(
        _ptr_array(xs, torch.float32, 4 * n), len(xs), _ptr(residual, torch.float32, 4 * n), n, chunk,
        _ptr(bits, torch.int32, _code_bytes(CODEC_SIGN1, n)), _ptr(scale, torch.float32, _meta_bytes(CODEC_SIGN1, n, chunk)),
        _stream(stream)))


def bagua_centralized_avg_fp(xs, out, stream=None):
    n = xs[0].numel()
    _check("bagua_centralized_avg_fp", _lib.bagua_centralized_avg_fp(_ptr_array(xs, torch.float32, 4 * n), len(xs), n,
                                                                     _ptr(out, torch.float32, 4 * n), _stream(stream)))


def bagua_decentralized_avg_peers(x_in, x_out, peer, stream=None):
    k, n = len(x_in), x_in[0].numel()
    if len(peer) != k:
        raise ValueError("peer must name one peer per worker")
    _same_len(k, x_out=x_out)
    pa = (ctypes.c_int * k)(*[int(p) for p in peer])
    _check("bagua_decentralized_avg_peers", _lib.bagua_decentralized_avg_peers(
        _ptr_array(x_in, torch.float32, 4 * n), _ptr_array(x_out, torch.float32, 4 * n), pa, k, n, _stream(stream)))


def bagua_decentralized_avg_peers_lp(x_in, x_out, xhat, codes, minmax, peer, chunk, stream=None):
    k, n = len(x_in), x_in[0].numel()
    if len(peer) != k:
        raise ValueError("peer must name one peer per worker")
    _same_len(k, x_out=x_out, xhat=xhat, codes=codes, minmax=minmax)
    pa = (ctypes.c_int * k)(*[int(p) for p in peer])
    _check("bagua_decentralized_avg_peers_lp", _lib.bagua_decentralized_avg_peers_lp(
        _ptr_array(x_in, torch.float32, 4 * n), _ptr_array(x_out, torch.float32, 4 * n),
        _ptr_array(xhat, torch.float32, 4 * n), _ptr_array(codes, torch.uint8, n),
        _ptr_array(minmax, torch.float32, 8 * num_chunks(n, chunk)), pa, k, n, chunk, _stream(stream)))


def bagua_decompress_adam_step(codec, codes, meta, n, chunk, param, m, v, lr, beta1=0.9, beta2=0.999, eps=1e-8,
                               weight_decay=0.0, variance_frozen=False, stream=None):
    _check("bagua_decompress_adam_step", _lib.bagua_decompress_adam_step(
        codec, _ptr(codes, None, _code_bytes(codec, n)), _ptr(meta, torch.float32, _meta_bytes(codec, n, chunk)), n, chunk,
        _ptr(param, torch.float32, 4 * n), _ptr(m, torch.float32, 4 * n), _ptr(v, torch.float32, 4 * n), lr, beta1, beta2, eps, weight_decay, int(bool(variance_frozen)), _stream(stream)))


def bagua_momentum_sign_compress_ef(g, m, beta1, residual, chunk, bits, scale, stream=None):
    _check("bagua_momentum_sign_compress_ef", _lib.bagua_momentum_sign_compress_ef(
        _ptr(g, torch.float32), _ptr(m, torch.float32, 4 * g.numel()), beta1, _ptr(residual, torch.float32, 4 * g.numel()),
        g.numel(), chunk, _ptr(bits, torch.int32, _code_bytes(CODEC_SIGN1, g.numel())),
        _ptr(scale, torch.float32, _meta_bytes(CODEC_SIGN1, g.numel(), chunk)), _stream(stream)))


def bagua_sign_compress_ef(x, residual, chunk, bits, scale, stream=None):
    _check("bagua_sign_compress_ef", _lib.bagua_sign_compress_ef(
        _ptr(x, torch.float32), _ptr(residual, torch.float32, 4 * x.numel()), x.numel(), chunk,
        _ptr(bits, torch.int32, _code_bytes(CODEC_SIGN1, x.numel())),
        _ptr(scale, torch.float32, _meta_bytes(CODEC_SIGN1, x.numel(), chunk)), _stream(stream)))


def bagua_decompress(codec, codes, meta, n, chunk, out, stream=None):
    _check("bagua_decompress", _lib.bagua_decompress(codec, _ptr(codes, None, _code_bytes(codec, n)),
                                                     _ptr(meta, torch.float32, _meta_bytes(codec, n, chunk)), n, chunk,
                                                     _ptr(out, torch.float32, 4 * n), _stream(stream)))


def bagua_decompress_sgd_step(codec, codes, meta, n, chunk, param, momentum_buf, lr, momentum=0.0, weight_decay=0.0,
                              stream=None):
    _check("bagua_decompress_sgd_step", _lib.bagua_decompress_sgd_step(
        codec, _ptr(codes, None, _code_bytes(codec, n)), _ptr(meta, torch.float32, _meta_bytes(codec, n, chunk)), n, chunk,
        _ptr(param, torch.float32, 4 * n), _ptr(momentum_buf, torch.float32, 4 * n), lr, momentum, weight_decay,
        _stream(stream)))


def bagua_decompress_sgd_step_topk(idx, val, n, chunk, keep, param, momentum_buf, lr, momentum=0.0, weight_decay=0.0,
                                   stream=None):
    _check("bagua_decompress_sgd_step_topk", _lib.bagua_decompress_sgd_step_topk(
        _ptr(idx, torch.int16, 2 * keep * num_chunks(n, chunk)), _ptr(val, torch.float32, 4 * keep * num_chunks(n, chunk)),
        n, chunk, keep, _ptr(param, torch.float32, 4 * n), _ptr(momentum_buf, torch.float32, 4 * n), lr, momentum,
        weight_decay, _stream(stream)))


def bagua_decompress_adam_step_topk(idx, val, n, chunk, keep, param, m, v, lr, beta1=0.9, beta2=0.999, eps=1e-8,
                                    weight_decay=0.0, variance_frozen=False, stream=None):
    _check("bagua_decompress_adam_step_topk", _lib.bagua_decompress_adam_step_topk(
        _ptr(idx, torch.int16, 2 * keep * num_chunks(n, chunk)), _ptr(val, torch.float32, 4 * keep * num_chunks(n, chunk)),
        n, chunk, keep, _ptr(param, torch.float32, 4 * n), _ptr(m, torch.float32, 4 * n), _ptr(v, torch.float32, 4 * n),
        lr, beta1, beta2, eps, weight_decay, int(bool(variance_frozen)), _stream(stream)))


def bagua_compress_topk_ef(x, residual, chunk, keep, idx, val, stream=None):
    _check("bagua_compress_topk_ef", _lib.bagua_compress_topk_ef(
        _ptr(x, torch.float32), _ptr(residual, torch.float32, 4 * x.numel()), x.numel(), chunk, keep,
        _ptr(idx, torch.int16, 2 * keep * num_chunks(x.numel(), chunk)),
        _ptr(val, torch.float32, 4 * keep * num_chunks(x.numel(), chunk)), _stream(stream)))


def bagua_decompress_reduce_recompress_topk(idx_in, val_in, keep, server_residual, n, chunk, idx_out, val_out,
                                            out_fp32=None, stream=None):
    _same_len(len(idx_in), val_in=val_in)
    _check("bagua_decompress_reduce_recompress_topk", _lib.bagua_decompress_reduce_recompress_topk(
        _ptr_array(idx_in, torch.int16, 2 * keep * num_chunks(n, chunk)),
        _ptr_array(val_in, torch.float32, 4 * keep * num_chunks(n, chunk)), len(idx_in), keep,
        _ptr(server_residual, torch.float32, 4 * n), n, chunk, _ptr(idx_out, torch.int16, 2 * keep * num_chunks(n, chunk)),
        _ptr(val_out, torch.float32, 4 * keep * num_chunks(n, chunk)), _ptr(out_fp32, torch.float32, 4 * n),
        _stream(stream)))


def bagua_decompress_topk(idx, val, n, chunk, keep, out, stream=None):
    _check("bagua_decompress_topk", _lib.bagua_decompress_topk(
        _ptr(idx, torch.int16, 2 * keep * num_chunks(n, chunk)), _ptr(val, torch.float32, 4 * keep * num_chunks(n, chunk)),
        n, chunk, keep, _ptr(out, torch.float32, 4 * n), _stream(stream)))


# ---------------------------------------------------------------------------------------------- batched forms
def bagua_batch_workspace_bytes(B, k=0):
    return int(_lib.bagua_batch_workspace_bytes(B, k))


def _sizes(ns):
    return (ctypes.c_size_t * len(ns))(*[int(v) for v in ns])


def _ws(workspace):
    return _ptr(workspace), workspace.numel() * workspace.element_size()


class PreparedCall:
    """A batched call with its pointer arrays already marshalled.  Marshalling thousands of tensors costs Python more
    time than the launch takes on the GPU; a caller whose buffers stay where they are prepares once (prepare=True) and
    then calls the object every step: that is only the C call (table build, upload launches, kernel launch)."""

    def __init__(self, name, fn, args, keep):
        self.name, self.fn, self.args, self.keep = name, fn, args, keep      # keep: the tensors behind the pointers

    def __call__(self, stream=None):
        _check(self.name, self.fn(*self.args, _stream(stream)))


def _run(prepare, name, fn, args, keep, stream):
    call = PreparedCall(name, fn, args, keep)
    if prepare:
        return call
    call(stream)
    return None


def bagua_compress_minmax_u8_batched(xs, residuals, chunk, codes, minmaxs, workspace, stream=None, prepare=False):
    """B buckets in one launch; xs/codes/minmaxs are lists of B tensors, residuals a list of B tensors or None.
    prepare=True returns a PreparedCall instead of launching (so do the other batched calls)."""
    B = len(xs)
    _same_len(B, residuals=residuals, codes=codes, minmaxs=minmaxs)
    ns = [x.numel() for x in xs]
    wp, wb = _ws(workspace)
    arrs = [_ptr(x, torch.float32) for x in xs]
    xa = (ctypes.c_void_p * B)(*[a.value for a in arrs])
    ra = None if residuals is None else (ctypes.c_void_p * B)(*[_ptr(r, torch.float32, 4 * n).value for r, n in zip(residuals, ns)])
    ca = (ctypes.c_void_p * B)(*[_ptr(c, torch.uint8, n).value for c, n in zip(codes, ns)])
    ma = (ctypes.c_void_p * B)(*[_ptr(m, torch.float32, 8 * num_chunks(n, chunk)).value for m, n in zip(minmaxs, ns)])
    return _run(prepare, "bagua_compress_minmax_u8_batched", _lib.bagua_compress_minmax_u8_batched,
                (xa, ra, _sizes(ns), B, chunk, ca, ma, wp, wb), (xs, residuals, codes, minmaxs, workspace), stream)


def bagua_sign_compress_ef_batched(xs, residuals, chunk, bits, scales, workspace, stream=None, prepare=False):
    B = len(xs)
    _same_len(B, residuals=residuals, bits=bits, scales=scales)
    ns = [x.numel() for x in xs]
    wp, wb = _ws(workspace)
    xa = (ctypes.c_void_p * B)(*[_ptr(x, torch.float32).value for x in xs])
    ra = None if residuals is None else (ctypes.c_void_p * B)(*[_ptr(r, torch.float32, 4 * n).value for r, n in zip(residuals, ns)])
    ba = (ctypes.c_void_p * B)(*[_ptr(b, torch.int32, _code_bytes(CODEC_SIGN1, n)).value for b, n in zip(bits, ns)])
    sa = (ctypes.c_void_p * B)(*[_ptr(s, torch.float32, _meta_bytes(CODEC_SIGN1, n, chunk)).value for s, n in zip(scales, ns)])
    return _run(prepare, "bagua_sign_compress_ef_batched", _lib.bagua_sign_compress_ef_batched,
                (xa, ra, _sizes(ns), B, chunk, ba, sa, wp, wb), (xs, residuals, bits, scales, workspace), stream)


def bagua_decompress_reduce_recompress_batched(codec, codes_in, meta_in, server_residuals, ns, chunk, codes_out, meta_out,
                                               outs, workspace, stream=None, prepare=False):
    """codes_in / meta_in: list over buckets of lists over the k workers."""
    B = len(ns)
    _same_len(B, codes_in=codes_in, meta_in=meta_in, server_residuals=server_residuals, codes_out=codes_out,
              meta_out=meta_out, outs=outs)
    k = len(codes_in[0])
    for b in range(B):
        _same_len(k, codes_in_b=codes_in[b], meta_in_b=meta_in[b])
    wp, wb = _ws(workspace)
    ci = (ctypes.c_void_p * (B * k))(*[_ptr(codes_in[b][j], None, _code_bytes(codec, ns[b])).value
                                       for b in range(B) for j in range(k)])
    mi = (ctypes.c_void_p * (B * k))(*[_ptr(meta_in[b][j], torch.float32, _meta_bytes(codec, ns[b], chunk)).value
                                       for b in range(B) for j in range(k)])
    ea = None if server_residuals is None else (ctypes.c_void_p * B)(*[_ptr(e, torch.float32, 4 * n).value for e, n in zip(server_residuals, ns)])
    co = (ctypes.c_void_p * B)(*[_ptr(c, None, _code_bytes(codec, n)).value for c, n in zip(codes_out, ns)])
    mo = (ctypes.c_void_p * B)(*[_ptr(m, torch.float32, _meta_bytes(codec, n, chunk)).value for m, n in zip(meta_out, ns)])
    oa = None if outs is None else (ctypes.c_void_p * B)(*[_ptr(o, torch.float32, 4 * n).value for o, n in zip(outs, ns)])
    return _run(prepare, "bagua_decompress_reduce_recompress_batched", _lib.bagua_decompress_reduce_recompress_batched,
                (codec, ci, mi, k, ea, _sizes(ns), B, chunk, co, mo, oa, wp, wb),
                (codes_in, meta_in, server_residuals, codes_out, meta_out, outs, workspace), stream)


def bagua_bucket_flatten_batched_run(plans, Ts, buckets, workspace, stream=None, prepare=False):
    B = len(plans)
    _same_len(B, Ts=Ts, buckets=buckets)
    wp, wb = _ws(workspace)
    pa = (ctypes.c_void_p * B)(*[_ptr(p).value for p in plans])
    ba = (ctypes.c_void_p * B)(*[_ptr(b, torch.float32).value for b in buckets])
    return _run(prepare, "bagua_bucket_flatten_batched_run", _lib.bagua_bucket_flatten_batched_run,
                (pa, _sizes(Ts), ba, _sizes([b.numel() for b in buckets]), B, wp, wb), (plans, buckets, workspace), stream)


# ---------------------------------------------------------------------------------------------- probes
def bagua_probe_read(x, tile_sums, stream=None):
    n = x.numel()
    _check("bagua_probe_read", _lib.bagua_probe_read(_ptr(x, torch.float32), n, _ptr(tile_sums, torch.float32, 4 * ((n + 4095) // 4096)),
                                                     _stream(stream)))


def bagua_probe_streams(ins, outs, bouts, nr, nw, nb, seq, n, stream=None):
    _same_len(seq * nr, ins=ins)
    _same_len(seq * nw, outs=outs)
    _same_len(seq * nb, bouts=bouts)
    _check("bagua_probe_streams", _lib.bagua_probe_streams(
        _ptr_array(ins, torch.float32, 4 * n), _ptr_array(outs, torch.float32, 4 * n) if outs else None,
        _ptr_array(bouts, torch.uint8, n) if bouts else None, nr, nw, nb, seq, n, _stream(stream)))


def raw():
    """The ctypes library object (tests call entry points with hand-made invalid arguments through it)."""
    return _lib
