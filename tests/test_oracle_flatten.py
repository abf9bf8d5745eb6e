"""Pins of the oracle's bucket flatten (Section 3.5, "Tensor Bucketing and Memory Flattening")."""
import numpy as np
import pytest


def test_flatten_matches_concatenate_with_gaps(oracle):
    r = np.random.default_rng(0)
    sizes = [1, 7, 64, 1000, 3, 4096, 0, 129]
    srcs = [r.standard_normal(s).astype(np.float32) for s in sizes]
    offs, pos = [], 0
    for i, s in enumerate(sizes):
        pos += (i % 3)              # leave some gaps
        offs.append(pos)
        pos += s
    total = pos + 50
    got = oracle.bucket_flatten(srcs, offs, total)
    want = np.zeros(total, np.float32)
    for s, o in zip(srcs, offs):
        want[o:o + s.size] = s
    assert got.tobytes() == want.tobytes()
    mask = np.ones(total, bool)
    for s, o in zip(srcs, offs):
        mask[o:o + s.size] = False
    assert not got[mask].view(np.uint32).any()      # pad is +0.0f bit pattern


def test_flatten_tight_is_concatenate(oracle):
    r = np.random.default_rng(1)
    srcs = [r.standard_normal(s).astype(np.float32) for s in (5, 11, 256, 30522)]
    offs = np.cumsum([0] + [s.size for s in srcs[:-1]]).tolist()
    got = oracle.bucket_flatten(srcs, offs, sum(s.size for s in srcs))
    assert got.tobytes() == np.concatenate(srcs).tobytes()


def test_flatten_rejects_overlap_and_overflow(oracle):
    a = np.zeros(10, np.float32)
    with pytest.raises(ValueError):
        oracle.bucket_flatten([a, a], [0, 5], 100)
    with pytest.raises(ValueError):
        oracle.bucket_flatten([a], [95], 100)


def test_unflatten_inverts_flatten(oracle):
    """Round trip: unflatten(flatten(tensors)) returns the tensors; gap elements of the bucket are ignored."""
    r = np.random.default_rng(4)
    sizes = [1, 7, 64, 0, 1000, 3, 4096, 129]
    srcs = [r.standard_normal(s).astype(np.float32) for s in sizes]
    offs, pos = [], 0
    for i, s in enumerate(sizes):
        pos += (i % 3)
        offs.append(pos)
        pos += s
    bucket = oracle.bucket_flatten(srcs, offs, pos + 9)
    bucket[[o - 1 for o, i in zip(offs, range(len(offs))) if i % 3]] = 123.0      # poison the gaps
    outs = [np.full(s, np.nan, np.float32) for s in sizes]
    oracle.bucket_unflatten(bucket, outs, offs)
    for a, b in zip(outs, srcs):
        assert a.tobytes() == b.tobytes()
    with pytest.raises(ValueError):
        oracle.bucket_unflatten(bucket, outs, [0] * len(offs))
