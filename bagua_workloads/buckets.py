"""Greedy bucket packing used by the benchmark configurations (host side, no arithmetic).

The paper decides buckets in its profiling phase with an unspecified heuristic (Section 3.1
"Bucketing", Section 3.5); the benchmark configurations say "25 MB buckets".  Rule used here:
tensors in definition order; a bucket is closed when the next tensor would push it over
25 MiB (6,553,600 fp32); a larger tensor is a bucket of its own; tensors are packed tightly;
the bucket length is rounded up to a multiple of k*chunk so that each of the k ScatterReduce
partitions (Section 3.4) is a whole number of chunks.
"""
from collections import namedtuple

from .shapes import numel

BUCKET_ELEMS = 25 * 1024 * 1024 // 4

# tensors: list of indices into the shape list; offsets: element offset of each in the bucket;
# n: payload elements; n_pad: padded bucket length.
Bucket = namedtuple("Bucket", "tensors offsets n n_pad")


def pack_buckets(shapes, k, chunk, cap=BUCKET_ELEMS):
    buckets = []
    cur, offs, fill = [], [], 0

    def close():
        nonlocal cur, offs, fill
        if cur:
            q = k * chunk
            buckets.append(Bucket(tuple(cur), tuple(offs), fill, (fill + q - 1) // q * q))
        cur, offs, fill = [], [], 0

    for idx, (_, shape) in enumerate(shapes):
        sz = numel(shape)
        if cur and fill + sz > cap:
            close()
        cur.append(idx)
        offs.append(fill)
        fill += sz
    close()
    return buckets
