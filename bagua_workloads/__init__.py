"""Seeded synthetic workloads shared by the tests, the smoke check and the benchmark.

This package holds layer shapes, the bucket packing rule and random-value generators only.
It contains none of the arithmetic of the compression / averaging primitives; both the CPU
oracle and the GPU library are fed from here so that they see bit-identical inputs.
"""
from .shapes import resnet50_shapes, bert_shapes  # noqa: F401
from .buckets import pack_buckets, Bucket, BUCKET_ELEMS  # noqa: F401
from .generators import seed_for, draw, layer_sigmas  # noqa: F401
