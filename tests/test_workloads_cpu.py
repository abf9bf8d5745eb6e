"""Host-side workload logic: layer shapes, greedy bucket packing, seeded generators (no GPU, no arithmetic of the method)."""
import numpy as np
import torch

from bagua_workloads import resnet50_shapes, bert_shapes, pack_buckets, draw, seed_for, layer_sigmas, BUCKET_ELEMS
from bagua_workloads.shapes import numel


def test_model_shapes_totals():
    r = resnet50_shapes()
    assert len(r) == 161 and sum(numel(s) for _, s in r) == 25557032
    bl = bert_shapes(24, 1024, 4096)
    assert len(bl) == 391 and sum(numel(s) for _, s in bl) == 335141888
    bb = bert_shapes(12, 768, 3072)
    assert len(bb) == 199 and sum(numel(s) for _, s in bb) == 109482240
    assert r[0][1] == (64, 3, 7, 7) and r[-2][1] == (1000, 2048) and bl[0][1] == (30522, 1024)


def test_bucket_packing_rule():
    for shapes, k, C in ((resnet50_shapes(), 8, 4096), (bert_shapes(24, 1024, 4096), 16, 8192)):
        buckets = pack_buckets(shapes, k, C)
        seen = []
        for b in buckets:
            seen += list(b.tensors)
            sizes = [numel(shapes[t][1]) for t in b.tensors]
            assert b.n == sum(sizes)
            assert list(b.offsets) == np.concatenate([[0], np.cumsum(sizes)[:-1]]).tolist()   # tight packing
            assert b.n_pad % (k * C) == 0 and 0 <= b.n_pad - b.n < k * C
            assert b.n <= BUCKET_ELEMS or len(b.tensors) == 1                              # oversize tensor alone
        assert seen == list(range(len(shapes)))                                            # definition order, once each
        # greedy: a bucket could not have taken the next tensor
        for b, nb in zip(buckets[:-1], buckets[1:]):
            assert b.n + numel(shapes[nb.tensors[0]][1]) > BUCKET_ELEMS
    # the BERT-large word embedding is an oversize bucket of its own
    assert pack_buckets(bert_shapes(24, 1024, 4096), 16, 8192)[0].tensors == (0,)


def test_generators_are_seeded_and_shaped():
    a = draw("normal", 1000, seed_for(1, 0, 3), "cpu", 1e-3)
    b = draw("normal", 1000, seed_for(1, 0, 3), "cpu", 1e-3)
    c = draw("normal", 1000, seed_for(1, 0, 4), "cpu", 1e-3)
    assert torch.equal(a, b) and not torch.equal(a, c)
    assert a.dtype == torch.float32 and abs(float(a.std()) - 1e-3) < 2e-4
    lap = draw("laplace", 200000, 5, "cpu", 1e-3)
    assert abs(float(lap.abs().mean()) - 1e-3) < 5e-5 and torch.isfinite(lap).all()
    t3 = draw("student_t3", 200000, 6, "cpu", 1e-3)
    assert torch.isfinite(t3).all() and float(t3.abs().max()) > 1e-2      # heavy tail
    sig = layer_sigmas(161, seed_for(1, 0, 99))
    assert len(sig) == 161 and min(sig) >= 1e-5 and max(sig) <= 1e-2
    assert seed_for(2, 1, 7) == 2107014990000 + 20000 + 100 + 7


def test_bench_refuses_more_than_one_gpu():
    """bench.py is the single-GPU share of the path: --gpus N with N > 1 exits with a message that says so (checked
    before anything touches a GPU, so this runs anywhere)."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode == 2
    assert "single-GPU" in res.stderr and "--gpus 1" in res.stderr


def test_bench_default_plan_names_the_largest_configurations():
    import bench
    primary = [name for name, layout, counts in bench.DEFAULT_PLAN if counts]
    assert primary == ["bert_large", "bert_base_ring", "onebit"]
    prims = [p for name in primary for p in bench.WORKLOADS[name]["prims"]]
    assert sorted(prims) == sorted(bench.ALL_PRIMS)          # every primitive exactly once in the headline
    assert bench.WORKLOADS["bert_large"]["k"] == 16 and bench.WORKLOADS["bert_large"]["chunk"] == 8192
    assert bench.WORKLOADS["onebit"]["sign_chunk"] == 2048 and bench.ONEBIT_N == 1500000000
