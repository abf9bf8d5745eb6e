"""Every element of the three largest benchmark configurations, at full size and in the launch configuration the
benchmark times, against the oracle streamed over the same bits (bench.py --verify-all runs the same three checks).
Bar: integer words equal, fp32 words bit-identical (which implies the 1e-6 relative / 1e-7 absolute tolerance)."""
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import bench
    import paper_2107_01499_amd as bg
    assert torch.cuda.is_available()
    return bench, bg


def check(cnt, min_words):
    assert cnt.c["int_words"] + cnt.c["fp32_words"] >= min_words, cnt.c       # nothing was skipped
    assert cnt.c["int_mismatch"] == 0 and cnt.c["fp32_not_bit_exact"] == 0 and cnt.c["fp32_out_of_tolerance"] == 0, cnt.c


def test_config3_bert_large_every_bucket(env):
    bench, bg = env
    print("configs[2]: 16 workers x 341M elements, flatten + compress + server step", flush=True)
    check(bench.verify_config2(torch, bg), 16 * 335141888 * 3)


def test_config4_ring_five_rounds_every_element(env):
    bench, bg = env
    print("configs[3]: 8 peers x 110M elements, 5 rounds FP and LP", flush=True)
    check(bench.verify_config3(torch, bg, rounds=5), 5 * 8 * 109482240 * 4)


def test_config5_onebit_every_element(env):
    bench, bg = env
    print("configs[4]: 8 workers x 1.5e9 elements, sign compression + server step", flush=True)
    check(bench.verify_config4(torch, bg), 8 * 1500000000)
