"""The benchmark's measurement utilities run and move what they say they move (no method arithmetic here)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def bg():
    import paper_2107_01499_amd as b
    assert torch.cuda.is_available()
    return b


def test_probe_read_tile_sums(bg):
    n = 3 * 4096 + 700
    x = torch.arange(n, dtype=torch.float32, device="cuda") % 7 - 3.0          # small integers: every order sums exactly
    sums = torch.full(((n + 4095) // 4096,), float("nan"), device="cuda")
    bg.bagua_probe_read(x, sums)
    want = [float(x[t * 4096:(t + 1) * 4096].double().sum()) for t in range(sums.numel())]
    assert sums.cpu().tolist() == want


def test_probe_streams_copies_rows(bg):
    n = 5 * 256
    a = torch.arange(n, dtype=torch.float32, device="cuda")
    b = torch.ones(n, device="cuda")
    out = [torch.empty(n, device="cuda") for _ in range(2)]
    byt = [torch.empty(n, dtype=torch.uint8, device="cuda")]
    bg.bagua_probe_streams([a, b], out, byt, 2, 2, 1, 1, n)
    torch.cuda.synchronize()
    assert torch.equal(out[0], a + b) and torch.equal(out[1], a + b)
    acc = b.clone()
    bg.bagua_probe_streams([a, acc], [acc], [], 2, 1, 0, 1, n)                  # in place, no byte stream
    torch.cuda.synchronize()
    assert torch.equal(acc, a + b)
    with pytest.raises(bg.binding.BaguaError):
        bg.bagua_probe_streams([a, b, a], [out[0]], [], 3, 1, 0, 1, n)       # combination outside the menu
