"""Hand-worked C_LP_S examples (tests/golden/c_lp_s_hand_examples.json) against the oracle."""
import json
import os

import numpy as np

G = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "c_lp_s_hand_examples.json")))


def test_two_workers_lossless(oracle):
    g = G["two_workers_lossless"]
    C = g["chunk"]
    i = np.arange(C, dtype=np.float32)
    xs = [i.copy(), (2 * (255 - i)).astype(np.float32)]
    want_codes = [np.arange(C, dtype=np.uint8), (255 - np.arange(C)).astype(np.uint8)]
    codes_in, mm_in = [], []
    for j in range(2):
        d = np.zeros(C, np.float32)
        c, m = oracle.compress_minmax_u8(xs[j], d, C)
        assert m.tolist() == g["worker_minmax"][j]
        np.testing.assert_array_equal(c, want_codes[j])
        assert not d.any()
        codes_in.append(c); mm_in.append(m)
    eps = np.zeros(C, np.float32)
    codes, mm, out = oracle.drr_minmax_u8(codes_in, mm_in, eps, C)
    assert mm.tolist() == g["server_minmax"]
    np.testing.assert_array_equal(codes, (255 - np.arange(C)).astype(np.uint8))
    np.testing.assert_array_equal(out, (255 - i / 2).astype(np.float32))
    assert not eps.any()


def test_error_feedback_three_iterations(oracle):
    g = G["error_feedback_three_iterations"]
    C = g["chunk"]
    x = np.zeros(C, np.float32)
    x[:3] = g["x_head"]
    d = np.zeros(C, np.float32)
    total = 0.0
    for t in range(3):
        codes, mm = oracle.compress_minmax_u8(x, d, C)
        assert mm.tolist() == [0.0, 255.0]
        assert codes[2] == g["codes_elem2"][t]
        assert d[2] == g["delta_elem2"][t]
        total += float(oracle.decompress_minmax_u8(codes, mm, C)[2])
    assert total == 3 * 100.25 - float(d[2]) == 301.0
