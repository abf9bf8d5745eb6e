"""Do the pins bite?  Each case plants ONE plausible mistake in a copy of the oracle's C source (a dropped term, a
wrong sign or index, a transposed operand, a wrong constant), builds that copy into a temporary library and runs the
oracle's pin tests against it in a child process.  The pins must reject every such build.  Nothing here touches the
GPU library: the mistakes live in the CPU oracle only, and the real oracle is never modified.

Not every line can be covered this way: mutants that only change a reading the paper leaves open in a way no outside
fact decides (the order of the sign codec's |v| sum, -0 against +0) are absent from the list on purpose.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
from oracle import build as oracle_build  # noqa: E402

PIN_FILES = ["test_oracle_minmax.py", "test_oracle_sign.py", "test_oracle_ring.py", "test_oracle_flatten.py",
             "test_oracle_golden.py", "test_oracle_sgd.py", "test_oracle_adam.py", "test_oracle_topk.py",
             "test_oracle_peers.py", "test_oracle_hierarchical.py"]

# (name, text in oracle/bagua_oracle.c, replacement, which occurrence of the text, pin file expected to object)
MUTANTS = [
    # MinMax-u8 codec
    ("minmax_256_levels_step", "return r / 255.0f;", "return r / 256.0f;", 0, "test_oracle_minmax.py"),
    ("minmax_256_levels_scale", "255.0f / r;", "256.0f / r;", 0, "test_oracle_minmax.py"),
    ("minmax_truncates", "float q = rintf(t);", "float q = floorf(t);", 0, "test_oracle_minmax.py"),
    ("minmax_offset_from_max", "float d = v[i] - mn;", "float d = v[i] - mx;", 0, "test_oracle_minmax.py"),
    ("minmax_max_never_updated", "if (v[i] > mx) mx = v[i];", ";", 0, "test_oracle_minmax.py"),
    ("minmax_dequant_from_max", "return mn + p;", "return mn - p;", 0, "test_oracle_minmax.py"),
    ("minmax_residual_sign", "residual[i] = v[i] - deq;", "residual[i] = deq - v[i];", 0, "test_oracle_minmax.py"),
    ("minmax_carry_in_subtracted", "v[i] = residual ? x[i] + residual[i] : x[i];",
     "v[i] = residual ? x[i] - residual[i] : x[i];", 0, "test_oracle_minmax.py"),
    ("minmax_residual_not_added", "v[i] = residual ? x[i] + residual[i] : x[i];", "v[i] = x[i];", 0,
     "test_oracle_minmax.py"),
    # server step
    ("drr_minmax_sum_not_average", "a[i] = s * inv_k;", "a[i] = s;", 0, "test_oracle_minmax.py"),
    ("drr_minmax_min_max_swapped", "float mn = minmax_in[j][2 * c], mx = minmax_in[j][2 * c + 1];",
     "float mx = minmax_in[j][2 * c], mn = minmax_in[j][2 * c + 1];", 0, "test_oracle_minmax.py"),
    ("drr_minmax_last_worker_only", "s = (j == 0) ? deq : s + deq;", "s = deq;", 0, "test_oracle_minmax.py"),
    ("drr_minmax_other_chunks_meta", "float mn = minmax_in[j][2 * c], mx = minmax_in[j][2 * c + 1];",
     "float mn = minmax_in[j][0], mx = minmax_in[j][1];", 0, "test_oracle_minmax.py"),
    ("drr_sign_sum_not_average", "a[i] = s * inv_k;", "a[i] = s;", 1, "test_oracle_sign.py"),
    ("drr_sign_last_worker_only", "s = (j == 0) ? deq : s + deq;", "s = deq;", 1, "test_oracle_sign.py"),
    ("drr_sign_polarity", "? sc : -sc;\n                s = ", "? -sc : sc;\n                s = ", 0,
     "test_oracle_sign.py"),
    # decentralised averaging
    ("ring_fp_left_neighbour", "const float* l = x_in[(i + k - 1) % k];", "const float* l = x_in[(i + k - 2) % k];",
     0, "test_oracle_ring.py"),
    ("ring_fp_right_is_self", "const float* r = x_in[(i + 1) % k];", "const float* r = x_in[i];", 0,
     "test_oracle_ring.py"),
    ("ring_fp_weight", "float third = 1.0f / 3.0f;", "float third = 0.5f;", 0, "test_oracle_ring.py"),
    ("ring_lp_weight", "float third = 1.0f / 3.0f;", "float third = 0.5f;", 1, "test_oracle_ring.py"),
    ("ring_lp_own_sign", "float own = x_in[i][e] - m[e];", "float own = m[e] - x_in[i][e];", 0,
     "test_oracle_ring.py"),
    ("ring_lp_own_dropped", "float own = x_in[i][e] - m[e];", "float own = 0.0f;", 0, "test_oracle_ring.py"),
    ("ring_lp_copy_replaced", "xhat[i][e] = xhat[i][e] + q[e];", "xhat[i][e] = q[e];", 0, "test_oracle_ring.py"),
    ("ring_lp_sends_replica", "d[e] = x_in[i][e] - xhat[i][e];", "d[e] = x_in[i][e];", 0, "test_oracle_ring.py"),
    ("ring_lp_right_neighbour", "const float* r = xhat[(i + 1) % k];", "const float* r = xhat[(i + 2) % k];", 0,
     "test_oracle_ring.py"),
    ("peer_fp_no_half", "x_out[i][e] = s * 0.5f;", "x_out[i][e] = s;", 0, "test_oracle_peers.py"),
    ("peer_fp_self", "const float* b = x_in[peer[i]];", "const float* b = x_in[i];", 0, "test_oracle_peers.py"),
    ("peer_lp_own_dropped", "float own = x_in[i][e] - a[e];", "float own = 0.0f;", 0, "test_oracle_peers.py"),
    ("peer_lp_copy_replaced", "xhat[i][e] = xhat[i][e] + q[e];", "xhat[i][e] = q[e];", 1, "test_oracle_peers.py"),
    ("peer_lp_self", "const float* b = xhat[peer[i]];", "const float* b = xhat[i];", 0, "test_oracle_peers.py"),
    # Sign-1bit codec
    ("sign_zero_is_negative", "int b = (v[i] >= 0.0f) ? 1 : 0;", "int b = (v[i] > 0.0f) ? 1 : 0;", 0,
     "test_oracle_sign.py"),
    ("sign_bit_order", "(uint32_t)1 << (g & 31);", "(uint32_t)1 << (31 - (g & 31));", 0, "test_oracle_sign.py"),
    ("sign_scale_without_abs", "e[t] = (i < len) ? fabsf(v[i]) : 0.0f;", "e[t] = (i < len) ? v[i] : 0.0f;", 0,
     "test_oracle_sign.py"),
    ("sign_scale_drops_a_quarter", "float g = p + q;", "float g = p + e[2];", 0, "test_oracle_sign.py"),
    ("sign_scale_half_butterfly", "for (int s = 1; s < 64; s <<= 1) {", "for (int s = 1; s < 32; s <<= 1) {", 0,
     "test_oracle_sign.py"),
    ("sign_tail_scale_by_chunk", "return s / (float)len;", "return s / (float)chunk;", 0, "test_oracle_sign.py"),
    ("sign_decode_polarity", "float deq = b ? scale : -scale;", "float deq = b ? -scale : scale;", 0,
     "test_oracle_sign.py"),
    ("sign_residual_sign", "residual[i] = v[i] - deq;", "residual[i] = deq - v[i];", 1, "test_oracle_sign.py"),
    ("sign_carry_in_subtracted", "v[i] = residual ? x[i] + residual[i] : x[i];",
     "v[i] = residual ? x[i] - residual[i] : x[i];", 1, "test_oracle_sign.py"),
    ("sign_decode_first_scale", "float s = scale[i / chunk];", "float s = scale[0];", 0, "test_oracle_sign.py"),
    # flatten
    ("flatten_reversed", "bucket[dst_offset[t] + e] = src[t][e];", "bucket[dst_offset[t] + e] = src[t][numel[t] - 1 - e];",
     0, "test_oracle_flatten.py"),
    ("flatten_gaps_not_cleared", "for (size_t e = 0; e < bucket_numel; ++e) bucket[e] = 0.0f;", ";", 0,
     "test_oracle_flatten.py"),
    ("unflatten_offset_ignored", "dst[t][e] = bucket[src_offset[t] + e];", "dst[t][e] = bucket[e];", 0,
     "test_oracle_flatten.py"),
    # optimizer steps
    ("sgd_ascent", "float s = lr * u;\n        param[i] = param[i] - s;", "float s = lr * u;\n        param[i] = param[i] + s;",
     0, "test_oracle_sgd.py"),
    ("sgd_momentum_sign", "float m = t + gi;", "float m = t - gi;", 0, "test_oracle_sgd.py"),
    ("sgd_decay_on_gradient", "float w = weight_decay * param[i];\n            gi = gi + w;",
     "float w = weight_decay * gi;\n            gi = gi + w;", 0, "test_oracle_sgd.py"),
    ("sgd_update_skips_momentum", "momentum_buf[i] = m;\n            u = m;", "momentum_buf[i] = m;", 0,
     "test_oracle_sgd.py"),
    ("adam_multiplies_by_denominator", "float u = mi / denom;", "float u = mi * denom;", 0, "test_oracle_adam.py"),
    ("adam_variance_of_d", "float dd = d[i] * d[i];", "float dd = d[i];", 0, "test_oracle_adam.py"),
    ("adam_no_square_root", "float root = sqrtf(vi);", "float root = vi;", 0, "test_oracle_adam.py"),
    ("adam_frozen_keeps_old_momentum", "mi = d[i];", "mi = m[i];", 0, "test_oracle_adam.py"),
    ("adam_betas_swapped", "float c = beta2 * vi;", "float c = beta1 * vi;", 0, "test_oracle_adam.py"),
    ("adam_eps_inside_root", "float root = sqrtf(vi);\n        float denom = root + eps;",
     "float root = vi + eps;\n        float denom = sqrtf(root);", 0, "test_oracle_adam.py"),
    ("momentum_compress_weights", "float b = omb1 * g[i];", "float b = beta1 * g[i];", 0, "test_oracle_adam.py"),
    # hierarchical / full precision
    ("reduce_compress_drops_worker_1", "for (int j = 1; j < k_local; ++j) s = s + x[j][i];",
     "for (int j = 2; j < k_local; ++j) s = s + x[j][i];", 0, "test_oracle_hierarchical.py"),
    ("reduce_compress_sum_not_average", "a[i] = s * inv;", "a[i] = s;", 0, "test_oracle_hierarchical.py"),
    ("centralized_sum_not_average", "out[i] = s * inv;", "out[i] = s;", 0, None),
    # top-K codec
    ("topk_keeps_smallest", "return x->key > y->key ? -1 : 1;", "return x->key > y->key ? 1 : -1;", 0,
     "test_oracle_topk.py"),
    ("topk_signed_compare", "items[i].key = bits & 0x7fffffffu;", "items[i].key = bits;", 0, "test_oracle_topk.py"),
    ("topk_tie_to_higher_index", "return x->pos < y->pos ? -1 : (x->pos > y->pos ? 1 : 0);",
     "return x->pos < y->pos ? 1 : (x->pos > y->pos ? -1 : 0);", 0, "test_oracle_topk.py"),
    ("topk_residual_inverted", "residual[i] = sel[i] ? 0.0f : v[i];", "residual[i] = sel[i] ? v[i] : 0.0f;", 0,
     "test_oracle_topk.py"),
    ("topk_drr_sum_not_average", "for (size_t i = 0; i < n; ++i) a[i] = a[i] * inv_k;", ";", 0, "test_oracle_topk.py"),
    ("topk_drr_last_worker_only", "a[i] = (j == 0) ? d[i] : a[i] + d[i];", "a[i] = d[i];", 0, "test_oracle_topk.py"),
    ("topk_decode_offset", "out[lo + p] = val[c * keep + s];", "out[lo + p] = val[c * keep];", 0, "test_oracle_topk.py"),
]


def _mutate(src, old, new, occurrence):
    at = -1
    for _ in range(occurrence + 1):
        at = src.find(old, at + 1)
        assert at >= 0, "mutation target not found (the oracle's source changed?): %r #%d" % (old, occurrence)
    return src[:at] + new + src[at + len(old):]


def _run_pins(lib_path, files):
    env = dict(os.environ, BAGUA_ORACLE_LIB=lib_path, PYTHONDONTWRITEBYTECODE="1")
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider", "--no-header"]
    cmd += [os.path.join(ROOT, "tests", f) for f in files]
    return subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)


def _build(src_text, workdir, name):
    c = os.path.join(workdir, name + ".c")
    so = os.path.join(workdir, name + ".so")
    with open(c, "w") as f:
        f.write(src_text)
    flags = [f for f in oracle_build.FLAGS if f not in ("-Wall", "-Wextra")]
    subprocess.run(["gcc"] + flags + [c, "-o", so, "-lm"], check=True, capture_output=True)
    return so


def test_unmodified_copy_passes_every_pin(tmp_path):
    """The harness itself: the same source, built the same way into another file, passes."""
    so = _build(open(oracle_build.SRC).read(), str(tmp_path), "identity")
    res = _run_pins(so, PIN_FILES)
    assert res.returncode == 0, res.stdout[-3000:]


def test_every_planted_mistake_is_rejected_by_a_pin(tmp_path):
    src = open(oracle_build.SRC).read()
    names = [m[0] for m in MUTANTS]
    assert len(set(names)) == len(names)

    def one(m):
        name, old, new, occ, expect = m
        so = _build(_mutate(src, old, new, occ), str(tmp_path), name)
        files = PIN_FILES if expect is None else [expect]
        res = _run_pins(so, files)
        if res.returncode == 0 and expect is not None:      # not where expected: anywhere?
            res = _run_pins(so, PIN_FILES)
        crashed = res.returncode < 0 or res.returncode >= 128
        return name, res.returncode, crashed

    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
        results = list(pool.map(one, MUTANTS))
    survived = [n for n, rc, _ in results if rc == 0]
    crashed = [n for n, _, cr in results if cr]
    assert not crashed, "mutants that crashed instead of failing a pin: %s" % crashed
    assert not survived, "no pin notices these mistakes: %s" % survived
