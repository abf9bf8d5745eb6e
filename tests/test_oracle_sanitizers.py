"""The oracle under AddressSanitizer + UndefinedBehaviorSanitizer (host code only): oracle/selftest.c runs every
oracle function on ragged sizes with exactly-sized heap buffers."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_is_clean_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_selftest")
    cmd = ["gcc", "-std=c11", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", "-fopenmp", "-ffp-contract=off",
           os.path.join(ROOT, "oracle", "selftest.c"), os.path.join(ROOT, "oracle", "bagua_oracle.c"), "-o", exe, "-lm"]
    subprocess.run(cmd, check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-4000:]
    assert "oracle selftest ok" in res.stdout
