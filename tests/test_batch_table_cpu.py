"""Host logic of the batched launches: the unit -> bucket lookup table (csrc/batch.hpp) against a linear scan, compiled
for the host only (no GPU code, no GPU needed)."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def test_bucket_lookup_matches_linear_scan(tmp_path):
    exe = str(tmp_path / "batch_table_check")
    cmd = [HIPCC, "--cuda-host-only", "-x", "hip", "-O1", "-I" + os.path.join(ROOT, "paper_2107_01499_amd", "csrc"),
           "-I" + os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "host", "batch_table_check.hip"), "-o", exe]
    subprocess.run(cmd, check=True)
    res = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-2000:]
    assert res.stdout.startswith("OK ")
