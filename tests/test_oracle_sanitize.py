"""Host-only: the oracle under the undefined-behaviour sanitizer (signed overflow, shifts, bounds
of fixed arrays, misaligned access, float-to-int range) on small awkward shapes."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_is_clean_under_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_ubsan")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fsanitize=undefined",
           "-fno-sanitize-recover=all", os.path.join(ROOT, "oracle", "dabnn_oracle.c"),
           os.path.join(ROOT, "tests", "host", "oracle_ubsan_main.c"), "-o", exe, "-lm"]
    subprocess.run(cmd, check=True)
    out = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    sys.stdout.write(out.stdout)
    sys.stderr.write(out.stderr)
    assert out.returncode == 0 and "oracle ubsan run ok" in out.stdout
