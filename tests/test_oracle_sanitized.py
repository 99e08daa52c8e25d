"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): a C
driver with exactly-sized buffers runs ref_gemm, ref_gemm_points, ref_rope and the scalar helpers
over small problems in every layout and storage type and checks them against integer sums."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "sanitize_oracle")
    cmd = ["gcc", "-std=c11", "-O1", "-g", "-fno-fast-math", "-ffp-contract=off", "-Wall", "-Wextra",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
           os.path.join(ROOT, "tests", "sanitize_oracle.c"), os.path.join(ROOT, "oracle", "ref_gemm.c"),
           os.path.join(ROOT, "oracle", "ref_rope.c"), "-lm", "-o", exe]
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    run = subprocess.run([exe], capture_output=True, text=True, env=dict(os.environ, ASAN_OPTIONS="detect_leaks=1"))
    assert run.returncode == 0, run.stdout + run.stderr
    assert "ok" in run.stdout and "runtime error" not in run.stderr, run.stdout + run.stderr
