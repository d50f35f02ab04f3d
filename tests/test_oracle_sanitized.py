"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer: oracle/fq_oracle.c is compiled together with
a small driver (tests/sanitize/oracle_walk.c) that walks every function through small ragged cases with exact-size
heap buffers; any out-of-bounds access, signed overflow or misaligned access ends the run with a report.  CPU only."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_walk_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_walk")
    cmd = ["gcc", "-std=c11", "-O1", "-g", "-fopenmp", "-ffp-contract=off", "-fno-omit-frame-pointer",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-o", exe,
           os.path.join(ROOT, "tests", "sanitize", "oracle_walk.c"), os.path.join(ROOT, "oracle", "fq_oracle.c"), "-lm"]
    subprocess.run(cmd, check=True)
    # the sanitizer runtime is linked statically; libraries preloaded into every process may precede it
    env = dict(os.environ, OMP_NUM_THREADS="2", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "oracle walk clean" in r.stdout
    assert "ERROR" not in r.stderr and "runtime error" not in r.stderr, r.stderr
