"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU): the C oracle walked
by a small driver over ragged problems with exactly-sized heap buffers."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_is_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_asan")
    cmd = ["gcc", "-O1", "-g", "-std=gnu11", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan",
           "-fno-omit-frame-pointer", "-Wall", "-Wextra", "-o", exe,
           os.path.join(ROOT, "tests", "sanitize_oracle_driver.c"), os.path.join(ROOT, "oracle", "fge_oracle.c"), "-lm"]
    subprocess.run(cmd, check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", OMP_NUM_THREADS="2")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, (r.returncode, r.stdout[-2000:], r.stderr[-4000:])
    assert r.stdout.startswith("checksum ") and "ERROR" not in r.stderr and "runtime error" not in r.stderr
