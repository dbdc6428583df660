"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer: oracle/prom_oracle.c is
compiled with -fsanitize=address,undefined together with a small C driver that calls every layer
function on heap buffers of exactly the documented sizes (odd image sizes, both strides, ragged
channel counts).  An access outside a tensor, a signed overflow or a bad shift in the oracle fails
the run.  Host code only; no GPU."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("gcc not available")
    exe = str(tmp_path / "oracle_sanitized")
    # the sanitizer runtimes are linked statically so that the run does not depend on the order of
    # preloaded libraries in the environment
    cmd = [gcc, "-O1", "-g", "-fno-omit-frame-pointer", "-fopenmp", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-static-libasan", "-static-libubsan", os.path.join(ROOT, "oracle", "prom_oracle.c"),
           os.path.join(ROOT, "tests", "oracle_sanitizer_driver.c"), "-o", exe]
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    env = dict(os.environ, OMP_NUM_THREADS="2", ASAN_OPTIONS="detect_leaks=0")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert run.returncode == 0, run.stdout + run.stderr
    assert run.stdout.strip().endswith("ok"), run.stdout + run.stderr
