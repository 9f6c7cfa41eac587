"""The oracle's C sources under AddressSanitizer and UndefinedBehaviorSanitizer: a small C driver
(oracle/sanitize_driver.c) runs every routine on tiny, exactly allocated cases; any access outside an
array, signed overflow or misaligned access stops it with a report."""
import os
import shutil
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = [os.path.join(ROOT, "oracle", f) for f in ("sanitize_driver.c", "qsr_oracle.c", "qsr_oracle_resmlp.c")]


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_runs_clean_under_address_and_undefined_behaviour_sanitizers():
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "sanitize_driver")
        # the sanitizer runtimes are linked statically: a preloaded library would otherwise come before them
        build = subprocess.run(["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-ffp-contract=off", "-fopenmp",
                                "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
                                "-static-libubsan", "-Wall", "-Wextra", "-o", exe] + SRC + ["-lm"],
                               capture_output=True, text=True, timeout=300)
        if build.returncode != 0 and "static-lib" in build.stderr:
            pytest.skip("no static sanitizer runtimes: " + build.stderr[-300:])
        assert build.returncode == 0, build.stderr[-3000:]
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
                   OMP_NUM_THREADS="2")
        run = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
        assert run.returncode == 0, (run.stdout + run.stderr)[-4000:]
        assert "sanitize_driver: ok" in run.stdout
        assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, run.stderr[-4000:]
