"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU involved).

`tests/native/oracle_sanitize.c` holds the inputs: the hand examples of tests/golden/ typed as
numbers, vocabularies that end inside a draw block in both input types with and without a
filter, trajectories stored back to back with clipped, empty and reversed extents, lengths
outside [0, T].  It is compiled together with `oracle/espo_oracle.c` by gcc with both sanitizers
and no recovery, and run as a plain host program; any finding ends it with a non-zero status.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           "-static-libasan",   # the runtime is linked in, so no preloaded library can come before it
           os.path.join(ROOT, "tests", "native", "oracle_sanitize.c"), os.path.join(ROOT, "oracle", "espo_oracle.c"),
           "-o", exe, "-lm"]
    build = subprocess.run(cmd, capture_output=True, text=True, timeout=300)
    assert build.returncode == 0, build.stderr
    env = {**os.environ, "ASAN_OPTIONS": "detect_leaks=1:abort_on_error=0", "UBSAN_OPTIONS": "print_stacktrace=1",
           "OMP_NUM_THREADS": "2"}
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "ran clean" in run.stdout
    assert "AddressSanitizer" not in run.stderr and "runtime error" not in run.stderr
