"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): the C
file is compiled together with a small driver (tests/oracle_sanitize_main.c) that calls every
routine on exactly-sized heap buffers, ragged shapes and the hand-worked cases; any
out-of-bounds access or undefined arithmetic ends the run with a report."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_is_clean_under_address_and_undefined_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    # the sanitizer runtime is linked statically: a preloaded library may then come first
    cmd = ["gcc", "-std=c11", "-O1", "-g", "-fno-omit-frame-pointer", "-fopenmp",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-static-libasan",
           "-Wall", "-Wextra", os.path.join(ROOT, "oracle", "jvoracle.c"),
           os.path.join(ROOT, "tests", "oracle_sanitize_main.c"), "-o", exe, "-lm"]
    build = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert build.returncode == 0, build.stdout
    env = dict(os.environ, OMP_NUM_THREADS="4",
               ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    sys.stdout.write(run.stdout[-2000:])
    assert run.returncode == 0, run.stdout[-4000:]
    assert "oracle sanitize run: ok" in run.stdout
