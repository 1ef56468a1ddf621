"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer: oracle/
sanitized_selfcheck.c calls every exported function on edge shapes in tightly sized heap
buffers and compares the oracle's forms of each quantity with each other.  Host code only."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = tmp_path / "oracle_selfcheck"
    build = subprocess.run(
        ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined",
         "-fno-sanitize-recover=all", "-Wall", "-Wextra",
         os.path.join(ROOT, "oracle", "sanitized_selfcheck.c"), "-o", str(exe), "-lm"],
        stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert build.returncode == 0, build.stdout
    assert "warning" not in build.stdout, build.stdout
    env = dict(os.environ)
    # libraries the environment preloads come before the sanitizer's runtime: not an error here;
    # the OpenMP runtime keeps its thread pool until exit, which the leak check would report
    env["ASAN_OPTIONS"] = "verify_asan_link_order=0:detect_leaks=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1"
    run = subprocess.run([str(exe)], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env,
                         timeout=300)
    assert run.returncode == 0, run.stdout[-4000:]
    assert "oracle self-check clean" in run.stdout
