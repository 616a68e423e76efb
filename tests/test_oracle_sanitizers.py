"""The oracle's C code under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): a driver
(tests/oracle_sanitize_main.c) calls every entry point on exact-size heap buffers over all formats, group sizes,
strides, ragged shapes and extreme inputs; an access past a buffer or an undefined operation aborts it."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", os.path.join(ROOT, "tests", "oracle_sanitize_main.c"),
           os.path.join(ROOT, "oracle", "amxfp4_ref.c"), "-lm", "-o", exe]
    built = subprocess.run(cmd, capture_output=True, text=True)
    if built.returncode != 0:
        pytest.skip("this gcc cannot link the sanitizer runtimes: " + built.stderr[-300:])
    # (the sanitizer runtime is linked statically, so whatever else the environment preloads does not matter)
    env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0 and run.stdout.strip() == "ok", (run.stdout + run.stderr)[-2000:]
