"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer: a C driver
(tests/oracle_sanitize_driver.c) calls every entry point on exactly-sized heap buffers; the
instrumented program aborts on any access outside them."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
pytestmark = pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")


def _build_and_run(tmp_path, name, extra):
    exe = tmp_path / name
    build = subprocess.run(
        ["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", *extra,
         os.path.join(ROOT, "oracle", "preft_oracle.c"), os.path.join(ROOT, "tests", "oracle_sanitize_driver.c"),
         "-lm", "-o", str(exe)], capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1", OMP_NUM_THREADS="4")
    return subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=120)


def test_oracle_is_clean_under_address_and_ub_sanitizers(tmp_path):
    run = _build_and_run(tmp_path, "driver", [])
    assert run.returncode == 0, run.stdout + run.stderr
    assert "ok" in run.stdout


def test_the_sanitized_run_notices_a_buffer_that_is_one_element_short(tmp_path):
    """The check of the check: with every matrix one element short the oracle reads past a heap
    block, and the instrumented build must say so."""
    run = _build_and_run(tmp_path, "driver_short", ["-DPLANT_SHORT_BUFFER"])
    assert run.returncode != 0
    assert "AddressSanitizer" in run.stderr and "heap-buffer-overflow" in run.stderr
