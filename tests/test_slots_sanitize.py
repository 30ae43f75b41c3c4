"""The slot manager's host logic under AddressSanitizer and UndefinedBehaviorSanitizer: hipcc builds
csrc/slots.hip with the host pass instrumented and links a C++ driver (tests/slots_sanitize_driver.cpp)
that runs the residency bookkeeping of managers without device memory -- no GPU needed."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
pytestmark = pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc")


def _build_and_run(tmp_path, name, extra):
    exe = tmp_path / name
    build = subprocess.run(
        ["hipcc", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
         "-Xarch_host", "-fno-sanitize-recover=all", *extra,
         os.path.join(ROOT, "paper_2605_14217_amd", "csrc", "slots.hip"),
         os.path.join(ROOT, "tests", "slots_sanitize_driver.cpp"), "-o", str(exe)],
        capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0")       # the HIP runtime keeps its own allocations
    return subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=120)


def test_slot_manager_host_logic_is_clean_under_sanitizers(tmp_path):
    run = _build_and_run(tmp_path, "driver", [])
    assert run.returncode == 0, run.stdout + run.stderr
    assert "ok" in run.stdout


def test_the_sanitized_run_notices_a_slot_array_that_is_one_entry_short(tmp_path):
    run = _build_and_run(tmp_path, "driver_short", ["-DPLANT_SHORT_OUTPUT"])
    assert run.returncode != 0
    assert "AddressSanitizer" in run.stderr
