"""The library's host code under AddressSanitizer + UndefinedBehaviorSanitizer, every kernel launch stubbed out.

tests/abi_host_driver.cpp defines the HIP runtime entry points the host code calls (launch, last error, device
queries), is compiled together with the library's sources with the sanitizers on the host side only, and walks the
argument validation and the complete host-side orchestration of the forward and backward passes with fake device
pointers.  It also arms the launch stub to report a failed launch and checks that every entry point maps it to
LP_ERR_HIP.  Nothing runs on a GPU, with or without one in the machine.
"""
import glob
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    if not os.path.exists(HIPCC):
        pytest.skip("hipcc is not installed")
    out = str(tmp_path_factory.mktemp("abi_sanitized") / "abi_host_driver")
    src = sorted(glob.glob(os.path.join(ROOT, "paper_2506_20818_amd", "csrc", "*.hip")))
    src += sorted(glob.glob(os.path.join(ROOT, "paper_2506_20818_amd", "csrc", "*.cpp")))
    src.append(os.path.join(ROOT, "tests", "abi_host_driver.cpp"))
    cmd = [HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2506_20818_amd", "csrc")] + src + ["-o", out]
    proc = subprocess.run(cmd, capture_output=True, text=True)
    assert proc.returncode == 0, proc.stdout + proc.stderr
    return out


def run(driver, *args):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    proc = subprocess.run([driver, *args], capture_output=True, text=True, env=env, timeout=120)
    text = proc.stdout + proc.stderr
    assert "AddressSanitizer" not in text and "runtime error" not in text, text
    assert proc.returncode == 0, text
    return text


def test_host_paths_are_clean_under_sanitizers_and_map_launch_failures(driver):
    text = run(driver)
    assert "0 checks failed" in text, text


def test_missing_scratch_symbol_is_reported_as_a_hip_error(driver):
    assert "status -5, 0 launches" in run(driver, "no-symbol")
