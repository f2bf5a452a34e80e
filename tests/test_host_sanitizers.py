"""Host logic of the library under AddressSanitizer and UBSan (no GPU needed).

The API source (descriptor validation, size formulas, problem tables, kernel choice) is compiled
for the host with both sanitizers and linked against stand-ins for the kernel launchers that
check every launch's parameters against what the kernels assume (tests/host/launcher_stubs.cpp).
A driver (tests/host/abi_host_check.cpp) then calls every entry point with every supported
representation, random mixes of matrices per launch, and 20,000 random descriptors.  Device code
is compiled without sanitizers: they are not available for the GPU here.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
pytestmark = pytest.mark.skipif(shutil.which(HIPCC) is None, reason="hipcc not available")

FLAGS = ["--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
         "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]
ENV = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=0:abort_on_error=0",
           UBSAN_OPTIONS="print_stacktrace=1")


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    out = tmp_path_factory.mktemp("host") / "abi_host_check"
    cmd = [HIPCC, *FLAGS,
           os.path.join(ROOT, "paper_2402_15319_amd", "csrc", "vq_api.hip"),
           os.path.join(ROOT, "tests", "host", "launcher_stubs.cpp"),
           os.path.join(ROOT, "tests", "host", "abi_host_check.cpp"), "-o", str(out)]
    res = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    assert res.returncode == 0, res.stderr[-3000:]
    return str(out)


def test_host_logic_is_clean_under_asan_and_ubsan(driver):
    res = subprocess.run([driver], capture_output=True, text=True, timeout=600, env=ENV)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-4000:]
    assert res.stdout.strip().endswith("host check ok")
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr


def test_a_planted_heap_overflow_is_reported(driver):
    res = subprocess.run([driver, "--plant-overflow"], capture_output=True, text=True, timeout=60, env=ENV)
    assert res.returncode != 0
    assert "AddressSanitizer" in res.stderr and "heap-buffer-overflow" in res.stderr


def test_a_planted_launch_mismatch_is_reported(driver):
    res = subprocess.run([driver, "--plant-launch"], capture_output=True, text=True, timeout=60, env=ENV)
    assert res.returncode != 0
    assert "launcher stub" in res.stderr and "violated" in res.stderr
