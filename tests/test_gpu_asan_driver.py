"""The device paths of the C ABI with the library's HOST code under AddressSanitizer and UBSan, on a real
GPU: tests/gpu_driver.cpp (built by paper_1902_01064_amd.build into tests/_bin/) walks contexts, every
gradient source, momentum, partial wave ranges, profiling, graph replay, data swaps and frees in awkward
orders.  Kernels are the product's own, uninstrumented."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
EXE = os.path.join(ROOT, "tests", "_bin", "gpu_asan_driver")


@pytest.mark.skipif(not os.path.exists(EXE), reason="tests/_bin/gpu_asan_driver not built (python -m paper_1902_01064_amd.build)")
def test_device_paths_host_code_is_clean_under_asan_and_ubsan():
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:verify_asan_link_order=0:protect_shadow_gap=0")
    out = subprocess.run([EXE], capture_output=True, text=True, env=env, timeout=240)
    assert out.returncode == 0, out.stdout[-2000:] + out.stderr[-4000:]
    assert out.stdout.strip().endswith("ok")
