"""The library's host simulator under AddressSanitizer and UBSan (host code only, no GPU): built with g++
together with a small driver that walks a grid of graphs, modes, frozen workers and latencies."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_simulator_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "sim_driver")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
           "-ffp-contract=off", "-I", os.path.join(ROOT, "include"),
           "-I", os.path.join(ROOT, "paper_1902_01064_amd", "csrc"),
           os.path.join(ROOT, "tests", "sim_driver.cpp"),
           os.path.join(ROOT, "paper_1902_01064_amd", "csrc", "hop_sim.cpp"), "-o", exe]
    subprocess.run(cmd, check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0")
    out = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert out.returncode == 0, out.stdout[-2000:] + out.stderr[-4000:]
    assert out.stdout.startswith("ok runs=")
    assert int(out.stdout.split("runs=")[1].split()[0]) > 200


@pytest.mark.skipif(shutil.which("g++") is None or not os.path.isdir("/opt/rocm/include"), reason="needs g++ and the HIP headers")
def test_c_abi_host_paths_are_clean_under_asan_and_ubsan(tmp_path):
    """hop_api.cpp + hop_sim.cpp built for the host with the sanitizers (kernel launchers stubbed: a context
    without device memory never reaches them): argument checking of every entry point, schedule views read
    to their full lengths, stalled runs, schedules freed before and after their context, leak check."""
    exe = str(tmp_path / "api_driver")
    csrc = os.path.join(ROOT, "paper_1902_01064_amd", "csrc")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
           "-ffp-contract=off", "-D__HIP_PLATFORM_AMD__", "-I", "/opt/rocm/include", "-I", os.path.join(ROOT, "include"),
           "-I", csrc, os.path.join(ROOT, "tests", "api_driver.cpp"), os.path.join(csrc, "hop_api.cpp"),
           os.path.join(csrc, "hop_sim.cpp"), "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib", "-o", exe]
    subprocess.run(cmd, check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0")
    out = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert out.returncode == 0, out.stdout[-2000:] + out.stderr[-4000:]
    assert out.stdout.startswith("ok total=")
