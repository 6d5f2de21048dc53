"""The lock-free ring and the proxy threads under ThreadSanitizer and
AddressSanitizer (host code only: a CPU producer stands in for the kernels and
speaks the same slot protocol)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = [os.path.join(ROOT, "paper_2512_19849_amd", "csrc", "proxy.cpp"),
       os.path.join(ROOT, "paper_2512_19849_amd", "csrc", "api.cpp"),
       os.path.join(ROOT, "tests", "native", "host_ring_driver.cpp")]


def _build_and_run(tmp_path, sanitizer, *args):
    if not shutil.which("g++") or not os.path.exists("/opt/rocm/include/hip/hip_runtime_api.h"):
        pytest.skip("g++ or the HIP headers are not available")
    exe = str(tmp_path / f"driver_{sanitizer}")
    cmd = ["g++", "-std=c++17", "-O1", "-g", f"-fsanitize={sanitizer}", "-fno-omit-frame-pointer",
           "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", *SRC, "-o", exe, "-L/opt/rocm/lib", "-lamdhip64",
           "-lpthread", "-lrt", "-Wl,-rpath,/opt/rocm/lib"]
    subprocess.run(cmd, check=True, capture_output=True, timeout=300)
    env = dict(os.environ, TSAN_OPTIONS="halt_on_error=0 report_signal_unsafe=0",
               ASAN_OPTIONS="detect_leaks=0 protect_shadow_gap=0")
    return subprocess.run([exe, *args], capture_output=True, text=True, timeout=300, env=env)


def test_ring_and_proxy_are_clean_under_thread_sanitizer(tmp_path):
    r = _build_and_run(tmp_path, "thread")
    assert r.returncode == 0, r.stdout + r.stderr
    assert "ThreadSanitizer" not in r.stderr, r.stderr[-3000:]
    assert r.stdout.count("rc 0") == 3


def test_proxy_policies_and_ring_channels_under_thread_sanitizer(tmp_path):
    r = _build_and_run(tmp_path, "thread", "policies")
    assert r.returncode == 0, r.stdout + r.stderr
    assert "ThreadSanitizer" not in r.stderr, r.stderr[-3000:]
    assert r.stdout.count("rc 0") == 3 and r.stdout.count("policies:") == 3


def test_proxy_policies_and_ring_channels_under_address_sanitizer(tmp_path):
    r = _build_and_run(tmp_path, "address,undefined", "policies")
    assert r.returncode == 0, r.stdout + r.stderr
    assert "AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-3000:]


def test_ring_and_proxy_are_clean_under_address_sanitizer(tmp_path):
    r = _build_and_run(tmp_path, "address,undefined")
    assert r.returncode == 0, r.stdout + r.stderr
    assert "AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-3000:]
