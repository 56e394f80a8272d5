"""The host side of the library (scheduler core, worker pool, lazy runtime, shared-memory front end) under
ThreadSanitizer and under AddressSanitizer + UBSan: tests/native/sched_stress.cpp drives them from
many threads on the null backend (no GPU code runs; sanitizers see host code only)."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CLANG = "/opt/rocm/llvm/bin/clang++"
SRCS = [os.path.join(HERE, "native", "sched_stress.cpp")] + [
    os.path.join(ROOT, "paper_2107_08538_amd", "csrc", f) for f in ("sched.cpp", "lazy.cpp", "ipc.cpp", "runner.cpp")]


def _build_and_run(tmp_path, name, flags, env=None):
    if not os.path.exists(CLANG) or not os.path.isdir("/opt/rocm/lib"):
        pytest.skip("ROCm clang++ not found")
    exe = str(tmp_path / name)
    cmd = [CLANG, "-std=c++17", "-O1", "-g", "-w", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include"] + flags + SRCS + [
        "-L/opt/rocm/lib", "-lamdhip64", "-lpthread", "-lrt", "-Wl,-rpath,/opt/rocm/lib", "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, text=True, timeout=600)
    e = dict(os.environ)
    e.update(env or {})
    r = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=e)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-6000:]
    assert "0 failed checks" in r.stdout
    assert "WARNING: ThreadSanitizer" not in r.stderr and "ERROR: AddressSanitizer" not in r.stderr
    assert "runtime error" not in r.stderr and "LeakSanitizer" not in r.stderr


def test_host_code_is_free_of_data_races(tmp_path):
    _build_and_run(tmp_path, "stress_tsan", ["-fsanitize=thread"], {"TSAN_OPTIONS": "halt_on_error=0 exitcode=66"})


def test_host_code_is_free_of_memory_errors_and_leaks(tmp_path):
    _build_and_run(tmp_path, "stress_asan", ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"],
                   {"ASAN_OPTIONS": "detect_leaks=1"})
