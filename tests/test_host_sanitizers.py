"""The library's host-only logic (packing plan of Sec. 4.1, planner of Alg. 1) under
AddressSanitizer and UBSan: tests/host_sanitize_driver.cpp feeds it random and damaged inputs and
checks the structure of what comes back; a memory error or undefined behaviour aborts the program.

Host code only: the translation unit holds no HIP call, so the host compiler builds it alone."""
from __future__ import annotations

import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2303_02868_amd", "csrc")


@pytest.mark.skipif(shutil.which("g++") is None, reason="no host C++ compiler")
def test_host_logic_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "host_sanitize")
    cmd = ["g++", "-std=c++17", "-g", "-O1", "-Wall", "-Wextra", "-Werror",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-static-libubsan",
           "-D__HIP_PLATFORM_AMD__", "-isystem", "/opt/rocm/include",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           os.path.join(ROOT, "tests", "host_sanitize_driver.cpp"), os.path.join(CSRC, "apm_host.cpp"),
           "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0:verify_asan_link_order=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1"
    r = subprocess.run([exe, "4000"], capture_output=True, text=True, env=env, timeout=300)
    if r.returncode != 0 and "unexpected memory mapping" in r.stderr:
        pytest.skip("the sanitizer runtime cannot map its shadow memory on this machine")
    assert r.returncode == 0, r.stdout + r.stderr
    assert r.stdout.strip() == "ok 4000"


@pytest.mark.skipif(shutil.which("g++") is None, reason="no host C++ compiler")
@pytest.mark.parametrize("sanitizer", ["thread", "address,undefined"])
def test_file_tier_thread_choreography_under_sanitizers(tmp_path, sanitizer):
    """The third tier's I/O thread pool and window chain (Alg. 2's fetch / update / offload, batch by
    batch) with a CPU loop in place of the kernel: results in the files after several passes, a
    failed read, a processing side that gives up -- under ThreadSanitizer, then ASan + UBSan."""
    exe = str(tmp_path / "host_tier")
    static = ["-static-libtsan"] if sanitizer == "thread" else ["-static-libasan", "-static-libubsan"]
    cmd = ["g++", "-std=c++17", "-g", "-O1", "-Wall", "-Wextra", "-Werror", "-pthread",
           f"-fsanitize={sanitizer}", "-fno-sanitize-recover=all"] + static + [
           "-I", CSRC, os.path.join(ROOT, "tests", "host_tier_driver.cpp"), "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr
    work = tmp_path / "files"
    work.mkdir()
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=1:verify_asan_link_order=0"
    env["TSAN_OPTIONS"] = "halt_on_error=1:second_deadlock_stack=1"
    r = subprocess.run([exe, str(work)], capture_output=True, text=True, env=env, timeout=600)
    if r.returncode != 0 and "unexpected memory mapping" in r.stderr:
        pytest.skip("the sanitizer runtime cannot map its shadow memory on this machine")
    assert r.returncode == 0, r.stdout + r.stderr
    assert r.stdout.strip().splitlines()[-1] == "ok"
