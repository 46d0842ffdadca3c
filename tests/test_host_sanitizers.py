"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer, on the CPU only (no GPU code is
sanitized): the library's pool / scheduler / buffer-recycling logic with stand-in HIP calls and
launchers that check every work list against what the kernels assume, and the C oracle on
exact-size buffers.  The drivers are tests/sanitize/*.c*; they are compiled here and run as
child processes."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def run(exe, *args):
    r = subprocess.run([exe, *args], capture_output=True, text=True, env=ENV, timeout=600)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-6000:]
    return r.stdout


@pytest.mark.skipif(shutil.which("g++") is None, reason="no host C++ compiler")
def test_host_logic_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "host_san")
    src = [os.path.join(ROOT, "tests", "sanitize", "host_san.cpp"),
           os.path.join(ROOT, "paper_2311_03285_amd", "csrc", "pool.cpp"),
           os.path.join(ROOT, "paper_2311_03285_amd", "csrc", "plan.cpp")]
    subprocess.check_call(["g++", "-std=c++17", *SAN, "-w", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
                           "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(ROOT, "paper_2311_03285_amd", "csrc"),
                           *src, "-o", exe])
    for seed in ("1", "2", "3", "4"):
        assert "host_san OK" in run(exe, seed)


@pytest.mark.skipif(shutil.which("gcc") is None, reason="no host C compiler")
def test_oracle_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    subprocess.check_call(["gcc", "-std=c11", *SAN, "-fopenmp", os.path.join(ROOT, "tests", "sanitize", "oracle_san.c"),
                           os.path.join(ROOT, "oracle", "slora_oracle.c"), "-o", exe, "-lm"])
    assert "oracle_san OK" in run(exe)
