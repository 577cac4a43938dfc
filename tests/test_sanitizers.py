"""Host sanitizers (no GPU): the CPU oracle and the schedule front end (parser, legality rules, lowering,
search) are compiled with -fsanitize=address,undefined together with small drivers under tests/sanitize/
and run; any report from a sanitizer fails the test."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2401_04836_amd", "csrc")
SAN = os.path.join(ROOT, "tests", "sanitize")


def _run(exe):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="4")
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300, env=env)
    assert r.returncode == 0, r.stdout[-4000:]
    assert "runtime error" not in r.stdout and "AddressSanitizer" not in r.stdout and "LeakSanitizer" not in r.stdout, r.stdout[-4000:]
    return r.stdout


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "san_oracle")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-static-libasan", os.path.join(ROOT, "oracle", "oracle.c"),
           os.path.join(SAN, "san_oracle.c"), "-lm", "-o", exe]
    subprocess.check_call(cmd)
    assert "san_oracle: ok" in _run(exe)


def test_schedule_front_end_under_sanitizers(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("hipcc is not installed")
    exe = str(tmp_path / "san_schedule")
    cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fno-omit-frame-pointer",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-I" + CSRC, "-x", "hip",
           os.path.join(CSRC, "schedule.cpp"), os.path.join(CSRC, "search.cpp"), os.path.join(SAN, "san_schedule.cpp"),
           "-o", exe]
    subprocess.check_call(cmd)
    assert "san_schedule: ok" in _run(exe)
