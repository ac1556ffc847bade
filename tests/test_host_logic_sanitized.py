"""The library's host logic under AddressSanitizer and UndefinedBehaviorSanitizer, without a GPU: the
context state machine, the unit planner, the segment builder, policy-chosen unit order, the
bookkeeping of an enqueued launch sequence (every other call, moe_destroy included, is refused while
it is pending) and the scheduler.  qmoe_api.hip and qsched.hip are compiled as plain C++ with g++
against a stand-in for the HIP runtime header and recording stubs of the kernel launchers
(tests/host_stub/); the driver host_test.cpp holds the checks."""
import os
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
STUB = os.path.join(HERE, "host_stub")
CSRC = os.path.join(ROOT, "paper_2503_09304_amd", "csrc")


def test_host_logic_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "host_test")
    cmd = ["g++", "-std=c++17", "-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-I", STUB, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           "-x", "c++", os.path.join(CSRC, "qmoe_api.hip"), os.path.join(CSRC, "qsched.hip"),
           os.path.join(STUB, "stub_launches.cpp"), os.path.join(STUB, "host_test.cpp"), "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0 and "sanitizer" in r.stderr.lower() and "cannot find" in r.stderr.lower():
        pytest.skip("no sanitizer runtime for g++ on this machine")
    assert r.returncode == 0, r.stderr[-4000:]
    # verify_asan_link_order=0: other preloaded libraries of the environment may come before the sanitizer runtime
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    print(r.stdout[-3000:])
    assert r.returncode == 0, (r.stdout[-3000:], r.stderr[-3000:])
    assert "all host-logic checks passed" in r.stdout


def test_oracle_under_asan_and_ubsan(tmp_path):
    """The oracle's C code through one small layer in both dtypes, every buffer a heap block of exactly
    the documented size (tests/host_stub/oracle_asan_test.c)."""
    exe = str(tmp_path / "oracle_asan_test")
    cmd = ["gcc", "-O1", "-g", "-fopenmp", "-fno-fast-math", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           os.path.join(ROOT, "oracle", "moe_oracle.c"), os.path.join(STUB, "oracle_asan_test.c"), "-o", exe, "-lm"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0 and "sanitizer" in r.stderr.lower() and "cannot find" in r.stderr.lower():
        pytest.skip("no sanitizer runtime for gcc on this machine")
    assert r.returncode == 0, r.stderr[-4000:]
    # leak detection off: the OpenMP runtime keeps its thread pool until exit
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="4")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    print(r.stdout[-2000:])
    assert r.returncode == 0, (r.stdout[-3000:], r.stderr[-3000:])
    assert "oracle ran clean under the sanitizers" in r.stdout
