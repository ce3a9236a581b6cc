"""AddressSanitizer + UndefinedBehaviorSanitizer runs of the CPU code: the oracle (C) and the library's host-side state
(stride policy, pager: plain C++ without device code).  Each driver is a small program next to this file that is
compiled with the code under test and run once; a report from either sanitizer (or a leak) ends it with a non-zero
status.  The GPU kernels cannot run under these sanitizers; their index arithmetic is covered by the parity tests and the
host-side launch checks."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
SAN = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all"]


def _build_and_run(tmp_path, compiler, args, src, timeout=240):
    if shutil.which(compiler) is None:
        pytest.skip(f"{compiler} not available")
    exe = str(tmp_path / "driver")
    probe = subprocess.run([compiler, *SAN, "-x", "c", "-", "-o", exe], input=b"int main(void){return 0;}", capture_output=True)
    if probe.returncode != 0:
        pytest.skip("the sanitizer runtimes are not installed for this compiler")
    subprocess.check_call([compiler, *SAN, *args, os.path.join(HERE, src), "-o", exe, "-lm"])
    # (verify_asan_link_order=0: the runtime need not be the first library of the process, whatever the environment preloads)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="2")
    r = subprocess.run([exe], capture_output=True, timeout=timeout, env=env)
    out = r.stdout.decode() + r.stderr.decode()
    assert r.returncode == 0 and out.startswith("ok"), out[-4000:]


def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    _build_and_run(tmp_path, "gcc", ["-std=c11", "-fopenmp"], "sanitize_oracle_main.c")


def test_host_state_runs_clean_under_asan_and_ubsan(tmp_path):
    _build_and_run(tmp_path, "g++", ["-std=c++17", "-x", "c++", "-I" + os.path.join(HERE, "..", "include")],
                   "sanitize_host_state_main.cpp")
