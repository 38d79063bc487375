"""The host-only code of the library (work planner, argument validation, the entry points that never touch a GPU, and
the scheduling library) built with g++ under the address and undefined-behaviour sanitizers, and the CPU tests of
those parts run against that build in a child process: any report (heap overflow in the planner's vectors, signed
overflow in the sizing arithmetic, misaligned or out-of-bounds reads of the caller's arrays) fails the run."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _preload_in_use():
    if os.environ.get("LD_PRELOAD"):
        return True
    try:
        return bool(open("/etc/ld.so.preload").read().strip())
    except OSError:
        return False


@pytest.mark.timeout(600)
def test_planner_validation_and_scheduler_run_clean_under_sanitizers():
    sys.path.insert(0, ROOT)
    from paper_2602_14516_amd.build import build_host_sanitized
    # the address sanitizer's runtime has to be the first library of the child process; where something else is
    # preloaded already, only the undefined-behaviour sanitizer (which needs no preload) is used
    address = not _preload_in_use()
    host_lib, sched_lib, runtime = build_host_sanitized(address=address)
    env = dict(os.environ, AMPD_LIB_PATH=host_lib, AMPD_HOST_ONLY="1", AMPD_SCHED_LIB_PATH=sched_lib,
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1",
               ASAN_OPTIONS="detect_leaks=0:halt_on_error=1:abort_on_error=0")
    if runtime:
        env["LD_PRELOAD"] = runtime
    # the two tests that push invalid arguments through ampd_kv_append need the GPU half of the library
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", os.path.join(ROOT, "tests", "test_host_abi.py"),
           os.path.join(ROOT, "tests", "test_sched.py"), os.path.join(ROOT, "tests", "test_simulator.py"),
           "-k", "not rejects_bad_arguments and not page_range_check and not exports_every_symbol"]
    res = subprocess.run(cmd, cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=580)
    out = res.stdout
    assert "AddressSanitizer" not in out and "runtime error:" not in out, out[-4000:]
    assert res.returncode == 0, out[-4000:]
    assert " passed" in out
