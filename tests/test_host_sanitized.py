"""Host robustness without a GPU: the plan code of the C ABI and the CPU oracle, each built with
sanitizers into an executable of its own and run here.

  * paper_1911_03458_amd/csrc/host_check.cpp against the host side of every library source
    (hipcc --cuda-host-only, seconds to build) under AddressSanitizer + UBSan: a seeded sweep of
    valid, odd and invalid shapes over every plan constructor, every query, tile requests, the
    error paths of every operation entry point (nothing is ever launched);
  * the same program under ThreadSanitizer with eight threads and one shared plan (merit.h:
    "a plan may be shared between threads");
  * oracle/oracle_check.c + merit_oracle.c under AddressSanitizer + UBSan: every ref_ function
    on exact-size buffers at the shapes where an index rule is most likely to slip.
"""
import os
import subprocess

import pytest

import oracle
from paper_1911_03458_amd import build as hip_build

# the sanitizer runtimes must not find another runtime preloaded in front of them complaining;
# the executables are self-contained, the environment is passed through unchanged
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
           UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1", TSAN_OPTIONS="halt_on_error=1")


def _run(cmd):
    proc = subprocess.run(cmd, capture_output=True, text=True, env=ENV, timeout=600)
    assert proc.returncode == 0, proc.stdout[-3000:] + proc.stderr[-6000:]
    assert "runtime error" not in proc.stderr and "Sanitizer" not in proc.stderr, proc.stderr[-6000:]
    return proc.stdout


def test_plan_code_under_address_and_undefined_behaviour_sanitizers():
    out = _run([hip_build.build_host_check("address,undefined")])
    assert "0 failed checks" in out and "plans made" in out, out


def test_plan_code_from_eight_threads_under_thread_sanitizer():
    out = _run([hip_build.build_host_check("thread"), "8"])
    assert "0 failed checks" in out and "8 thread(s)" in out, out


def test_oracle_under_address_and_undefined_behaviour_sanitizers():
    out = _run([oracle.build_sanitized_check()])
    assert "0 failed checks" in out, out
