"""The library's host shell under AddressSanitizer and UndefinedBehaviorSanitizer (host code only; device code is built
as usual).  paper_2604_26555_amd/build.py:build_host_checked compiles csrc/som_api.hip with both sanitizers, links it
with the ordinary objects into libsom_hostsan.so and builds tests/host_shell_check.cpp against it; the driver exits
non-zero on a failed expectation, and a sanitizer report ends it with an error of its own.

Without a GPU the driver covers what needs no device (error strings, null contexts, creation on a missing device).  On
the GPU machine it goes on to one context on device 0: streamed epochs from memory and from a file with several reader
threads, the short-file and bad-argument paths, a resident epoch, create / destroy twice."""
import os
import subprocess

import pytest

from paper_2604_26555_amd import build as libbuild

ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:protect_shadow_gap=0:abort_on_error=0",
           UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")


def run_driver(*args, timeout):
    r = subprocess.run([libbuild.HOST_CHECKED_DRIVER, *args], env=ENV, capture_output=True, text=True, timeout=timeout)
    print(r.stdout[-2000:], r.stderr[-6000:], flush=True)
    assert r.returncode == 0, f"host_shell_check {' '.join(args)} ended with status {r.returncode}"
    assert "host_shell_check: ok" in r.stdout
    assert "ERROR: AddressSanitizer" not in r.stderr and "runtime error:" not in r.stderr


def test_host_shell_without_a_device():
    objs = [os.path.join(libbuild.HERE, "_build", s.replace(".hip", ".o")) for s in libbuild.SOURCES]
    if not all(os.path.exists(o) for o in objs):
        libbuild.build(verbose=False)
    libbuild.build_host_checked(verbose=False)
    run_driver(timeout=60)


@pytest.mark.gpu
def test_host_shell_on_the_device():
    if not os.path.exists(libbuild.HOST_CHECKED_DRIVER):
        pytest.skip("the instrumented driver has not been built (__graft_entry__.build() builds it)")
    run_driver("--device", timeout=110)
