"""The host side of the library under AddressSanitizer and UndefinedBehaviorSanitizer: tests/host_sanitize_driver.cpp
is built with the library's sources into one executable whose host code is instrumented (__graft_entry__.
build_sanitize_driver; device code is not instrumented) and exercises the C ABI directly.  Without a GPU it runs the
argument checks and host-only routines of every entry point; with one, every kind of call on tiny random models.
A sanitizer report aborts the run, a failed check makes the exit status 1."""
import os
import subprocess

import pytest

import __graft_entry__ as entry

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SOURCES = [os.path.join(ROOT, "paper_2407_19947_amd", "csrc", n) for n in
           ("stairs_kernels.hip", "stairs_kernels.h", "stairs_api.hip")] + \
          [os.path.join(ROOT, "include", "stairs.h"), entry.SANITIZE_DRIVER + ".cpp"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")


def _run(timeout):
    res = subprocess.run([entry.SANITIZE_DRIVER], capture_output=True, text=True, env=ENV, timeout=timeout)
    print(res.stdout[-2000:], res.stderr[-6000:], flush=True)
    return res


def test_argument_checks_under_host_sanitizers():
    """No GPU: (re)build the instrumented driver when it is missing or older than a source, run part 1."""
    exe = entry.SANITIZE_DRIVER
    if not os.path.exists(exe) or any(os.path.getmtime(s) > os.path.getmtime(exe) for s in SOURCES):
        entry.build_sanitize_driver()
    res = _run(120)
    assert res.returncode == 0
    assert "part 1 (no GPU): 0 failed checks" in res.stdout


@pytest.mark.gpu
def test_every_kind_of_call_under_host_sanitizers():
    """GPU: the prebuilt driver (built on the CPU beforehand, never here) through prefill, generation, batches,
    sampling, end token, encoder-decoder and the diagnostics."""
    if not os.path.exists(entry.SANITIZE_DRIVER):
        pytest.skip("instrumented driver not built (python -c 'import __graft_entry__ as g; g.build()' builds it)")
    res = _run(300)
    assert res.returncode == 0
    assert "part 2 (encoder-decoder): 0 failed checks in all" in res.stdout
