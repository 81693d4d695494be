"""Host side of the library under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only): argument checks and
size arithmetic of every entry point, driven with extreme and invalid arguments by tests/host/host_check.cpp.  No call
gets past its checks, so nothing touches a device; device code is not instrumented."""
import os
import subprocess

from paper_2603_25702_amd import build


def test_argument_checks_and_size_arithmetic_are_clean_under_asan_and_ubsan():
    exe = build.build_host_check()
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    env.pop("LD_PRELOAD", None)   # the sanitizer runtime has to come first in the library list
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120, env=env)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
    assert "host_check: 0 failed expectation(s)" in r.stdout
