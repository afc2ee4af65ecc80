"""The C ABI's host logic under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only, no GPU is touched):
csrc/api.hip is compiled with the host sanitizers, linked with the ordinary objects of the other sources and with
tests/host_check/abi_host_check.cpp, which sweeps the size queries over many configurations, feeds every entry point
arguments it must refuse before any launch, and runs the host-side penalty-weight feedback.  A sanitizer report or a
wrong status fails the run."""
import os
import subprocess

from paper_2510_20787_amd import binding as B
from paper_2510_20787_amd import build


def test_abi_host_logic_under_sanitizers():
    B.lib()      # builds the library (and with it the objects the executable links) when nothing is built yet
    exe = build.build_host_check(verbose=False)
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout[-3000:] + "\n" + r.stderr[-6000:]
    assert "0 failures" in r.stdout
