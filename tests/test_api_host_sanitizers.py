"""The library's HOST code under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU; the device code is not sanitized).

The sources are compiled a second time with the sanitizers on the host pass, and a child process with the sanitizer runtime
preloaded drives the paths of the C ABI that end before or at the first device call: descriptors of every rank and every way
to get one wrong, sp_pack's argument checks, null handles everywhere, the status strings.  A report (out-of-bounds access,
use after free, a load of an invalid enumeration value, signed overflow ...) aborts the child and fails this test.
"""
import os
import subprocess
import sys

from paper_2202_04305_amd import build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_paths_of_the_abi_under_asan_and_ubsan():
    lib = build.build_host_sanitized()
    runtime = build.sanitizer_runtime()
    assert runtime, "no AddressSanitizer runtime next to hipcc's clang"
    env = dict(os.environ, LD_PRELOAD=runtime, ASAN_OPTIONS="detect_leaks=0:abort_on_error=1:halt_on_error=1",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = subprocess.run([sys.executable, os.path.join(ROOT, "tests", "host_sanitizer_child.py"), lib], cwd=ROOT, env=env,
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, timeout=600)
    text = r.stdout.decode(errors="replace")
    assert r.returncode == 0, text[-3000:]
    assert "host paths ok" in text and "runtime error:" not in text and "ERROR: AddressSanitizer" not in text, text[-3000:]
