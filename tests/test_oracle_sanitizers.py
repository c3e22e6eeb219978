"""The CPU checker under AddressSanitizer and UndefinedBehaviorSanitizer (host code only, no GPU).

oracle.c is compiled a second time with -fsanitize=address,undefined (every finding aborts) and the checker's own
pins run against that build in a child process that has the sanitizer runtime preloaded: the paper's worked examples,
the enumerated-dense-tensor rebuilds, the error paths (bad rank, level type, ordering, width, coordinates, duplicates),
the products and their closed forms.  An out-of-bounds access, a use after free or a signed overflow anywhere on those
paths fails this test.
"""
import os
import subprocess
import sys

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_checker_pins_pass_under_asan_and_ubsan():
    oracle.build_sanitized()
    runtime = subprocess.check_output(["gcc", "-print-file-name=libasan.so"]).decode().strip()
    assert os.path.isabs(runtime) and os.path.exists(runtime), "no AddressSanitizer runtime next to gcc"
    env = dict(os.environ, ORACLE_SANITIZED="1", LD_PRELOAD=runtime,
               ASAN_OPTIONS="detect_leaks=0:abort_on_error=1:halt_on_error=1", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    which = subprocess.run([sys.executable, "-c", "import oracle; print(oracle.lib()._name)"], cwd=ROOT, env=env, stdout=subprocess.PIPE,
                           stderr=subprocess.STDOUT, timeout=120)
    assert which.returncode == 0 and which.stdout.decode().strip().endswith("liboracle_sanitized.so"), which.stdout.decode()
    files = ["tests/test_oracle_pack.py", "tests/test_oracle_matmul.py", "tests/test_oracle_sddmm.py", "tests/test_oracle_mttkrp.py",
             "tests/test_oracle_spgemm.py", "tests/test_oracle_add.py"]
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu"] + files, cwd=ROOT, env=env,
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, timeout=900)
    tail = r.stdout.decode(errors="replace")[-3000:]
    assert r.returncode == 0, "the checker's pins failed under the sanitizers:\n" + tail
    assert " passed" in tail and "ERROR: AddressSanitizer" not in tail and "runtime error:" not in tail, tail
