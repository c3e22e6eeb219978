"""The library used from plain C: tests/c_client/client.c is compiled with gcc against include/spmi.h (the build step
does that) and run here.  It relies on the library's default allocator (hipMalloc / hipFree)."""
import os
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
CLIENT = os.path.join(HERE, "c_client", "client")


def test_header_compiles_as_c_with_warnings_as_errors(tmp_path):
    """No GPU needed: the public header alone, as C99 and as C++17, pedantic."""
    inc = os.path.join(os.path.dirname(HERE), "include")
    src = tmp_path / "only_header.c"
    src.write_text('#include "spmi.h"\nint main(void) { return (int)SP_OK; }\n')
    subprocess.check_call(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", inc, "-c", str(src), "-o", str(tmp_path / "a.o")])
    subprocess.check_call(["g++", "-std=c++17", "-pedantic", "-Wall", "-Wextra", "-Werror", "-x", "c++", "-I", inc, "-c", str(src), "-o", str(tmp_path / "b.o")])


@pytest.mark.gpu
def test_c_client_runs():
    if not os.path.exists(CLIENT):      # normally built by __graft_entry__.build(); a one-second gcc step otherwise
        try:
            from paper_2202_04305_amd import build as hipbuild
            hipbuild.build_c_client()
        except Exception as e:          # no compiler or no ROCm headers here: nothing to run
            pytest.skip("the C client is not built and cannot be built here: %s" % e)
    r = subprocess.run([CLIENT], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, timeout=120)
    out = r.stdout.decode()
    print(out, flush=True)
    assert r.returncode == 0 and "c client ok" in out, out
