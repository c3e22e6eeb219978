"""Compiles the HIP sources under csrc/ into libspmi.so (gfx950 only), next to this file."""
import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libspmi.so")
SOURCES = sorted(glob.glob(os.path.join(HERE, "csrc", "*.hip")))
HEADERS = sorted(glob.glob(os.path.join(HERE, "csrc", "*.h"))) + [os.path.join(ROOT, "include", "spmi.h"), os.path.join(ROOT, "include", "spmi_bench.h")]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-fp32 instructions off (device pass only; the host pass warns that it ignores it)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-munsafe-fp-atomics",            # hardware floating-point atomic adds for the scatter kernels
    "-Wno-unused-command-line-argument",
]


def is_stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


def build(verbose=False):
    """Always compiles.  Objects are built in parallel, then linked."""
    bdir = os.path.join(HERE, "_build")
    os.makedirs(bdir, exist_ok=True)
    procs, objs = [], []
    for src in SOURCES:
        obj = os.path.join(bdir, os.path.basename(src) + ".o")
        objs.append(obj)
        cmd = ["hipcc", "-c", src, "-o", obj, "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc")] + \
              [f for f in FLAGS if f != "-shared"]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)))
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.decode().splitlines() if "packed-fp32-ops" not in l and l.strip())
        if p.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, out))
        if verbose and out:
            print(out)
    tmp = LIB + ".tmp%d" % os.getpid()
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs)
    os.replace(tmp, LIB)
    return LIB


HOSTSAN_LIB = os.path.join(HERE, "libspmi_hostsan.so")


def sanitizer_runtime():
    """The AddressSanitizer runtime of the clang that hipcc drives (to preload into a process that loads HOSTSAN_LIB)."""
    out = subprocess.check_output(["hipcc", "--offload-arch=gfx950", "-print-file-name=libclang_rt.asan-x86_64.so"]).decode().strip()
    if os.path.isabs(out) and os.path.exists(out):
        return out
    hits = sorted(glob.glob(os.path.join(os.environ.get("ROCM_PATH", "/opt/rocm"), "lib", "llvm", "lib", "clang", "*", "lib", "linux",
                                         "libclang_rt.asan-x86_64.so")))
    return hits[-1] if hits else None


def build_host_sanitized():
    """The same library with its HOST code under AddressSanitizer and UndefinedBehaviorSanitizer (the device code is built as
    usual: GPU sanitizers are not used).  For the CPU test that drives the host-only paths of the ABI; never loaded otherwise."""
    bdir = os.path.join(HERE, "_build", "hostsan")
    os.makedirs(bdir, exist_ok=True)
    san = []
    for f in ("-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"):
        san += ["-Xarch_host", f]
    procs, objs = [], []
    for src in SOURCES:
        obj = os.path.join(bdir, os.path.basename(src) + ".o")
        objs.append(obj)
        cmd = ["hipcc", "-c", src, "-o", obj, "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc")] + \
              [f for f in FLAGS if f not in ("-shared", "-O3")] + ["-O1", "-g"] + san
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)))
    for src, p in procs:
        out, _ = p.communicate()
        if p.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, out.decode()))
    tmp = HOSTSAN_LIB + ".tmp%d" % os.getpid()
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address,undefined", "-shared-libsan", "-o", tmp] + objs)
    os.replace(tmp, HOSTSAN_LIB)
    return HOSTSAN_LIB


C_CLIENT_SRC = os.path.join(ROOT, "tests", "c_client", "client.c")
C_CLIENT = os.path.join(ROOT, "tests", "c_client", "client")


def build_c_client():
    """The plain-C client of the ABI used by the tests: gcc, the public header as C, linked against libspmi.so."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    tmp = C_CLIENT + ".tmp%d" % os.getpid()
    subprocess.check_call(["gcc", "-std=c99", "-O1", "-Wall", "-Wextra", "-Werror", "-D__HIP_PLATFORM_AMD__", "-isystem", os.path.join(rocm, "include"),
                           "-I", os.path.join(ROOT, "include"), C_CLIENT_SRC, "-o", tmp, "-L", HERE, "-lspmi",
                           "-L", os.path.join(rocm, "lib"), "-lamdhip64",
                           "-Wl,-rpath,$ORIGIN/../../paper_2202_04305_amd", "-Wl,-rpath," + os.path.join(rocm, "lib")])
    os.replace(tmp, C_CLIENT)
    return C_CLIENT


if __name__ == "__main__":
    print(build(verbose=True))
    print(build_c_client())
