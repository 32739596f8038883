"""Builds libepara.so (HIP kernels + host planner) for gfx950, in-tree next to this file."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SOURCES = [os.path.join(HERE, "csrc", "epara_kernels.hip"), os.path.join(HERE, "csrc", "epara_rows.hip"),
           os.path.join(HERE, "csrc", "epara_probe.hip"), os.path.join(HERE, "csrc", "epara_host.cpp")]
HEADER = os.path.join(ROOT, "include", "epara.h")
CAST_HEADER = os.path.join(HERE, "csrc", "epara_cast.h")
LIB = os.path.join(HERE, "libepara.so")

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed fp32 VALU forms
         "-I" + os.path.join(ROOT, "include")]


def is_stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in SOURCES + [HEADER, CAST_HEADER])


def build(force=True, verbose=False):
    """Compile with hipcc (cross-compiles without a GPU).  Returns the library path."""
    if not force and not is_stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + ".tmp%d" % os.getpid()
    cmd = [hipcc] + FLAGS + SOURCES + ["-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
