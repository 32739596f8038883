"""Builds libepara.so (HIP kernels + host planner) for gfx950, in-tree next to this file.

Every translation unit is compiled on its own (in parallel) and the objects are linked into one
shared library."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
UNITS = ["epara_k_bf16_plain.hip", "epara_k_bf16_gated.hip", "epara_k_fp8_plain.hip", "epara_k_fp8_gated.hip",
         "epara_c_bf16_plain.hip", "epara_c_bf16_ffn.hip", "epara_c_fp8_plain.hip", "epara_c_fp8_ffn.hip",
         "epara_k_f32.hip", "epara_launch.hip", "epara_rows.hip", "epara_block.hip", "epara_host.cpp"]
SOURCES = [os.path.join(CSRC, u) for u in UNITS]
HEADERS = [os.path.join(ROOT, "include", "epara.h")] + [os.path.join(CSRC, h) for h in (
    "epara_cast.h", "epara_device.h", "epara_internal.h", "epara_panel.h", "epara_stream.h", "epara_f32.h", "epara_grouped.h")]
LIB = os.path.join(HERE, "libepara.so")
OBJ_DIR = os.path.join(ROOT, "_build", "obj")

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed fp32 VALU forms
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def is_stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


def _compile(src, obj, hipcc, extra, verbose):
    cmd = [hipcc] + FLAGS + list(extra) + ["-c", src, "-o", obj]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s" % (src, out))
    return out


def build(force=True, verbose=False, jobs=None, extra=(), lib=None, csrc=None):
    """Compile with hipcc (cross-compiles without a GPU).  Returns the library path.
    lib / csrc: build another library from another copy of the sources (experiments)."""
    lib = lib or LIB
    if not force and lib == LIB and not is_stale():
        return lib
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    obj_dir = OBJ_DIR + ("" if lib == LIB else "_" + os.path.basename(lib))
    os.makedirs(obj_dir, exist_ok=True)
    sources = SOURCES if csrc is None else [os.path.join(csrc, u) for u in UNITS]
    if csrc is not None:
        extra = ["-I" + csrc] + list(extra)
    objs = [os.path.join(obj_dir, os.path.basename(s) + ".o") for s in sources]
    jobs = jobs or min(len(sources), max(1, min(16, os.cpu_count() or 1)))
    with ThreadPoolExecutor(jobs) as pool:
        outs = list(pool.map(lambda so: _compile(so[0], so[1], hipcc, extra, verbose), zip(sources, objs)))
    if verbose:
        print("\n".join(o for o in outs if o), flush=True)
    tmp = lib + ".tmp%d" % os.getpid()
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", tmp])
    os.replace(tmp, lib)
    return lib


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
