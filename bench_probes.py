"""Builds and loads the benchmark's measurement probes (bench_probes.hip -> libbench_probes.so beside
bench.py).  They are measurement tooling, not part of libepara: bandwidth / matrix-rate ceilings and a
copy kernel of known traffic for calibrating profiler counters."""
import ctypes
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "bench_probes.hip")
LIB = os.path.join(HERE, "libbench_probes.so")
_lib = None


def build(force=False):
    if force or not os.path.exists(LIB) or os.path.getmtime(LIB) < os.path.getmtime(SRC):
        tmp = LIB + ".tmp%d" % os.getpid()
        subprocess.check_call([os.environ.get("HIPCC", "/opt/rocm/bin/hipcc"), "--offload-arch=gfx950", "-O3", "-std=c++17",
                               "-fPIC", "-shared", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", SRC, "-o", tmp],
                              stderr=subprocess.DEVNULL)
        os.replace(tmp, LIB)
    return LIB


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        L.probe_read.argtypes = [vp, i64, vp, i32, vp]
        L.probe_copy.argtypes = [vp, vp, i64, vp]
        L.probe_mfma.argtypes = [vp, i32, vp, i32, vp]
        for name in ("probe_read", "probe_copy", "probe_mfma"):
            getattr(L, name).restype = i32
        _lib = L
    return _lib


def _check(rc, what):
    if rc != 0:
        raise RuntimeError("%s failed with status %d" % (what, rc))


def probe_read(d_buf, nbytes, d_sink, n_workgroups, stream=0):
    _check(lib().probe_read(int(d_buf), int(nbytes), int(d_sink), int(n_workgroups), int(stream) or None), "probe_read")


def probe_copy(d_src, d_dst, nbytes, stream=0):
    _check(lib().probe_copy(int(d_src), int(d_dst), int(nbytes), int(stream) or None), "probe_copy")


def probe_mfma(d_operands, iters, d_sink, n_workgroups, stream=0):
    _check(lib().probe_mfma(int(d_operands), int(iters), int(d_sink), int(n_workgroups), int(stream) or None), "probe_mfma")
