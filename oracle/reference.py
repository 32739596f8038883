"""numpy front end of the fp64 C oracle (test infrastructure only).

Every function takes the LOGICAL operands: X [M,K], W [K,N] (row-major, as the
formula Y = act(s * X W + b) reads), b [N].  Low-precision operands arrive as
their bit patterns (uint16 bfloat16, uint8 E4M3) and are decoded here, by the
oracle's own decoders, to the exact values they represent.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dense_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

ACT = {"none": 0, "relu": 1, "gelu_erf": 2, "gelu_tanh": 3, "silu": 4}

_lib = None


def build(force=False):
    """Compile dense_oracle.c with gcc (-O2, OpenMP) next to its source."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", _SRC, "-o", tmp, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        dp = ctypes.POINTER(ctypes.c_double)
        i64, f64, i32 = ctypes.c_int64, ctypes.c_double, ctypes.c_int
        L.oracle_dense_forward.argtypes = [dp, dp, dp, i64, i64, i64, f64, i32, dp]
        L.oracle_dense_forward.restype = None
        L.oracle_swiglu_hidden.argtypes = [dp, dp, dp, i64, i64, i64, f64, f64, dp]
        L.oracle_swiglu_hidden.restype = None
        L.oracle_act_array.argtypes = [dp, i64, i32, dp]
        L.oracle_act_array.restype = None
        L.oracle_bf16_decode.argtypes = [ctypes.POINTER(ctypes.c_uint16), i64, dp]
        L.oracle_bf16_decode.restype = None
        L.oracle_bf16_encode.argtypes = [ctypes.POINTER(ctypes.c_float), i64, ctypes.POINTER(ctypes.c_uint16)]
        L.oracle_bf16_encode.restype = None
        L.oracle_e4m3_decode.argtypes = [ctypes.POINTER(ctypes.c_uint8), i64, f64, dp]
        L.oracle_e4m3_decode.restype = None
        L.oracle_e4m3_encode.argtypes = [dp, i64, f64, ctypes.POINTER(ctypes.c_uint8)]
        L.oracle_e4m3_encode.restype = None
        L.oracle_threads.argtypes = []
        L.oracle_threads.restype = i32
        _lib = L
    return _lib


def threads():
    """Number of OpenMP threads the C loops will use."""
    return int(lib().oracle_threads())


def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _dp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def act(z, name):
    z = _f64(z)
    out = np.empty_like(z)
    lib().oracle_act_array(_dp(z), z.size, ACT[name], _dp(out))
    return out


def dense_forward(X, W, b=None, act="none", s=1.0):
    """Y = act(s * X W + b) in fp64 by the naive triple loop.  X [M,K], W [K,N], b [N] or None."""
    X, W = _f64(X), _f64(W)
    M, K = X.shape
    K2, N = W.shape
    if K != K2:
        raise ValueError("inner dimensions differ")
    Y = np.empty((M, N), dtype=np.float64)
    bp = None
    if b is not None:
        b = _f64(b)
        if b.shape != (N,):
            raise ValueError("bias shape")
        bp = _dp(b)
    lib().oracle_dense_forward(_dp(X), _dp(W), bp, M, K, N, float(s), ACT[act], _dp(Y))
    return Y


def swiglu_hidden(X, Wgate, Wup, s_gate=1.0, s_up=1.0):
    """H = SiLU(s_gate * X Wgate) * (s_up * X Wup) in fp64."""
    X, Wgate, Wup = _f64(X), _f64(Wgate), _f64(Wup)
    M, K = X.shape
    if Wgate.shape != Wup.shape or Wgate.shape[0] != K:
        raise ValueError("shape mismatch")
    F = Wgate.shape[1]
    H = np.empty((M, F), dtype=np.float64)
    lib().oracle_swiglu_hidden(_dp(X), _dp(Wgate), _dp(Wup), M, K, F, float(s_gate), float(s_up), _dp(H))
    return H


def ffn_swiglu(X, Wgate, Wup, Wdown, s_gate=1.0, s_up=1.0, s_down=1.0, h_scale=None):
    """Y = (SiLU(X Wgate) * (X Wup)) Wdown.  Returns (H, Y).

    h_scale=None keeps H in fp64.  With h_scale = s_h the hidden activations are
    requantised to E4M3 (q = sat(RNE(H / s_h))) before the down projection, as the
    fp8 path stores them; then H is returned as the dequantised values s_h * q and
    s_down must already include s_h.
    """
    return ffn_swiglu_down(swiglu_hidden(X, Wgate, Wup, s_gate, s_up), Wdown, s_down, h_scale)


def ffn_swiglu_down(H, Wdown, s_down=1.0, h_scale=None):
    """Second half of ffn_swiglu from given hidden activations H (fp64): returns (H as stored, Y)."""
    if h_scale is not None:
        H = e4m3_decode(e4m3_encode(H, h_scale), 1.0)       # codes as values, scale folded in s_down
        Y = dense_forward(H, Wdown, None, "none", s_down)
        return H * h_scale, Y
    return H, dense_forward(H, Wdown, None, "none", s_down)


def mlp_chain(X, layers):
    """layers: list of (W, b, act).  Returns the list of every layer's output."""
    outs, cur = [], X
    for W, b, a in layers:
        cur = dense_forward(cur, W, b, a)
        outs.append(cur)
    return outs


def bf16_decode(bits):
    bits = np.ascontiguousarray(np.asarray(bits, dtype=np.uint16))
    out = np.empty(bits.shape, dtype=np.float64)
    lib().oracle_bf16_decode(bits.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)), bits.size, _dp(out))
    return out


def bf16_encode(x):
    x = np.ascontiguousarray(np.asarray(x, dtype=np.float32))
    out = np.empty(x.shape, dtype=np.uint16)
    lib().oracle_bf16_encode(x.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), x.size,
                             out.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)))
    return out


def e4m3_decode(codes, scale=1.0):
    codes = np.ascontiguousarray(np.asarray(codes, dtype=np.uint8))
    out = np.empty(codes.shape, dtype=np.float64)
    lib().oracle_e4m3_decode(codes.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)), codes.size, float(scale), _dp(out))
    return out


def e4m3_encode(x, scale=1.0):
    x = _f64(x)
    out = np.empty(x.shape, dtype=np.uint8)
    lib().oracle_e4m3_encode(_dp(x), x.size, float(scale), out.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)))
    return out
