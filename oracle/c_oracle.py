"""ctypes front end of ``shflbw_oracle.c`` (test infrastructure only).

``build()`` compiles the C file with gcc into ``oracle/_build/``;
the wrappers load it on first use and compile it if it is not there.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "shflbw_oracle.c")
_OUT_DIR = os.path.join(_HERE, "_build")
_LIB_PATH = os.path.join(_OUT_DIR, "libshflbw_oracle.so")
_lib = None


def build(force=True):
    """Compile the oracle (gcc -O2 -fopenmp, no BLAS)."""
    os.makedirs(_OUT_DIR, exist_ok=True)
    if not force and os.path.exists(_LIB_PATH) and \
            os.path.getmtime(_LIB_PATH) >= os.path.getmtime(_SRC):
        return _LIB_PATH
    tmp = _LIB_PATH + ".tmp.%d" % os.getpid()
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                           "-Wall", "-o", tmp, _SRC, "-lm"])
    os.replace(tmp, _LIB_PATH)
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        path = build(force=False)
        lib = ctypes.CDLL(path)
        i64, vp = ctypes.c_int64, ctypes.c_void_p
        lib.oracle_half_to_double.restype = ctypes.c_double
        lib.oracle_half_to_double.argtypes = [ctypes.c_uint16]
        lib.oracle_bfloat16_to_double.restype = ctypes.c_double
        lib.oracle_bfloat16_to_double.argtypes = [ctypes.c_uint16]
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_spmm_fmt.restype = ctypes.c_int
        lib.oracle_spmm_fmt.argtypes = [vp, vp, vp, i64, i64, i64, vp, vp, ctypes.c_int]
        lib.oracle_conv2d_fmt.restype = ctypes.c_int
        lib.oracle_conv2d_fmt.argtypes = [vp, vp, vp] + [i64] * 11 + [ctypes.c_int, vp, vp, ctypes.c_int]
        _lib = lib
    return _lib


def _ptr(a):
    return ctypes.c_void_p(a.ctypes.data)


def _bits(a):
    """(bit patterns, format): float16 arrays are binary16 (format 0); uint16
    arrays hold bfloat16 bit patterns (format 1; numpy has no such dtype)."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        return a.view(np.uint16), 0
    if a.dtype == np.uint16:
        return a, 1
    raise TypeError("expected float16, or uint16 holding bfloat16 bits, got %s" % a.dtype)


def num_threads():
    return int(_load().oracle_num_threads())


def half_to_double(bits):
    return float(_load().oracle_half_to_double(int(bits)))


def bfloat16_to_double(bits):
    return float(_load().oracle_bfloat16_to_double(int(bits)))


def spmm(W, mask, X, want_scale=True):
    """Y (float64, M x N) and S = |W.mask| |X| for W (M x K), X (K x N), both
    float16 or both uint16 arrays of bfloat16 bit patterns."""
    (Wb, fmt), (Xb, fx) = _bits(W), _bits(X)
    if fmt != fx:
        raise TypeError("W and X must have the same format")
    m = np.ascontiguousarray(mask, dtype=np.uint8)
    M, K = Wb.shape
    K2, N = Xb.shape
    if K2 != K or m.shape != (M, K):
        raise ValueError("shape mismatch")
    Y = np.empty((M, N), dtype=np.float64)
    S = np.empty((M, N), dtype=np.float64) if want_scale else None
    rc = _load().oracle_spmm_fmt(_ptr(Wb), _ptr(m), _ptr(Xb), M, K, N, _ptr(Y),
                                 _ptr(S) if want_scale else None, fmt)
    if rc != 0:
        raise MemoryError("oracle_spmm rc=%d" % rc)
    return (Y, S) if want_scale else Y


def conv2d(Wt, mask, inp, R, S, stride=(1, 1), pad=(0, 0), layout="NCHW", want_scale=True):
    """Masked conv2d.  Wt, mask: (Cout, Cin*R*S), k = (c*R + r)*S + s.
    inp: (B, Cin, H, W) for NCHW or (Cin, H, W, B) for CHWN; the result uses
    the same layout."""
    (Wb, fmt), (Ib, fi) = _bits(Wt), _bits(inp)
    if fmt != fi:
        raise TypeError("weights and input must have the same format")
    m = np.ascontiguousarray(mask, dtype=np.uint8)
    lay = {"NCHW": 0, "CHWN": 1}[layout]
    if lay == 0:
        B, Cin, H, Wd = Ib.shape
    else:
        Cin, H, Wd, B = Ib.shape
    Cout, K = Wb.shape
    if K != Cin * R * S or m.shape != (Cout, K):
        raise ValueError("shape mismatch")
    sh, sw = stride
    ph, pw = pad
    Ho = (H + 2 * ph - R) // sh + 1
    Wo = (Wd + 2 * pw - S) // sw + 1
    shape = (B, Cout, Ho, Wo) if lay == 0 else (Cout, Ho, Wo, B)
    out = np.empty(shape, dtype=np.float64)
    sc = np.empty(shape, dtype=np.float64) if want_scale else None
    rc = _load().oracle_conv2d_fmt(_ptr(Wb), _ptr(m), _ptr(Ib), B, Cin, H, Wd, Cout, R, S,
                                   sh, sw, ph, pw, lay, _ptr(out),
                                   _ptr(sc) if want_scale else None, fmt)
    if rc != 0:
        raise RuntimeError("oracle_conv2d rc=%d" % rc)
    return (out, sc) if want_scale else out
