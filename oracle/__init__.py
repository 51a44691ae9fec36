"""ctypes access to the CPU oracle (oracle/oracle.c).

Test infrastructure only: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  It never imports the HIP package.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force=False):
    """Compile oracle.c with gcc (-O2 -fopenmp) into oracle/liboracle.so."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        L.oracle_fp16_to_double.restype = ctypes.c_double
        L.oracle_fp16_to_double.argtypes = [ctypes.c_uint16]
        L.oracle_truncate_index.restype = ctypes.c_uint
        L.oracle_truncate_index.argtypes = [ctypes.c_uint, ctypes.c_int, ctypes.c_int]
        L.oracle_gemv.restype = ctypes.c_int
        L.oracle_gemv.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                  ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_int,
                                  ctypes.c_void_p, ctypes.c_void_p]
        L.oracle_dequantize.restype = ctypes.c_int
        L.oracle_dequantize.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                        ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
        L.oracle_anyprecision_bytes.restype = ctypes.c_double
        L.oracle_anyprecision_bytes.argtypes = [ctypes.c_double, ctypes.c_double, ctypes.c_uint,
                                                ctypes.c_double]
        L.oracle_num_threads.restype = ctypes.c_int
        L.oracle_num_threads.argtypes = []
        _lib = L
    return _lib


def _u16(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    assert a.dtype == np.uint16
    return a


def num_threads():
    return lib().oracle_num_threads()


def fp16_to_double(bits):
    return lib().oracle_fp16_to_double(int(bits))


def truncate_index(idx_n, n, b):
    return lib().oracle_truncate_index(int(idx_n), int(n), int(b))


def gemv(idx, lut, b, x, n=8):
    """Return (y, mag): float64 arrays of shape (batch, M).

    idx: (M, K) uint8; lut: (M, 2**b) float16 (or uint16 bit patterns); x: (batch, K) float16.
    """
    idx = np.ascontiguousarray(idx, dtype=np.uint8)
    M, K = idx.shape
    lut = _u16(lut)
    x = _u16(x)
    if x.ndim == 1:
        x = x[None, :]
    assert lut.shape == (M, 1 << b) and x.shape[1] == K
    batch = x.shape[0]
    y = np.empty((batch, M), dtype=np.float64)
    mag = np.empty((batch, M), dtype=np.float64)
    rc = lib().oracle_gemv(idx.ctypes.data, M, K, n, lut.ctypes.data, b, x.ctypes.data, batch,
                           y.ctypes.data, mag.ctypes.data)
    if rc != 0:
        raise ValueError("oracle_gemv rejected its arguments")
    return y, mag


def dequantize(idx, lut, b, n=8):
    idx = np.ascontiguousarray(idx, dtype=np.uint8)
    M, K = idx.shape
    lut = _u16(lut)
    W = np.empty((M, K), dtype=np.float64)
    rc = lib().oracle_dequantize(idx.ctypes.data, M, K, n, lut.ctypes.data, b, W.ctypes.data)
    if rc != 0:
        raise ValueError("oracle_dequantize rejected its arguments")
    return W


def anyprecision_bytes(n_weights, n_rows, bit_widths, other_bytes):
    mask = 0
    for b in bit_widths:
        mask |= 1 << b
    return lib().oracle_anyprecision_bytes(float(n_weights), float(n_rows), mask, float(other_bytes))
