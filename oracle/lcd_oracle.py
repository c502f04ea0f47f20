"""ctypes front end of the plain-C fp64 oracle (``lcd_oracle.c``).  TEST INFRASTRUCTURE ONLY.

The oracle evaluates the definition of the smoothed table-lookup product
(paper Sec. 3.2 for W' = centroid, Sec. 3.4 for the division by the smoothing factor,
Sec. 4.2 for lookup-and-accumulate) in fp64 with a sequential sum over k.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "lcd_oracle.c"
_LIB = _HERE / "liblcd_oracle.so"
_lib = None


def build_oracle(force: bool = False) -> Path:
    """Compile the C oracle with gcc (-O2 -fopenmp).  Building the checker is not using it."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(".so.tmp%d" % os.getpid())
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fno-fast-math", "-shared", "-fPIC", "-o", str(tmp), str(_SRC), "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build_oracle()
        lib = ctypes.CDLL(str(_LIB))
        u16p = ctypes.POINTER(ctypes.c_uint16)
        u8p = ctypes.POINTER(ctypes.c_uint8)
        f32p = ctypes.POINTER(ctypes.c_float)
        f64p = ctypes.POINTER(ctypes.c_double)
        i32p = ctypes.POINTER(ctypes.c_int32)
        ci = ctypes.c_int
        lib.oracle_half_to_double.restype = ctypes.c_double
        lib.oracle_half_to_double.argtypes = [ctypes.c_uint16]
        lib.oracle_num_threads.restype = ci
        lib.oracle_dequant.restype = ci
        lib.oracle_dequant.argtypes = [u16p, u8p, ci, ci, ci, f64p]
        lib.oracle_smooth.restype = None
        lib.oracle_smooth.argtypes = [u16p, f32p, ci, ci, f64p]
        for name in ("oracle_lut_matmul", "oracle_bucket_matmul"):
            fn = getattr(lib, name)
            fn.restype = ci
            fn.argtypes = [u16p, u8p, u16p, f32p, ci, ci, ci, ci, f64p]
        lib.oracle_input_transform.restype = None
        lib.oracle_input_transform.argtypes = [u16p, f32p, ctypes.c_double, ci, ci, ci, i32p]
        lib.oracle_input_transform_f32.restype = None
        lib.oracle_input_transform_f32.argtypes = [u16p, f32p, ctypes.c_float, ci, ci, ci, i32p]
        _lib = lib
    return _lib


def _p(a: np.ndarray, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def _as_half_bits(a: np.ndarray) -> np.ndarray:
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    if a.dtype != np.uint16:
        raise TypeError("expected float16 or uint16 (fp16 bit patterns)")
    return np.ascontiguousarray(a)


def _check(codebook, idx, x, s, bits):
    cb = _as_half_bits(codebook)
    ix = np.ascontiguousarray(idx, dtype=np.uint8)
    xx = _as_half_bits(x)
    ss = np.ascontiguousarray(s, dtype=np.float32)
    N, K = ix.shape
    M = xx.shape[0]
    if cb.shape != (N, 1 << bits) or xx.shape != (M, K) or ss.shape != (K,):
        raise ValueError("shape mismatch")
    return cb, ix, xx, ss, M, N, K


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def half_to_double(bits16: int) -> float:
    return float(_load().oracle_half_to_double(ctypes.c_uint16(int(bits16))))


def dequant(codebook, idx, bits: int) -> np.ndarray:
    cb = _as_half_bits(codebook)
    ix = np.ascontiguousarray(idx, dtype=np.uint8)
    N, K = ix.shape
    out = np.empty((N, K), dtype=np.float64)
    bad = _load().oracle_dequant(_p(cb, ctypes.c_uint16), _p(ix, ctypes.c_uint8), N, K, bits,
                                 _p(out, ctypes.c_double))
    if bad:
        raise ValueError("index >= 2**bits")
    return out


def smooth(x, s) -> np.ndarray:
    xx = _as_half_bits(x)
    ss = np.ascontiguousarray(s, dtype=np.float32)
    M, K = xx.shape
    out = np.empty((M, K), dtype=np.float64)
    _load().oracle_smooth(_p(xx, ctypes.c_uint16), _p(ss, ctypes.c_float), M, K, _p(out, ctypes.c_double))
    return out


def _matmul(name, codebook, idx, x, s, bits):
    cb, ix, xx, ss, M, N, K = _check(codebook, idx, x, s, bits)
    Y = np.empty((M, N), dtype=np.float64)
    bad = getattr(_load(), name)(_p(cb, ctypes.c_uint16), _p(ix, ctypes.c_uint8), _p(xx, ctypes.c_uint16),
                                 _p(ss, ctypes.c_float), M, N, K, bits, _p(Y, ctypes.c_double))
    if bad:
        raise ValueError("index >= 2**bits")
    return Y


def lut_matmul(codebook, idx, x, s, bits: int) -> np.ndarray:
    """Y[m,n] = sum_k (x[m,k]/s[k]) * C[n, idx[n,k]] (fp64, sequential k)."""
    return _matmul("oracle_lut_matmul", codebook, idx, x, s, bits)


def bucket_matmul(codebook, idx, x, s, bits: int) -> np.ndarray:
    """Same result in centroid-bucket order (Sec. 4.2)."""
    return _matmul("oracle_bucket_matmul", codebook, idx, x, s, bits)


def input_transform(x, s_m, s_q: float, b: int = 8, single_precision: bool = False) -> np.ndarray:
    """q = clip(round(x/(s_m*s_q))) to the b-bit symmetric range (Sec. 4.1, Eq. 10-11).

    single_precision=False: fp64 throughout.  True: every step in binary32 (d = s_m*s_q, v = x/d,
    round half to even), the precision in which a single-precision kernel takes the rounding decision."""
    xx = _as_half_bits(x)
    ss = np.ascontiguousarray(s_m, dtype=np.float32)
    M, K = xx.shape
    q = np.empty((M, K), dtype=np.int32)
    fn = _load().oracle_input_transform_f32 if single_precision else _load().oracle_input_transform
    fn(_p(xx, ctypes.c_uint16), _p(ss, ctypes.c_float), float(s_q), int(b), M, K, _p(q, ctypes.c_int32))
    return q


def quantised_lut_matmul(codebook, idx, x, s_m, s_q: float, bits: int, b: int = 8) -> np.ndarray:
    """The product with the input transformation of Sec. 4.1 in front of it:
    Y = s_q * sum_k q[m][k] * C[n][idx[n][k]], q from input_transform in single precision (fp64 sum)."""
    q = input_transform(x, s_m, s_q, b, single_precision=True)
    qh = q.astype(np.float16)                       # |q| <= 128: exact
    assert np.array_equal(qh.astype(np.int32), q)
    ones = np.ones(q.shape[1], dtype=np.float32)
    return float(np.float32(s_q)) * lut_matmul(codebook, idx, qh, ones, bits)
