"""ctypes front end of oracle/quant_oracle.c.  TEST INFRASTRUCTURE ONLY (imported by tests/ alone)."""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "quant_oracle.c")
_LIB = os.path.join(_HERE, "libquantorc.so")
_lib = None


def build(force: bool = False) -> str:
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        # -ffp-contract=off: the 32-bit product c * x must be rounded on its own, as written
        subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        L.orc_quant_blockwise.restype = C.c_int
        L.orc_quant_blockwise.argtypes = [vp, i64, i32, i32, vp, vp]
        L.orc_dequant_blockwise.restype = C.c_int
        L.orc_dequant_blockwise.argtypes = [vp, vp, i64, i32, i32, vp]
        L.orc_dequant_linear.restype = C.c_int
        L.orc_dequant_linear.argtypes = [vp, i32, i32, vp, vp, i32, i32, i32, vp]
        _lib = L
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def quant(x: np.ndarray, block: int, bits: int):
    """x (any shape, float32, quantised as one flat tensor) -> (codes int8 [n] or packed [(n+1)//2], consts float32)."""
    x = np.ascontiguousarray(x, dtype=np.float32).ravel()
    n = x.size
    codes = np.zeros(n if bits == 8 else (n + 1) // 2, dtype=np.int8)
    consts = np.zeros((n + block - 1) // block, dtype=np.float32)
    assert lib().orc_quant_blockwise(_p(x), n, block, bits, _p(codes), _p(consts)) == 0
    return codes, consts


def dequant(codes: np.ndarray, consts: np.ndarray, n: int, block: int, bits: int) -> np.ndarray:
    out = np.zeros(n, dtype=np.float32)
    assert lib().orc_dequant_blockwise(_p(np.ascontiguousarray(codes)), _p(np.ascontiguousarray(consts)), n, block,
                                       bits, _p(out)) == 0
    return out


def unpack(codes: np.ndarray, n: int, bits: int) -> np.ndarray:
    """Integer codes as int32 [n] (test helper: plain bit handling, no arithmetic of the method)."""
    if bits == 8:
        return codes.astype(np.int32)[:n]
    b = codes.view(np.uint8).astype(np.int32)
    nib = np.stack([b & 0xf, b >> 4], axis=1).ravel()[:n]
    return np.where(nib >= 8, nib - 16, nib)


def dequant_linear(x: np.ndarray, codes: np.ndarray, consts: np.ndarray, N: int, block: int, bits: int) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    M, K = x.shape
    y = np.zeros((M, N), dtype=np.float64)
    assert lib().orc_dequant_linear(_p(x), M, K, _p(np.ascontiguousarray(codes)), _p(np.ascontiguousarray(consts)), N,
                                    block, bits, _p(y)) == 0
    return y
