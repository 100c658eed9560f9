"""ctypes front end of the weight-GEMV CPU oracle (oracle/akw_oracle.c).

TEST INFRASTRUCTURE, NOT A PRODUCT PATH: only tests, the smoke check and a
benchmark's CPU leg may import this module.  It holds no arithmetic of the
method (that is all in the C file); it marshals numpy arrays.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "akw_oracle.c")
_LIB = os.path.join(_HERE, "libakw_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C99, no contraction of a*b+c)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-std=c99", "-O2", "-ffp-contract=off", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC,
             "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.akwo_pack.restype = C.c_int
        _lib.akwo_pack.argtypes = [C.c_int, C.c_int] + [C.c_void_p] * 5
        _lib.akwo_unpack.restype = C.c_int
        _lib.akwo_unpack.argtypes = [C.c_int, C.c_int] + [C.c_void_p] * 4
        _lib.akwo_levels.restype = C.c_int
        _lib.akwo_levels.argtypes = [C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p]
        _lib.akwo_gemv.restype = C.c_int
        _lib.akwo_gemv.argtypes = ([C.c_int] * 3 + [C.c_void_p] * 5 + [C.c_int, C.c_int] + [C.c_void_p] * 3)
        _lib.akwo_half_to_double.restype = C.c_double
        _lib.akwo_half_to_double.argtypes = [C.c_uint16]
        _lib.akwo_read_at_level.restype = C.c_uint16
        _lib.akwo_read_at_level.argtypes = [C.c_uint16, C.c_int]
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _chk(a, dtype, shape=None):
    assert isinstance(a, np.ndarray) and a.dtype == dtype and a.flags["C_CONTIGUOUS"], (a.dtype, dtype)
    if shape is not None:
        assert tuple(a.shape) == tuple(shape), (a.shape, shape)
    return a


@dataclass
class Weights:
    """Host copy of one weight matrix in split planes."""
    K: int
    N: int
    hi: np.ndarray      # uint8  [K, N]
    mid: np.ndarray     # uint8  [K, N/2]
    lo: np.ndarray      # uint8  [K, N/2]
    rowmax: np.ndarray  # uint16 [K]


def pack(W: np.ndarray) -> Weights:
    """W: uint16 (fp16 bits) [K, N], N even."""
    K, N = W.shape
    _chk(W, np.uint16)
    w = Weights(K, N, np.zeros((K, N), np.uint8), np.zeros((K, N // 2), np.uint8), np.zeros((K, N // 2), np.uint8),
                np.zeros((K,), np.uint16))
    if lib().akwo_pack(K, N, _p(W), _p(w.hi), _p(w.mid), _p(w.lo), _p(w.rowmax)) != 0:
        raise ValueError("akwo_pack: bad arguments")
    return w


def unpack(w: Weights) -> np.ndarray:
    out = np.empty((w.K, w.N), np.uint16)
    assert lib().akwo_unpack(w.K, w.N, _p(w.hi), _p(w.mid), _p(w.lo), _p(out)) == 0
    return out


def levels(x: np.ndarray, rowmax: np.ndarray, guard_bits: int = 0, force_level: int = -1) -> np.ndarray:
    """x: uint16 (fp16 bits) [B, K]; rowmax: uint16 [K].  Level (0, 1, 2) each row of W is read at."""
    B, K = x.shape
    _chk(x, np.uint16)
    _chk(rowmax, np.uint16, (K,))
    lvl = np.zeros((K,), np.uint8)
    assert lib().akwo_levels(B, K, _p(x), _p(rowmax), guard_bits, force_level, _p(lvl)) == 0
    return lvl


@dataclass
class GemvResult:
    y: np.ndarray        # float64 [B, N]
    lvl: np.ndarray      # uint8   [K]
    abs_sum: np.ndarray  # float64 [B, N]  sum_k |x_k w~_kn|


def gemv(w: Weights, x: np.ndarray, guard_bits: int = 0, force_level: int = -1) -> GemvResult:
    """x: uint16 (fp16 bits) [B, K]."""
    B, K = x.shape
    _chk(x, np.uint16, (B, w.K))
    r = GemvResult(np.zeros((B, w.N), np.float64), np.zeros((K,), np.uint8), np.zeros((B, w.N), np.float64))
    rc = lib().akwo_gemv(B, K, w.N, _p(w.hi), _p(w.mid), _p(w.lo), _p(w.rowmax), _p(x), guard_bits, force_level,
                         _p(r.y), _p(r.lvl), _p(r.abs_sum))
    if rc != 0:
        raise ValueError("akwo_gemv: bad arguments")
    return r


def half_to_double(h: int) -> float:
    return lib().akwo_half_to_double(h)


def read_at_level(h: int, level: int) -> int:
    return lib().akwo_read_at_level(h, level)
