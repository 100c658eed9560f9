"""ctypes front end of the AlignedKV CPU oracle (oracle/akv_oracle.c).

TEST INFRASTRUCTURE, NOT A PRODUCT PATH: only tests, the smoke check and the
benchmark's cpu_baseline leg may import this module.  It holds no arithmetic of
the method (that is all in the C file); it marshals numpy arrays.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "akv_oracle.c")
_LIB = os.path.join(_HERE, "libakv_oracle.so")
TB = 256  # tokens per K block (layout constant of the cache)


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C99, no contraction of a*b+c)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-std=c99", "-O2", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Debug(C.Structure):
    _fields_ = [("lvlK", C.c_void_p), ("logits", C.c_void_p), ("a", C.c_void_p), ("sel", C.c_void_p),
                ("oest", C.c_void_p), ("Ehat", C.c_void_p), ("needV", C.c_void_p), ("appliedV", C.c_void_p),
                ("counts", C.c_void_p)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.akvo_half_to_double.restype = C.c_double
        _lib.akvo_half_to_double.argtypes = [C.c_uint16]
        _lib.akvo_read_at_level.restype = C.c_uint16
        _lib.akvo_read_at_level.argtypes = [C.c_uint16, C.c_int]
        _lib.akvo_level_for_mantissa_bits.restype = C.c_int
        _lib.akvo_level_for_mantissa_bits.argtypes = [C.c_int]
        _lib.akvo_append.restype = C.c_int
        _lib.akvo_append.argtypes = [C.c_int] * 4 + [C.c_void_p] * 11 + [C.c_int]
        _lib.akvo_unpack.restype = C.c_int
        _lib.akvo_unpack.argtypes = [C.c_int] * 4 + [C.c_void_p] * 8
        _lib.akvo_decode_attention.restype = C.c_int
        _lib.akvo_decode_attention.argtypes = ([C.c_int] * 5 + [C.c_void_p] * 9 + [C.c_float, C.c_int, C.c_int, C.c_int]
                                               + [C.c_void_p, C.POINTER(_Debug)])
        _lib.akvo_fp16_attention.restype = C.c_int
        _lib.akvo_fp16_attention.argtypes = [C.c_int] * 5 + [C.c_void_p] * 4 + [C.c_float, C.c_void_p]
        _lib.akvo_v_granule_counts.restype = C.c_int
        _lib.akvo_v_granule_counts.argtypes = [C.c_int] * 4 + [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p]
        _lib.akvo_k_levels_per_block.restype = C.c_int
        _lib.akvo_k_levels_per_block.argtypes = [C.c_int] * 5 + [C.c_void_p] * 5 + [C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        _lib.akvo_max_threads.restype = C.c_int
        _lib.akvo_set_threads.restype = None
        _lib.akvo_set_threads.argtypes = [C.c_int]
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _chk(a, dtype, shape=None):
    assert isinstance(a, np.ndarray) and a.dtype == dtype and a.flags["C_CONTIGUOUS"], (a.dtype, dtype)
    if shape is not None:
        assert tuple(a.shape) == tuple(shape), (a.shape, shape)
    return a


@dataclass
class Cache:
    """Host copy of the split-plane cache (all numpy, zero-initialised)."""
    B: int
    Hkv: int
    D: int
    Ncap: int
    k_hi: np.ndarray
    k_mid: np.ndarray
    k_lo: np.ndarray
    v_hi: np.ndarray
    v_mid: np.ndarray
    v_lo: np.ndarray
    colmax: np.ndarray
    lens: np.ndarray

    @staticmethod
    def empty(B, Hkv, D, Ncap) -> "Cache":
        assert Ncap % TB == 0
        NB = Ncap // TB
        z = np.zeros
        return Cache(B, Hkv, D, Ncap,
                     z((B, Hkv, NB, D, TB), np.uint8), z((B, Hkv, NB, D, TB // 2), np.uint8),
                     z((B, Hkv, NB, D, TB // 2), np.uint8),
                     z((B, Hkv, Ncap, D), np.uint8), z((B, Hkv, Ncap, D // 2), np.uint8),
                     z((B, Hkv, Ncap, D // 2), np.uint8),
                     z((B, Hkv, D), np.uint16), z((B,), np.int32))

    def planes(self):
        return (self.k_hi, self.k_mid, self.k_lo, self.v_hi, self.v_mid, self.v_lo)


def append(cache: Cache, k_new: np.ndarray, v_new: np.ndarray, n_new: np.ndarray | None = None) -> int:
    """k_new, v_new: uint16 (fp16 bits) [B, Hkv, n, D].  Returns #sequences refused for capacity."""
    n = k_new.shape[2]
    _chk(k_new, np.uint16, (cache.B, cache.Hkv, n, cache.D))
    _chk(v_new, np.uint16, (cache.B, cache.Hkv, n, cache.D))
    if n_new is not None:
        _chk(n_new, np.int32, (cache.B,))
    r = lib().akvo_append(cache.B, cache.Hkv, cache.D, cache.Ncap, *[_p(x) for x in cache.planes()],
                          _p(cache.colmax), _p(cache.lens), _p(k_new), _p(v_new), _p(n_new), n)
    if r < 0:
        raise ValueError("akvo_append: bad arguments")
    return r


def unpack(cache: Cache):
    k = np.empty((cache.B, cache.Hkv, cache.Ncap, cache.D), np.uint16)
    v = np.empty_like(k)
    r = lib().akvo_unpack(cache.B, cache.Hkv, cache.D, cache.Ncap, *[_p(x) for x in cache.planes()], _p(k), _p(v))
    assert r == 0
    return k, v


@dataclass
class DecodeResult:
    out: np.ndarray        # float64 [B, Hq, D]
    lvlK: np.ndarray       # uint8   [B, Hkv, D]
    logits: np.ndarray     # float32 [B, Hq, Ncap]  (entries t >= len are 0)
    a: np.ndarray          # int8    [B, Hq, Ncap]
    sel: np.ndarray        # int32   [B, Hq, topk]
    oest: np.ndarray       # float32 [B, Hq, D]
    Ehat: np.ndarray       # int16   [B, Hkv, D]
    needV: np.ndarray | None     # uint8 [B, Hkv, Ncap, D]
    appliedV: np.ndarray   # uint8   [B, Hkv, Ncap]
    counts: np.ndarray     # uint64  [9]


def decode_attention(cache: Cache, q: np.ndarray, *, scale: float = 0.0, topk: int = 32, guard_bits: int = 0,
                     force_level: int = -1, want_needV: bool = True) -> DecodeResult:
    """q: uint16 (fp16 bits) [B, Hq, D]."""
    B, Hq, D = q.shape
    _chk(q, np.uint16, (cache.B, Hq, cache.D))
    Hkv, Ncap = cache.Hkv, cache.Ncap
    out = np.zeros((B, Hq, D), np.float64)
    res = DecodeResult(out, np.zeros((B, Hkv, D), np.uint8), np.zeros((B, Hq, Ncap), np.float32),
                       np.zeros((B, Hq, Ncap), np.int8), np.full((B, Hq, topk), -1, np.int32),
                       np.zeros((B, Hq, D), np.float32), np.zeros((B, Hkv, D), np.int16),
                       np.zeros((B, Hkv, Ncap, D), np.uint8) if want_needV else None,
                       np.zeros((B, Hkv, Ncap), np.uint8), np.zeros((9,), np.uint64))
    dbg = _Debug(_p(res.lvlK), _p(res.logits), _p(res.a), _p(res.sel), _p(res.oest), _p(res.Ehat), _p(res.needV),
                 _p(res.appliedV), _p(res.counts))
    r = lib().akvo_decode_attention(B, Hq, Hkv, D, Ncap, *[_p(x) for x in cache.planes()], _p(cache.colmax),
                                    _p(cache.lens), _p(q), float(scale), topk, guard_bits, force_level, _p(out),
                                    C.byref(dbg))
    if r != 0:
        raise ValueError("akvo_decode_attention: bad arguments")
    return res


def fp16_attention(k: np.ndarray, v: np.ndarray, lens: np.ndarray, q: np.ndarray, scale: float = 0.0) -> np.ndarray:
    """Textbook fp64 attention on plain fp16-bit tensors k, v [B, Hkv, Ncap, D]; q [B, Hq, D]."""
    B, Hkv, Ncap, D = k.shape
    Hq = q.shape[1]
    _chk(k, np.uint16)
    _chk(v, np.uint16, k.shape)
    _chk(q, np.uint16, (B, Hq, D))
    _chk(lens, np.int32, (B,))
    out = np.zeros((B, Hq, D), np.float64)
    r = lib().akvo_fp16_attention(B, Hq, Hkv, D, Ncap, _p(k), _p(v), _p(lens), _p(q), float(scale), _p(out))
    if r != 0:
        raise ValueError("akvo_fp16_attention: bad arguments")
    return out


def v_granule_counts(cache: Cache, needV: np.ndarray, tt: int, cc: int) -> np.ndarray:
    """V elements read at level 0 / 1 / 2 if the fetch unit were tt tokens x cc channels (uint64 [3])."""
    _chk(needV, np.uint8, (cache.B, cache.Hkv, cache.Ncap, cache.D))
    counts = np.zeros(3, np.uint64)
    r = lib().akvo_v_granule_counts(cache.B, cache.Hkv, cache.D, cache.Ncap, _p(needV), _p(cache.lens), tt, cc, _p(counts))
    if r != 0:
        raise ValueError("akvo_v_granule_counts: bad arguments")
    return counts


def k_levels_per_block(cache: Cache, q: np.ndarray, block: int, guard_bits: int = 0):
    """Rule 1 with one column maximum per `block` tokens: (levels uint8 [B, Hkv, ceil(Ncap/block), D], counts uint64 [3])."""
    B, Hq, D = q.shape
    _chk(q, np.uint16, (cache.B, Hq, cache.D))
    nb = (cache.Ncap + block - 1) // block
    lvl = np.zeros((B, cache.Hkv, nb, D), np.uint8)
    counts = np.zeros(3, np.uint64)
    r = lib().akvo_k_levels_per_block(B, Hq, cache.Hkv, D, cache.Ncap, _p(cache.k_hi), _p(cache.k_mid), _p(cache.k_lo),
                                      _p(cache.lens), _p(q), guard_bits, block, _p(lvl), _p(counts))
    if r != 0:
        raise ValueError("akvo_k_levels_per_block: bad arguments")
    return lvl, counts


def max_threads() -> int:
    return lib().akvo_max_threads()


def set_threads(n: int) -> None:
    """Threads used by the loops over (sequence, head) from now on."""
    lib().akvo_set_threads(int(n))
