"""ctypes binding of the C ABI in ``include/akv.h`` and ``include/akw.h`` -- argument marshalling only.

Every function has the name of its C entry point and hands torch device pointers and the current
HIP stream to it; no step of the path runs here.  If ``libakv.so`` has not been built the import of
the library fails loudly: there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass, field

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libakv.so")

AKV_OK, AKV_EINVAL, AKV_EWORKSPACE, AKV_EHIP, AKV_ECAPACITY = 0, 1, 2, 3, 4
AKV_TB = 256
AKV_NFLAGS = 4
AKV_FLAG_OVERFLOW, AKV_FLAG_MAXLEN = 0, 1
AKV_MAX_TOPK = 64
AKV_NEVENTS = 5
AKV_STATIC_SCRATCH_BYTES = 48 << 20
EXPORTS = ["akv_version", "akv_last_error", "akv_layout_sizes", "akv_cache_reset", "akv_append", "akv_check_capacity_sync",
           "akv_workspace_init",
           "akv_decode_attention", "akv_decode_path", "akv_decode_attention_static", "akv_append_decode_attention", "akv_unpack", "akv_fp16_decode_attention", "akv_stream_read",
           "akw_layout_sizes", "akw_workspace_init", "akw_pack", "akw_unpack", "akw_gemv"]
AKW_MAX_B = 4


class AkvError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"akv status {status}: {msg}")
        self.status = status


class akv_shape(C.Structure):
    _fields_ = [("B", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("D", C.c_int32), ("Ncap", C.c_int32)]


class akv_sizes(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in ("k_hi", "k_mid", "k_lo", "v_hi", "v_mid", "v_lo", "colmax", "lens", "flags",
                                          "workspace", "fp16_workspace")]


class akv_cache(C.Structure):
    _fields_ = [("shape", akv_shape)] + [(n, C.c_void_p) for n in ("k_hi", "k_mid", "k_lo", "v_hi", "v_mid", "v_lo",
                                                                   "colmax", "lens", "flags")]


class akv_debug(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("lvlK", "logits", "a", "sel", "oest", "Ehat", "needV", "appliedV")]


class akv_stats(C.Structure):
    _fields_ = [("k_elems", C.c_uint64 * 3), ("v_row_elems", C.c_uint64 * 3), ("v_need_elems", C.c_uint64 * 3)]


class akv_params(C.Structure):
    _fields_ = [("scale", C.c_float), ("topk", C.c_int32), ("guard_bits", C.c_int32), ("force_level", C.c_int32),
                ("out_dtype", C.c_int32), ("max_len", C.c_int32), ("dbg", C.POINTER(akv_debug)),
                ("events", C.POINTER(C.c_void_p)), ("path", C.c_int32), ("stats", C.c_void_p)]


class akw_weights(C.Structure):
    _fields_ = [("K", C.c_int32), ("N", C.c_int32)] + [(n, C.c_void_p) for n in ("hi", "mid", "lo", "rowmax")]


class akw_sizes(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in ("hi", "mid", "lo", "rowmax", "workspace")]


class akw_params(C.Structure):
    _fields_ = [("guard_bits", C.c_int32), ("force_level", C.c_int32), ("lvl_out", C.c_void_p)]


_lib = None


def lib() -> C.CDLL:
    """Load libakv.so (built by ``python -m paper_2409_16546_amd.build`` / ``__graft_entry__.build()``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build the HIP library first (python -m paper_2409_16546_amd.build); "
                              "there is no CPU fallback")
        L = C.CDLL(LIB_PATH)
        L.akv_version.restype = C.c_int
        L.akv_last_error.restype = C.c_char_p
        L.akv_layout_sizes.restype = C.c_int
        L.akv_layout_sizes.argtypes = [C.POINTER(akv_shape), C.POINTER(akv_sizes)]
        L.akv_cache_reset.restype = C.c_int
        L.akv_cache_reset.argtypes = [C.POINTER(akv_cache), C.c_void_p]
        L.akv_append.restype = C.c_int
        L.akv_append.argtypes = [C.POINTER(akv_cache), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]
        L.akv_check_capacity_sync.restype = C.c_int
        L.akv_check_capacity_sync.argtypes = [C.POINTER(akv_cache), C.c_int32, C.c_void_p]
        L.akv_workspace_init.restype = C.c_int
        L.akv_workspace_init.argtypes = [C.POINTER(akv_shape), C.c_void_p, C.c_size_t, C.c_void_p]
        L.akv_decode_attention.restype = C.c_int
        L.akv_decode_attention.argtypes = [C.POINTER(akv_cache), C.c_void_p, C.c_void_p, C.POINTER(akv_params), C.c_void_p,
                                           C.c_size_t, C.c_void_p]
        L.akv_decode_path.restype = C.c_int32
        L.akv_decode_path.argtypes = [C.POINTER(akv_shape), C.c_int32]
        L.akv_decode_attention_static.restype = C.c_int
        L.akv_decode_attention_static.argtypes = [C.POINTER(akv_cache), C.c_void_p, C.c_void_p, C.POINTER(akv_params), C.c_void_p]
        L.akv_append_decode_attention.restype = C.c_int
        L.akv_append_decode_attention.argtypes = [C.POINTER(akv_cache), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                                  C.POINTER(akv_params), C.c_void_p, C.c_size_t, C.c_void_p]
        L.akv_stream_read.restype = C.c_int
        L.akv_stream_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        L.akv_unpack.restype = C.c_int
        L.akv_unpack.argtypes = [C.POINTER(akv_cache), C.c_void_p, C.c_void_p, C.c_void_p]
        L.akv_fp16_decode_attention.restype = C.c_int
        L.akv_fp16_decode_attention.argtypes = [C.POINTER(akv_shape), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                                C.c_void_p, C.c_float, C.c_int32, C.c_int32, C.c_void_p, C.c_size_t,
                                                C.c_void_p]
        L.akw_layout_sizes.restype = C.c_int
        L.akw_layout_sizes.argtypes = [C.c_int32, C.c_int32, C.POINTER(akw_sizes)]
        L.akw_workspace_init.restype = C.c_int
        L.akw_workspace_init.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p]
        L.akw_pack.restype = C.c_int
        L.akw_pack.argtypes = [C.POINTER(akw_weights), C.c_void_p, C.c_void_p]
        L.akw_unpack.restype = C.c_int
        L.akw_unpack.argtypes = [C.POINTER(akw_weights), C.c_void_p, C.c_void_p]
        L.akw_gemv.restype = C.c_int
        L.akw_gemv.argtypes = [C.POINTER(akw_weights), C.c_void_p, C.c_int32, C.c_void_p, C.POINTER(akw_params), C.c_void_p,
                               C.c_size_t, C.c_void_p]
        _lib = L
    return _lib


def _check(st: int):
    if st != AKV_OK:
        raise AkvError(st, lib().akv_last_error().decode())


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t: torch.Tensor | None) -> int | None:
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensors only"
    return t.data_ptr()


def akv_version() -> int:
    return lib().akv_version()


def akv_layout_sizes(B: int, Hq: int, Hkv: int, D: int, Ncap: int) -> akv_sizes:
    shp, out = akv_shape(B, Hq, Hkv, D, Ncap), akv_sizes()
    _check(lib().akv_layout_sizes(C.byref(shp), C.byref(out)))
    return out


@dataclass
class Cache:
    """Caller-owned device buffers of one split-plane cache (torch owns the memory)."""
    B: int
    Hq: int
    Hkv: int
    D: int
    Ncap: int
    k_hi: torch.Tensor = field(repr=False, default=None)
    k_mid: torch.Tensor = field(repr=False, default=None)
    k_lo: torch.Tensor = field(repr=False, default=None)
    v_hi: torch.Tensor = field(repr=False, default=None)
    v_mid: torch.Tensor = field(repr=False, default=None)
    v_lo: torch.Tensor = field(repr=False, default=None)
    colmax: torch.Tensor = field(repr=False, default=None)
    lens: torch.Tensor = field(repr=False, default=None)
    flags: torch.Tensor = field(repr=False, default=None)
    workspace: torch.Tensor = field(repr=False, default=None)
    sizes: akv_sizes = field(repr=False, default=None)
    _struct: akv_cache = field(repr=False, default=None)

    @staticmethod
    def allocate(B: int, Hq: int, Hkv: int, D: int, Ncap: int, device="cuda:0") -> "Cache":
        sz = akv_layout_sizes(B, Hq, Hkv, D, Ncap)
        u8 = lambda n: torch.empty(n, dtype=torch.uint8, device=device)
        c = Cache(B, Hq, Hkv, D, Ncap, u8(sz.k_hi), u8(sz.k_mid), u8(sz.k_lo), u8(sz.v_hi), u8(sz.v_mid), u8(sz.v_lo),
                  torch.empty(B * Hkv * D, dtype=torch.int16, device=device),
                  torch.empty(B, dtype=torch.int32, device=device),
                  torch.empty(AKV_NFLAGS + B, dtype=torch.int32, device=device), u8(sz.workspace), sz)
        akv_cache_reset(c)
        akv_workspace_init(c, c.workspace)
        return c

    def struct(self) -> akv_cache:
        if self._struct is None:   # the tensors never change after allocation
            self._struct = akv_cache(akv_shape(self.B, self.Hq, self.Hkv, self.D, self.Ncap), _ptr(self.k_hi),
                                     _ptr(self.k_mid), _ptr(self.k_lo), _ptr(self.v_hi), _ptr(self.v_mid),
                                     _ptr(self.v_lo), _ptr(self.colmax), _ptr(self.lens), _ptr(self.flags))
        return self._struct


def akv_cache_reset(cache: Cache) -> None:
    s = cache.struct()
    _check(lib().akv_cache_reset(C.byref(s), _stream()))


def akv_workspace_init(cache: Cache, workspace: torch.Tensor) -> None:
    """Zero the control words of a decode workspace (once per workspace, before its first use)."""
    shp = akv_shape(cache.B, cache.Hq, cache.Hkv, cache.D, cache.Ncap)
    _check(lib().akv_workspace_init(C.byref(shp), _ptr(workspace), workspace.numel(), _stream()))


def akv_append(cache: Cache, k_new: torch.Tensor, v_new: torch.Tensor, n_new: torch.Tensor | None = None) -> None:
    """k_new, v_new: fp16 [B, Hkv, n, D] on the device; n_new: int32 [B] on the device or None."""
    assert k_new.dtype == torch.float16 and v_new.dtype == torch.float16
    n = k_new.shape[2]
    assert tuple(k_new.shape) == (cache.B, cache.Hkv, n, cache.D) == tuple(v_new.shape)
    if n_new is not None:
        assert n_new.dtype == torch.int32 and tuple(n_new.shape) == (cache.B,)
    s = cache.struct()
    _check(lib().akv_append(C.byref(s), _ptr(k_new), _ptr(v_new), _ptr(n_new), n, _stream()))


def akv_check_capacity_sync(cache: Cache, n: int) -> None:
    """Debugging aid (synchronises): raises AkvError(AKV_ECAPACITY) if n more tokens would not fit some sequence."""
    s = cache.struct()
    _check(lib().akv_check_capacity_sync(C.byref(s), n, _stream()))


def akv_stream_read(buf: torch.Tensor, sink: torch.Tensor) -> None:
    """Read the bytes of `buf` once with the library's plain streaming kernel (a measurement aid)."""
    _check(lib().akv_stream_read(_ptr(buf), buf.numel() * buf.element_size(), _ptr(sink), _stream()))


def akv_unpack(cache: Cache) -> tuple[torch.Tensor, torch.Tensor]:
    k = torch.empty(cache.B, cache.Hkv, cache.Ncap, cache.D, dtype=torch.float16, device=cache.k_hi.device)
    v = torch.empty_like(k)
    s = cache.struct()
    _check(lib().akv_unpack(C.byref(s), _ptr(k), _ptr(v), _stream()))
    return k, v


@dataclass
class DebugBuffers:
    """Device tensors receiving the decisions of one akv_decode_attention call."""
    lvlK: torch.Tensor
    logits: torch.Tensor
    a: torch.Tensor
    sel: torch.Tensor
    oest: torch.Tensor
    Ehat: torch.Tensor
    needV: torch.Tensor | None
    appliedV: torch.Tensor

    @staticmethod
    def allocate(cache: Cache, topk: int = 32, want_needV: bool = True) -> "DebugBuffers":
        dev = cache.k_hi.device
        B, Hq, Hkv, D, N = cache.B, cache.Hq, cache.Hkv, cache.D, cache.Ncap
        z = lambda shape, dt: torch.zeros(shape, dtype=dt, device=dev)
        return DebugBuffers(z((B, Hkv, D), torch.uint8), z((B, Hq, N), torch.float32), z((B, Hq, N), torch.int8),
                            torch.full((B, Hq, topk), -1, dtype=torch.int32, device=dev), z((B, Hq, D), torch.float32),
                            z((B, Hkv, D), torch.int16), z((B, Hkv, N, D), torch.uint8) if want_needV else None,
                            z((B, Hkv, N), torch.uint8))

    def struct(self) -> akv_debug:
        return akv_debug(_ptr(self.lvlK), _ptr(self.logits), _ptr(self.a), _ptr(self.sel), _ptr(self.oest),
                         _ptr(self.Ehat), _ptr(self.needV), _ptr(self.appliedV))


def akv_decode_path(B: int, Hq: int, Hkv: int, D: int, Ncap: int, max_len: int = 0) -> int:
    """1 (head-per-workgroup kernel), 3 (the same, logits kept in LDS) or 2 (token-split kernels): what path=0 takes."""
    shp = akv_shape(B, Hq, Hkv, D, Ncap)
    return int(lib().akv_decode_path(C.byref(shp), max_len))


def new_stats(device="cuda:0") -> torch.Tensor:
    """Zeroed device counters for the `stats` argument of the decode calls: int64 [9] = k_elems[3], v_row_elems[3],
    v_need_elems[3] (the fields of akv_stats in order); every call adds to them."""
    return torch.zeros(9, dtype=torch.int64, device=device)


def _params(out, scale, topk, guard_bits, force_level, max_len, d, events, path, stats) -> akv_params:
    if stats is not None:
        assert stats.dtype == torch.int64 and stats.numel() == 9
    return akv_params(scale, topk, guard_bits, force_level, 0 if out.dtype == torch.float32 else 1, max_len,
                      C.pointer(d) if d is not None else None, events, path, _ptr(stats))


def akv_decode_attention(cache: Cache, q: torch.Tensor, out: torch.Tensor | None = None, *, scale: float = 0.0,
                         topk: int = 32, guard_bits: int = 0, force_level: int = -1, max_len: int = 0,
                         dbg: DebugBuffers | None = None, workspace: torch.Tensor | None = None,
                         events=None, path: int = 0, stats: torch.Tensor | None = None) -> torch.Tensor:
    """q: fp16 [B, Hq, D] on the device; out: float32 or fp16 [B, Hq, D] (allocated if None).
    events: None or a ctypes array of AKV_NEVENTS hipEvent_t handles the library records around its kernels.
    path: 0 choose, 1 head-per-workgroup kernel, 2 token-split kernels.  stats: see new_stats()."""
    assert q.dtype == torch.float16 and tuple(q.shape) == (cache.B, cache.Hq, cache.D)
    if out is None:
        out = torch.empty(cache.B, cache.Hq, cache.D, dtype=torch.float32, device=q.device)
    assert out.dtype in (torch.float32, torch.float16) and tuple(out.shape) == tuple(q.shape)
    ws = cache.workspace if workspace is None else workspace
    d = dbg.struct() if dbg is not None else None
    p = _params(out, scale, topk, guard_bits, force_level, max_len, d, events, path, stats)
    s = cache.struct()
    _check(lib().akv_decode_attention(C.byref(s), _ptr(q), _ptr(out), C.byref(p), _ptr(ws), ws.numel(), _stream()))
    return out


def akv_decode_attention_static(cache: Cache, q: torch.Tensor, out: torch.Tensor, *, scale: float = 0.0,
                                topk: int = 32, guard_bits: int = 0, force_level: int = -1, max_len: int = 0,
                                dbg: DebugBuffers | None = None, events=None, path: int = 0,
                                stats: torch.Tensor | None = None) -> torch.Tensor:
    """akv_decode_attention on the library's own static scratch array: the call allocates nothing (out is the
    caller's); shapes beyond AKV_STATIC_SCRATCH_BYTES are refused."""
    assert q.dtype == torch.float16 and tuple(q.shape) == (cache.B, cache.Hq, cache.D)
    assert out.dtype in (torch.float32, torch.float16) and tuple(out.shape) == tuple(q.shape)
    d = dbg.struct() if dbg is not None else None
    p = _params(out, scale, topk, guard_bits, force_level, max_len, d, events, path, stats)
    s = cache.struct()
    _check(lib().akv_decode_attention_static(C.byref(s), _ptr(q), _ptr(out), C.byref(p), _stream()))
    return out


def akv_append_decode_attention(cache: Cache, k_new: torch.Tensor, v_new: torch.Tensor, q: torch.Tensor,
                                out: torch.Tensor | None = None, *, scale: float = 0.0, topk: int = 32,
                                guard_bits: int = 0, force_level: int = -1, max_len: int = 0,
                                dbg: DebugBuffers | None = None, workspace: torch.Tensor | None = None, events=None,
                                path: int = 0, stats: torch.Tensor | None = None) -> torch.Tensor:
    """One decode step: append k_new, v_new (fp16 [B, Hkv, 1, D] or [B, Hkv, D]) and attend with q."""
    assert k_new.dtype == torch.float16 and v_new.dtype == torch.float16 and k_new.numel() == cache.B * cache.Hkv * cache.D
    assert v_new.numel() == k_new.numel()
    assert q.dtype == torch.float16 and tuple(q.shape) == (cache.B, cache.Hq, cache.D)
    if out is None:
        out = torch.empty(cache.B, cache.Hq, cache.D, dtype=torch.float32, device=q.device)
    assert out.dtype in (torch.float32, torch.float16) and tuple(out.shape) == tuple(q.shape)
    ws = cache.workspace if workspace is None else workspace
    d = dbg.struct() if dbg is not None else None
    p = _params(out, scale, topk, guard_bits, force_level, max_len, d, events, path, stats)
    s = cache.struct()
    _check(lib().akv_append_decode_attention(C.byref(s), _ptr(k_new), _ptr(v_new), _ptr(q), _ptr(out), C.byref(p),
                                             _ptr(ws), ws.numel(), _stream()))
    return out


def akv_fp16_decode_attention(k: torch.Tensor, v: torch.Tensor, lens: torch.Tensor, q: torch.Tensor,
                              out: torch.Tensor | None = None, *, scale: float = 0.0, max_len: int = 0,
                              workspace: torch.Tensor | None = None) -> torch.Tensor:
    """k, v: fp16 [B, Hkv, Ncap, D]; lens: int32 [B]; q: fp16 [B, Hq, D] -- all on the device."""
    B, Hkv, Ncap, D = k.shape
    Hq = q.shape[1]
    assert k.dtype == v.dtype == q.dtype == torch.float16 and lens.dtype == torch.int32 and v.shape == k.shape
    if out is None:
        out = torch.empty(B, Hq, D, dtype=torch.float32, device=q.device)
    if workspace is None:
        workspace = torch.empty(akv_layout_sizes(B, Hq, Hkv, D, Ncap).fp16_workspace, dtype=torch.uint8, device=q.device)
    shp = akv_shape(B, Hq, Hkv, D, Ncap)
    _check(lib().akv_fp16_decode_attention(C.byref(shp), _ptr(k), _ptr(v), _ptr(lens), _ptr(q), _ptr(out), scale,
                                           0 if out.dtype == torch.float32 else 1, max_len, _ptr(workspace),
                                           workspace.numel(), _stream()))
    return out


# ------------------------------------------------------------------------------------------ weight GEMV (akw.h)

def akw_layout_sizes(K: int, N: int) -> akw_sizes:
    out = akw_sizes()
    _check(lib().akw_layout_sizes(K, N, C.byref(out)))
    return out


@dataclass
class Weights:
    """Caller-owned device buffers of one weight matrix in split planes (torch owns the memory)."""
    K: int
    N: int
    hi: torch.Tensor = field(repr=False, default=None)
    mid: torch.Tensor = field(repr=False, default=None)
    lo: torch.Tensor = field(repr=False, default=None)
    rowmax: torch.Tensor = field(repr=False, default=None)
    workspace: torch.Tensor = field(repr=False, default=None)

    @staticmethod
    def allocate(K: int, N: int, device="cuda:0") -> "Weights":
        sz = akw_layout_sizes(K, N)
        u8 = lambda n: torch.empty(n, dtype=torch.uint8, device=device)
        w = Weights(K, N, u8(sz.hi), u8(sz.mid), u8(sz.lo), torch.empty(K, dtype=torch.int16, device=device),
                    u8(sz.workspace))
        akw_workspace_init(w, w.workspace)
        return w

    def struct(self) -> akw_weights:
        return akw_weights(self.K, self.N, _ptr(self.hi), _ptr(self.mid), _ptr(self.lo), _ptr(self.rowmax))


def akw_workspace_init(w: Weights, workspace: torch.Tensor) -> None:
    _check(lib().akw_workspace_init(w.K, w.N, _ptr(workspace), workspace.numel(), _stream()))


def akw_pack(w: Weights, W: torch.Tensor) -> None:
    """W: fp16 [K, N] on the device."""
    assert W.dtype == torch.float16 and tuple(W.shape) == (w.K, w.N)
    s = w.struct()
    _check(lib().akw_pack(C.byref(s), _ptr(W), _stream()))


def akw_unpack(w: Weights) -> torch.Tensor:
    out = torch.empty(w.K, w.N, dtype=torch.float16, device=w.hi.device)
    s = w.struct()
    _check(lib().akw_unpack(C.byref(s), _ptr(out), _stream()))
    return out


def akw_gemv(w: Weights, x: torch.Tensor, y: torch.Tensor | None = None, *, guard_bits: int = 0, force_level: int = -1,
             lvl_out: torch.Tensor | None = None, workspace: torch.Tensor | None = None) -> torch.Tensor:
    """x: fp16 [B, K] on the device; returns y: float32 [B, N].  lvl_out: uint8 [K] receiving the row levels."""
    assert x.dtype == torch.float16 and x.dim() == 2 and x.shape[1] == w.K
    B = x.shape[0]
    if y is None:
        y = torch.empty(B, w.N, dtype=torch.float32, device=x.device)
    assert y.dtype == torch.float32 and tuple(y.shape) == (B, w.N)
    if lvl_out is not None:
        assert lvl_out.dtype == torch.uint8 and lvl_out.numel() == w.K
    ws = w.workspace if workspace is None else workspace
    s, p = w.struct(), akw_params(guard_bits, force_level, _ptr(lvl_out))
    _check(lib().akw_gemv(C.byref(s), _ptr(x), B, _ptr(y), C.byref(p), _ptr(ws), ws.numel(), _stream()))
    return y
