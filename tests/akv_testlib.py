"""Shared helpers of the GPU parity tests: build the same cache on both sides, compare every export."""
from __future__ import annotations

import numpy as np
import torch

from oracle import akv_oracle as O
from paper_2409_16546_amd import binding as A

MAX_ABS = 2e-3      # tolerance of the attention output against the oracle (the benchmark spec)
REL_L2 = 1e-3
LOGIT_C = 1.0       # constant of the derived bound below


def out_tolerance(r: O.DecodeResult, lens, scale: float = 0.0) -> np.ndarray:
    """Absolute bound per (sequence, query head), shape [B, Hq], for the comparison of the kernel's output with the
    oracle's.

    Wherever the head's max|out| <= 1 the bound is the literal 2e-3.  Where the output is larger it is derived from the
    head's own logits: the kernel's softmax weights come from logits accumulated in binary32 (the contract of the
    decision path -- those are the bits the masks are decided from), the oracle's from binary64.  A sum of D = 128
    addends rounded at every step carries an error of up to about sqrt(D) units in the last place of the largest logit
    (a few standard deviations of D independent roundings), the weight 2^((l - M) * scale * log2 e) then a relative
    error of that times scale, and the normalised sum over V a deviation of that relative error times the magnitude of
    the output:
        bound = max(2e-3, LOGIT_C * sqrt(D) * ulp32(max|l|) * scale * max|out|)      (per head).
    """
    lens = np.asarray(lens)
    B, Hq, D = r.out.shape
    sc = scale if scale > 0 else 1.0 / np.sqrt(D)
    bound = np.full((B, Hq), MAX_ABS)
    for b, n in enumerate(lens):
        if n <= 0:
            continue
        lmax = np.abs(r.logits[b, :, :int(n)]).max(axis=1).astype(np.float64)      # [Hq]
        omax = np.abs(r.out[b]).max(axis=1)                                          # [Hq]
        ulp = np.exp2(np.floor(np.log2(np.maximum(lmax, 1e-30))) - 23)
        derived = LOGIT_C * np.sqrt(D) * ulp * sc * omax
        bound[b] = np.where(omax <= 1.0, MAX_ABS, np.maximum(MAX_ABS, derived))
    return bound


def bits(t: torch.Tensor) -> np.ndarray:
    """fp16 torch tensor -> contiguous uint16 numpy array of its bit patterns."""
    return np.ascontiguousarray(t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16))


def oracle_cache(k: torch.Tensor, v: torch.Tensor, lens, Ncap: int) -> O.Cache:
    B, Hkv, N, D = k.shape
    c = O.Cache.empty(B, Hkv, D, Ncap)
    assert O.append(c, bits(k), bits(v), np.asarray(lens, np.int32)) == 0
    return c


def gpu_cache(k: torch.Tensor, v: torch.Tensor, lens, Hq: int, Ncap: int, dev="cuda:0") -> A.Cache:
    B, Hkv, N, D = k.shape
    c = A.Cache.allocate(B, Hq, Hkv, D, Ncap, dev)
    A.akv_append(c, k.to(dev), v.to(dev), torch.as_tensor(np.asarray(lens, np.int32)).to(dev))
    return c


def assert_cache_equal(g: A.Cache, o: O.Cache):
    for name in ("k_hi", "k_mid", "k_lo", "v_hi", "v_mid", "v_lo"):
        got = getattr(g, name).cpu().numpy()
        assert np.array_equal(got, getattr(o, name).reshape(-1)), f"plane {name} differs"
    assert np.array_equal(g.colmax.cpu().numpy().view(np.uint16), o.colmax.reshape(-1)), "colmax differs"
    assert np.array_equal(g.lens.cpu().numpy(), o.lens), "lens differ"


def rel_l2(x, ref):
    return float(np.linalg.norm((x - ref).ravel()) / max(np.linalg.norm(ref.ravel()), 1e-30))


def assert_decode_equal(g_out: torch.Tensor, d: A.DebugBuffers, r: O.DecodeResult, lens, G: int, what="", scale: float = 0.0):
    """Bit-exact decisions, output within tolerance.  Only tokens t < len and sequences with len > 0 count."""
    lens = np.asarray(lens)
    out = g_out.float().cpu().numpy().astype(np.float64)
    lvlK, logits, a, sel = d.lvlK.cpu().numpy(), d.logits.cpu().numpy(), d.a.cpu().numpy(), d.sel.cpu().numpy()
    oest, Ehat, appl = d.oest.cpu().numpy(), d.Ehat.cpu().numpy(), d.appliedV.cpu().numpy()
    needV = d.needV.cpu().numpy() if d.needV is not None else None
    for b, n in enumerate(lens):
        n = int(n)
        if n == 0:
            assert not out[b].any(), f"{what} b={b}: empty sequence must give zeros"
            continue
        assert np.array_equal(lvlK[b], r.lvlK[b]), f"{what} b={b}: lvlK differs"
        assert np.array_equal(logits[b, :, :n].view(np.uint32), r.logits[b, :, :n].view(np.uint32)), \
            f"{what} b={b}: logits differ in bits"
        assert np.array_equal(a[b, :, :n], r.a[b, :, :n]), f"{what} b={b}: score exponents differ"
        assert np.array_equal(sel[b], r.sel[b]), f"{what} b={b}: top-k selection differs"
        assert np.array_equal(oest[b].view(np.uint32), r.oest[b].view(np.uint32)), f"{what} b={b}: O_est differs in bits"
        assert np.array_equal(Ehat[b], r.Ehat[b]), f"{what} b={b}: result exponents differ"
        assert np.array_equal(appl[b, :, :n], r.appliedV[b, :, :n]), f"{what} b={b}: appliedV differs"
        if needV is not None and r.needV is not None:
            assert np.array_equal(needV[b, :, :n], r.needV[b, :, :n]), f"{what} b={b}: needV differs"
    err_h = np.abs(out - r.out).max(axis=2)                                          # [B, Hq]
    err = float(err_h.max())
    rl2 = rel_l2(out, r.out)
    bound = out_tolerance(r, lens, scale)
    worst = np.unravel_index(np.argmax(err_h / bound), err_h.shape)
    print(f"    {what}: max-abs {err:.3e}; worst head {worst}: {err_h[worst]:.3e} of its bound {bound[worst]:.3e} "
          f"(max|out| of that head {np.abs(r.out[worst]).max():.4g}; {int((bound > MAX_ABS).sum())} of {bound.size} heads "
          f"above the literal {MAX_ABS}) rel-L2 {rl2:.2e}", flush=True)
    assert np.all(err_h <= bound), f"{what}: head {worst}: max-abs {err_h[worst]:.3e} > {bound[worst]:.3e}"
    assert rl2 <= REL_L2, f"{what}: rel-L2 {rl2:.3e} > {REL_L2}"
    return err, rl2


def assert_stats_equal(stats: torch.Tensor, r: O.DecodeResult, what=""):
    """The library's device counters (akv_stats) against the oracle's counts: K elements per level, V elements per
    level as fetched (row granule), V elements per level as needed."""
    got = stats.cpu().numpy().astype(np.uint64)
    assert np.array_equal(got, r.counts), f"{what}: akv_stats {got.tolist()} != oracle counts {r.counts.tolist()}"


def run_both(k, v, q, lens, Ncap=None, dev="cuda:0", path=0, **params):
    """Build both caches from the same host tensors, decode on both sides with every export on.
    path: 0 library's choice, 1 head-per-workgroup kernel, 2 token-split kernels (GPU side only).
    The device counters of the call are compared with the oracle's counts on the way."""
    B, Hkv, N, D = k.shape
    Hq = q.shape[1]
    Ncap = Ncap or ((N + 255) // 256) * 256
    oc = oracle_cache(k, v, lens, Ncap)
    gc = gpu_cache(k, v, lens, Hq, Ncap, dev)
    topk = params.get("topk", 32)
    dbg = A.DebugBuffers.allocate(gc, topk=topk)
    stats = A.new_stats(dev)
    out = A.akv_decode_attention(gc, q.to(dev), dbg=dbg, path=path, stats=stats, **params).clone()
    # the same call with nothing exported runs the kernels as a caller gets them (no export code compiled in): the
    # exports must not change a bit of the result
    plain = A.akv_decode_attention(gc, q.to(dev), path=path, **params)
    torch.cuda.synchronize()
    assert torch.equal(plain, out), f"path {path}: the output without exports differs from the one with them"
    r = O.decode_attention(oc, bits(q), **params)
    assert_stats_equal(stats, r, f"path {path}")
    return gc, oc, out, dbg, r
