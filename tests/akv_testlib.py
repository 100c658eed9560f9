"""Shared helpers of the GPU parity tests: build the same cache on both sides, compare every export."""
from __future__ import annotations

import numpy as np
import torch

from oracle import akv_oracle as O
from paper_2409_16546_amd import binding as A

MAX_ABS = 2e-3      # tolerance of the attention output against the oracle (the benchmark spec), for outputs
REL_L2 = 1e-3       # of unit scale: where |out| exceeds 1 (outlier channels x20 on top of channel scales up to 10) the
                    # absolute bound is taken relative to max|out| -- the kernel's logits are fp32 (by the contract of
                    # the decision path), so a weight 2^x carries a relative error of about ulp(logit) * log2(e)/sqrt(D),
                    # which is 4e-5 for logits in the thousands, times the magnitude of the output


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


def assert_decode_equal(g_out: torch.Tensor, d: A.DebugBuffers, r: O.DecodeResult, lens, G: int, what=""):
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
    err = np.abs(out - r.out).max()
    rl2 = rel_l2(out, r.out)
    bound = MAX_ABS * max(1.0, float(np.abs(r.out).max()))
    assert err <= bound, f"{what}: max-abs {err:.3e} > {bound:.3e} (max|out| {np.abs(r.out).max():.3g})"
    assert rl2 <= REL_L2, f"{what}: rel-L2 {rl2:.3e} > {REL_L2}"
    return err, rl2


def run_both(k, v, q, lens, Ncap=None, dev="cuda:0", path=0, **params):
    """Build both caches from the same host tensors, decode on both sides with every export on.
    path: 0 library's choice, 1 head-per-workgroup kernel, 2 token-split kernels (GPU side only)."""
    B, Hkv, N, D = k.shape
    Hq = q.shape[1]
    Ncap = Ncap or ((N + 255) // 256) * 256
    oc = oracle_cache(k, v, lens, Ncap)
    gc = gpu_cache(k, v, lens, Hq, Ncap, dev)
    topk = params.get("topk", 32)
    dbg = A.DebugBuffers.allocate(gc, topk=topk)
    out = A.akv_decode_attention(gc, q.to(dev), dbg=dbg, path=path, **params)
    torch.cuda.synchronize()
    r = O.decode_attention(oc, bits(q), **params)
    return gc, oc, out, dbg, r
