"""Synthetic analogues of the paper's bit-width curve and relative-error table ("Experiments": average bit width
of the KV cache against context length; relative error of QK^T and SV against a uniformly truncated cache).

Run on the GPU:  python -m paper_2409_16546_amd.analysis [--cfg 2] [--heads 8] [--batch 2]
Data: the generator of the chosen benchmark configuration at a reduced batch / head count (the statistics are per
head).  For every context length it prints the average number of bits read per K element and per V element (by
the exported masks), and the relative error |R - R16| / |R16| of the logits and of the attention output against
the same kernel reading all 16 bits, for the aligned cache (guard 0, 1, 2) and for uniform truncation to 12 and
to 8 bits (force_level 1 and 0).

A second table estimates what a finer granule of the K rule would save: Rule 1 evaluated with a column maximum per
256-token block instead of one per sequence ("Quantization of K-Cache": the columns are only roughly uniform along
the tokens).  This is an estimate of bytes from the data, computed here in torch; no kernel reads K that way."""
from __future__ import annotations

import argparse

import numpy as np
import torch

from . import binding as A
from . import workloads


def rel_err(x: torch.Tensor, ref: torch.Tensor) -> np.ndarray:
    ref = ref.double().flatten()
    x = x.double().flatten()
    keep = ref != 0
    return ((x[keep] - ref[keep]).abs() / ref[keep].abs()).cpu().numpy()


def bits_k_with_block_colmax(k: torch.Tensor, q: torch.Tensor, n: int, guard_bits: int, block: int) -> float:
    """Average bits per K element over the first n tokens if Rule 1 took its column maxima per `block` tokens
    (block >= n: one maximum per sequence, the rule the kernels implement).  k: [B, H, N, D] fp16, q: [B, H, D] fp16."""
    kk = k[:, :, :n].float().abs()
    B, H, _, D = kk.shape
    total, weight = 0.0, 0
    for t0 in range(0, n, block):
        t1 = min(n, t0 + block)
        cm = kk[:, :, t0:t1].amax(dim=2).clamp_min(2.0 ** -14)          # [B, H, D]
        P = q.float() * cm                                                 # exact in fp32 (11-bit x 11-bit mantissas)
        e = torch.frexp(P)[1].float()
        e = torch.where(P != 0, e, torch.full_like(e, -1e9))
        m = 10 + guard_bits - (e.amax(dim=-1, keepdim=True) - e)
        lvl = torch.where(P != 0, (m > 2).float() + (m > 6).float(), torch.zeros_like(m))
        total += float((8 + 4 * lvl).sum()) * (t1 - t0)
        weight += B * H * D * (t1 - t0)
    return total / weight


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--cfg", type=int, default=2)
    ap.add_argument("--heads", type=int, default=8)
    ap.add_argument("--batch", type=int, default=2)
    ap.add_argument("--lengths", type=int, nargs="+", default=[512, 1024, 2048, 4096, 8192, 16384, 32768])
    args = ap.parse_args()
    dev = "cuda:0"
    nmax = max(args.lengths)
    w = workloads.make(args.cfg, B=args.batch, Hq=args.heads, Hkv=args.heads, N=nmax)
    kd, vd, qd = w.k.to(dev), w.v.to(dev), w.q.to(dev)
    modes = [("aligned g0", dict(guard_bits=0)), ("aligned g1", dict(guard_bits=1)), ("aligned g2", dict(guard_bits=2)),
             ("uniform 12", dict(force_level=1)), ("uniform 8", dict(force_level=0))]
    print(f"data: config {args.cfg}, batch {args.batch}, {args.heads} heads (MHA), seed {1000 + args.cfg}")
    print("| context | mode | bits K | bits V | logits: median / p99 rel. err | output: median / p99 rel. err | output rel-L2 |")
    print("|---|---|---|---|---|---|---|")
    for n in args.lengths:
        ncap = (n + 255) // 256 * 256
        c = A.Cache.allocate(w.B, w.Hq, w.Hkv, w.D, ncap, dev)
        A.akv_append(c, kd[:, :, :n].contiguous(), vd[:, :, :n].contiguous())
        dbg = A.DebugBuffers.allocate(c, want_needV=False)
        ref = A.akv_decode_attention(c, qd, force_level=2, dbg=dbg).clone()
        ref_logits = dbg.logits[:, :, :n].clone()
        for name, kw in modes:
            out = A.akv_decode_attention(c, qd, dbg=dbg, **kw)
            torch.cuda.synchronize()
            lv = dbg.lvlK.float()
            ap_ = dbg.appliedV[:, :, :n].float()
            bits_k = float((8 + 4 * (lv >= 1).float() + 4 * (lv >= 2).float()).mean())
            bits_v = float((8 + 4 * (ap_ >= 1).float() + 4 * (ap_ >= 2).float()).mean())
            el = rel_err(dbg.logits[:, :, :n], ref_logits)
            eo = rel_err(out, ref)
            rl2 = float((out.double() - ref.double()).norm() / ref.double().norm())
            print(f"| {n} | {name} | {bits_k:.2f} | {bits_v:.2f} | {np.median(el):.1e} / {np.percentile(el, 99):.1e} | "
                  f"{np.median(eo):.1e} / {np.percentile(eo, 99):.1e} | {rl2:.1e} |", flush=True)
        del c, dbg
    print()
    print("| context | guard | bits K, one colmax per sequence | bits K, one colmax per 256-token block | per 64-token block |")
    print("|---|---|---|---|---|")
    for n in args.lengths:
        for g in (0, 1, 2):
            whole = bits_k_with_block_colmax(kd, qd, n, g, 1 << 30)
            print(f"| {n} | {g} | {whole:.2f} | {bits_k_with_block_colmax(kd, qd, n, g, 256):.2f} | "
                  f"{bits_k_with_block_colmax(kd, qd, n, g, 64):.2f} |", flush=True)


if __name__ == "__main__":
    main()
