"""Synthetic analogues of the paper's bit-width curve and relative-error table ("Experiments": average bit width
of the KV cache against context length; relative error of QK^T and SV against a uniformly truncated cache), and the
study of other fetch granules ("Dynamic Quantization", data re-arrangement: the hardware reads in units of bytes;
"Quantization of K-Cache": the columns are only roughly uniform along the tokens).

Run on the GPU:  python -m paper_2409_16546_amd.analysis [--cfg 2] [--heads 8] [--batch 2]
Data: the generator of the chosen benchmark configuration at a reduced batch / head count (the statistics are per
head).  For every context length it prints the average number of bits read per K element and per V element (from the
library's device counters), and the relative error |R - R16| / |R16| of the logits and of the attention output against
the same kernels reading all 16 bits, for the aligned cache (guard 0, 1, 2) and for uniform truncation to 12 and to
8 bits (force_level 1 and 0).

Two further tables are estimates of bytes, computed here from the masks the library exports and from the data; no
kernel reads the cache that way: what V would read if its fetch unit were tt tokens x cc channels instead of one token
row, and what K would read if Rule 1 took its column maxima per block of tokens instead of per sequence.  Both are
checked against the CPU oracle's own evaluation of the same granules in the tests."""
from __future__ import annotations

import argparse

import numpy as np
import torch

from . import binding as A
from . import workloads

V_GRANULES = [(1, 128), (1, 64), (1, 32), (2, 128), (2, 64), (4, 32), (8, 16), (4, 128)]


def rel_err(x: torch.Tensor, ref: torch.Tensor) -> np.ndarray:
    """|x - ref| / |ref| over the elements with ref != 0 (the paper's formula with |R_normal| in the denominator)."""
    ref = ref.double().flatten()
    x = x.double().flatten()
    keep = ref != 0
    return ((x[keep] - ref[keep]).abs() / ref[keep].abs()).cpu().numpy()


def bits_from_counts(cnt) -> float:
    cnt = [int(x) for x in cnt]
    return (8 * cnt[0] + 12 * cnt[1] + 16 * cnt[2]) / max(sum(cnt), 1)


def measure(c: A.Cache, q: torch.Tensor, n: int, ref: torch.Tensor, ref_logits: torch.Tensor, dbg: A.DebugBuffers, **kw) -> dict:
    """One decode call with the given parameters on cache c (sequences of n tokens): bits per element from the device
    counters, relative errors against ref / ref_logits (the same kernels reading all 16 bits)."""
    st = A.new_stats(q.device)
    out = A.akv_decode_attention(c, q, dbg=dbg, stats=st, **kw)
    torch.cuda.synchronize()
    s = st.cpu().numpy()
    el = rel_err(dbg.logits[:, :, :n], ref_logits)
    eo = rel_err(out, ref)
    return {"bits_k": bits_from_counts(s[0:3]), "bits_v": bits_from_counts(s[3:6]), "bits_v_needed": bits_from_counts(s[6:9]),
            "logits_median": float(np.median(el)), "logits_p99": float(np.percentile(el, 99)),
            "logits_zero_frac": float((el == 0).mean()),
            "out_median": float(np.median(eo)), "out_p99": float(np.percentile(eo, 99)),
            "out_rel_l2": float((out.double() - ref.double()).norm() / ref.double().norm()), "out": out}


def v_counts_for_granule(needV: torch.Tensor, lens, tt: int, cc: int) -> list[int]:
    """Elements read at level 0 / 1 / 2 if V's fetch unit were tt tokens x cc channels: the maximum of the exported
    per-element needs over each unit, counted over the tokens of each sequence.  needV: uint8 [B, Hkv, Ncap, D]."""
    B, Hkv, Ncap, D = needV.shape
    counts = [0, 0, 0]
    for b in range(B):
        n = int(lens[b])
        need = needV[b].clone()
        need[:, n:] = 0
        unit = need.view(Hkv, Ncap // tt, tt, D // cc, cc).amax(dim=(2, 4))
        ntok = (torch.arange(Ncap, device=needV.device) < n).view(Ncap // tt, tt).sum(dim=1)
        for lvl in range(3):
            counts[lvl] += int(((unit == lvl) * ntok[None, :, None]).sum()) * cc
    return counts


def k_counts_with_block_colmax(k: torch.Tensor, q: torch.Tensor, lens, guard_bits: int, block: int) -> list[int]:
    """K elements read at level 0 / 1 / 2 if Rule 1 took its column maxima per `block` tokens (block >= the sequence: the
    rule the kernels implement).  k: fp16 [B, Hkv, N, D], q: fp16 [B, Hq, D]; query heads of a group take the maximum level."""
    B, Hkv, _, D = k.shape
    G = q.shape[1] // Hkv
    counts = [0, 0, 0]
    for b in range(B):
        n = int(lens[b])
        kk = k[b, :, :n].float().abs()
        qq = q[b].float().view(Hkv, G, D)
        for t0 in range(0, n, block):
            t1 = min(n, t0 + block)
            cm = kk[:, t0:t1].amax(dim=1).clamp_min(2.0 ** -14)               # [Hkv, D]
            P = qq * cm[:, None, :]                                            # exact in fp32 (11-bit x 11-bit significands)
            e = torch.frexp(P)[1].float()
            e = torch.where(P != 0, e, torch.full_like(e, -1e9))
            m = 10 + guard_bits - (e.amax(dim=-1, keepdim=True) - e)
            lvl = torch.where(P != 0, (m > 2).float() + (m > 6).float(), torch.zeros_like(m)).amax(dim=1)   # [Hkv, D]
            for l in range(3):
                counts[l] += int((lvl == l).sum()) * (t1 - t0)
    return counts


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--cfg", type=int, default=2)
    ap.add_argument("--heads", type=int, default=8, help="KV heads")
    ap.add_argument("--group", type=int, default=1, help="query heads per KV head")
    ap.add_argument("--batch", type=int, default=2)
    ap.add_argument("--lengths", type=int, nargs="+", default=[512, 1024, 2048, 4096, 8192, 16384, 32768])
    args = ap.parse_args()
    dev = "cuda:0"
    nmax = max(args.lengths)
    w = workloads.make(args.cfg, B=args.batch, Hq=args.heads * args.group, Hkv=args.heads, N=nmax)
    kd, vd, qd = w.k.to(dev), w.v.to(dev), w.q.to(dev)
    modes = [("aligned g0", dict(guard_bits=0)), ("aligned g1", dict(guard_bits=1)), ("aligned g2", dict(guard_bits=2)),
             ("uniform 12", dict(force_level=1)), ("uniform 8", dict(force_level=0))]
    print(f"data: config {args.cfg}, batch {args.batch}, {args.heads} KV heads x {args.group} query heads, seed {1000 + args.cfg}")
    print("| context | mode | bits K | bits V | logits: median / p99 rel. err (share exactly 0) | output: median / p99 rel. err | output rel-L2 |")
    print("|---|---|---|---|---|---|---|")
    gran = {}
    for n in args.lengths:
        ncap = (n + 255) // 256 * 256
        c = A.Cache.allocate(w.B, w.Hq, w.Hkv, w.D, ncap, dev)
        A.akv_append(c, kd[:, :, :n].contiguous(), vd[:, :, :n].contiguous())
        dbg = A.DebugBuffers.allocate(c, want_needV=True)
        ref = A.akv_decode_attention(c, qd, force_level=2, dbg=dbg).clone()
        ref_logits = dbg.logits[:, :, :n].clone()
        for name, kw in modes:
            m = measure(c, qd, n, ref, ref_logits, dbg, **kw)
            print(f"| {n} | {name} | {m['bits_k']:.2f} | {m['bits_v']:.2f} | {m['logits_median']:.1e} / {m['logits_p99']:.1e} "
                  f"({m['logits_zero_frac']:.0%}) | {m['out_median']:.1e} / {m['out_p99']:.1e} | {m['out_rel_l2']:.1e} |", flush=True)
            if name == "aligned g0":
                lens = [n] * w.B
                gran[n] = {g: bits_from_counts(v_counts_for_granule(dbg.needV, lens, *g)) for g in V_GRANULES}
                gran[n]["per element"] = m["bits_v_needed"]
        del c, dbg
    print()
    print("V: bits per element read if the fetch unit were (tokens x channels); (1 x 128) is the cache's token row")
    print("| context | per element | " + " | ".join(f"{t} x {c_}" for t, c_ in V_GRANULES) + " |")
    print("|---|---|" + "---|" * len(V_GRANULES))
    for n in args.lengths:
        print(f"| {n} | {gran[n]['per element']:.2f} | " + " | ".join(f"{gran[n][g]:.2f}" for g in V_GRANULES) + " |")
    print()
    print("K: bits per element read if Rule 1 took one column maximum per block of tokens")
    print("| context | guard | per sequence | per 256-token block | per 64-token block |")
    print("|---|---|---|---|---|")
    for n in args.lengths:
        lens = [n] * w.B
        for g in (0, 1, 2):
            row = [bits_from_counts(k_counts_with_block_colmax(kd, qd, lens, g, blk)) for blk in (1 << 30, 256, 64)]
            print(f"| {n} | {g} | {row[0]:.2f} | {row[1]:.2f} | {row[2]:.2f} |", flush=True)


if __name__ == "__main__":
    main()
