"""Decode attention on every benchmark configuration (1..5), one JSON line each: time of the library's own choice of
path, of each path where it applies, of the fp16 kernels of the same design and of the control group (the same kernels
reading all 16 bits); bytes read by plane from the exported decisions; effective bandwidth against the 8 TB/s peak.

Run on the GPU:  python -m paper_2409_16546_amd.bench_configs [--configs 1 3 4 5] [--steps 50]
``bench.py`` at the repository root is the benchmark of record (configuration 2, one appended token per step,
rotating cache copies); this module is the survey over the other shapes.  The calls rotate over as many cache copies as it takes to pass 2 GB (a single copy of a small configuration would sit
in the 256-MB memory-side cache, and two copies of configuration 2 still hit it in part).
"""
from __future__ import annotations

import argparse
import json
import time

import numpy as np
import torch

from . import binding as A
from . import workloads

HBM_PEAK_GBS = 8000.0


def timed(fn, n: int) -> float:
    for i in range(10):
        fn(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(n):
        fn(i)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e6 / n


def measure(cfg: int, steps: int = 50, dev: str = "cuda:0") -> dict:
    w = workloads.make(cfg)
    N, G = w.Ncap, w.Hq // w.Hkv
    fp16_cache_bytes = 2 * w.B * w.Hkv * N * w.D * 2
    R = max(1, min(64, -(-(2 << 30) // fp16_cache_bytes)))       # copies, so that the rotating footprint passes 2 GB, eight times the memory-side cache
    kd, vd, qd, lens = w.k.to(dev), w.v.to(dev), w.q.to(dev), w.lens.to(dev)
    caches = []
    for _ in range(R):
        c = A.Cache.allocate(w.B, w.Hq, w.Hkv, w.D, N, dev)
        A.akv_append(c, kd, vd, lens)
        caches.append(c)
    maxlen = int(w.lens.max())
    dbg = A.DebugBuffers.allocate(caches[0], want_needV=False)
    A.akv_decode_attention(caches[0], qd, max_len=maxlen, dbg=dbg)
    torch.cuda.synchronize()
    lv = dbg.lvlK.cpu().numpy().astype(np.int64)
    ap = dbg.appliedV.cpu().numpy().astype(np.int64)
    L = w.lens.numpy().astype(np.int64)
    k_bytes = sum(int(L[b]) * float((1 + 0.5 * (lv[b] >= 1) + 0.5 * (lv[b] >= 2)).sum()) for b in range(w.B))
    v_bytes = sum(int((128 + 64 * (ap[b, :, :L[b]] >= 1) + 64 * (ap[b, :, :L[b]] >= 2)).sum()) for b in range(w.B))
    logits_bytes = int(L.sum()) * w.Hq * 12                      # written once, read by the mid step and by the V side
    elems = int(L.sum()) * w.Hkv * w.D
    fp16_bytes = elems * 4
    total = k_bytes + v_bytes + logits_bytes
    del dbg
    o = torch.empty(w.B, w.Hq, w.D, dtype=torch.float32, device=dev)
    res = {"metric": "decode-attention us/step + effective HBM GB/s (% of peak) vs fp16 kernel", "unit": "us/step",
           "higher_is_better": False, "dtype": "f32", "data": "synthetic",
           "config": {"workload": w.name, "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "D": w.D, "Ncap": N,
                      "lens": [int(x) for x in L[:8]], "cache_copies_rotated": R},
           "bytes": {"K": int(k_bytes), "V": int(v_bytes), "logits": int(logits_bytes), "fp16": int(fp16_bytes),
                     "avg_bits_K": round(8.0 * k_bytes / elems, 2), "avg_bits_V_rows": round(8.0 * v_bytes / elems, 2),
                     "reduction_vs_fp16": round(1.0 - total / fp16_bytes, 4)}}
    t_end = time.perf_counter() + 0.3                           # the device reaches its working clocks before anything is timed
    while time.perf_counter() < t_end:
        A.akv_decode_attention(caches[0], qd, o, max_len=maxlen)
        torch.cuda.synchronize()
    paths = {}
    for path, name in ((0, "library_choice"), (1, "head_path"), (2, "token_split_path")):
        if path == 1 and G > 4:
            continue
        paths[name] = round(timed(lambda i: A.akv_decode_attention(caches[i % R], qd, o, max_len=maxlen, path=path), steps), 1)
    res["value"] = paths["library_choice"]
    res["us_by_path"] = paths
    res["control_group_16bit_us"] = round(timed(lambda i: A.akv_decode_attention(caches[i % R], qd, o, max_len=maxlen,
                                                                                force_level=2), steps), 1)
    if cfg == 3:
        # this configuration is defined with the append in the step: one more token per sequence is stored and attended
        # to.  Timed over consecutive steps that end at the configuration's context (the library's own choice of path,
        # which here stores the token with its append kernel before the four decode kernels)
        nsteps = min(steps, 100)
        first = N - 5 - nsteps
        grow = A.Cache.allocate(w.B, w.Hq, w.Hkv, w.D, N, dev)
        A.akv_append(grow, kd[:, :, :first].contiguous(), vd[:, :, :first].contiguous())
        kn = [kd[:, :, first + i].contiguous() for i in range(5 + nsteps)]
        vn = [vd[:, :, first + i].contiguous() for i in range(5 + nsteps)]
        for i in range(5):
            A.akv_append_decode_attention(grow, kn[i], vn[i], qd, o, max_len=N)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(5, 5 + nsteps):
            A.akv_append_decode_attention(grow, kn[i], vn[i], qd, o, max_len=N)
        torch.cuda.synchronize()
        res["fused_append_step_us"] = round((time.perf_counter() - t0) * 1e6 / nsteps, 1)
        res["fused_append_step_contexts"] = [first + 6, N]
        assert int(grow.lens.max()) == N and int(grow.flags[0]) == 0
        del grow, kn, vn
    gbps = total / paths["library_choice"] / 1e3
    res["roofline"] = {"bound": "hbm", "achieved": round(gbps, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                       "frac": round(gbps / HBM_PEAK_GBS, 4), "traffic": None, "algorithmic_bytes_per_step": int(total)}
    del caches
    torch.cuda.empty_cache()
    plain = [(kd, vd)] + [(kd.clone(), vd.clone()) for _ in range(R - 1)]
    ws16 = torch.empty(A.akv_layout_sizes(w.B, w.Hq, w.Hkv, w.D, N).fp16_workspace, dtype=torch.uint8, device=dev)
    f16 = timed(lambda i: A.akv_fp16_decode_attention(plain[i % R][0], plain[i % R][1], lens, qd, o, max_len=maxlen,
                                                      workspace=ws16), steps)
    res["fp16_kernel_us"] = round(f16, 1)
    res["fp16_kernel_GBps"] = round(fp16_bytes / f16 / 1e3, 1)
    res["speedup_vs_fp16_kernel"] = round(f16 / paths["library_choice"], 3)
    return res


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--configs", type=int, nargs="+", default=[1, 2, 3, 4, 5])
    ap.add_argument("--steps", type=int, default=50)
    args = ap.parse_args()
    for cfg in args.configs:
        print(json.dumps(measure(cfg, args.steps)), flush=True)
        torch.cuda.empty_cache()


if __name__ == "__main__":
    main()
