"""Timing of the precision-aligned weight GEMV (include/akw.h) on the projection shapes of the paper's model.

Run on the GPU:  python -m paper_2409_16546_amd.bench_weights [--shapes attn_proj mlp_up mlp_down] [--B 1] [--steps 200]
One JSON line per shape: microseconds per call, the bytes the levels make the kernel read (algorithmic bytes: the
planes of every row at its level, x, rowmax, y), the effective bandwidth against the 8 TB/s peak, the same kernel
reading all 16 bits (control group), uniform 8 bits, and the fp16 product of the BLAS library torch calls
(``torch.matmul``) on the same matrices.  The calls rotate over enough copies of the matrix that no copy is still
in a cache when its turn comes again.
"""
from __future__ import annotations

import argparse
import json
import time

import torch

from . import binding as A
from . import workloads

HBM_PEAK_GBS = 8000.0
FOOTPRINT = 768 << 20   # bytes the rotating copies cover at least (L2 and the memory-side cache hold less)


def measure(shape: str, B: int = 1, steps: int = 200, guard_bits: int = 0, dev: str = "cuda:0") -> dict:
    wl = workloads.make_weights(shape, B)
    K, N = wl.K, wl.N
    R = max(2, -(-FOOTPRINT // (K * N * 2)))
    Wd, xd = wl.W.to(dev), wl.x.to(dev)
    packed = []
    for _ in range(R):
        w = A.Weights.allocate(K, N, dev)
        A.akw_pack(w, Wd)
        packed.append(w)
    plain = [Wd.clone() for _ in range(R)]
    y = torch.empty(B, N, dtype=torch.float32, device=dev)
    lvl = torch.empty(K, dtype=torch.uint8, device=dev)
    A.akw_gemv(packed[0], xd, y, guard_bits=guard_bits, lvl_out=lvl)
    torch.cuda.synchronize()
    lv = lvl.cpu().numpy()
    plane_bytes = float(((1.0 + 0.5 * (lv >= 1) + 0.5 * (lv >= 2)) * N).sum())
    alg_bytes = plane_bytes + 2.0 * K * (B + 1) + 4.0 * B * N
    fp16_bytes = 2.0 * K * N + 2.0 * K * B + 4.0 * B * N

    def timed(fn):
        for i in range(10):
            fn(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            fn(i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e6 / steps

    us = timed(lambda i: A.akw_gemv(packed[i % R], xd, y, guard_bits=guard_bits))
    ctl_us = timed(lambda i: A.akw_gemv(packed[i % R], xd, y, force_level=2))
    u8_us = timed(lambda i: A.akw_gemv(packed[i % R], xd, y, force_level=0))
    y16 = torch.empty(B, N, dtype=torch.float16, device=dev)
    blas_us = timed(lambda i: torch.matmul(xd, plain[i % R], out=y16))
    ref = xd.double() @ Wd.double()
    A.akw_gemv(packed[0], xd, y, guard_bits=guard_bits)
    rel = float((y.double() - ref).norm() / ref.norm())
    gbps = alg_bytes / us / 1e3
    return {
        "metric": "weight GEMV us/call + effective HBM GB/s (% of peak) vs the same kernel at 16 bits", "value": round(us, 2),
        "unit": "us/call", "higher_is_better": False, "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name, "K": K, "N": N, "B": B, "guard_bits": guard_bits, "copies_rotated": R},
        "roofline": {"bound": "hbm", "kernel": f"akv::gemv_kernel<{B}>", "achieved": round(gbps, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(gbps / HBM_PEAK_GBS, 4), "traffic": None,
                     "algorithmic_bytes_per_launch": int(alg_bytes)},
        "bytes": {"aligned": int(alg_bytes), "fp16": int(fp16_bytes), "reduction_vs_fp16": round(1 - alg_bytes / fp16_bytes, 4),
                  "avg_bits_W": round(8.0 * plane_bytes / (K * N), 2),
                  "rows_at_8_12_16_bits": [int((lv == i).sum()) for i in range(3)]},
        "control_group_16bit_us": round(ctl_us, 2), "uniform_8bit_us": round(u8_us, 2),
        "control_group_GBps": round(fp16_bytes / ctl_us / 1e3, 1), "speedup_vs_control_group": round(ctl_us / us, 3),
        "blas_fp16_matmul_us": round(blas_us, 2), "speedup_vs_blas_fp16": round(blas_us / us, 3),
        "rel_l2_vs_exact_product": rel,
    }


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--shapes", nargs="+", default=list(workloads.WEIGHT_SHAPES))
    ap.add_argument("--B", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--guard-bits", type=int, default=0)
    args = ap.parse_args()
    for shape in args.shapes:
        print(json.dumps(measure(shape, args.B, args.steps, args.guard_bits)), flush=True)
        torch.cuda.empty_cache()


if __name__ == "__main__":
    main()
