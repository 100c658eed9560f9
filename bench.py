#!/usr/bin/env python3
"""Benchmark of the AlignedKV decode step on one MI355X.

A step = one pass of the whole hot path over one batch: append one new token per sequence into the
split-plane cache and decode attention (Rule 1 levels, q.K~ pass, mid step, Rule 2 + S.V~ pass, final
division) for one query token per sequence -- one call of akv_append_decode_attention, one kernel.
Workload: benchmark configuration 2 (Llama-2-7B-shaped layer, batch 8, 32 heads, head_dim 128, context 4096,
synthetic fp16 K/V with per-channel log-uniform scales).  Inputs are resident in HBM before the timed
region; the steps rotate over several cache copies so that no copy is still in the L2 / Infinity Cache
when it is read again.  The tokens the steps append are the workload's own last tokens, so the last step
of every copy attends over exactly the workload (context 4096).

Prints ONE JSON line (metric, value, roofline of the dominant kernel, cpu_baseline, ...); progress goes to
stderr.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth
KERNEL = "akv::head_kernel<1, 1024, false>"


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class HipEvents:
    """hipEvent_t handles from the HIP runtime torch has loaded (same soname, same instance)."""

    def __init__(self):
        self.hip = C.CDLL("libamdhip64.so.7")
        self.hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self.hip.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [C.c_void_p]
        self.hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]

    def create(self, n):
        arr = (C.c_void_p * n)()
        for i in range(n):
            ev = C.c_void_p()
            assert self.hip.hipEventCreate(C.byref(ev)) == 0
            arr[i] = ev
        return arr

    def record(self, ev, stream):
        assert self.hip.hipEventRecord(ev, stream) == 0

    def elapsed_ms(self, e0, e1):
        assert self.hip.hipEventSynchronize(e1) == 0
        ms = C.c_float()
        assert self.hip.hipEventElapsedTime(C.byref(ms), e0, e1) == 0
        return float(ms.value)


def measured_traffic():
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary, or None."""
    path = os.path.join(ROOT, "profiles", "head_kernel_cfg2_pmc.txt")
    try:
        m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read(), flags=re.M)
        return int(float(m.group(1))) if m else None
    except OSError:
        return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--copies", type=int, default=8, help="cache copies the steps rotate over")
    ap.add_argument("--guard-bits", type=int, default=0)
    ap.add_argument("--clock-warmup-ms", type=float, default=300.0,
                    help="untimed decode calls (no append, the caches are left as they are) before the warm-up steps, "
                         "so that a fresh device is at its working clocks when the timed region starts")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the fp16 / control-group legs")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy three times (known traffic, for scaling rocprofv3 counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus must be 1")
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2409_16546_amd import binding as A, workloads

    dev = "cuda:0"
    torch.cuda.set_device(0)
    t_start = time.time()
    w = workloads.make(2)
    B, Hq, Hkv, D, N = w.B, w.Hq, w.Hkv, w.D, 4096
    steps, warmup = args.steps, args.warmup
    R = max(args.copies, (steps + warmup + 255) // 256)
    visits = (steps + warmup + R - 1) // R          # times each cache copy is stepped
    N0 = N - visits                                 # tokens in each copy before its first step
    Ncap = N
    log(f"[bench] workload {w.name}; {R} cache copies, each stepped {visits} times from context {N0 + 1} to {N}; "
        f"generated in {time.time() - t_start:.1f}s")

    kd, vd, qd = w.k.to(dev), w.v.to(dev), w.q.to(dev)
    caches = []
    for r in range(R):
        c = A.Cache.allocate(B, Hq, Hkv, D, Ncap, dev)
        A.akv_append(c, kd[:, :, :N0].contiguous(), vd[:, :, :N0].contiguous())
        caches.append(c)
    kn = [kd[:, :, N0 + i].contiguous() for i in range(visits)]   # the workload's own tokens N0 .. N-1
    vn = [vd[:, :, N0 + i].contiguous() for i in range(visits)]
    outs = [torch.empty(B, Hq, D, dtype=torch.float32, device=dev) for _ in range(R)]
    visit_of = [0] * R

    def step(i):
        r = i % R
        vi = visit_of[r]
        visit_of[r] += 1
        A.akv_append_decode_attention(caches[r], kn[vi], vn[vi], qd, outs[r], guard_bits=args.guard_bits, max_len=Ncap)

    # ---------------------------------------------------------------- the timed region
    ev = HipEvents()
    stream = torch.cuda.current_stream().cuda_stream
    e0, e1 = ev.create(2)
    t_warm = time.perf_counter() + args.clock_warmup_ms * 1e-3
    while time.perf_counter() < t_warm:
        for r in range(R):
            A.akv_decode_attention(caches[r], qd, outs[r], guard_bits=args.guard_bits, max_len=Ncap)
        torch.cuda.synchronize()
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev.record(e0, stream)                            # HIP events on the stream the kernels are launched on
    for i in range(warmup, warmup + steps):
        step(i)
    ev.record(e1, stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps
    kern_us = ev.elapsed_ms(e0, e1) * 1e3 / steps    # one kernel launch per step: average launch duration
    log(f"[bench] {steps} steps: {ms_per_step * 1e3:.1f} us/step wall clock, {kern_us:.1f} us per launch by HIP events "
        f"(contexts {N0 + 1}..{N})")

    # ---------------------------------------------------------------- algorithmic bytes (from the exported decisions)
    for c in caches:                                     # every copy now holds exactly the workload's N tokens
        c.lens.fill_(N)
    c0 = caches[0]
    dbg = A.DebugBuffers.allocate(c0, want_needV=False)
    out_dbg = A.akv_decode_attention(c0, qd, guard_bits=args.guard_bits, max_len=Ncap, dbg=dbg).clone()
    torch.cuda.synchronize()
    lvlK = dbg.lvlK.cpu().numpy()
    appl = dbg.appliedV.cpu().numpy()[:, :, :N]
    # per (sequence, KV head) and token: K columns at 1 / 1.5 / 2 bytes, V rows at 128 / 192 / 256 bytes
    k_plane_bytes = float(((1.0 + 0.5 * (lvlK >= 1) + 0.5 * (lvlK >= 2)).sum()) * N)
    v_plane_bytes = float((128.0 + 64.0 * (appl >= 1) + 64.0 * (appl >= 2)).sum())
    logits_bytes = 3 * 4.0 * B * Hq * N                  # written by the K side, read by the mid step and by the V side
    oest_bytes = float(B * Hq * 32 * D * 2)              # the top-k rows of V at 16 bits
    small_bytes = B * Hq * D * 2 + B * Hkv * D * 2 + B * Hq * D * 4 + 2 * B * Hkv * D * 2 * 2   # q, colmax, out, new K/V token
    akv_bytes = k_plane_bytes + v_plane_bytes + logits_bytes + oest_bytes + small_bytes
    fp16_bytes = 2.0 * B * Hkv * N * D * 2 + B * Hq * D * 2 + B * Hq * D * 4
    kbits = 8.0 * k_plane_bytes / (B * Hkv * N * D)
    vbits = 8.0 * v_plane_bytes / (B * Hkv * N * D)
    achieved = akv_bytes / (kern_us * 1e-6) / 1e9
    log(f"[bench] K {kbits:.2f} bits/elem, V {vbits:.2f} bits/elem; algorithmic bytes/step {akv_bytes / 1e6:.1f} MB vs fp16 "
        f"{fp16_bytes / 1e6:.1f} MB; {achieved:.0f} GB/s = {achieved / HBM_PEAK_GBS:.1%} of peak")

    result = {
        "metric": "decode-attention us/step + effective HBM GB/s (% of peak) vs fp16 kernel",
        "value": round(ms_per_step * 1e3, 2), "unit": "us/step", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "BASELINE config 2: Llama-2-7B-shaped layer, batch 8, 32 heads (MHA), head_dim 128, "
                               "context 4096 (each timed step appends one token; the contexts of the timed steps end at "
                               "4096), fp16 K/V N(0,1) x per-channel log-uniform scales in [0.1,10], q N(0,1), seed 1002",
                   "B": B, "Hq": Hq, "Hkv": Hkv, "D": D, "context": N, "guard_bits": args.guard_bits, "topk": 32,
                   "cache_copies_rotated": R,
                   "step": "akv_append_decode_attention: append 1 token/seq + decode attention, one kernel launch"},
        "roofline": {"bound": "hbm", "kernel": KERNEL, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": measured_traffic(),
                     "algorithmic_bytes_per_launch": int(akv_bytes), "avg_launch_us": round(kern_us, 2)},
        "bytes_per_step": {"alignedkv": int(akv_bytes), "fp16": int(fp16_bytes),
                           "reduction_vs_fp16": round(1.0 - akv_bytes / fp16_bytes, 4),
                           "avg_bits_K": round(kbits, 2), "avg_bits_V_rows": round(vbits, 2)},
        "effective_GBps": {"fetched": round(akv_bytes / (ms_per_step * 1e-3) / 1e9, 1),
                           "fp16_equivalent": round(fp16_bytes / (ms_per_step * 1e-3) / 1e9, 1)},
        "paper_context": "paper reports 25% less KV memory access and up to 1.3x attention speedup on one V100 (Llama-2-7B); "
                         "other hardware, not a target",
    }

    def timed(fn, n):
        for i in range(min(warmup, 10)):
            fn(i)
        torch.cuda.synchronize()
        a = time.perf_counter()
        for i in range(n):
            fn(i)
        torch.cuda.synchronize()
        return (time.perf_counter() - a) * 1e6 / n

    if not args.no_extras:
        # ------------------------------------------------------------ fp16 yardstick and control group, timed the same way
        kp = [kd.clone() for _ in range(R)]
        vp = [vd.clone() for _ in range(R)]
        lens_n = torch.full((B,), N, dtype=torch.int32, device=dev)
        ws16 = torch.empty(A.akv_layout_sizes(B, Hq, Hkv, D, Ncap).fp16_workspace, dtype=torch.uint8, device=dev)
        o16 = torch.empty(B, Hq, D, dtype=torch.float32, device=dev)
        fp16_us = timed(lambda i: A.akv_fp16_decode_attention(kp[i % R], vp[i % R], lens_n, qd, o16, max_len=Ncap,
                                                             workspace=ws16), steps)
        ctl_us = timed(lambda i: A.akv_decode_attention(caches[i % R], qd, outs[i % R], force_level=2, max_len=Ncap), steps)
        akv_only_us = timed(lambda i: A.akv_decode_attention(caches[i % R], qd, outs[i % R], guard_bits=args.guard_bits,
                                                             max_len=Ncap), steps)
        g2_us = timed(lambda i: A.akv_decode_attention(caches[i % R], qd, outs[i % R], guard_bits=2, max_len=Ncap), steps)
        split_us = timed(lambda i: A.akv_decode_attention(caches[i % R], qd, outs[i % R], guard_bits=args.guard_bits,
                                                          max_len=Ncap, path=2), steps)
        # "hot": one cache copy over and over (its planes partly stay in the 256-MB memory-side cache); the figures
        # above are the "cold" ones, over the rotating copies
        hot_us = timed(lambda i: A.akv_decode_attention(caches[0], qd, outs[0], guard_bits=args.guard_bits, max_len=Ncap), steps)
        hot16_us = timed(lambda i: A.akv_fp16_decode_attention(kp[0], vp[0], lens_n, qd, o16, max_len=Ncap, workspace=ws16), steps)
        log(f"[bench] attention only (context {N}): AlignedKV {akv_only_us:.1f} us, control(16-bit) {ctl_us:.1f} us, "
            f"fp16 kernel {fp16_us:.1f} us, guard2 {g2_us:.1f} us, token-split path {split_us:.1f} us")
        # the read ceiling of this device, by the library's plain streaming kernel over the same rotating footprint
        sink = torch.zeros(1, dtype=torch.int32, device=dev)
        stream_us = timed(lambda i: A.akv_stream_read(kp[i % R], sink), steps)
        stream_gbps = kp[0].numel() * 2 / stream_us / 1e3
        log(f"[bench] plain streaming read of {kp[0].numel() * 2 / 1e6:.0f} MB: {stream_us:.1f} us = {stream_gbps:.0f} GB/s")
        o16 = A.akv_fp16_decode_attention(kp[0], vp[0], lens_n, qd, max_len=Ncap, workspace=ws16)
        torch.cuda.synchronize()
        dev16 = (out_dbg - o16).double()
        result["streaming_read_ceiling"] = {
            "GBps": round(stream_gbps, 1), "frac_of_peak": round(stream_gbps / HBM_PEAK_GBS, 4),
            "step_frac_of_ceiling": round(akv_bytes / (ms_per_step * 1e-3) / 1e9 / stream_gbps, 4),
            "how": "akv_stream_read (16-byte non-temporal loads, four in flight per lane, 1-MB blocks dealt over the XCDs) over the K tensors of the rotating fp16 copies, timed like a step"}
        result["vs_fp16_kernel"] = {
            "fp16_kernel_us": round(fp16_us, 2), "fp16_kernel_GBps": round(fp16_bytes / fp16_us / 1e3, 1),
            "fp16_kernel_frac_of_peak": round(fp16_bytes / fp16_us / 1e3 / HBM_PEAK_GBS, 4),
            "one_copy_repeated_us": {"alignedkv": round(hot_us, 2), "fp16_kernel": round(hot16_us, 2)},
            "alignedkv_attention_only_us": round(akv_only_us, 2), "control_group_16bit_us": round(ctl_us, 2),
            "alignedkv_guard2_us": round(g2_us, 2), "alignedkv_token_split_path_us": round(split_us, 2),
            "speedup_vs_fp16_kernel": round(fp16_us / akv_only_us, 3), "speedup_vs_control_group": round(ctl_us / akv_only_us, 3),
            "deviation_from_fp16_attention": {"max_abs": float(dev16.abs().max()),
                                              "rel_l2": float(dev16.norm() / o16.double().norm())}}
        del kp, vp
        # ------------------------------------------------------------ the second workload (weight GEMV under Rule 1), briefly
        torch.cuda.empty_cache()
        from paper_2409_16546_amd import bench_weights
        gemv = {}
        for shape in ("attn_proj", "mlp_up", "mlp_down"):
            m = bench_weights.measure(shape, 1, steps)
            gemv[shape] = {"K": m["config"]["K"], "N": m["config"]["N"], "us": m["value"],
                           "avg_bits_W": m["bytes"]["avg_bits_W"], "GBps": m["roofline"]["achieved"],
                           "frac_of_peak": m["roofline"]["frac"], "control_group_16bit_us": m["control_group_16bit_us"],
                           "blas_fp16_matmul_us": m["blas_fp16_matmul_us"]}
            torch.cuda.empty_cache()
        log("[bench] weight GEMV (B=1): " + ", ".join(f"{k} {v['us']} us ({v['avg_bits_W']} bits, 16-bit control "
                                                       f"{v['control_group_16bit_us']} us, BLAS {v['blas_fp16_matmul_us']} us)"
                                                       for k, v in gemv.items()))
        result["weight_gemv"] = gemv

    if args.pmc_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        log("[bench] calibration: 3 device copies of 268435456 bytes (read 268435456, write 268435456 each)")

    if not args.no_cpu_baseline:
        # ------------------------------------------------------------ the CPU oracle, as it stands, on the host cores
        from oracle import akv_oracle as O
        bits = lambda t: np.ascontiguousarray(t.contiguous().view(torch.int16).numpy().view(np.uint16))
        oc = O.Cache.empty(B, Hkv, D, N)
        O.append(oc, bits(w.k), bits(w.v), np.full(B, N - 1, np.int32))
        nrep = 3
        ta = time.perf_counter()
        for rep in range(nrep):                          # the same step three times (about 15-20 s of CPU work in all)
            oc.lens[:] = N - 1
            O.append(oc, bits(w.k[:, :, N - 1:N]), bits(w.v[:, :, N - 1:N]))
            ref = O.decode_attention(oc, bits(w.q), guard_bits=args.guard_bits, want_needV=False)
        cpu_us = (time.perf_counter() - ta) * 1e6 / nrep
        # the same step on ONE thread, on the first sequence only (32 of the 256 pairs), scaled to the whole batch
        nthreads = O.max_threads()
        o1 = O.Cache.empty(1, Hkv, D, N)
        O.append(o1, bits(w.k[:1]), bits(w.v[:1]), np.full(1, N - 1, np.int32))
        O.set_threads(1)
        tb = time.perf_counter()
        O.append(o1, bits(w.k[:1, :, N - 1:N]), bits(w.v[:1, :, N - 1:N]))
        O.decode_attention(o1, bits(w.q[:1]), guard_bits=args.guard_bits, want_needV=False)
        cpu1_us = (time.perf_counter() - tb) * 1e6 * B
        O.set_threads(nthreads)
        got = out_dbg.cpu().numpy().astype(np.float64)
        err = float(np.abs(got - ref.out).max())
        rl2 = float(np.linalg.norm(got - ref.out) / np.linalg.norm(ref.out))
        planes_equal = all(np.array_equal(getattr(c0, n).cpu().numpy(), getattr(oc, n).reshape(-1))
                           for n in ("k_hi", "k_mid", "k_lo", "v_hi", "v_mid", "v_lo"))
        masks_equal = bool(np.array_equal(lvlK, ref.lvlK) and np.array_equal(appl, ref.appliedV[:, :, :N]))
        log(f"[bench] oracle: {cpu_us / 1e6:.2f} s/step on {nthreads} threads, {cpu1_us / 1e6:.2f} s/step on one (extrapolated from one sequence); GPU vs oracle max-abs {err:.2e} "
            f"rel-L2 {rl2:.2e}; masks equal {masks_equal}; cache bytes equal {planes_equal}")
        result["cpu_baseline"] = {"value": round(cpu_us, 1), "unit": "us/step", "cores": O.max_threads(), "kind": "oracle",
                                  "sample": "the whole config-2 step (all 256 (sequence, head) pairs: append 1 token + decode "
                                            "attention over 4096), mean of 3 runs, OpenMP over (sequence, head)",
                                  "one_thread": {"value": round(cpu1_us, 1), "unit": "us/step", "cores": 1,
                                                 "sample": "the step of the first sequence (32 of the 256 pairs), once, "
                                                           "times 8: extrapolated"}}
        result["parity_vs_oracle"] = {"max_abs": err, "rel_l2": rl2, "masks_bit_exact": masks_equal,
                                      "cache_bytes_bit_exact": bool(planes_equal)}

    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
