#!/usr/bin/env python3
"""Benchmark of the AlignedKV decode step on one MI355X.

A step = one pass of the whole hot path over one batch: append one new token per sequence into the split-plane cache
and decode attention (Rule 1 levels, q.K~ pass, mid step, Rule 2 + S.V~ pass, combination) for one query token per
sequence -- one call of akv_append_decode_attention.

Headline workload: benchmark configuration 3, the largest of the five that is defined on one GPU's share (Llama-2-7B-
shaped layer, batch 16, 32 heads, head_dim 128, context 8192, 1 % token outliers, one token appended per sequence
inside the timed step).  Inputs are resident in HBM before the timed region; the steps rotate over cache copies far
larger than the L2 and the memory-side cache.  The tokens the steps append are the workload's own last tokens, so the
last step of every copy attends over exactly the workload.

The JSON line also carries a "configs" object with one entry per benchmark configuration 1..5 (attention as each is
defined: only configuration 3 includes the append): time of the library's own choice of path, time per phase from HIP
events the library records around its kernels, algorithmic bytes from the library's device counters (akv_stats),
fraction of the 8 TB/s peak, the fp16 kernels of the same design, the 16-bit control group, and the CPU oracle timed
on a stated sample.

Prints ONE JSON line; progress goes to stderr.
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
HEADLINE = 3
MIN_LEG_MS = 50.0       # every side leg is timed for at least this long, whatever --steps says
WORKLOAD_TEXT = {
    1: "BASELINE config 1: batch 1, 32 heads (MHA), head_dim 128, context 1024, fp16 Q/K/V N(0,1) with 4 outlier channels "
       "per head x20, seed 1001",
    2: "BASELINE config 2: Llama-2-7B-shaped layer, batch 8, 32 heads (MHA), head_dim 128, context 4096, fp16 K/V N(0,1) x "
       "per-channel log-uniform scales in [0.1,10], q N(0,1), seed 1002",
    3: "BASELINE config 3: Llama-2-7B-shaped layer, batch 16, 32 heads (MHA), head_dim 128, context 8192, fp16 K/V as config 2 "
       "plus 1% token rows x30, q N(0,1), seed 1003; each step appends 1 new token per sequence, then attends (the contexts "
       "of the timed steps end at 8192)",
    4: "BASELINE config 4: Llama-3-8B-shaped GQA layer, batch 8, 32 query / 8 KV heads, head_dim 128, context 32768, fp16 K/V "
       "with per-channel log-uniform scales and 4 outlier channels x20, seed 1004",
    5: "BASELINE config 5: long-context stress, batch 4, 32 query / 8 KV heads, head_dim 128, capacity 131072, lengths uniform in "
       "[32K,128K], fp16 K/V Student-t(3), seed 1005",
}


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
        self.hip.hipEventDestroy.argtypes = [C.c_void_p]

    def create(self, n):
        arr = (C.c_void_p * n)()
        for i in range(n):
            ev = C.c_void_p()
            assert self.hip.hipEventCreate(C.byref(ev)) == 0
            arr[i] = ev
        return arr

    def destroy(self, arr):
        for e in arr:
            self.hip.hipEventDestroy(e)

    def record(self, ev, stream):
        assert self.hip.hipEventRecord(ev, stream) == 0

    def elapsed_ms(self, e0, e1):
        assert self.hip.hipEventSynchronize(e1) == 0
        ms = C.c_float()
        assert self.hip.hipEventElapsedTime(C.byref(ms), e0, e1) == 0
        return float(ms.value)


def measured_traffic(kernel_tag: str, cfg: int):
    """HBM bytes per launch of a kernel from the committed rocprofv3 --pmc summary of that kernel and configuration
    (profiles/<kernel_tag>_cfg<cfg>_pmc.txt), or None.  Not measured in this run: counters need rocprofv3."""
    path = os.path.join(ROOT, "profiles", f"{kernel_tag}_cfg{cfg}_pmc.txt")
    try:
        m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read(), flags=re.M)
        return (int(float(m.group(1))), os.path.relpath(path, ROOT)) if m else (None, None)
    except OSError:
        return None, None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--guard-bits", type=int, default=0)
    ap.add_argument("--clock-warmup-ms", type=float, default=300.0,
                    help="untimed decode calls (no append, the caches are left as they are) before the warm-up steps, "
                         "so that a fresh device is at its working clocks when the timed region starts")
    ap.add_argument("--configs", type=int, nargs="*", default=[1, 2, 3, 4, 5],
                    help="configurations of the 'configs' object (the headline configuration is always run)")
    ap.add_argument("--headline", type=int, default=HEADLINE, help="configuration the headline value is measured on (profiling aid)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the fp16 / control-group / other-path legs and the weight GEMV")
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
    ev = HipEvents()
    stream = torch.cuda.current_stream().cuda_stream
    bits = lambda t: np.ascontiguousarray(t.contiguous().view(torch.int16).numpy().view(np.uint16))

    def timed(fn, n):
        """us per call: at least n calls and at least MIN_LEG_MS of device time, after a few untimed calls."""
        for i in range(5):
            fn(i)
        torch.cuda.synchronize()
        total, done = 0.0, 0
        while done < n or total < MIN_LEG_MS * 1e-3:
            t0 = time.perf_counter()
            for i in range(done, done + n):
                fn(i)
            torch.cuda.synchronize()
            total += time.perf_counter() - t0
            done += n
        return total * 1e6 / done

    def clock_warmup(fn):
        t_end = time.perf_counter() + args.clock_warmup_ms * 1e-3
        while time.perf_counter() < t_end:
            for i in range(4):
                fn(i)
            torch.cuda.synchronize()

    def event_gap_us(n=50):
        """Stream time between two events recorded back to back (what an event adds to the segment in front of it)."""
        pairs = [ev.create(2) for _ in range(n)]
        for a, b in pairs:
            ev.record(a, stream)
            ev.record(b, stream)
        torch.cuda.synchronize()
        gap = sum(ev.elapsed_ms(a, b) for a, b in pairs) * 1e3 / n
        for pr in pairs:
            ev.destroy(pr)
        return gap

    def bytes_from_stats(st, w, lens, with_append, logits_in_memory=True):
        """Algorithmic bytes of one step from the library's device counters (elements per level).  logits_in_memory:
        false where the head-per-workgroup kernel keeps its logits in LDS (akv_decode_path() == 3)."""
        k, v = st[0:3], st[3:6]
        k_planes = int(k.sum()) + int(k[1] + k[2]) // 2 + int(k[2]) // 2
        v_planes = int(v.sum()) + int(v[1] + v[2]) // 2 + int(v[2]) // 2
        ntok = int(sum(lens))
        logits_w = 4 * ntok * w.Hq if logits_in_memory else 0   # written by the K side
        logits_r = 4 * ntok * w.Hq if logits_in_memory else 0   # read by the V side (the mid step's read is served by the caches)
        oest = w.B * w.Hq * 32 * w.D * 2                 # the top-k rows of V at 16 bits
        small = w.B * w.Hq * w.D * 2 + w.B * w.Hkv * w.D * 2 + w.B * w.Hq * w.D * 4
        if with_append:
            small += 2 * w.B * w.Hkv * w.D * 2 * 2       # the new K / V token, read and stored
        elems = ntok * w.Hkv * w.D
        return {"k_planes": k_planes, "v_planes": v_planes, "logits_written": logits_w, "logits_read": logits_r,
                "oest_rows": oest, "small": small, "total": k_planes + v_planes + logits_w + logits_r + oest + small,
                "k_kernel": k_planes + logits_w + w.B * w.Hq * w.D * 2 + w.B * w.Hkv * w.D * 2,
                "v_kernel": v_planes + logits_r,
                "fp16": 4 * elems + w.B * w.Hq * w.D * 2 + w.B * w.Hq * w.D * 4,
                "avg_bits_K": round(8.0 * k_planes / elems, 2), "avg_bits_V_rows": round(8.0 * v_planes / elems, 2),
                "avg_bits_V_needed": round(float(8 * st[6] + 12 * st[7] + 16 * st[8]) / max(elems, 1), 2)}

    def run_config(cfg, steps, warmup, headline):
        """Measure one configuration; returns (entry of the 'configs' object, extras for the headline)."""
        t_gen = time.time()
        w = workloads.make(cfg)
        B, Hq, Hkv, D, N = w.B, w.Hq, w.Hkv, w.D, w.Ncap
        lens = w.lens.tolist()
        maxlen = max(lens)
        append = w.append_last
        plane_bytes = 2 * B * Hkv * N * D * 2
        R = max(2, min(64, -(-(2 << 30) // plane_bytes)))       # copies: the rotating footprint passes 2 GB
        path = A.akv_decode_path(B, Hq, Hkv, D, N, maxlen)      # the library's own choice for this shape
        prof_steps = 0 if path != 2 else max(10, min(steps, 50))  # second pass with events between the kernels (token-split path)
        if headline:
            R = max(R, (steps + warmup + prof_steps + 255) // 256)
        visits = (steps + warmup + prof_steps + R - 1) // R if append else 0  # times each cache copy is stepped
        log(f"[bench] cfg{cfg}: {w.name}; generated in {time.time() - t_gen:.1f}s; {R} cache copies"
            + (f", each stepped {visits} times up to context {N}" if append else ""))
        kd, vd, qd, lens_d = w.k.to(dev), w.v.to(dev), w.q.to(dev), w.lens.to(dev)
        caches = []
        for r in range(R):
            c = A.Cache.allocate(B, Hq, Hkv, D, N, dev)
            if append:
                A.akv_append(c, kd[:, :, :N - visits].contiguous(), vd[:, :, :N - visits].contiguous())
            else:
                A.akv_append(c, kd, vd, lens_d)
            caches.append(c)
        outs = [torch.empty(B, Hq, D, dtype=torch.float32, device=dev) for _ in range(R)]
        kw = dict(guard_bits=args.guard_bits, max_len=maxlen)
        clock_warmup(lambda i: A.akv_decode_attention(caches[i % R], qd, outs[i % R], **kw))

        entry = {"workload": WORKLOAD_TEXT[cfg], "B": B, "Hq": Hq, "Hkv": Hkv, "D": D, "Ncap": N,
                 "lens": lens if len(set(lens)) > 1 else lens[0], "cache_copies_rotated": R,
                 "step": "akv_append_decode_attention (append 1 token/seq + attention)" if append else "akv_decode_attention"}
        # ------------------------------------------------------------ the timed region
        if append:
            kn = [kd[:, :, N - visits + i].contiguous() for i in range(visits)]
            vn = [vd[:, :, N - visits + i].contiguous() for i in range(visits)]
            visit_of = [0] * R

            def step(i, events=None):
                r = i % R
                vi = visit_of[r]
                visit_of[r] += 1
                A.akv_append_decode_attention(caches[r], kn[vi], vn[vi], qd, outs[r], events=events, **kw)
        else:
            def step(i, events=None):
                A.akv_decode_attention(caches[i % R], qd, outs[i % R], events=events, **kw)
        e0, e1 = ev.create(2)
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
        us_step = (t1 - t0) * 1e6 / steps
        us_events = ev.elapsed_ms(e0, e1) * 1e3 / steps  # on the head-per-workgroup path: one launch per step, its average duration
        # Token-split path: the same steps once more with the library's events between its kernels.  An event costs
        # about 4.5 us of stream time, which is why these steps are not the timed ones; that cost, measured here between
        # events recorded back to back, is taken off every segment (a segment = one kernel, or the slice + selection kernels).
        seg = None
        if prof_steps:
            evs = [ev.create(A.AKV_NEVENTS) for _ in range(prof_steps)]
            for i in range(prof_steps):
                step(warmup + steps + i, evs[i])
            torch.cuda.synchronize()
            gap = event_gap_us()
            seg = [max(0.0, sum(ev.elapsed_ms(e[k], e[k + 1]) for e in evs) * 1e3 / prof_steps - gap) for k in range(A.AKV_NEVENTS - 1)]
            for e in evs:
                ev.destroy(e)
        one_kernel = path != 2
        if append:
            for c in caches:
                assert int(c.flags[0]) == 0 and int(c.flags[1]) == 0
                c.lens.fill_(N)                          # every copy now holds the workload's N tokens (extra steps of the last round aside)
        # ------------------------------------------------------------ bytes from the device counters (one untimed call)
        st = A.new_stats(dev)
        out_stats = A.akv_decode_attention(caches[0], qd, stats=st, **kw).clone()
        torch.cuda.synchronize()
        by = bytes_from_stats(st.cpu().numpy().astype(np.int64), w, lens, append, logits_in_memory=path != 3)
        entry["us_per_step"] = round(us_step, 2)
        entry["us_per_step_hip_events"] = round(us_events, 2)
        if one_kernel:
            entry["path"] = "head-per-workgroup (one kernel" + ("; logits in LDS)" if path == 3 else ")")
            entry["kernel_us"] = {"head_kernel": round(us_events, 2)}
            dom_name = f"akv::head_kernel<{Hq // Hkv}, {1024 if Hq == Hkv else 512}, false, {'true' if path == 3 else 'false'}>"
            dom_tag, dom_us, dom_bytes = "head_kernel", us_events, by["total"]
        else:
            entry["path"] = "token-split (K, slice, selection, V kernels" + ("; append kernel in front)" if append else ")")
            entry["kernel_us"] = {"append": round(seg[0], 2), "k_kernel": round(seg[1], 2), "slice_and_selection": round(seg[2], 2),
                                  "v_kernel": round(seg[3], 2),
                                  "how": f"HIP events recorded by the library between its kernels, mean over {prof_steps} steps run right "
                                         f"after the timed ones, minus the {gap:.2f} us two back-to-back events lie apart"}
            if by["k_kernel"] >= by["v_kernel"]:
                dom_name, dom_tag, dom_us, dom_bytes = f"akv::split_k_kernel<{Hq // Hkv}>", "split_k_kernel", seg[1], by["k_kernel"]
            else:
                dom_name, dom_tag, dom_us, dom_bytes = f"akv::split_v_kernel<{Hq // Hkv}, false>", "split_v_kernel", seg[3], by["v_kernel"]
            entry["kernel_frac_of_peak"] = {"k_kernel": round(by["k_kernel"] / seg[1] / 1e3 / HBM_PEAK_GBS, 4),
                                            "v_kernel": round(by["v_kernel"] / seg[3] / 1e3 / HBM_PEAK_GBS, 4)}
        entry["algorithmic_bytes"] = by
        entry["reduction_vs_fp16"] = round(1.0 - by["total"] / by["fp16"], 4)
        entry["step_GBps"] = round(by["total"] / us_step / 1e3, 1)
        entry["step_frac_of_peak"] = round(by["total"] / us_step / 1e3 / HBM_PEAK_GBS, 4)
        traffic, traffic_src = measured_traffic(dom_tag, cfg)
        roof = {"bound": "hbm", "kernel": dom_name, "achieved": round(dom_bytes / dom_us / 1e3, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(dom_bytes / dom_us / 1e3 / HBM_PEAK_GBS, 4), "traffic": traffic,
                "traffic_source": (traffic_src + " (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a plain copy; a committed "
                                   "figure, not measured in this run)") if traffic else None,
                "algorithmic_bytes_per_launch": int(dom_bytes), "avg_launch_us": round(dom_us, 2),
                "logits_bytes_counted": ("4 B per (query head, token) written by the K side and 4 B read by the V side; the mid "
                                         "step's read of the same logits is left out (served by the caches)") if path != 3 else
                                        "none: the kernel keeps its logits in LDS"}
        entry["roofline"] = roof
        log(f"[bench] cfg{cfg}: {us_step:.1f} us/step ({entry['path']}); kernels {entry['kernel_us']}; K {by['avg_bits_K']} / V "
            f"{by['avg_bits_V_rows']} bits; {by['total'] / 1e6:.1f} MB vs fp16 {by['fp16'] / 1e6:.1f} MB "
            f"(-{entry['reduction_vs_fp16']:.1%}); step {entry['step_frac_of_peak']:.1%} of peak, {dom_name} {roof['frac']:.1%}")

        extras = {}
        if not args.no_extras:
            # -------------------------------------------------------- attention only, control group, other path, fp16 kernels
            n = max(20, min(steps, 100))
            att = timed(lambda i: A.akv_decode_attention(caches[i % R], qd, outs[i % R], **kw), n)
            ctl = timed(lambda i: A.akv_decode_attention(caches[i % R], qd, outs[i % R], force_level=2, max_len=maxlen), n)
            other = None
            G = Hq // Hkv
            if G <= 4:
                other_path = 2 if one_kernel else 1
                other = timed(lambda i: A.akv_decode_attention(caches[i % R], qd, outs[i % R], path=other_path, **kw), max(5, n // 4))
            g2 = timed(lambda i: A.akv_decode_attention(caches[i % R], qd, outs[i % R], guard_bits=2, max_len=maxlen), max(5, n // 4))
            st2 = A.new_stats(dev)
            A.akv_decode_attention(caches[0], qd, guard_bits=2, max_len=maxlen, stats=st2)
            torch.cuda.synchronize()
            by2 = bytes_from_stats(st2.cpu().numpy().astype(np.int64), w, lens, False, logits_in_memory=path != 3)
            hot = timed(lambda i: A.akv_decode_attention(caches[0], qd, outs[0], **kw), n)
            keep = caches[0]
            del caches[1:]
            torch.cuda.empty_cache()
            kp = [kd] + [kd.clone() for _ in range(R - 1)]
            vp = [vd] + [vd.clone() for _ in range(R - 1)]
            if kd.shape[2] < N:                              # the fp16 kernels take [B, Hkv, Ncap, D]
                raise AssertionError("workload shorter than its capacity")
            ws16 = torch.empty(A.akv_layout_sizes(B, Hq, Hkv, D, N).fp16_workspace, dtype=torch.uint8, device=dev)
            o16 = torch.empty(B, Hq, D, dtype=torch.float32, device=dev)
            f16 = timed(lambda i: A.akv_fp16_decode_attention(kp[i % R], vp[i % R], lens_d, qd, o16, max_len=maxlen, workspace=ws16), n)
            ref16 = A.akv_fp16_decode_attention(kp[0], vp[0], lens_d, qd, max_len=maxlen, workspace=ws16).clone()
            torch.cuda.synchronize()
            dev16 = (out_stats - ref16).double()
            entry.update({
                "attention_only_us": round(att, 2), "control_group_16bit_us": round(ctl, 2), "fp16_kernel_us": round(f16, 2),
                "fp16_kernel_frac_of_peak": round(by["fp16"] / f16 / 1e3 / HBM_PEAK_GBS, 4),
                "other_path_us": None if other is None else round(other, 2),
                "guard2": {"us": round(g2, 2), "reduction_vs_fp16": round(1.0 - by2["total"] / by2["fp16"], 4),
                           "avg_bits_K": by2["avg_bits_K"], "avg_bits_V_rows": by2["avg_bits_V_rows"]},
                "one_copy_repeated_us": round(hot, 2),
                "speedup_vs_fp16_kernel": round(f16 / att, 3), "speedup_vs_control_group": round(ctl / att, 3),
                "deviation_from_fp16_attention": {"max_abs": float(dev16.abs().max()),
                                                  "rel_l2": float(dev16.norm() / ref16.double().norm())}})
            log(f"[bench] cfg{cfg}: attention only {att:.1f} us, control(16-bit) {ctl:.1f} us, fp16 kernels {f16:.1f} us "
                f"({entry['fp16_kernel_frac_of_peak']:.1%} of peak), other path {other}, guard2 {g2:.1f} us")
            if headline:                                     # the read ceiling of this device, by the library's plain streaming kernel
                sink = torch.zeros(1, dtype=torch.int32, device=dev)
                s_us = timed(lambda i: A.akv_stream_read(kp[i % R], sink), n)
                gbps = kp[0].numel() * 2 / s_us / 1e3
                extras["stream"] = {"GBps": round(gbps, 1), "frac_of_peak": round(gbps / HBM_PEAK_GBS, 4),
                                    "step_frac_of_ceiling": round(by["total"] / us_step / 1e3 / gbps, 4),
                                    "how": "akv_stream_read (16-byte non-temporal loads, four in flight per lane, 1-MB blocks dealt "
                                           "over the XCDs) over the K tensors of the rotating fp16 copies, timed like a step"}
                log(f"[bench] plain streaming read of {kp[0].numel() * 2 / 1e6:.0f} MB: {s_us:.1f} us = {gbps:.0f} GB/s")
            del kp, vp
            caches[:] = [keep]

        if not args.no_cpu_baseline:
            # -------------------------------------------------------- the CPU oracle as it stands, on a stated sample
            from oracle import akv_oracle as O
            G = Hq // Hkv
            pairs = B * Hkv
            target_tokens = (2 if headline else 0.5) * 1024 * 1024           # (query head, token) products: about 15 s / 4 s of core time
            order = [(b, h) for h in range(Hkv) for b in range(B)]           # sequences first: ragged lengths are all represented
            sample, tok = [], 0
            for b, h in order:
                sample.append((b, h))
                tok += lens[b] * G
                if tok >= target_tokens:
                    break
            full = len(sample) == pairs
            oc = O.Cache.empty(len(sample), 1, D, N)
            ks = torch.stack([w.k[b, h] for b, h in sample]).unsqueeze(1)
            vs = torch.stack([w.v[b, h] for b, h in sample]).unsqueeze(1)
            qs = torch.stack([w.q[b, h * G:(h + 1) * G] for b, h in sample])
            slens = np.array([lens[b] for b, _ in sample], np.int32)
            O.append(oc, bits(ks), bits(vs), slens - (1 if append else 0))
            ta = time.perf_counter()
            if append:
                last = torch.stack([ks[i, :, slens[i] - 1:slens[i]] for i in range(len(sample))])
                lastv = torch.stack([vs[i, :, slens[i] - 1:slens[i]] for i in range(len(sample))])
                O.append(oc, bits(last), bits(lastv))
            ref = O.decode_attention(oc, bits(qs), guard_bits=args.guard_bits, want_needV=False)
            cpu_s = time.perf_counter() - ta
            scale_up = float(sum(lens[b] for b in range(B)) * Hkv) / float(slens.sum())
            got = torch.stack([out_stats[b, h * G:(h + 1) * G] for b, h in sample]).cpu().numpy().astype(np.float64)
            err = float(np.abs(got - ref.out).max())
            rl2 = float(np.linalg.norm(got - ref.out) / np.linalg.norm(ref.out))
            entry["cpu_oracle"] = {"value": round(cpu_s * scale_up * 1e6, 1), "unit": "us/step", "cores": O.max_threads(), "kind": "oracle",
                                   "sample": ("the whole step" if full else
                                              f"{len(sample)} of the {pairs} (sequence, KV head) pairs ({int(slens.sum())} of "
                                              f"{sum(lens) * Hkv} pair-tokens), scaled to the whole step: extrapolated") +
                                             ", once, OpenMP over the pairs",
                                   "measured_seconds": round(cpu_s, 3)}
            entry["parity_vs_oracle_on_the_sample"] = {"max_abs": err, "rel_l2": rl2, "max_abs_out": float(np.abs(ref.out).max())}
            log(f"[bench] cfg{cfg}: oracle {cpu_s:.2f} s on the sample ({entry['cpu_oracle']['sample']}) -> {cpu_s * scale_up:.2f} s/step; "
                f"GPU vs oracle max-abs {err:.2e} rel-L2 {rl2:.2e}")
        del caches, kd, vd
        torch.cuda.empty_cache()
        return entry, extras

    # ---------------------------------------------------------------- all configurations; the headline one with --steps / --warmup
    t_all = time.time()
    configs = {}
    head_entry, head_extras = None, None
    for cfg in sorted(set(args.configs) | {args.headline}):
        is_head = cfg == args.headline
        entry, extras = run_config(cfg, args.steps if is_head else max(20, min(args.steps, 50)), args.warmup if is_head else 5, is_head)
        configs[f"config{cfg}"] = entry
        if is_head:
            head_entry, head_extras = entry, extras
    log(f"[bench] all configurations in {time.time() - t_all:.0f} s")

    e = head_entry
    result = {
        "metric": "decode-attention us/step + effective HBM GB/s (% of peak) vs fp16 kernel",
        "value": e["us_per_step"], "unit": "us/step", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(e["us_per_step"] / 1e3, 5), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": WORKLOAD_TEXT[args.headline], "B": e["B"], "Hq": e["Hq"], "Hkv": e["Hkv"], "D": e["D"],
                   "context": e["Ncap"], "guard_bits": args.guard_bits, "topk": 32, "cache_copies_rotated": e["cache_copies_rotated"],
                   "step": e["step"], "path": e["path"]},
        "roofline": e["roofline"],
        "step_roofline": {"algorithmic_bytes_per_step": e["algorithmic_bytes"]["total"], "GBps": e["step_GBps"],
                          "frac_of_peak": e["step_frac_of_peak"], "kernel_us": e["kernel_us"]},
        "bytes_per_step": {"alignedkv": e["algorithmic_bytes"]["total"], "fp16": e["algorithmic_bytes"]["fp16"],
                           "reduction_vs_fp16": e["reduction_vs_fp16"], "avg_bits_K": e["algorithmic_bytes"]["avg_bits_K"],
                           "avg_bits_V_rows": e["algorithmic_bytes"]["avg_bits_V_rows"]},
        "paper_context": "paper reports 25% less KV memory access and up to 1.3x attention speedup on one V100 (Llama-2-7B); "
                         "other hardware, not a target",
    }
    if "stream" in head_extras:
        result["streaming_read_ceiling"] = head_extras["stream"]
    if "fp16_kernel_us" in e:
        result["vs_fp16_kernel"] = {k: e[k] for k in ("attention_only_us", "fp16_kernel_us", "fp16_kernel_frac_of_peak",
                                                      "control_group_16bit_us", "speedup_vs_fp16_kernel", "speedup_vs_control_group",
                                                      "deviation_from_fp16_attention")}
    if "cpu_oracle" in e:
        result["cpu_baseline"] = e["cpu_oracle"]
        result["parity_vs_oracle"] = e["parity_vs_oracle_on_the_sample"]
    result["configs"] = configs

    if not args.no_extras:
        # ------------------------------------------------------------ the second workload (weight GEMV under Rule 1), briefly
        from paper_2409_16546_amd import bench_weights
        gemv = {}
        for shape in ("attn_proj", "mlp_up", "mlp_down"):
            m = bench_weights.measure(shape, 1, 200)
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

    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
