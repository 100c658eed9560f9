"""The study module (paper_2409_16546_amd/analysis.py: bits per element, relative-error statistics, other fetch
granules) against the same quantities from the CPU oracle.  The estimates that need no GPU run here on CPU tensors;
the figures that come from library calls are checked in the GPU test below."""
import numpy as np
import pytest
import torch


def bits(t):
    return np.ascontiguousarray(t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16))


def test_block_colmax_estimate_equals_the_oracles_per_block_rule(oracle):
    from paper_2409_16546_amd import analysis, workloads
    for cfg, G, guard in ((2, 1, 0), (3, 1, 1), (4, 2, 0), (5, 4, 2)):
        w = workloads.make(cfg, B=2, Hq=2 * G, Hkv=2, N=1100)
        lens = [1100, 700]
        oc = oracle.Cache.empty(2, 2, 128, 1280)
        oracle.append(oc, bits(w.k), bits(w.v), np.array(lens, np.int32))
        for block in (64, 256, 1 << 20):
            _, cnt = oracle.k_levels_per_block(oc, bits(w.q), min(block, 1280), guard)
            assert analysis.k_counts_with_block_colmax(w.k, w.q, lens, guard, block) == [int(x) for x in cnt], (cfg, block)


def test_v_granule_estimate_equals_the_oracles_on_cpu_tensors(oracle):
    from paper_2409_16546_amd import analysis, workloads
    w = workloads.make(2, B=2, Hq=4, Hkv=2, N=900)
    lens = [900, 411]
    oc = oracle.Cache.empty(2, 2, 128, 1024)
    oracle.append(oc, bits(w.k), bits(w.v), np.array(lens, np.int32))
    r = oracle.decode_attention(oc, bits(w.q))
    need = torch.from_numpy(r.needV)
    for tt, cc in analysis.V_GRANULES:
        assert analysis.v_counts_for_granule(need, lens, tt, cc) == [int(x) for x in oracle.v_granule_counts(oc, r.needV, tt, cc)]


@pytest.mark.gpu
@pytest.mark.parametrize("kw", [dict(guard_bits=0), dict(guard_bits=2), dict(force_level=1), dict(force_level=0)],
                         ids=["aligned-g0", "aligned-g2", "uniform-12", "uniform-8"])
def test_bit_width_and_relative_error_figures_against_the_oracle(oracle, kw):
    """"Experiments": bits per element and the relative error of QK^T and of the output against 16-bit reads, as the
    study module derives them from library calls, against the oracle's counts, logits, out and its fp64 fp16 attention."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2409_16546_amd import analysis, workloads, binding as A
    dev = "cuda:0"
    n = 1500
    w = workloads.make(2, B=2, Hq=4, Hkv=4, N=n)
    print(f"analysis vs oracle: cfg2 B2 H4 N{n} {kw}", flush=True)
    c = A.Cache.allocate(w.B, w.Hq, w.Hkv, w.D, 1536, dev)
    A.akv_append(c, w.k.to(dev), w.v.to(dev))
    qd = w.q.to(dev)
    dbg = A.DebugBuffers.allocate(c)
    ref = A.akv_decode_attention(c, qd, force_level=2, dbg=dbg).clone()
    ref_logits = dbg.logits[:, :, :n].clone()
    m = analysis.measure(c, qd, n, ref, ref_logits, dbg, **kw)
    oc = oracle.Cache.empty(w.B, w.Hkv, w.D, 1536)
    oracle.append(oc, bits(w.k), bits(w.v))
    r = oracle.decode_attention(oc, bits(w.q), **kw)
    r16 = oracle.decode_attention(oc, bits(w.q), force_level=2)
    kp = np.zeros((w.B, w.Hkv, 1536, w.D), np.uint16); kp[:, :, :n] = bits(w.k)
    vp = np.zeros((w.B, w.Hkv, 1536, w.D), np.uint16); vp[:, :, :n] = bits(w.v)
    ref16 = oracle.fp16_attention(kp, vp, oc.lens, bits(w.q))
    assert np.abs(r16.out - ref16).max() < 1e-12                              # the reference of the study is fp16 attention
    # bits per element: exactly the oracle's counts
    assert m["bits_k"] == analysis.bits_from_counts(r.counts[0:3])
    assert m["bits_v"] == analysis.bits_from_counts(r.counts[3:6])
    assert m["bits_v_needed"] == analysis.bits_from_counts(r.counts[6:9])
    # QK^T: the kernel's logits are the oracle's bit for bit, so are the error statistics
    lo, lo16 = r.logits[:, :, :n].astype(np.float64), r16.logits[:, :, :n].astype(np.float64)
    el = (np.abs(lo - lo16) / np.abs(lo16))[lo16 != 0]
    assert m["logits_median"] == float(np.median(el)) and m["logits_p99"] == float(np.percentile(el, 99))
    assert m["logits_zero_frac"] == float((el == 0).mean())
    # output: the kernel's fp32 sums against the oracle's fp64 ones
    eo = (np.abs(r.out - ref16) / np.abs(ref16))[ref16 != 0]
    rl2 = float(np.linalg.norm(r.out - ref16) / np.linalg.norm(ref16))
    assert abs(m["out_rel_l2"] - rl2) <= 0.02 * rl2 + 1e-6
    assert abs(m["out_median"] - float(np.median(eo))) <= 0.05 * float(np.median(eo)) + 1e-6
    assert abs(m["out_p99"] - float(np.percentile(eo, 99))) <= 0.10 * float(np.percentile(eo, 99)) + 1e-5
    # other fetch granules from the exported needs: exactly the oracle's evaluation
    if kw.get("guard_bits") == 0:
        for tt, cc in analysis.V_GRANULES:
            got = analysis.v_counts_for_granule(dbg.needV, [n] * w.B, tt, cc)
            assert got == [int(x) for x in oracle.v_granule_counts(oc, r.needV, tt, cc)], (tt, cc)
