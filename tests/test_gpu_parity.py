"""GPU parity: the HIP library (through its C ABI) against the CPU oracle on the same seeded inputs.
Cache bytes, K levels, logits, score exponents, top-k, O_est, result exponents and V masks are compared
bit for bit; the attention output within max-abs 2e-3 and rel-L2 1e-3."""
import math

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(scope="module")
def T():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from oracle import akv_oracle
    akv_oracle.build()
    import akv_testlib
    return akv_testlib


def say(msg):
    print(msg, flush=True)


# ------------------------------------------------------------------------------------------ append / unpack

def test_append_bulk_matches_oracle_bytes_and_unpack_is_lossless(T):
    from paper_2409_16546_amd import workloads, binding as A
    say("append: edge bit patterns B2 Hkv3 N700 Ncap768, ragged")
    k, v = workloads.edge_patterns(2, 3, 700)
    lens = [700, 389]
    oc = T.oracle_cache(k, v, lens, 768)
    gc = T.gpu_cache(k, v, lens, 3, 768)
    torch.cuda.synchronize()
    T.assert_cache_equal(gc, oc)
    ku, vu = A.akv_unpack(gc)
    kb, vb = T.bits(ku), T.bits(vu)
    for b, n in enumerate(lens):
        assert np.array_equal(kb[b, :, :n], T.bits(k)[b, :, :n]) and np.array_equal(vb[b, :, :n], T.bits(v)[b, :, :n])
        assert not kb[b, :, n:].any() and not vb[b, :, n:].any()


def test_append_token_by_token_and_capacity_flag(T):
    from paper_2409_16546_amd import workloads, binding as A
    from oracle import akv_oracle as O
    say("append: token by token, ragged counts, overflow refusal")
    B, Hkv, D, Ncap = 3, 2, 128, 256
    k, v = workloads.edge_patterns(B, Hkv, 300, seed=11)
    oc = O.Cache.empty(B, Hkv, D, Ncap)
    gc = A.Cache.allocate(B, 2, Hkv, D, Ncap, DEV)
    pos = 0
    rng = np.random.default_rng(5)
    for step, n in enumerate([1, 1, 1, 2, 5, 1, 64, 1, 130, 1, 1]):
        n_new = rng.integers(0, n + 1, size=B).astype(np.int32) if step % 3 == 2 else np.full(B, n, np.int32)
        kn, vn = k[:, :, pos:pos + n].contiguous(), v[:, :, pos:pos + n].contiguous()
        O.append(oc, T.bits(kn), T.bits(vn), n_new)
        A.akv_append(gc, kn.to(DEV), vn.to(DEV), torch.from_numpy(n_new).to(DEV))
        pos += n
    torch.cuda.synchronize()
    T.assert_cache_equal(gc, oc)
    assert int(gc.flags.cpu()[0]) == 0
    # an append that does not fit leaves the sequence unchanged and raises the flag
    kn, vn = k[:, :, :200].contiguous(), v[:, :, :200].contiguous()
    n_new = np.array([200, 1, 0], np.int32)
    refused = O.append(oc, T.bits(kn), T.bits(vn), n_new)
    A.akv_append(gc, kn.to(DEV), vn.to(DEV), torch.from_numpy(n_new).to(DEV))
    torch.cuda.synchronize()
    assert refused >= 1 and int(gc.flags.cpu()[0]) == refused
    T.assert_cache_equal(gc, oc)
    # the synchronising debug helper says the same on the host, before anything is enqueued
    A.akv_check_capacity_sync(gc, Ncap - int(oc.lens.max()))
    with pytest.raises(A.AkvError) as e:
        A.akv_check_capacity_sync(gc, Ncap - int(oc.lens.max()) + 1)
    assert e.value.status == A.AKV_ECAPACITY and "capacity" in str(e.value)


def test_append_prefill_after_unaligned_lengths(T):
    """A long append onto sequences that end inside a K block: a partly covered first block, whole blocks through the
    transposing path, a partly covered last block, ragged counts, K_colmax merged with what was there."""
    from paper_2409_16546_amd import workloads, binding as A
    from oracle import akv_oracle as O
    say("append: prefill of up to 900 tokens after lengths 100 / 255 / 256 / 513")
    B, Hkv, Ncap = 4, 2, 1536
    k, v = workloads.edge_patterns(B, Hkv, 1500, seed=23)
    lens0 = [100, 255, 256, 513]
    oc = T.oracle_cache(k[:, :, :513], v[:, :, :513], lens0, Ncap)
    gc = T.gpu_cache(k[:, :, :513], v[:, :, :513], lens0, 2, Ncap)
    n_new = np.array([900, 770, 512, 300], np.int32)
    kn, vn = k[:, :, 600:1500].contiguous(), v[:, :, 600:1500].contiguous()
    assert O.append(oc, T.bits(kn), T.bits(vn), n_new) == 0
    A.akv_append(gc, kn.to(DEV), vn.to(DEV), torch.from_numpy(n_new).to(DEV))
    torch.cuda.synchronize()
    T.assert_cache_equal(gc, oc)
    assert not gc.flags.cpu().any()


# ------------------------------------------------------------------------------------------ decode parity

CASES = [
    # name, cfg, overrides, lens (None = full), params
    ("cfg1-small", 1, dict(B=1, Hq=4, Hkv=4, N=1024), None, {}),
    ("cfg2-ragged", 2, dict(B=3, Hq=4, Hkv=4, N=1500), [1500, 1237, 513], {}),
    ("cfg2-guard2", 2, dict(B=2, Hq=2, Hkv=2, N=1100), [1100, 777], dict(guard_bits=2)),
    ("cfg3-token-outliers", 3, dict(B=2, Hq=4, Hkv=4, N=2304), [2304, 2303], {}),
    ("cfg4-gqa4", 4, dict(B=2, Hq=8, Hkv=2, N=2600), [2600, 1999], {}),
    ("cfg4-gqa2-topk8", 4, dict(B=1, Hq=4, Hkv=2, N=900), None, dict(topk=8)),
    ("cfg4-gqa8", 4, dict(B=1, Hq=8, Hkv=1, N=700), None, {}),
    ("cfg5-student-t", 5, dict(B=3, Hq=8, Hkv=2, N=3000), None, {}),
    ("cfg1-force0", 1, dict(B=1, Hq=2, Hkv=2, N=600), None, dict(force_level=0)),
    ("cfg1-force1", 1, dict(B=1, Hq=2, Hkv=2, N=600), None, dict(force_level=1)),
    ("cfg1-force2-control", 1, dict(B=1, Hq=2, Hkv=2, N=600), None, dict(force_level=2)),
    ("cfg2-scale", 2, dict(B=1, Hq=2, Hkv=2, N=520), None, dict(scale=0.05)),
    # several blocks per wave and several chunks of the mid step on the head-per-workgroup kernel; 4096 is the
    # longest sequence whose logits it keeps in registers
    ("cfg2-mha-long", 2, dict(B=3, Hq=2, Hkv=2, N=5000), [5000, 4097, 4096], {}),
    ("cfg4-gqa2-long", 4, dict(B=2, Hq=4, Hkv=2, N=4300), [4300, 2048], {}),
    # groups of four and eight heads over several rounds of the V kernel's shared mode, with a ragged last round
    ("cfg4-gqa8-long", 4, dict(B=2, Hq=16, Hkv=2, N=2300), [2300, 1029], {}),
    ("cfg2-gqa4-guard1", 2, dict(B=2, Hq=8, Hkv=2, N=3100), [3100, 65], dict(guard_bits=1)),
]


@pytest.mark.parametrize("path", [1, 2], ids=["head-path", "split-path"])
@pytest.mark.parametrize("name,cfg,over,lens,params", CASES, ids=[c[0] for c in CASES])
def test_decode_matches_oracle(T, name, cfg, over, lens, params, path):
    from paper_2409_16546_amd import workloads
    w = workloads.make(cfg, **over)
    if path == 1 and w.Hq // w.Hkv > 4:
        pytest.skip("the head-per-workgroup kernel covers Hq/Hkv <= 4")
    say(f"decode parity: {name} cfg={cfg} {over} lens={lens} params={params} path={path}")
    lens = w.lens.tolist() if lens is None else lens
    gc, oc, out, dbg, r = T.run_both(w.k, w.v, w.q, lens, path=path, **params)
    T.assert_cache_equal(gc, oc)
    err, rl2 = T.assert_decode_equal(out, dbg, r, lens, w.Hq // w.Hkv, name, scale=params.get("scale", 0.0))
    say(f"  max-abs {err:.2e} rel-L2 {rl2:.2e} levels K {np.bincount(r.lvlK.ravel(), minlength=3)} "
        f"V rows {r.counts[3:6] // 128}")


def test_decode_random_shapes_lengths_and_parameters(T):
    """Seeded sweep over what the targeted cases fix by hand: group size, head and batch counts, capacity, ragged lengths
    (empty, one token, block and chunk edges, full), guard bits, top-k, scale, both paths, adaptive and append-then-decode."""
    from paper_2409_16546_amd import workloads, binding as A
    from oracle import akv_oracle as O
    rng = np.random.default_rng(20240916)
    edges = [0, 1, 2, 15, 16, 17, 255, 256, 257, 511, 512, 513, 1023, 1024, 1025]
    for case in range(24):
        G = int(rng.choice([1, 1, 2, 4, 8]))
        Hkv, B = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        Ncap = int(rng.choice([256, 512, 1024, 1280, 2304]))
        lens = [int(rng.choice(edges)) if rng.random() < 0.5 else int(rng.integers(0, Ncap + 1)) for _ in range(B)]
        lens = [min(n, Ncap) for n in lens]
        params = dict(guard_bits=int(rng.integers(0, 3)), topk=int(rng.choice([1, 5, 32, 64])))
        if rng.random() < 0.3:
            params["scale"] = float(rng.choice([0.02, 0.3]))
        path = 2 if G > 4 else int(rng.integers(1, 3))
        cfg = int(rng.choice([1, 2, 3, 4]))
        w = workloads.make(cfg, B=B, Hq=Hkv * G, Hkv=Hkv, N=max(max(lens), 1), seed=1000 + case)
        say(f"random case {case}: cfg{cfg} G{G} Hkv{Hkv} B{B} Ncap{Ncap} lens{lens} {params} path{path}")
        gc, oc, out, dbg, r = T.run_both(w.k, w.v, w.q, lens, Ncap=Ncap, path=path, **params)
        T.assert_cache_equal(gc, oc)
        T.assert_decode_equal(out, dbg, r, lens, G, f"random case {case}", scale=params.get("scale", 0.0))
        # one more token where there is room, appended and attended to in one call
        room = [n < Ncap for n in lens]
        if any(room):
            gen = torch.Generator().manual_seed(case)
            kn = torch.randn(B, Hkv, 1, 128, generator=gen).half()
            vn = torch.randn(B, Hkv, 1, 128, generator=gen).half()
            O.append(oc, T.bits(kn), T.bits(vn), np.array([1] * B, np.int32))          # full sequences are refused on both sides
            out2 = A.akv_append_decode_attention(gc, kn.to(DEV), vn.to(DEV), w.q.to(DEV), dbg=dbg, path=path, **params)
            torch.cuda.synchronize()
            r2 = O.decode_attention(oc, T.bits(w.q), **params)
            T.assert_cache_equal(gc, oc)
            T.assert_decode_equal(out2, dbg, r2, oc.lens.tolist(), G, f"random case {case} + 1 token", scale=params.get("scale", 0.0))


@pytest.mark.parametrize("B,Hkv,G", [(3, 7, 1), (5, 5, 2), (9, 2, 4)])
def test_head_path_with_pair_counts_that_do_not_divide_by_eight(T, B, Hkv, G):
    """The head-per-workgroup kernel pads its grid to a multiple of eight workgroups and gives every XCD a run of
    consecutive (sequence, head) pairs: 21, 25 and 18 pairs leave padding workgroups and uneven runs; ragged lengths
    (with an empty and a one-token sequence) make some waves' ranges of V batches empty.  Then one token more, fused."""
    from paper_2409_16546_amd import workloads, binding as A
    from oracle import akv_oracle as O
    say(f"head path, {B * Hkv} pairs (B{B} Hkv{Hkv} G{G}), ragged")
    Ncap = 768
    rng = np.random.default_rng(100 * B + Hkv)
    lens = [int(x) for x in rng.integers(2, Ncap, size=B)]
    lens[0], lens[1] = 0, 1
    w = workloads.make(2, B=B, Hq=Hkv * G, Hkv=Hkv, N=max(lens), seed=4242 + B)
    gc, oc, out, dbg, r = T.run_both(w.k, w.v, w.q, lens, Ncap=Ncap, path=1)
    T.assert_cache_equal(gc, oc)
    T.assert_decode_equal(out, dbg, r, lens, G, f"{B * Hkv} pairs")
    gen = torch.Generator().manual_seed(B)
    kn = torch.randn(B, Hkv, 1, 128, generator=gen).half()
    vn = torch.randn(B, Hkv, 1, 128, generator=gen).half()
    O.append(oc, T.bits(kn), T.bits(vn), np.array([1] * B, np.int32))
    out2 = A.akv_append_decode_attention(gc, kn.to(DEV), vn.to(DEV), w.q.to(DEV), dbg=dbg, path=1)
    torch.cuda.synchronize()
    r2 = O.decode_attention(oc, T.bits(w.q))
    T.assert_cache_equal(gc, oc)
    T.assert_decode_equal(out2, dbg, r2, oc.lens.tolist(), G, f"{B * Hkv} pairs + 1 token")


def test_decode_edge_lengths_empty_one_and_smallest_capacity(T):
    from paper_2409_16546_amd import workloads
    say("decode parity: lens 0 / 1 / 255 / 256, Ncap 256")
    w = workloads.make(2, B=4, Hq=4, Hkv=2, N=256)
    lens = [0, 1, 255, 256]
    for path in (1, 2):
        gc, oc, out, dbg, r = T.run_both(w.k, w.v, w.q, lens, Ncap=256, path=path)
        T.assert_decode_equal(out, dbg, r, lens, 2, f"edge-lens path {path}")


def test_decode_raw_bit_patterns_with_zeros_and_subnormals(T):
    from paper_2409_16546_amd import workloads
    say("decode parity: K, V of random finite bit patterns (zeros, subnormals, 65504)")
    k, v = workloads.edge_patterns(1, 2, 640, seed=3)
    k = (k.float() * 2.0 ** -12).to(torch.float16)     # keep logits finite in fp32 and fp16 ranges sane
    v = (v.float().clamp(-100, 100)).to(torch.float16)
    q = workloads.make(1, B=1, Hq=2, Hkv=2, N=256).q
    lens = [640]
    for path in (1, 2):
        gc, oc, out, dbg, r = T.run_both(k, v, q, lens, path=path)
        T.assert_cache_equal(gc, oc)
        T.assert_decode_equal(out, dbg, r, lens, 1, f"raw-bits path {path}")


@pytest.mark.parametrize("path", [1, 2], ids=["head-path", "split-path"])
def test_append_decode_in_one_call_matches_oracle_step_by_step(T, path):
    """Several decode steps in a row (append one token, attend), also into a sequence that is full."""
    from paper_2409_16546_amd import workloads, binding as A
    from oracle import akv_oracle as O
    say(f"append + decode in one call, 6 steps, path {path}")
    B, Hq, Hkv, Ncap = 3, 4, 2, 512
    w = workloads.make(2, B=B, Hq=Hq, Hkv=Hkv, N=512)
    lens0 = [250, 506, 0]                       # sequence 1 fills up after 6 steps; sequence 2 starts empty
    oc = T.oracle_cache(w.k[:, :, :506], w.v[:, :, :506], lens0, Ncap)
    gc = T.gpu_cache(w.k[:, :, :506], w.v[:, :, :506], lens0, Hq, Ncap)
    gen = torch.Generator().manual_seed(9)
    refused = 0
    for step in range(8):
        kn = (torch.randn(B, Hkv, 1, 128, generator=gen) * 3).to(torch.float16)
        vn = torch.randn(B, Hkv, 1, 128, generator=gen).to(torch.float16)
        q = torch.randn(B, Hq, 128, generator=gen).to(torch.float16)
        refused += O.append(oc, T.bits(kn), T.bits(vn))
        r = O.decode_attention(oc, T.bits(q))
        dbg = A.DebugBuffers.allocate(gc)
        out = A.akv_append_decode_attention(gc, kn.to(DEV), vn.to(DEV), q.to(DEV), dbg=dbg, path=path)
        torch.cuda.synchronize()
        T.assert_cache_equal(gc, oc)
        T.assert_decode_equal(out, dbg, r, oc.lens.tolist(), Hq // Hkv, f"step {step}")
    assert refused == 2 and int(gc.flags.cpu()[0]) == 2
    assert not gc.flags.cpu()[A.AKV_NFLAGS:].any()          # the arrival counters are back at zero


def test_decode_is_deterministic_and_fp16_output(T):
    from paper_2409_16546_amd import workloads, binding as A
    say("decode: run twice, bitwise equal; fp16 output = rounded fp32 output")
    w = workloads.make(2, B=2, Hq=4, Hkv=4, N=1024)
    gc = T.gpu_cache(w.k, w.v, w.lens.tolist(), w.Hq, 1024)
    q = w.q.to(DEV)
    for path in (1, 2):
        o1 = A.akv_decode_attention(gc, q, path=path).clone()
        o2 = A.akv_decode_attention(gc, q, path=path).clone()
        o16 = A.akv_decode_attention(gc, q, out=torch.empty_like(q), path=path)
        torch.cuda.synchronize()
        assert torch.equal(o1, o2)
        assert torch.equal(o16, o1.to(torch.float16))


@pytest.mark.parametrize("Hq,Hkv", [(2, 2), (8, 2), (8, 1)], ids=["mha", "gqa4", "gqa8"])
def test_max_len_hint_gives_the_same_result(T, Hq, Hkv):
    from paper_2409_16546_amd import workloads, binding as A
    say(f"decode: max_len hint bounds the launch, same result (Hq {Hq}, Hkv {Hkv})")
    w = workloads.make(2, B=2, Hq=Hq, Hkv=Hkv, N=700)
    gc = T.gpu_cache(w.k, w.v, [700, 300], w.Hq, 4096)
    q = w.q.to(DEV)
    for path in ((1, 2) if Hq // Hkv <= 4 else (2,)):
        o1 = A.akv_decode_attention(gc, q, path=path).clone()
        o2 = A.akv_decode_attention(gc, q, max_len=700, path=path).clone()
        torch.cuda.synchronize()
        assert torch.equal(o1, o2)


def test_max_len_hint_below_a_length_attends_the_first_max_len_tokens_on_both_paths(T):
    """A bound below a sequence's length: both paths attend to the first max_len tokens of that sequence (the oracle on
    the truncated lengths), count the sequence in flags[AKV_FLAG_MAXLEN], and leave nothing stale for the next call.
    With an append in the same call the bound is on the lengths after the append: one too small leaves the new token
    out of the attention (it is stored all the same)."""
    from paper_2409_16546_amd import workloads, binding as A
    from oracle import akv_oracle as O
    say("decode: max_len below a length, both paths, then a correct call; fp16 kernels the same")
    w = workloads.make(2, B=2, Hq=4, Hkv=2, N=3000)
    lens = [3000, 1500]
    q = w.q.to(DEV)
    oc_cut = T.oracle_cache(w.k, w.v, lens, 4096)
    oc_cut.lens[:] = 1100                  # K_colmax stays the running maximum over everything that was stored
    r_cut = O.decode_attention(oc_cut, T.bits(w.q))
    for path in (1, 2):
        gc = T.gpu_cache(w.k, w.v, lens, w.Hq, 4096)
        ref = A.akv_decode_attention(gc, q, path=path).clone()
        dbg = A.DebugBuffers.allocate(gc)
        short = A.akv_decode_attention(gc, q, max_len=1100, path=path, dbg=dbg).clone()
        again = A.akv_decode_attention(gc, q, path=path).clone()
        torch.cuda.synchronize()
        T.assert_decode_equal(short, dbg, r_cut, [1100, 1100], 2, f"max_len 1100 path {path}")
        assert torch.equal(ref, again)
        assert int(gc.flags.cpu()[A.AKV_FLAG_MAXLEN]) == 2          # both sequences exceeded the bound, one call
        # append + decode with the bound of the lengths BEFORE the append: the new token is stored, not attended
        gen = torch.Generator().manual_seed(3)
        kn = torch.randn(2, 2, 1, 128, generator=gen).half()
        vn = torch.randn(2, 2, 1, 128, generator=gen).half()
        gc2 = T.gpu_cache(w.k[:, :, :1100], w.v[:, :, :1100], [1100, 1100], w.Hq, 4096)
        dbg2 = A.DebugBuffers.allocate(gc2)
        out2 = A.akv_append_decode_attention(gc2, kn.to(DEV), vn.to(DEV), q, max_len=1100, path=path, dbg=dbg2)
        torch.cuda.synchronize()
        oc2 = T.oracle_cache(w.k[:, :, :1100], w.v[:, :, :1100], [1100, 1100], 4096)
        O.append(oc2, T.bits(kn), T.bits(vn))
        T.assert_cache_equal(gc2, oc2)
        assert gc2.lens.cpu().tolist() == [1101, 1101] and int(gc2.flags.cpu()[A.AKV_FLAG_MAXLEN]) == 2
        oc2.lens[:] = 1100                 # attended: the first 1100 tokens, K_colmax counting the new token
        r2 = O.decode_attention(oc2, T.bits(w.q))
        T.assert_decode_equal(out2, dbg2, r2, [1100, 1100], 2, f"append with max_len of before, path {path}")
    gc = T.gpu_cache(w.k, w.v, lens, w.Hq, 4096)
    ku, vu = A.akv_unpack(gc)
    lens_d = torch.tensor(lens, dtype=torch.int32, device=DEV)
    f_ref = A.akv_fp16_decode_attention(ku, vu, lens_d, q).clone()
    f_short = A.akv_fp16_decode_attention(ku, vu, lens_d, q, max_len=1100).clone()
    f_again = A.akv_fp16_decode_attention(ku, vu, lens_d, q).clone()
    torch.cuda.synchronize()
    assert torch.equal(f_ref, f_again)
    # the fp16 kernels with the short hint attend to exactly the first 1100 tokens
    f_cut = A.akv_fp16_decode_attention(ku, vu, torch.tensor([1100, 1100], dtype=torch.int32, device=DEV), q)
    torch.cuda.synchronize()
    assert torch.equal(f_short, f_cut)


def test_stream_read_runs_and_checks_its_arguments(T):
    from paper_2409_16546_amd import binding as A
    say("stream read: 64 MiB + ragged tail, misaligned size refused")
    buf = torch.zeros((64 << 20) + 48, dtype=torch.uint8, device=DEV)
    sink = torch.zeros(1, dtype=torch.int32, device=DEV)
    A.akv_stream_read(buf, sink)
    A.akv_stream_read(buf[:16], sink)
    torch.cuda.synchronize()
    assert int(sink.cpu()[0]) == 0
    with pytest.raises(A.AkvError) as e:
        A.akv_stream_read(buf[:24], sink)
    assert e.value.status == A.AKV_EINVAL


def test_bad_arguments_are_refused_on_the_host(T):
    from paper_2409_16546_amd import binding as A
    say("errors: bad shape / params / workspace -> status codes, nothing launched")
    with pytest.raises(A.AkvError) as e:
        A.akv_layout_sizes(1, 4, 4, 64, 256)
    assert e.value.status == A.AKV_EINVAL
    with pytest.raises(A.AkvError):
        A.akv_layout_sizes(1, 4, 4, 128, 300)
    gc = A.Cache.allocate(1, 2, 2, 128, 256, DEV)
    q = torch.zeros(1, 2, 128, dtype=torch.float16, device=DEV)
    for bad in (dict(topk=65), dict(guard_bits=13), dict(force_level=3), dict(max_len=257), dict(path=3)):
        with pytest.raises(A.AkvError) as e:
            A.akv_decode_attention(gc, q, **bad)
        assert e.value.status == A.AKV_EINVAL
    with pytest.raises(A.AkvError) as e:
        A.akv_decode_attention(gc, q, workspace=torch.empty(256, dtype=torch.uint8, device=DEV))
    assert e.value.status == A.AKV_EWORKSPACE
    torch.cuda.synchronize()


# ------------------------------------------------------------------------------------------ fp16 yardstick

@pytest.mark.parametrize("G", [1, 4])
def test_fp16_yardstick_matches_textbook_attention(T, G):
    from paper_2409_16546_amd import workloads, binding as A
    from oracle import akv_oracle as O
    say(f"fp16 yardstick: G={G} ragged, against fp64 textbook attention")
    w = workloads.make(2, B=3, Hq=2 * G, Hkv=2, N=1300)
    lens = np.array([1300, 511, 0], np.int32)
    Ncap = 1536
    kp = torch.zeros(3, 2, Ncap, 128, dtype=torch.float16)
    vp = torch.zeros_like(kp)
    kp[:, :, :1300], vp[:, :, :1300] = w.k, w.v
    out = A.akv_fp16_decode_attention(kp.to(DEV), vp.to(DEV), torch.from_numpy(lens).to(DEV), w.q.to(DEV))
    torch.cuda.synchronize()
    ref = O.fp16_attention(T.bits(kp), T.bits(vp), lens, T.bits(w.q))
    got = out.cpu().numpy().astype(np.float64)
    assert np.abs(got - ref).max() <= T.MAX_ABS and T.rel_l2(got, ref) <= T.REL_L2
    assert not got[2].any()


@pytest.mark.parametrize("G", [1, 2])
def test_fp16_yardstick_head_per_workgroup_variant(T, G):
    from paper_2409_16546_amd import workloads, binding as A
    from oracle import akv_oracle as O
    say(f"fp16 yardstick, many heads (one workgroup per head): G={G}, ragged lengths incl. 0 and 1")
    B, Hkv, N, Ncap = 24, 8, 700, 768
    w = workloads.make(2, B=B, Hq=Hkv * G, Hkv=Hkv, N=N)
    rng = np.random.default_rng(3)
    lens = rng.integers(1, N + 1, size=B).astype(np.int32)
    lens[0], lens[1], lens[2] = N, 0, 1
    kp = torch.zeros(B, Hkv, Ncap, 128, dtype=torch.float16)
    vp = torch.zeros_like(kp)
    kp[:, :, :N], vp[:, :, :N] = w.k, w.v
    out = A.akv_fp16_decode_attention(kp.to(DEV), vp.to(DEV), torch.from_numpy(lens).to(DEV), w.q.to(DEV))
    torch.cuda.synchronize()
    ref = O.fp16_attention(T.bits(kp), T.bits(vp), lens, T.bits(w.q))
    got = out.cpu().numpy().astype(np.float64)
    assert np.abs(got - ref).max() <= T.MAX_ABS and T.rel_l2(got, ref) <= T.REL_L2
    assert not got[1].any()


# ------------------------------------------------------------------------------------------ full bench size, sampled

@pytest.mark.parametrize("G", [1, 2])
def test_append_decode_in_one_call_across_block_chunk_and_prefetch_boundaries(T, G):
    """The one-call decode step on the head-per-workgroup kernel while the lengths cross 256 (new K block), 512 (the
    rows its waves fetch ahead), 1024, 2048 and 4096 (one chunk of the mid step for 512 / 1024 threads)."""
    from paper_2409_16546_amd import workloads, binding as A
    from oracle import akv_oracle as O
    lens0 = [254, 510, 1022, 2046, 4094]
    B, Hkv, Ncap = len(lens0), 2, 4352
    Hq = Hkv * G
    say(f"append + decode in one call across boundaries, G={G}, lens {lens0}")
    w = workloads.make(2, B=B, Hq=Hq, Hkv=Hkv, N=4094)
    oc = T.oracle_cache(w.k, w.v, lens0, Ncap)
    gc = T.gpu_cache(w.k, w.v, lens0, Hq, Ncap)
    gen = torch.Generator().manual_seed(11 + G)
    for step in range(4):
        kn = (torch.randn(B, Hkv, 1, 128, generator=gen) * 2).to(torch.float16)
        vn = torch.randn(B, Hkv, 1, 128, generator=gen).to(torch.float16)
        q = torch.randn(B, Hq, 128, generator=gen).to(torch.float16)
        assert O.append(oc, T.bits(kn), T.bits(vn)) == 0
        r = O.decode_attention(oc, T.bits(q))
        dbg = A.DebugBuffers.allocate(gc)
        out = A.akv_append_decode_attention(gc, kn.to(DEV), vn.to(DEV), q.to(DEV), dbg=dbg, path=1)
        torch.cuda.synchronize()
        T.assert_cache_equal(gc, oc)
        T.assert_decode_equal(out, dbg, r, oc.lens.tolist(), G, f"G={G} step {step}")
        # the same step without the exports (the kernel variant that is timed)
        gc2_out = A.akv_decode_attention(gc, q.to(DEV), path=1)
        torch.cuda.synchronize()
        assert torch.equal(gc2_out, out)


@pytest.mark.parametrize("cfg,path", [(1, 0), (2, 0), (3, 0), (3, 2), (4, 0), (5, 0)],
                         ids=["cfg1", "cfg2", "cfg3", "cfg3-split-path", "cfg4", "cfg5"])
def test_full_size_configurations_against_the_oracle_everywhere(T, cfg, path):
    """The five benchmark configurations at full size, in the launch configuration the benchmark times (max_len = the
    longest sequence, the library's choice of path, no exports in the timed call; config 3 with its last token appended
    inside the step -- the library takes the head-per-workgroup kernel there: fused append, two rounds of pairs, two
    blocks per wave, logits in LDS -- and also on the token-split kernels).  The oracle runs the
    WHOLE configuration: every plane byte, every lvlK, logit, score exponent, selection, O_est, result exponent, needV
    and appliedV of every (sequence, head) is compared bit for bit, every output within the tolerance, and the device
    counters with the oracle's counts."""
    from paper_2409_16546_amd import workloads, binding as A
    from oracle import akv_oracle as O
    w = workloads.make(cfg)
    G, N = w.Hq // w.Hkv, w.Ncap
    lens = w.lens.tolist()
    say(f"full size: cfg{cfg} B{w.B} H{w.Hq}/{w.Hkv} Ncap{N} lens {lens[:4]}... path {path}")
    q = w.q.to(DEV)
    stats = A.new_stats(DEV)
    if w.append_last:
        before = [n - 1 for n in lens]
        gc = T.gpu_cache(w.k, w.v, before, w.Hq, N)
        kn = torch.stack([w.k[b, :, lens[b] - 1:lens[b]] for b in range(w.B)]).contiguous()
        vn = torch.stack([w.v[b, :, lens[b] - 1:lens[b]] for b in range(w.B)]).contiguous()
        dbg = A.DebugBuffers.allocate(gc)
        out = A.akv_append_decode_attention(gc, kn.to(DEV), vn.to(DEV), q, max_len=max(lens), dbg=dbg, path=path, stats=stats)
    else:
        gc = T.gpu_cache(w.k, w.v, lens, w.Hq, N)
        dbg = A.DebugBuffers.allocate(gc)
        out = A.akv_decode_attention(gc, q, max_len=max(lens), dbg=dbg, path=path, stats=stats)
    plain = A.akv_decode_attention(gc, q, max_len=max(lens), path=path)           # the launch without exports
    torch.cuda.synchronize()
    assert torch.equal(plain, out)                                                  # exports do not change the result
    assert gc.lens.cpu().tolist() == lens and not gc.flags.cpu()[:A.AKV_NFLAGS].any()
    say("  GPU done; oracle on the whole configuration ...")
    oc = T.oracle_cache(w.k, w.v, lens, N)
    r = O.decode_attention(oc, T.bits(w.q))
    say("  oracle done; comparing")
    T.assert_cache_equal(gc, oc)
    err, rl2 = T.assert_decode_equal(out, dbg, r, lens, G, f"cfg{cfg}")
    T.assert_stats_equal(stats, r, f"cfg{cfg}")
    bits_k = (8 * r.counts[0] + 12 * r.counts[1] + 16 * r.counts[2]) / r.counts[0:3].sum()
    bits_v = (8 * r.counts[3] + 12 * r.counts[4] + 16 * r.counts[5]) / r.counts[3:6].sum()
    say(f"  cfg{cfg}: max-abs {err:.2e} rel-L2 {rl2:.2e}; bits read per element K {bits_k:.2f} V {bits_v:.2f}")
    if cfg == 2:   # the other path gives the same masks; its sums run in another order
        out_other = A.akv_decode_attention(gc, q, max_len=max(lens), path=2)
        torch.cuda.synchronize()
        assert (plain - out_other).abs().max().item() <= 1e-4
