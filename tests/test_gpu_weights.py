"""GPU parity of the precision-aligned weight GEMV (include/akw.h) against its CPU oracle on the same seeded
inputs: plane bytes, rowmax and row levels bit for bit; y within the accumulation tolerance.

Tolerance: the kernel adds K exact products in binary32 (8 rows per lane in row order, the 8 row lanes, the 8 waves,
then the K/512 slabs), the oracle in binary64.  Each binary32 addition rounds by at most 2^-24 of the running sum,
which is at most S_n = sum_k |x_k w~_kn|; a product passes through at most 8 + 3 + 8 + K/512 additions, so
|y - y_oracle| <= (19 + K/512) * 2^-24 * S_n  (2.5e-6 * S_n at K = 11008).  The test allows 1e-5 * S_n."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
TOL = 1e-5


@pytest.fixture(scope="module")
def T():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from oracle import akw_oracle
    akw_oracle.build()
    return akw_oracle


def say(msg):
    print(msg, flush=True)


def bits(t):
    return np.ascontiguousarray(t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16))


def both(T, wl, **kw):
    from paper_2409_16546_amd import binding as A
    ow = T.pack(bits(wl.W))
    gw = A.Weights.allocate(wl.K, wl.N, DEV)
    A.akw_pack(gw, wl.W.to(DEV))
    lvl = torch.full((wl.K,), 255, dtype=torch.uint8, device=DEV)
    y = A.akw_gemv(gw, wl.x.to(DEV), lvl_out=lvl, **kw)
    torch.cuda.synchronize()
    r = T.gemv(ow, bits(wl.x), **kw)
    return gw, ow, y.cpu().numpy().astype(np.float64), lvl.cpu().numpy(), r


def check(y, lvl, r, what):
    assert np.array_equal(lvl, r.lvl), f"{what}: row levels differ"
    err = np.abs(y - r.y)
    bound = TOL * r.abs_sum + 1e-30
    assert np.all(err <= bound), f"{what}: max err/bound {np.max(err / bound):.3f}"
    return float(np.max(err / (r.abs_sum + 1e-300)))


def test_pack_matches_oracle_bytes_and_unpack_is_lossless(T):
    from paper_2409_16546_amd import binding as A, workloads
    say("weights: pack edge bit patterns K=72 N=1040")
    k, _ = workloads.edge_patterns(1, 1, 585, seed=3)           # 585 * 128 = 72 * 1040 raw finite patterns
    W = k.reshape(72, 1040).contiguous()
    ow = T.pack(bits(W))
    gw = A.Weights.allocate(72, 1040, DEV)
    A.akw_pack(gw, W.to(DEV))
    torch.cuda.synchronize()
    assert np.array_equal(gw.hi.cpu().numpy(), ow.hi.reshape(-1))
    assert np.array_equal(gw.mid.cpu().numpy(), ow.mid.reshape(-1))
    assert np.array_equal(gw.lo.cpu().numpy(), ow.lo.reshape(-1))
    assert np.array_equal(gw.rowmax.cpu().numpy().view(np.uint16), ow.rowmax)
    assert np.array_equal(bits(A.akw_unpack(gw)), bits(W))


CASES = [
    # name, (K, N), B, kwargs -- several column tiles, a ragged last tile, a ragged last slab, one slab only
    ("small-one-slab", (64, 1024), 1, {}),
    ("ragged-tile-and-slab", (200, 2576), 2, {}),
    ("tiles-and-slabs", (1032, 3088), 1, {}),
    ("batch3-guard2", (512, 2064), 3, dict(guard_bits=2)),
    ("batch4", (384, 1536), 4, {}),
    ("uniform-8", (256, 1040), 2, dict(force_level=0)),
    ("uniform-12", (256, 1040), 1, dict(force_level=1)),
    ("control-16", (256, 1040), 1, dict(force_level=2)),
]


@pytest.mark.parametrize("name,shape,B,kw", CASES, ids=[c[0] for c in CASES])
def test_gemv_matches_oracle(T, name, shape, B, kw):
    from paper_2409_16546_amd import workloads
    say(f"gemv: {name} K{shape[0]} N{shape[1]} B{B} {kw}")
    wl = workloads.make_weights(shape, B, outliers=4, seed=[c[0] for c in CASES].index(name) + 1)
    _, _, y, lvl, r = both(T, wl, **kw)
    rel = check(y, lvl, r, name)
    if not kw:
        assert len(set(r.lvl.tolist())) > 1, "the case should exercise several levels"
    say(f"  levels {np.bincount(r.lvl, minlength=3).tolist()}  max err / S_n {rel:.2e}")


def test_gemv_random_shapes_and_parameters(T):
    """Seeded sweep over shapes (ragged strips and slabs, a single strip, a single slab), batch and guard bits."""
    from paper_2409_16546_amd import workloads
    rng = np.random.default_rng(424242)
    for case in range(16):
        K = int(rng.choice([8, 64, 504, 512, 520, 1000, 1536, 2056]))
        N = int(rng.choice([16, 112, 128, 144, 1024, 2064, 4112]))
        B = int(rng.integers(1, 5))
        kw = dict(guard_bits=int(rng.integers(0, 4)))
        say(f"gemv random case {case}: K{K} N{N} B{B} {kw}")
        wl = workloads.make_weights((K, N), B, outliers=int(rng.integers(0, 5)), seed=3000 + case)
        _, _, y, lvl, r = both(T, wl, **kw)
        check(y, lvl, r, f"random case {case}")


def test_gemv_zero_rows_subnormals_and_zero_activations(T):
    from paper_2409_16546_amd import workloads
    say("gemv: zero / subnormal rows, zero activations")
    wl = workloads.make_weights((128, 1024), 2, outliers=2, seed=77)
    wl.W[5] = 0
    wl.W[9] = 3e-6
    wl.W[17, ::3] = 6e-8
    wl.x[0, 11] = 0
    wl.x[1] = 0                                                  # an all-zero activation row
    _, _, y, lvl, r = both(T, wl)
    check(y, lvl, r, "edge rows")
    assert not y[1].any()


def test_gemv_is_deterministic_and_reusable(T):
    """The slabs are added in slab order by whichever workgroup finishes last: the result does not depend on timing,
    and the counters are back at zero for the next call on the same workspace."""
    from paper_2409_16546_amd import binding as A, workloads
    say("gemv: repeated calls give identical bits")
    wl = workloads.make_weights((2048, 4096), 2, seed=5)
    gw = A.Weights.allocate(wl.K, wl.N, DEV)
    A.akw_pack(gw, wl.W.to(DEV))
    x = wl.x.to(DEV)
    first = A.akw_gemv(gw, x).clone()
    for _ in range(5):
        assert torch.equal(A.akw_gemv(gw, x), first)
    torch.cuda.synchronize()


@pytest.mark.parametrize("shape", ["attn_proj", "mlp_up", "mlp_down"])
def test_full_size_projection_matrices_sampled_against_oracle(T, shape):
    """The three projection shapes of the paper's model at full size: every row level against the oracle, and y on the
    whole output (the oracle needs a few seconds per matrix)."""
    from paper_2409_16546_amd import workloads
    say(f"gemv: full size {shape}")
    wl = workloads.make_weights(shape, 1)
    _, _, y, lvl, r = both(T, wl)
    rel = check(y, lvl, r, shape)
    bits_avg = float(np.mean(8 + 4 * r.lvl.astype(np.float64)))
    say(f"  levels {np.bincount(r.lvl, minlength=3).tolist()}  average bits {bits_avg:.2f}  max err / S_n {rel:.2e}")


def test_bad_arguments_are_refused_on_the_host(T):
    from paper_2409_16546_amd import binding as A
    say("gemv errors: B out of range, guard, workspace")
    gw = A.Weights.allocate(64, 1024, DEV)
    x = torch.zeros(5, 64, dtype=torch.float16, device=DEV)
    with pytest.raises(A.AkvError) as e:
        A.akw_gemv(gw, x)
    assert e.value.status == A.AKV_EINVAL
    x = x[:1].contiguous()
    for bad in (dict(guard_bits=13), dict(force_level=3)):
        with pytest.raises(A.AkvError) as e:
            A.akw_gemv(gw, x, **bad)
        assert e.value.status == A.AKV_EINVAL
    with pytest.raises(A.AkvError) as e:
        A.akw_gemv(gw, x, workspace=torch.empty(256, dtype=torch.uint8, device=DEV))
    assert e.value.status == A.AKV_EWORKSPACE
    torch.cuda.synchronize()
