"""CPU pins of the weight-GEMV oracle ("Precision Alignment in Uncertainty Calculation": A W = A (W_quant +- dW);
"A Framework for Aligning Precision": Rule 1, and the bit width of an addend is the bit width of its weight).
Every part is checked against something other than itself: numpy bit slices, read-outs written out by hand,
brute force over every level assignment, the error bound the rule promises, numpy's fp64 product."""
import itertools
import math

import numpy as np
import pytest

MBITS = (2, 6, 10)      # mantissa bits kept at level 0 / 1 / 2
RBITS = (8, 12, 16)     # bits read at level 0 / 1 / 2


@pytest.fixture(scope="module")
def wo():
    from oracle import akw_oracle
    akw_oracle.build()
    return akw_oracle


def f16bits(x):
    return np.ascontiguousarray(np.asarray(x, np.float16)).view(np.uint16)


def exp2floor(x):
    m, e = math.frexp(abs(x))
    return e - 1


def tiny(rng, B, K, N, spread=6):
    x = (rng.normal(size=(B, K)) * np.exp2(rng.integers(-spread, spread + 1, size=(B, K)))).astype(np.float16)
    W = (rng.normal(size=(K, N)) * np.exp2(rng.integers(-spread, spread + 1, size=(K, 1)))).astype(np.float16)
    return x, W


def test_pack_unpack_every_pattern_and_planes_against_numpy_bit_slices(wo):
    # every fp16 pattern once, shuffled so that neighbouring columns differ in every plane
    h = np.ascontiguousarray(np.random.default_rng(0).permutation(65536).astype(np.uint16).reshape(64, 1024))
    w = wo.pack(h)
    assert np.array_equal(wo.unpack(w), h)
    assert np.array_equal(w.hi, (h >> 8).astype(np.uint8))
    mid, lo = (h >> 4) & 15, h & 15
    assert np.array_equal(w.mid, (mid[:, 0::2] | (mid[:, 1::2] << 4)).astype(np.uint8))
    assert np.array_equal(w.lo, (lo[:, 0::2] | (lo[:, 1::2] << 4)).astype(np.uint8))
    assert np.array_equal(w.rowmax, (h & 0x7FFF).max(axis=1))


def test_rowmax_is_the_largest_magnitude_of_the_row(wo):
    rng = np.random.default_rng(1)
    W = rng.normal(size=(37, 50)).astype(np.float16)
    W[3] = 0
    W[5, 7] = np.float16(-9.5)                                        # a negative entry is the largest
    w = wo.pack(f16bits(W))
    assert np.array_equal(w.rowmax.view(np.float16), np.abs(W).max(axis=1))


# "Dynamic Quantization": the first 8 / first 12 / all 16 bits, the rest filled with 100...; written out by hand
HAND = [
    # pattern, level, value read
    (0x3C00, 2, 1.0), (0x3C00, 1, 1.0 + 2.0 ** -7), (0x3C00, 0, 1.0 + 2.0 ** -3),      # 1.0: below the kept bits sits 100...
    (0x3FFF, 1, 1.0 + 1016 / 1024), (0x3FFF, 0, 1.0 + 896 / 1024),                     # 1.999: (m & ~15) | 8, (m & ~255) | 128
    (0xC2A5, 0, -(2.0 + 2.0 * 640 / 1024)), (0xC2A5, 1, -(2.0 + 2.0 * 680 / 1024)),    # negative, exponent 1
    (0x0013, 0, 128 * 2.0 ** -24), (0x0013, 1, 24 * 2.0 ** -24),                       # subnormal: same rule on the bits
]


@pytest.mark.parametrize("h,level,value", HAND)
def test_read_outs_written_out_by_hand(wo, h, level, value):
    assert wo.half_to_double(wo.read_at_level(h, level)) == value


@pytest.mark.parametrize("guard", [0, 1, 2])
@pytest.mark.parametrize("B", [1, 2])
def test_level_rule_is_the_cheapest_assignment_that_aligns_every_addend(wo, guard, B):
    """Rule 1: every addend x_k * W_kn keeps at least the last place of the coarsest addend (the one of the largest
    magnitude, bounded through rowmax); among all assignments of 8 / 12 / 16 bits to the rows that do so for every
    activation row, the rule's is the one that reads the fewest bits."""
    rng = np.random.default_rng(100 + guard + 7 * B)
    K, N = 6, 8
    for _ in range(40):
        x, W = tiny(rng, B, K, N)
        w = wo.pack(f16bits(W))
        lvl = wo.levels(f16bits(x), w.rowmax, guard_bits=guard)
        rowmax = np.maximum(np.abs(W).max(axis=1).astype(np.float64), 2.0 ** -14)
        best, best_cost = None, None
        for assign in itertools.product(range(3), repeat=K):
            ok = True
            for b in range(B):
                P = [float(x[b, k]) * rowmax[k] for k in range(K)]
                es = [exp2floor(p) for p in P if p != 0]
                if not es:
                    continue
                target = max(es) - 10 - guard
                for k in range(K):
                    if P[k] == 0 or assign[k] == 2:
                        continue
                    if exp2floor(P[k]) - MBITS[assign[k]] > target:
                        ok = False
            cost = sum(RBITS[a] for a in assign)
            if ok and (best_cost is None or cost < best_cost):
                best, best_cost = assign, cost
        assert tuple(int(v) for v in lvl) == best


@pytest.mark.parametrize("guard", [0, 2])
def test_rule_keeps_the_result_within_the_aligned_place(wo, guard):
    """Reading a row at fewer bits moves each of its addends by at most half of the last kept place, which the rule
    keeps at or below the last place of the coarsest addend, 2^(emax - 10 - guard): the result moves by at most that
    times the number of rows read below 16 bits."""
    rng = np.random.default_rng(200 + guard)
    B, K, N = 2, 96, 40
    for _ in range(5):
        x, W = tiny(rng, B, K, N, spread=5)
        w = wo.pack(f16bits(W))
        r = wo.gemv(w, f16bits(x), guard_bits=guard)
        assert len(set(r.lvl.tolist())) > 1
        exact = x.astype(np.float64) @ W.astype(np.float64)
        rowmax = np.maximum(np.abs(W).max(axis=1).astype(np.float64), 2.0 ** -14)
        ntrunc = int(np.sum(r.lvl < 2))
        for b in range(B):
            P = np.abs(x[b].astype(np.float64)) * rowmax
            emax = max(exp2floor(p) for p in P if p != 0)
            bound = ntrunc * 2.0 ** (emax - 10 - guard)
            assert np.all(np.abs(r.y[b] - exact[b]) <= bound + 1e-12 * np.abs(exact[b]).max())


def test_all_16_bit_reads_reproduce_the_fp64_product(wo):
    rng = np.random.default_rng(300)
    x, W = tiny(rng, 3, 200, 64, spread=3)
    w = wo.pack(f16bits(W))
    r = wo.gemv(w, f16bits(x), force_level=2)
    assert np.all(r.lvl == 2)
    exact = x.astype(np.float64) @ W.astype(np.float64)
    scale = np.abs(x.astype(np.float64)) @ np.abs(W.astype(np.float64))
    assert np.all(np.abs(r.y - exact) <= 1e-13 * scale)               # both are fp64 sums of exact products
    assert np.allclose(r.abs_sum, scale, rtol=1e-13)


def test_uniform_truncation_is_the_forced_level(wo):
    rng = np.random.default_rng(301)
    x, W = tiny(rng, 1, 50, 32, spread=2)
    bits = f16bits(W)
    w = wo.pack(bits)
    for level, mask, fill in ((0, 0xFF00, 0x0080), (1, 0xFFF0, 0x0008)):
        r = wo.gemv(w, f16bits(x), force_level=level)
        Wt = ((bits & mask) | fill).view(np.float16).astype(np.float64)
        assert np.all(r.lvl == level)
        assert np.allclose(r.y, x.astype(np.float64) @ Wt, rtol=0, atol=1e-12 * np.abs(r.abs_sum).max())


def test_rule_invariances(wo):
    rng = np.random.default_rng(302)
    x, W = tiny(rng, 2, 128, 16, spread=3)
    w = wo.pack(f16bits(W))
    base = wo.levels(f16bits(x), w.rowmax)
    assert 0 < np.count_nonzero(base < 2) < base.size
    # scaling the activations by a power of two changes no level
    for j in (-3, 2):
        assert np.array_equal(wo.levels(f16bits(x * np.float16(2.0 ** j)), w.rowmax), base)
    # moving a power of two from a row of W into its activation changes no level and no result
    s = np.exp2(rng.integers(-2, 3, size=128)).astype(np.float16)
    w2 = wo.pack(f16bits(W * s[:, None]))
    assert np.array_equal(wo.levels(f16bits(x / s), w2.rowmax), base)
    assert np.array_equal(wo.gemv(w2, f16bits(x / s)).y, wo.gemv(w, f16bits(x)).y)
    # more guard bits never lower a level, and enough of them read everything
    prev = base
    for guard in (1, 2, 3, 12):
        cur = wo.levels(f16bits(x), w.rowmax, guard_bits=guard)
        assert np.all(cur >= prev)
        prev = cur
    assert np.all(prev == 2)
    # several activation rows: a row of W is read once, at the largest of their needs
    each = [wo.levels(f16bits(x[b:b + 1]), w.rowmax) for b in range(2)]
    assert np.array_equal(base, np.maximum(each[0], each[1]))


def test_zero_and_subnormal_rows_and_zero_activations(wo):
    rng = np.random.default_rng(303)
    x, W = tiny(rng, 1, 64, 16, spread=1)
    W[5] = 0                        # all-zero row: bounded by the smallest normal exponent
    W[9] = np.float16(3e-6)         # subnormal row
    x[0, 11] = 0                    # the addends of this row are exactly zero
    w = wo.pack(f16bits(W))
    r = wo.gemv(w, f16bits(x))
    assert r.lvl[5] == 0 and r.lvl[9] == 0 and r.lvl[11] == 0
    # an all-zero activation row reads every row at 8 bits and gives zeros
    z = wo.gemv(w, f16bits(np.zeros((1, 64), np.float16)))
    assert np.all(z.lvl == 0) and not z.y.any()


def test_a_subnormal_row_counts_at_the_smallest_normal_exponent(wo):
    """The places of a subnormal fp16 are those of the exponent 2^-14: a row whose largest entry is subnormal is
    treated like a row whose largest entry is 2^-14.  Levels written out by hand: with x = 1 everywhere the coarsest
    addend is row 2 (2^-10); rows 0 and 1 sit 4 exponents below and need 10 - 4 = 6 mantissa bits, the first 12 bits."""
    W = np.zeros((3, 4), np.float16)
    W[0, 1] = 2.0 ** -14
    W[1, 2] = 2.0 ** -20
    W[2, 0] = 2.0 ** -10
    w = wo.pack(f16bits(W))
    assert wo.levels(f16bits(np.ones((1, 3), np.float16)), w.rowmax).tolist() == [1, 1, 2]


def test_bad_shapes_are_refused(wo):
    with pytest.raises(ValueError):
        wo.pack(np.zeros((4, 7), np.uint16))
