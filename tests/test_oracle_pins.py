"""CPU pins of the oracle: every part is checked against something other than itself --
numpy's own fp16, exhaustive enumeration, brute force over every precision choice,
the numerical error bound the rule promises, exact sorting, textbook fp64 attention.
Citations name the paper's sections."""
import itertools
import math
import os
import re
from fractions import Fraction

import numpy as np
import pytest
import torch

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_facts.txt")
MBITS = (2, 6, 10)      # mantissa bits kept at level 0 / 1 / 2
RBITS = (8, 12, 16)     # bits read at level 0 / 1 / 2


def paper_facts():
    facts = {}
    for line in open(GOLD):
        line = line.split("#")[0].strip()
        if line:
            k, v = [s.strip() for s in line.split("=")]
            facts[k] = v
    return facts


def finite_patterns():
    h = np.arange(65536, dtype=np.uint32)
    return h[(h & 0x7C00) != 0x7C00].astype(np.uint16)


def fill_cache(oracle, k16, v16, Ncap=None, lens=None):
    """k16, v16: uint16 [B, Hkv, N, D]; appended in one call (or ragged with lens)."""
    B, Hkv, N, D = k16.shape
    Ncap = Ncap or ((N + 255) // 256) * 256
    c = oracle.Cache.empty(B, Hkv, D, Ncap)
    n_new = None if lens is None else np.asarray(lens, np.int32)
    assert oracle.append(c, np.ascontiguousarray(k16), np.ascontiguousarray(v16), n_new) == 0
    return c


def f16bits(x):
    return np.ascontiguousarray(np.asarray(x, np.float16)).view(np.uint16)


# ----------------------------------------------------------------------------------------------
# fp16 format and conversions ("Precision Alignment in Floating-Point Addition": 1 / 5 / 10 bits)
# ----------------------------------------------------------------------------------------------

def test_paper_format_facts_are_what_the_oracle_uses(oracle):
    f = paper_facts()
    assert int(f["fp16_sign_bits"]) + int(f["fp16_exponent_bits"]) + int(f["fp16_mantissa_bits"]) == 16
    assert (int(f["read_bits_least"]), int(f["read_bits_less"]), int(f["read_bits_important"])) == RBITS
    # bits read minus sign and exponent = mantissa bits kept
    hdr = int(f["fp16_sign_bits"]) + int(f["fp16_exponent_bits"])
    assert tuple(r - hdr for r in RBITS) == MBITS
    # the fill is a one followed by zeros, in both truncated widths
    assert f["fill_pattern"].startswith("100")
    L = oracle.lib()
    assert L.akvo_read_at_level(0x0000, 0) == 0x0080 and L.akvo_read_at_level(0xFFFF, 0) == 0xFF80
    assert L.akvo_read_at_level(0x0000, 1) == 0x0008 and L.akvo_read_at_level(0xFFFF, 1) == 0xFFF8
    assert int(f["head_dim"]) == 128


def test_half_to_double_matches_numpy_on_every_pattern(oracle):
    L = oracle.lib()
    h = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    ref = h.view(np.float16).astype(np.float64)
    got = np.array([L.akvo_half_to_double(int(x)) for x in h])
    fin = np.isfinite(ref)
    assert np.array_equal(got[fin], ref[fin])
    assert np.array_equal(np.isnan(got), np.isnan(ref)) and np.array_equal(np.isinf(got), np.isinf(ref))
    assert np.array_equal(np.signbit(got[fin]), np.signbit(ref[fin]))


# ----------------------------------------------------------------------------------------------
# truncation + fill ("Dynamic Quantization")
# ----------------------------------------------------------------------------------------------

def test_truncation_error_is_half_a_kept_ulp_on_every_finite_pattern(oracle):
    L = oracle.lib()
    h = finite_patterns()
    x = h.view(np.float16).astype(np.float64)
    e = np.maximum((h >> 10) & 31, 1).astype(np.int64) - 15          # exponent whose places the number has
    for level in (0, 1, 2):
        r = np.array([L.akvo_read_at_level(int(p), level) for p in h], dtype=np.uint16)
        xr = r.view(np.float16).astype(np.float64)
        assert np.all(np.isfinite(xr))                                 # never Inf / NaN
        assert np.array_equal(r >> (16 - RBITS[level]), h >> (16 - RBITS[level]))   # the bits read are kept
        if level == 2:
            assert np.array_equal(r, h)
        else:
            bound = np.ldexp(1.0, e - MBITS[level] - 1)
            assert np.all(np.abs(xr - x) <= bound)
            assert np.any(np.abs(xr - x) == bound)                    # and the bound is attained


def test_fill_100_minimises_the_worst_case_error_over_every_fill():
    # brute force over every fill pattern of the dropped bits, every value of the dropped bits
    for nd in (4, 8):
        worst = [max(abs(fill - low) for low in range(1 << nd)) for fill in range(1 << nd)]
        best = min(worst)
        assert worst[1 << (nd - 1)] == best                           # 100...0 is optimal
        assert [f for f in range(1 << nd) if worst[f] == best] == [(1 << (nd - 1)) - 1, 1 << (nd - 1)]


# ----------------------------------------------------------------------------------------------
# uncertainty calculus and the alignment criterion ("Precision Alignment in Uncertainty Calculation")
# ----------------------------------------------------------------------------------------------

def test_uncertainty_rules_hold_on_intervals():
    rng = np.random.default_rng(0)
    for _ in range(2000):
        s, x, y = rng.normal(size=3) * 10
        dx, dy = np.abs(rng.normal(size=2))
        for sx in (-1, 1):
            for sy in (-1, 1):
                # s (x +- dx) = sx +- s dx
                assert abs(s * (x + sx * dx) - s * x) <= abs(s) * dx * (1 + 1e-12)
                # (x +- dx) + (y +- dy) = (x + y) +- (dx + dy)
                assert abs((x + sx * dx) + (y + sy * dy) - (x + y)) <= (dx + dy) * (1 + 1e-12) + 1e-300


def test_equal_uncertainties_minimise_the_sum_at_fixed_bit_budget():
    # cost ~ -log2(dx) - log2(dy) fixed  <=>  bx + by fixed; dx + dy = 2^-bx + 2^-by is minimal at bx = by
    for budget in range(2, 41, 2):
        sums = {bx: Fraction(1, 2 ** bx) + Fraction(1, 2 ** (budget - bx)) for bx in range(budget + 1)}
        assert min(sums, key=sums.get) == budget // 2
        assert all(sums[budget // 2] < v for b, v in sums.items() if b != budget // 2)


def test_digits_below_the_coarser_addend_barely_move_an_fp16_sum():
    # "Precision Alignment in Floating-Point Addition": digits of the smaller addend that have no
    # counterpart in the larger addend are wasted -- changing them moves RN16(x + y) by <= 1 ulp.
    rng = np.random.default_rng(1)
    for gap in range(1, 11):
        ex, ey = 20, 20 - gap
        mx = rng.integers(0, 1024, 256).astype(np.uint16)
        my = rng.integers(0, 1024, 256).astype(np.uint16)
        x = ((ex << 10) | mx).astype(np.uint16).view(np.float16)
        y0 = ((ey << 10) | my).astype(np.uint16)
        base = (x + y0.view(np.float16)).view(np.uint16).astype(np.int64)
        for low in range(1 << gap):                                   # every setting of the wasted digits
            y = ((y0 & ~np.uint16((1 << gap) - 1)) | np.uint16(low)).view(np.float16)
            s = (x + y).view(np.uint16).astype(np.int64)
            assert np.all(np.abs(s - base) <= 1)


# ----------------------------------------------------------------------------------------------
# storage: planes, K_colmax ("Dynamic Quantization", "Quantization of K-Cache")
# ----------------------------------------------------------------------------------------------

def test_pack_unpack_every_pattern_and_planes_against_numpy_bit_slices(oracle):
    h = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    rng = np.random.default_rng(2)
    k = rng.permutation(h).reshape(1, 1, 512, 128)
    v = rng.permutation(h).reshape(1, 1, 512, 128)
    c = fill_cache(oracle, k, v)
    ku, vu = oracle.unpack(c)
    assert np.array_equal(ku, k) and np.array_equal(vu, v)            # lossless
    kb = k.reshape(2, 256, 128).transpose(0, 2, 1)                    # [blk][d][j]
    assert np.array_equal(c.k_hi[0, 0], (kb >> 8).astype(np.uint8))
    for plane, sh in ((c.k_mid, 4), (c.k_lo, 0)):
        nib = ((kb >> sh) & 15).astype(np.uint8)
        assert np.array_equal(plane[0, 0], nib[..., 0::2] | (nib[..., 1::2] << 4))
    assert np.array_equal(c.v_hi[0, 0], (v[0, 0] >> 8).astype(np.uint8))
    for plane, sh in ((c.v_mid, 4), (c.v_lo, 0)):
        nib = ((v[0, 0] >> sh) & 15).astype(np.uint8)
        assert np.array_equal(plane[0, 0], nib[..., 0::2] | (nib[..., 1::2] << 4))
    assert c.lens[0] == 512


def test_colmax_is_the_running_column_maximum_of_abs_k(oracle):
    rng = np.random.default_rng(3)
    B, H, N, D = 2, 3, 300, 128
    k = (rng.normal(size=(B, H, N, D)) * np.exp(rng.normal(size=(1, H, 1, D)) * 3)).astype(np.float16)
    v = rng.normal(size=(B, H, N, D)).astype(np.float16)
    c = oracle.Cache.empty(B, H, D, 512)
    done = 0
    for n in (1, 7, 255, 37):                                          # appended in ragged pieces
        oracle.append(c, f16bits(k[:, :, done:done + n]), f16bits(v[:, :, done:done + n]))
        done += n
        ref = np.abs(k[:, :, :done]).max(axis=2)
        assert np.array_equal(c.colmax.view(np.float16), ref)
    assert np.all(c.lens == N)
    ku, vu = oracle.unpack(c)
    assert np.array_equal(ku[:, :, :N], f16bits(k)) and np.array_equal(vu[:, :, :N], f16bits(v))
    assert not ku[:, :, N:].any() and not vu[:, :, N:].any()          # untouched slots stay zero


def test_append_respects_capacity_and_per_sequence_counts(oracle):
    rng = np.random.default_rng(4)
    c = oracle.Cache.empty(2, 1, 128, 256)
    k = f16bits(rng.normal(size=(2, 1, 200, 128)))
    assert oracle.append(c, k, k, np.array([200, 100], np.int32)) == 0
    assert list(c.lens) == [200, 100]
    before = [x.copy() for x in c.planes()] + [c.colmax.copy()]
    assert oracle.append(c, k[:, :, :100].copy(), k[:, :, :100].copy()) == 1   # sequence 0 would overflow
    assert list(c.lens) == [200, 200]
    for x, y in zip(before, list(c.planes()) + [c.colmax]):
        assert np.array_equal(x[0], y[0])                              # sequence 0 untouched


# ----------------------------------------------------------------------------------------------
# K rule (Rule 1) -- brute force over every level assignment, error bound, invariances
# ----------------------------------------------------------------------------------------------

def exp2floor(x):
    """floor(log2 |x|) of a nonzero python float, exactly."""
    m, e = math.frexp(abs(x))
    return e - 1


def tiny_case(rng, G, N, D, spread=6.0):
    q = (rng.normal(size=(1, G, D)) * np.exp2(rng.integers(-spread, spread + 1, size=(1, G, D)))).astype(np.float16)
    k = (rng.normal(size=(1, 1, N, D)) * np.exp2(rng.integers(-spread, spread + 1, size=(1, 1, 1, D)))).astype(np.float16)
    v = (rng.normal(size=(1, 1, N, D)) * np.exp2(rng.integers(-spread, spread + 1, size=(1, 1, N, 1)))).astype(np.float16)
    return q, k, v


@pytest.mark.parametrize("guard", [0, 1, 2])
@pytest.mark.parametrize("G", [1, 2])
def test_k_rule_is_the_cheapest_assignment_that_aligns_every_addend(oracle, guard, G):
    rng = np.random.default_rng(10 + guard + 7 * G)
    D, N = 6, 9
    for _ in range(40):
        q, k, v = tiny_case(rng, G, N, D)
        c = fill_cache(oracle, f16bits(k), f16bits(v))
        r = oracle.decode_attention(c, f16bits(q), guard_bits=guard)
        colmax = np.maximum(np.abs(k[0, 0]).max(axis=0).astype(np.float64), 2.0 ** -14)
        best, best_cost = None, None
        for assign in itertools.product(range(3), repeat=D):          # every precision choice
            ok = True
            for g in range(G):
                P = [float(q[0, g, d]) * colmax[d] for d in range(D)]
                es = [exp2floor(p) for p in P if p != 0]
                if not es:
                    continue
                target = max(es) - 10 - guard                          # last place of the coarsest addend
                for d in range(D):
                    if P[d] == 0 or assign[d] == 2:
                        continue
                    if exp2floor(P[d]) - MBITS[assign[d]] > target:   # last place kept by this choice
                        ok = False
            cost = sum(RBITS[a] for a in assign)
            if ok and (best_cost is None or cost < best_cost):
                best, best_cost = assign, cost
        assert tuple(int(x) for x in r.lvlK[0, 0]) == best


@pytest.mark.parametrize("guard", [0, 2])
def test_k_rule_keeps_the_logit_error_within_the_aligned_place(oracle, guard):
    rng = np.random.default_rng(20 + guard)
    G, N, D = 2, 64, 128
    for _ in range(5):
        q, k, v = tiny_case(rng, G, N, D, spread=5)
        c = fill_cache(oracle, f16bits(k), f16bits(v))
        r = oracle.decode_attention(c, f16bits(q), guard_bits=guard)
        lvl = r.lvlK[0, 0]
        assert len(set(lvl.tolist())) > 1                              # the case exercises several levels
        colmax = np.maximum(np.abs(k[0, 0]).max(axis=0).astype(np.float64), 2.0 ** -14)
        exact = q[0].astype(np.float64) @ k[0, 0].astype(np.float64).T       # [G, N]
        for g in range(G):
            P = np.abs(q[0, g].astype(np.float64)) * colmax
            emax = max(exp2floor(p) for p in P if p != 0)
            ntrunc = int(np.sum(lvl < 2))
            bound = ntrunc * 2.0 ** (emax - 10 - guard)
            err = np.abs(r.logits[0, g, :N].astype(np.float64) - exact[g])
            fp32_slack = 128 * 2.0 ** -24 * np.abs(exact[g]).max() + 1e-30
            assert np.all(err <= bound + fp32_slack)


def test_k_rule_invariances(oracle):
    rng = np.random.default_rng(30)
    G, N, D = 2, 16, 128
    q, k, v = tiny_case(rng, G, N, D, spread=3)
    base = oracle.decode_attention(fill_cache(oracle, f16bits(k), f16bits(v)), f16bits(q)).lvlK
    # scaling q by a power of two changes no level
    for j in (-3, 2):
        r = oracle.decode_attention(fill_cache(oracle, f16bits(k), f16bits(v)), f16bits(q * np.float16(2.0 ** j)))
        assert np.array_equal(r.lvlK, base)
    # moving a power of two from a K column into q changes no level
    s = np.exp2(rng.integers(-2, 3, size=D)).astype(np.float16)
    r = oracle.decode_attention(fill_cache(oracle, f16bits(k * s), f16bits(v)), f16bits(q / s))
    assert np.array_equal(r.lvlK, base)
    # more guard bits never lower a level; the control group reads everything at 16 bits
    prev = base
    for guard in (1, 2, 3, 12):
        cur = oracle.decode_attention(fill_cache(oracle, f16bits(k), f16bits(v)), f16bits(q), guard_bits=guard).lvlK
        assert np.all(cur >= prev)
        prev = cur
    assert np.all(prev == 2)
    r = oracle.decode_attention(fill_cache(oracle, f16bits(k), f16bits(v)), f16bits(q), force_level=2)
    assert np.all(r.lvlK == 2) and np.all(r.appliedV[0, 0, :N] == 2)


def test_k_rule_zero_and_subnormal_columns(oracle):
    rng = np.random.default_rng(31)
    q, k, v = tiny_case(rng, 1, 8, 128, spread=1)
    k[..., 5] = 0                      # all-zero column: bounded by the smallest normal exponent
    k[..., 9] = np.float16(3e-6)       # subnormal column
    q[..., 11] = 0                     # zero query channel: the addend is exactly zero
    r = oracle.decode_attention(fill_cache(oracle, f16bits(k), f16bits(v)), f16bits(q))
    assert r.lvlK[0, 0, 5] == 0 and r.lvlK[0, 0, 9] == 0 and r.lvlK[0, 0, 11] == 0
    exact = q[0].astype(np.float64) @ k[0, 0].astype(np.float64).T
    P = np.abs(q[0, 0].astype(np.float64)) * np.maximum(np.abs(k[0, 0]).max(axis=0).astype(np.float64), 2.0 ** -14)
    bound = 128 * 2.0 ** (max(exp2floor(p) for p in P if p != 0) - 10)
    assert np.all(np.abs(r.logits[0, 0, :8] - exact[0]) <= bound)


def test_logits_match_a_float32_numpy_accumulation_in_channel_order(oracle):
    rng = np.random.default_rng(32)
    G, N, D = 2, 300, 128
    q, k, v = tiny_case(rng, G, N, D, spread=4)
    c = fill_cache(oracle, f16bits(k), f16bits(v))
    r = oracle.decode_attention(c, f16bits(q))
    kb = f16bits(k)[0, 0].astype(np.uint16)                            # [N, D]
    lvl = r.lvlK[0, 0]
    kq = np.where(lvl == 2, kb, np.where(lvl == 1, (kb & 0xFFF0) | 0x0008, (kb & 0xFF00) | 0x0080)).astype(np.uint16)
    kq = kq.view(np.float16).astype(np.float32)
    for g in range(G):
        acc = np.zeros(N, np.float32)
        for d in range(D):
            acc = acc + np.float32(q[0, g, d]) * kq[:, d]
        assert np.array_equal(acc, r.logits[0, g, :N])


# ----------------------------------------------------------------------------------------------
# score exponents and the approximate top-k ("Quantization of V-Cache")
# ----------------------------------------------------------------------------------------------

def test_score_exponents_bracket_the_true_weights_and_ignore_a_common_shift(oracle):
    rng = np.random.default_rng(40)
    G, N, D = 1, 200, 128
    q, k, v = tiny_case(rng, G, N, D, spread=2)
    r = oracle.decode_attention(fill_cache(oracle, f16bits(k), f16bits(v)), f16bits(q), force_level=2)
    l = r.logits[0, 0, :N].astype(np.float64)
    x = (l - l.max()) / math.sqrt(128) * math.log2(math.e)
    a = r.a[0, 0, :N].astype(np.int64)
    assert a.max() == 0 and a.min() >= -64
    far = np.abs(x - np.round(x)) > 1e-4                               # away from bucket edges
    assert np.array_equal(a[far], np.maximum(np.floor(x[far]), -64).astype(np.int64))
    # a constant added to every logit (here: an extra channel pair that contributes the same to all
    # tokens) leaves the exponents unchanged -- softmax shift invariance
    k2 = k.copy(); q2 = q.copy()
    k2[..., 0] = np.float16(1.0); q2[..., 0] = np.float16(8.0)
    k3 = k2.copy(); q3 = q2.copy(); q3[..., 0] = np.float16(-16.0)
    r2 = oracle.decode_attention(fill_cache(oracle, f16bits(k2), f16bits(v)), f16bits(q2), force_level=2)
    r3 = oracle.decode_attention(fill_cache(oracle, f16bits(k3), f16bits(v)), f16bits(q3), force_level=2)
    x2 = (r2.logits[0, 0, :N].astype(np.float64) - float(r2.logits[0, 0, :N].max())) / math.sqrt(128) * math.log2(math.e)
    clear = np.abs(x2 - np.round(x2)) > 1e-3                           # the shift only moves rounding errors
    assert clear.mean() > 0.9
    assert np.array_equal(r2.a[0, 0, :N][clear], r3.a[0, 0, :N][clear])


@pytest.mark.parametrize("topk", [1, 4, 32])
def test_topk_against_an_exact_sort(oracle, topk):
    rng = np.random.default_rng(41 + topk)
    for N in (3, 40, 500):
        q, k, v = tiny_case(rng, 2, N, 128, spread=1)
        q = (q.astype(np.float32) * 0.3).astype(np.float16)            # flatter softmax: crowded buckets
        r = oracle.decode_attention(fill_cache(oracle, f16bits(k), f16bits(v)), f16bits(q), topk=topk)
        for g in range(2):
            kk = min(topk, N)
            sel = r.sel[0, g]
            chosen = sel[sel >= 0]
            assert len(chosen) == kk and np.all(np.diff(chosen) > 0)   # exactly k', ascending, distinct
            assert np.all(sel[kk:] == -1)
            a = r.a[0, g, :N].astype(np.int64)
            cut = a[chosen].min()                                       # bucket that was cut
            assert set(np.flatnonzero(a > cut)) <= set(chosen)          # every bucket above the cut is taken whole
            rest = np.setdiff1d(np.arange(N), chosen)
            if len(rest):
                assert a[rest].max() <= cut                             # nothing unselected outranks the cut
                in_cut_sel = chosen[a[chosen] == cut]
                in_cut_rest = rest[a[rest] == cut]
                if len(in_cut_rest):
                    assert in_cut_sel.max() < in_cut_rest.min()         # ties are taken by position
            exact = np.argsort(-r.logits[0, g, :N], kind="stable")[:kk]
            missed = np.setdiff1d(exact, chosen)
            assert np.all(a[missed] == cut)                              # only the cut bucket is approximate


def test_oest_is_the_weighted_sum_of_the_selected_full_precision_rows(oracle):
    rng = np.random.default_rng(45)
    G, N = 2, 120
    q, k, v = tiny_case(rng, G, N, 128, spread=2)
    r = oracle.decode_attention(fill_cache(oracle, f16bits(k), f16bits(v)), f16bits(q), topk=8)
    for g in range(G):
        sel = r.sel[0, g]
        l = r.logits[0, g, :N].astype(np.float64)
        x = (l - l.max()) / math.sqrt(128) * math.log2(math.e)
        a = np.maximum(np.floor(x), -64)
        phat = (1 + (x - np.floor(x))) * np.exp2(a)                     # piecewise-linear 2^x
        ref = phat[sel] @ v[0, 0, sel].astype(np.float64)
        scale = np.abs(phat[sel, None] * v[0, 0, sel].astype(np.float64)).sum(axis=0)
        assert np.all(np.abs(r.oest[0, g] - ref) <= 1e-5 * scale + 1e-30)
        assert np.all(phat >= np.exp2(x) * (1 - 1e-6)) and np.all(phat <= np.exp2(x) * 1.0616)   # chord of 2^x


# ----------------------------------------------------------------------------------------------
# V rule (Rule 2)
# ----------------------------------------------------------------------------------------------

@pytest.mark.parametrize("guard", [0, 1, 2])
@pytest.mark.parametrize("G", [1, 2])
def test_v_rule_is_the_cheapest_choice_that_aligns_every_addend_to_the_result(oracle, guard, G):
    rng = np.random.default_rng(50 + guard + 5 * G)
    D, N = 6, 5
    for it in range(60):
        q, k, v = tiny_case(rng, G, N, D, spread=4)
        if it >= 40:                                                    # zeros and subnormals in V
            v = (v.astype(np.float32) * 2.0 ** -17).astype(np.float16)
            v[0, 0, rng.integers(N), rng.integers(D)] = 0
            q = (q.astype(np.float32) * 0.25).astype(np.float16)
        c = fill_cache(oracle, f16bits(k), f16bits(v))
        r = oracle.decode_attention(c, f16bits(q), guard_bits=guard, topk=2)
        Ahat = r.a[0, :, :N].astype(np.int64).max(axis=0)               # heads sharing the KV head
        E = np.array([[exp2floor(float(r.oest[0, g, d])) if r.oest[0, g, d] != 0 else -127 for d in range(D)]
                      for g in range(G)])
        Ehat = E.min(axis=0)
        assert np.array_equal(r.Ehat[0, 0].astype(np.int64), Ehat)
        for t in range(N):
            for d in range(D):
                ev = max(exp2floor(float(v[0, 0, t, d])) if v[0, 0, t, d] != 0 else -99, -14)   # places of v
                tau = int(Ahat[t]) + ev                                  # exponent of the addend weight * v
                target = int(Ehat[d]) - 10 - guard                      # last place of the result
                feas = [lvl for lvl in range(3) if lvl == 2 or tau - MBITS[lvl] <= target]
                assert r.needV[0, 0, t, d] == min(feas)                 # cheapest feasible of all three choices
            assert r.appliedV[0, 0, t] == r.needV[0, 0, t].max()       # fetch granule = one token row


@pytest.mark.parametrize("guard", [0, 2])
def test_v_rule_keeps_the_output_error_within_the_aligned_place(oracle, guard):
    rng = np.random.default_rng(60 + guard)
    G, N, D = 2, 400, 128
    for _ in range(4):
        q, k, v = tiny_case(rng, G, N, D, spread=3)
        c = fill_cache(oracle, f16bits(k), f16bits(v))
        r = oracle.decode_attention(c, f16bits(q), guard_bits=guard)
        ap = r.appliedV[0, 0, :N]
        assert (ap < 2).any() and (ap > 0).any()
        vb = f16bits(v)[0, 0]
        vq = np.where(ap[:, None] == 2, vb, np.where(ap[:, None] == 1, (vb & 0xFFF0) | 8, (vb & 0xFF00) | 0x80))
        dv = vq.astype(np.uint16).view(np.float16).astype(np.float64) - v[0, 0].astype(np.float64)
        for g in range(G):
            l = r.logits[0, g, :N].astype(np.float64)
            w = np.exp2((l - l.max()) / math.sqrt(128) * math.log2(math.e))     # unnormalised weights
            err = np.abs(w @ dv)
            bound = np.sum(ap < 2) * np.exp2(r.Ehat[0, 0].astype(np.float64) - 10 - guard)
            assert np.all(err <= bound * (1 + 1e-5))


def test_v_rule_invariances_and_zero_result(oracle):
    rng = np.random.default_rng(70)
    G, N = 1, 300
    q, k, v = tiny_case(rng, G, N, 128, spread=3)
    base = oracle.decode_attention(fill_cache(oracle, f16bits(k), f16bits(v)), f16bits(q))
    for j in (-4, 3):                                                   # V times a power of two: same masks
        r = oracle.decode_attention(fill_cache(oracle, f16bits(k), f16bits(v * np.float16(2.0 ** j))), f16bits(q))
        assert np.array_equal(r.needV, base.needV) and np.array_equal(r.appliedV, base.appliedV)
        assert np.array_equal(r.Ehat, base.Ehat + j)
    prev = base.needV
    for guard in (1, 2, 4):
        cur = oracle.decode_attention(fill_cache(oracle, f16bits(k), f16bits(v)), f16bits(q), guard_bits=guard).needV
        assert np.all(cur >= prev)
        prev = cur
    v0 = v.copy(); v0[..., 17] = 0                                      # a result that is exactly zero
    r = oracle.decode_attention(fill_cache(oracle, f16bits(k), f16bits(v0)), f16bits(q))
    assert r.oest[0, 0, 17] == 0 and r.Ehat[0, 0, 17] == -127 and np.all(r.needV[0, 0, :N, 17] == 2)


# ----------------------------------------------------------------------------------------------
# values: the control group is textbook attention ("Runtime of AlignedKV")
# ----------------------------------------------------------------------------------------------

def torch_attention(q, k, v, lens, G):
    out = np.zeros(q.shape, np.float64)
    for b in range(q.shape[0]):
        n = int(lens[b])
        if n == 0:
            continue
        kk = torch.from_numpy(k[b, :, :n].astype(np.float64)).repeat_interleave(G, dim=0)
        vv = torch.from_numpy(v[b, :, :n].astype(np.float64)).repeat_interleave(G, dim=0)
        qq = torch.from_numpy(q[b].astype(np.float64))
        s = torch.softmax(torch.einsum("hd,htd->ht", qq, kk) / math.sqrt(q.shape[-1]), dim=-1)
        out[b] = torch.einsum("ht,htd->hd", s, vv).numpy()
    return out


@pytest.mark.parametrize("G", [1, 4])
def test_all_16_bit_reads_reproduce_textbook_fp64_attention(oracle, G):
    rng = np.random.default_rng(80 + G)
    B, Hkv, N, D = 3, 2, 333, 128
    q = rng.normal(size=(B, Hkv * G, D)).astype(np.float16)
    k = (rng.normal(size=(B, Hkv, N, D)) * np.exp(rng.normal(size=(1, Hkv, 1, D)))).astype(np.float16)
    v = rng.normal(size=(B, Hkv, N, D)).astype(np.float16)
    lens = np.array([333, 1, 0], np.int32)
    c = fill_cache(oracle, f16bits(k), f16bits(v), lens=lens)
    ref = torch_attention(q, k, v, lens, G)
    r = oracle.decode_attention(c, f16bits(q), force_level=2)
    assert np.abs(r.out - ref).max() < 1e-12
    assert not r.out[2].any()                                            # empty sequence -> zeros
    kp = np.zeros((B, Hkv, 512, D), np.float16); kp[:, :, :N] = k
    vp = np.zeros((B, Hkv, 512, D), np.float16); vp[:, :, :N] = v
    assert np.abs(oracle.fp16_attention(f16bits(kp), f16bits(vp), lens, f16bits(q)) - ref).max() < 1e-12
    # adaptive reads stay close to it, and guard bits bring them closer
    e0 = np.abs(oracle.decode_attention(c, f16bits(q)).out - ref).max()
    e4 = np.abs(oracle.decode_attention(c, f16bits(q), guard_bits=4).out - ref).max()
    assert e0 < 5e-2 and e4 <= e0


def read_bits_np(h, lvl):
    """fp16 bit patterns h read at levels lvl (broadcast): the kept bits, then 100... ("Dynamic Quantization")."""
    h = h.astype(np.uint16)
    r = np.where(lvl == 2, h, np.where(lvl == 1, (h & 0xFFF0) | 0x0008, (h & 0xFF00) | 0x0080)).astype(np.uint16)
    return r.view(np.float16).astype(np.float64)


def mixed_level_case(seed, G, N):
    """Data on which Rule 1 leaves K columns, and Rule 2 leaves V rows, at all three levels: channel scales over a
    few octaves for K; a flat softmax (small q), a spread of row scales and a nonzero mean (no result channel cancels
    to almost nothing) for V."""
    rng = np.random.default_rng(seed)
    D = 128
    q = (rng.normal(size=(1, G, D)) * 0.05).astype(np.float16)
    k = (rng.normal(size=(1, 1, N, D)) * np.exp2(rng.integers(-5, 6, size=(1, 1, 1, D)))).astype(np.float16)
    v = ((rng.normal(size=(1, 1, N, D)) + 3.0) * np.exp2(rng.integers(-13, 1, size=(1, 1, N, 1)))).astype(np.float16)
    return q, k, v


@pytest.mark.parametrize("force", [-1, 0, 1])
@pytest.mark.parametrize("G", [1, 2])
def test_out_is_attention_over_the_values_as_they_were_read(oracle, G, force):
    """"Runtime of AlignedKV": S = QK^T/sqrt(128); softmax; O = SV, on the operands "Dynamic Quantization" hands over:
    K column d read at lvlK[d], V row t read at appliedV[t].  Recomputed in numpy fp64 from the exported masks; a value
    path that reads either operand at any other level than the exported one fails here."""
    N, D = 200, 128
    q, k, v = mixed_level_case(100 + G, G, N)
    c = fill_cache(oracle, f16bits(k), f16bits(v))
    r = oracle.decode_attention(c, f16bits(q), force_level=force)
    lvlK, appl = r.lvlK[0, 0], r.appliedV[0, 0, :N]
    if force < 0:
        assert set(lvlK.tolist()) == {0, 1, 2} and set(appl.tolist()) == {0, 1, 2}    # every level is exercised
    else:
        assert np.all(lvlK == force) and np.all(appl == force)
    kt = read_bits_np(f16bits(k)[0, 0], lvlK[None, :])                       # [N, D]
    vt = read_bits_np(f16bits(v)[0, 0], appl[:, None])                       # [N, D]
    full_k, full_v = k[0, 0].astype(np.float64), v[0, 0].astype(np.float64)
    ref = np.zeros((G, D))
    wrongK = np.zeros((G, D))
    wrongV = np.zeros((G, D))
    for g in range(G):
        qg = q[0, g].astype(np.float64)
        for kk, vv, dst in ((kt, vt, ref), (full_k, vt, wrongK), (kt, full_v, wrongV)):
            s = (kk @ qg) / math.sqrt(D)
            w = np.exp(s - s.max())
            dst[g] = (w / w.sum()) @ vv
    assert np.abs(r.out[0] - ref).max() <= 1e-12 * max(1.0, np.abs(ref).max())
    if force != 2:
        # the pin discriminates: the same sums over operands read at 16 bits are far outside the tolerance
        assert np.abs(wrongK - ref).max() > 1e-7 and np.abs(wrongV - ref).max() > 1e-7


# ----------------------------------------------------------------------------------------------
# other fetch granules (studies): "Dynamic Quantization", data re-arrangement -- the hardware reads in units
# ----------------------------------------------------------------------------------------------

def test_v_granule_counts_against_numpy_block_maxima(oracle):
    rng = np.random.default_rng(120)
    B, Hkv, G, N, D = 2, 2, 2, 512, 128
    q = (rng.normal(size=(B, Hkv * G, D)) * 0.3).astype(np.float16)
    k = rng.normal(size=(B, Hkv, N, D)).astype(np.float16)
    v = ((rng.normal(size=(B, Hkv, N, D)) + 1.0) * np.exp2(rng.integers(-8, 1, size=(B, Hkv, N, 1)))
         * np.exp2(rng.integers(-3, 4, size=(B, Hkv, 1, D)))).astype(np.float16)
    lens = np.array([512, 333], np.int32)                                   # a ragged sequence: the last unit is partly valid
    c = fill_cache(oracle, f16bits(k), f16bits(v), lens=lens)
    r = oracle.decode_attention(c, f16bits(q))
    assert len(set(r.needV[0, 0, :512].ravel().tolist())) == 3              # every level occurs
    # the cache's own unit (a token row) and the per-element need are the two counts the decode call reports
    assert np.array_equal(oracle.v_granule_counts(c, r.needV, 1, D), r.counts[3:6])
    assert np.array_equal(oracle.v_granule_counts(c, r.needV, 1, 1), r.counts[6:9])
    bits = lambda cnt: float(8 * cnt[0] + 12 * cnt[1] + 16 * cnt[2]) / float(cnt.sum())
    for tt, cc in ((2, 128), (2, 64), (4, 32), (8, 16), (1, 64), (1, 32), (16, 128), (256, 128)):
        got = oracle.v_granule_counts(c, r.needV, tt, cc)
        want = np.zeros(3, np.uint64)
        for b in range(B):
            n = int(lens[b])
            need = r.needV[b].copy()
            need[:, n:] = 0                                                  # slots past the sequence ask for nothing
            ntok = (np.arange(c.Ncap) < n).reshape(c.Ncap // tt, tt).sum(axis=1)            # valid tokens per unit
            unit = need.reshape(Hkv, c.Ncap // tt, tt, D // cc, cc).max(axis=(2, 4))         # [Hkv, units, channel groups]
            for lvl in range(3):
                want[lvl] += np.uint64(((unit == lvl) * ntok[None, :, None]).sum() * cc)
        assert np.array_equal(got, want), (tt, cc)
        assert got.sum() == r.counts[3:6].sum()
        assert bits(got) >= bits(r.counts[6:9])                              # no unit reads less than the elements need
    # a unit made of whole smaller units never reads less than they do
    chain = [(1, 32), (1, 64), (1, 128), (2, 128), (4, 128), (16, 128)]
    b_ = [bits(oracle.v_granule_counts(c, r.needV, tt, cc)) for tt, cc in chain]
    assert all(x <= y for x, y in zip(b_, b_[1:]))
    with pytest.raises(ValueError):
        oracle.v_granule_counts(c, r.needV, 3, 128)


@pytest.mark.parametrize("guard", [0, 2])
def test_k_levels_per_block_against_a_frexp_rewrite_and_the_promised_bound(oracle, guard):
    rng = np.random.default_rng(130 + guard)
    G, N, D = 2, 700, 128
    q, k, v = tiny_case(rng, G, N, D, spread=4)
    k[0, 0, 100:140, :16] *= np.float16(16.0)                                # a stretch where 16 columns are large: its blocks decide differently
    k = k.astype(np.float16)
    c = fill_cache(oracle, f16bits(k), f16bits(v))
    r = oracle.decode_attention(c, f16bits(q), guard_bits=guard)
    # one block over the whole sequence is the rule of the decode call
    lvl, cnt = oracle.k_levels_per_block(c, f16bits(q), c.Ncap, guard)
    assert np.array_equal(lvl[0, 0, 0], r.lvlK[0, 0]) and np.array_equal(cnt, r.counts[0:3])
    for block in (64, 256):
        lvl, cnt = oracle.k_levels_per_block(c, f16bits(q), block, guard)
        exact = q[0].astype(np.float64) @ k[0, 0].astype(np.float64).T       # [G, N]
        want_cnt = np.zeros(3, np.uint64)
        for bi, t0 in enumerate(range(0, N, block)):
            t1 = min(N, t0 + block)
            cm = np.maximum(np.abs(k[0, 0, t0:t1]).max(axis=0).astype(np.float64), 2.0 ** -14)
            want = np.zeros(D, np.int64)
            emaxs = []
            for g in range(G):
                P = np.abs(q[0, g].astype(np.float64)) * cm
                es = np.array([exp2floor(x) if x != 0 else -10 ** 6 for x in P])
                emax = es.max()
                emaxs.append(emax)
                m = 10 + guard - (emax - es)
                want = np.maximum(want, np.where(P != 0, (m > 2).astype(np.int64) + (m > 6), 0))
            assert np.array_equal(lvl[0, 0, bi], want), (block, bi)
            for lv_ in range(3):
                want_cnt[lv_] += np.uint64((want == lv_).sum() * (t1 - t0))
            # the block's own promise: every addend reaches the last place of the block's coarsest addend
            kt = read_bits_np(f16bits(k)[0, 0, t0:t1], want[None, :])
            for g in range(G):
                err = np.abs(kt @ q[0, g].astype(np.float64) - exact[g, t0:t1])
                assert np.all(err <= int((want < 2).sum()) * 2.0 ** (emaxs[g] - 10 - guard))
        assert np.array_equal(cnt, want_cnt)
        assert block == 256 or lvl[0, 0, 1].tolist() != lvl[0, 0, 5].tolist()   # the large stretch changes its block's levels


def test_counts_add_up(oracle):
    rng = np.random.default_rng(90)
    q, k, v = tiny_case(rng, 2, 100, 128, spread=3)
    r = oracle.decode_attention(fill_cache(oracle, f16bits(k), f16bits(v)), f16bits(q))
    cnt = r.counts.astype(np.int64)
    assert cnt[0:3].sum() == cnt[3:6].sum() == cnt[6:9].sum() == 100 * 128
    assert [int((r.lvlK == i).sum()) * 100 for i in range(3)] == cnt[0:3].tolist()
    assert [int((r.appliedV[0, 0, :100] == i).sum()) * 128 for i in range(3)] == cnt[3:6].tolist()
    assert [int((r.needV[0, 0, :100] == i).sum()) for i in range(3)] == cnt[6:9].tolist()
