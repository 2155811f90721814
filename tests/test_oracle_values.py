"""Pins for the value side of the CPU oracle (Algorithm 1, Eq. 2-3, Phases 1-3, decoder phases 3-4).

Each pin checks the oracle against something other than itself: Python's correctly rounded
math.fsum, exact rational arithmetic, the paper's worked example, or a stated invariant.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import ref
from tests.streamparse import exact_code, parse

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def golden(name):
    out = {}
    for line in open(os.path.join(GOLDEN, name)):
        line = line.strip()
        if line and not line.startswith("#"):
            k, v = line.split("=", 1)
            out[k.strip()] = v.strip()
    return out


def f32(x):
    return np.asarray(x, dtype=np.float32)


def bits_to_f32(b):
    return np.asarray(b, dtype=np.uint32).view(np.float32)


# ----------------------------------------------------------------------------- abs-sum
def wide_values(rng, n):
    """float32 values whose exponents span the whole finite range, denormals and zeros included."""
    e = rng.integers(0, 255, n).astype(np.uint32)
    m = rng.integers(0, 1 << 23, n).astype(np.uint32)
    s = rng.integers(0, 2, n).astype(np.uint32)
    return ((s << 31) | (e << 23) | m).view(np.float32)


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_abs_sum_equals_fsum_wide_exponents(seed):
    rng = np.random.default_rng(seed)
    v = wide_values(rng, 5000)
    bad, s = ref.abs_sum(v)
    assert not bad
    assert s == math.fsum(abs(float(x)) for x in v)


@pytest.mark.parametrize("lo,hi", [(0, 40), (100, 140), (230, 254), (0, 3)])
def test_abs_sum_equals_fsum_narrow_windows(lo, hi):
    rng = np.random.default_rng(lo)
    n = 20000
    e = rng.integers(lo, hi + 1, n).astype(np.uint32)
    m = rng.integers(0, 1 << 23, n).astype(np.uint32)
    v = ((e << 23) | m).view(np.float32)
    bad, s = ref.abs_sum(v)
    assert not bad and s == math.fsum(float(x) for x in v)


def test_abs_sum_rounds_ties_to_even_and_sticky():
    # 2^60 + 2^7 is exactly half an ulp (ulp of 2^60 in binary64 is 2^8): tie -> even -> 2^60.
    assert ref.abs_sum(f32([2.0 ** 60, 2.0 ** 7]))[1] == 2.0 ** 60
    # a sticky bit below the tie pushes it up
    assert ref.abs_sum(f32([2.0 ** 60, 2.0 ** 7, 2.0 ** -20]))[1] == 2.0 ** 60 + 2.0 ** 8
    # odd mantissa + tie rounds up to even
    assert ref.abs_sum(f32([2.0 ** 60, 2.0 ** 8, 2.0 ** 7]))[1] == 2.0 ** 60 + 2.0 ** 9
    # smallest denormal alone, and with a huge partner (lost to rounding, but only once)
    tiny = np.uint32(1).view(np.float32)
    assert ref.abs_sum(f32([tiny]))[1] == 2.0 ** -149
    assert ref.abs_sum(f32([3.0e38, tiny]))[1] == float(np.float32(3.0e38))


def test_abs_sum_order_independent_and_signs():
    rng = np.random.default_rng(7)
    v = wide_values(rng, 3000)
    s0 = ref.abs_sum(v)[1]
    for k in range(5):
        assert ref.abs_sum(rng.permutation(v))[1] == s0
    assert ref.abs_sum(-v)[1] == s0
    assert ref.abs_sum(np.zeros(0, np.float32)) == (False, 0.0)
    assert ref.abs_sum(f32([0.0, -0.0]))[1] == 0.0


def test_abs_sum_many_equal_values_carry_chain():
    # 2^20 copies of the largest finite float: exercises long carries; exact answer known.
    big = np.float32(3.4028234663852886e38)
    v = np.full(1 << 20, big, np.float32)
    assert ref.abs_sum(v)[1] == float(big) * 2.0 ** 20


@pytest.mark.parametrize("badval", [np.nan, np.inf, -np.inf])
def test_abs_sum_flags_nonfinite(badval):
    v = f32([1.0, 2.0, badval, 3.0])
    assert ref.abs_sum(v)[0] is True
    rc, st = ref.compress(np.arange(4), v, ref.params())
    assert rc == ref.ERR_NONFINITE and st.size == 0


# ----------------------------------------------------------------------------- tables
@pytest.mark.parametrize("S,b,tau", [(100.25, 1.1, 128), (3.7e-4, 1.0371, 128), (1e30, 2.0, 128),
                                     (2.0 ** -140, 1.5, 128), (12345.678, 16.0, 128), (1.0, 1.000001, 64),
                                     (1e40, 1.5, 128)])
def test_tables_against_exact_rationals(S, b, tau):
    B, V = ref.tables(S, b, tau)
    Sf, bf = Fraction(S), Fraction(b)
    FLT_MAX = Fraction(float(np.finfo(np.float32).max))
    for c in range(1, tau + 1):
        t = Sf / bf ** c                       # the real-number boundary sum / b^c
        Bc, Vc = bits_to_f32(B[c]), bits_to_f32(V[c])
        if t > FLT_MAX * 2:
            assert np.isinf(Bc)
            continue
        if t < Fraction(2.0 ** -149) / 4:
            assert B[c] in (0, 1, 2)
            continue
        # the float64 recipe carries at most ~c+2 roundings of 2^-53 each
        tol = Fraction(c + 3, 2 ** 52)
        if np.isfinite(Bc):
            up, dn = Fraction(float(Bc)), Fraction(float(bits_to_f32(max(int(B[c]) - 1, 0))))
            assert up >= t * (1 - tol)           # boundary rounded up ...
            assert dn <= t * (1 + tol)           # ... and to the very next float32
        assert int(V[c]) in (int(B[c]), int(B[c]) - 1)   # nearest is the boundary or the float below
        assert float(Vc) <= float(Bc)
        if np.isfinite(Bc) and int(B[c]) > 0:
            # ... whichever of the two is nearer to the real boundary (up to the recipe's own rounding)
            other = dn if int(V[c]) == int(B[c]) else up
            assert abs(Fraction(float(Vc)) - t) <= abs(other - t) + 2 * tol * t


def test_tables_monotone_and_tau_e():
    B, V = ref.tables(100.25, 1.1, 128)
    assert np.all(np.diff(B[1:129].astype(np.int64)) < 0)      # strictly decreasing boundaries
    assert np.all(np.diff(V[1:129].astype(np.int64)) < 0)
    # Algorithm 1 line 2: tau_e = sum / b^tau
    tau_e = float(bits_to_f32(B[128]))
    assert tau_e == pytest.approx(100.25 / 1.1 ** 128, rel=1e-6)


# ----------------------------------------------------------------------------- codes
def codes_of(values, p):
    keys = np.arange(len(values), dtype=np.uint32)
    rc, st = ref.compress(keys, f32(values), p)
    assert rc == ref.OK
    info = parse(st)
    return info


def test_fig2_worked_example():
    g = golden("fig2_logquant.txt")
    b, D = float(g["base"]), int(g["D"])
    # six values whose first reciprocal value is the paper's 6.1: v1 = 1, the rest add up to 5.1
    v = f32([1.0, 1.7, -0.9, 0.5, 1.2, 0.8])
    assert len(v) == D
    S = ref.abs_sum(v)[1]
    assert S / 1.0 == pytest.approx(float(g["R_first"]), rel=1e-6)
    info = codes_of(v, ref.params(b, 128, 2, 1024))
    assert info["d"] == D
    assert (info["codes"][0] & 0x7F) + 1 == int(g["L_first"])
    # and every other code is ceil(log_2(S/|v|)) too, sign in bit 7
    for x, byte in zip(v, info["codes"]):
        assert (byte & 0x7F) + 1 == max(1, math.ceil(math.log2(S / abs(float(x)))))
        assert (byte >> 7) == (1 if x < 0 else 0)


@pytest.mark.parametrize("seed,b,tau", [(0, 1.1, 128), (1, 1.05, 128), (2, 2.0, 40), (3, 1.3, 64),
                                        (4, 1.0371, 128), (5, 16.0, 9)])
def test_codes_match_exact_rational_log(seed, b, tau):
    """Brute force: L = ceil(log_b(sum/|v|)) with exact rationals; kept iff L <= tau (Phase 3)."""
    rng = np.random.default_rng(seed)
    n = 300
    v = (rng.laplace(0, 1, n) * np.exp(rng.uniform(-12, 0, n))).astype(np.float32)
    S = ref.abs_sum(v)[1]
    assert S == math.fsum(abs(float(x)) for x in v)
    info = codes_of(v, ref.params(b, tau, 2, 1024))
    got = dict(zip(info["keys"], info["codes"]))
    checked = 0
    for j, x in enumerate(v):
        if x == 0:
            assert j not in got
            continue
        c, margin = exact_code(abs(float(x)), S, b, limit=tau + 2)
        if c is not None and margin < 1e-9:
            continue                      # on a boundary to within float64 round-off: recipe decides
        if c is None or c > tau:
            assert j not in got, (j, x, c)
        else:
            assert j in got, (j, x, c)
            assert (got[j] & 0x7F) + 1 == max(c, 1)
            assert (got[j] >> 7) == (1 if x < 0 else 0)
            checked += 1
    assert checked > 20


def test_codes_nonincreasing_in_magnitude_and_R_at_least_one():
    rng = np.random.default_rng(11)
    v = np.sort(np.abs(rng.laplace(0, 1e-3, 2000)).astype(np.float32))
    info = codes_of(v, ref.params(1.08, 128, 2, 1024))
    c = np.array([(x & 0x7F) + 1 for x in info["codes"]])
    assert c.min() >= 1                                   # R >= 1  =>  L >= 0, stored >= 1
    assert np.all(np.diff(c) <= 0)                        # bigger |v|  =>  smaller code
    # survivors are exactly the top of the sorted order (order reversal, Phase 3)
    assert info["keys"] == list(range(2000 - info["d"], 2000))


def test_kept_set_is_threshold_test():
    rng = np.random.default_rng(12)
    v = rng.laplace(0, 1e-3, 5000).astype(np.float32)
    b, tau = 1.07, 128
    S = math.fsum(abs(float(x)) for x in v)
    info = codes_of(v, ref.params(b, tau, 2, 1024))
    thr = Fraction(S) / Fraction(b) ** tau
    expect = [j for j, x in enumerate(v) if Fraction(abs(float(x))) >= thr * (1 + Fraction(1, 10 ** 9))]
    maybe = [j for j, x in enumerate(v) if Fraction(abs(float(x))) >= thr * (1 - Fraction(1, 10 ** 9))]
    assert set(expect) <= set(info["keys"]) <= set(maybe)


def test_power_of_two_scaling_leaves_codes_unchanged():
    rng = np.random.default_rng(13)
    v = rng.laplace(0, 1e-3, 3000).astype(np.float32)
    p = ref.params(1.09, 128, 2, 1024)
    a = codes_of(v, p)
    for k in (-20, 7, 30):
        s = codes_of(v * np.float32(2.0 ** k), p)
        assert s["codes"] == a["codes"] and s["keys"] == a["keys"]
        assert s["S"] == a["S"] * 2.0 ** k


def test_single_element_code_clamped_to_one():
    info = codes_of([-0.37], ref.params(1.1, 128, 2, 1024))
    assert info["d"] == 1 and info["codes"] == [0x80 | 0]   # L = 0 stored as code 1, negative


def test_zero_and_empty_inputs():
    p = ref.params()
    rc, st = ref.compress(np.zeros(0, np.uint32), np.zeros(0, np.float32), p)
    assert rc == ref.OK and st.size == 64 and parse(st)["d"] == 0
    rc, st = ref.compress(np.arange(10), np.zeros(10, np.float32), p)
    assert rc == ref.OK and st.size == 64 and parse(st)["n"] == 10
    info = codes_of([0.0, 1.0, -0.0, 2.0], p)
    assert info["keys"] == [1, 3]                          # zeros never survive


# ----------------------------------------------------------------------------- decode
@pytest.mark.parametrize("seed,b", [(0, 1.1), (1, 1.07), (2, 3.0)])
def test_decode_underestimates_within_one_base_step(seed, b):
    rng = np.random.default_rng(seed)
    n = 4000
    keys = np.sort(rng.choice(10 * n, n, replace=False)).astype(np.uint32)
    v = rng.laplace(0, 1e-3, n).astype(np.float32)
    p = ref.params(b, 128, 2, 256)
    rc, st = ref.compress(keys, v, p)
    assert rc == ref.OK
    rc, k2, v2 = ref.decompress(st)
    assert rc == ref.OK
    info = parse(st)
    assert list(k2) == info["keys"]
    orig = v[np.searchsorted(keys, k2)]
    assert np.all(np.sign(v2) == np.sign(orig))
    a, o = np.abs(v2).astype(np.float64), np.abs(orig).astype(np.float64)
    clamped = np.array([(c & 0x7F) == 0 for c in info["codes"]], dtype=bool)
    assert info["d"] > 100
    assert np.all(a <= o)                                   # never over-estimates
    assert np.all((o / b < a * (1 + 2.0 ** -22)) | clamped)  # and by less than one base step
    # decoded magnitude is sum / b^code
    S = info["S"]
    c = np.array([(x & 0x7F) + 1 for x in info["codes"]], dtype=np.float64)
    assert np.allclose(a, S / b ** c, rtol=1e-6)


def test_decoded_magnitude_stays_in_its_own_bucket():
    """The decoded magnitude of code c lies between the boundaries of c+1 and c (at most one
    float32 below its own boundary), so re-quantizing a decoded value moves it by at most one code."""
    rng = np.random.default_rng(5)
    v = rng.laplace(0, 1e-3, 3000).astype(np.float32)
    b, tau = 1.1, 128
    rc, st = ref.compress(np.arange(3000), v, ref.params(b, tau, 2, 1024))
    info = parse(st)
    rc, k2, v2 = ref.decompress(st)
    B, V = ref.tables(info["S"], b, tau)
    a = np.abs(v2).view(np.uint32)
    for x, byte in zip(a, info["codes"]):
        c = (byte & 0x7F) + 1
        # the decoded magnitude lies in (B[c+1], B[c]]: one ulp below B[c] at most
        assert x <= B[c] and (c == tau or x >= B[c + 1])


def boundary_gradient(tau=10, reps=8):
    """Values whose sum is exactly 2^20 with base 2, so that every boundary sum / 2^c is a power of two
    (Eq. 3 evaluated without rounding): elements sit exactly on boundaries, one ulp below and one ulp
    above them.  Returns (keys, values, expected codes, kept mask)."""
    f = np.float32
    vals, codes = [], []
    for c in range(tau - 3, tau + 3):                 # boundaries 2^(20-c); c > tau lies below the threshold
        t = f(2.0 ** (20 - c))
        below, above = np.nextafter(t, f(0)), np.nextafter(t, f(np.inf))
        for x, cx in ((t, c), (above, c), (below, c + 1)):
            for s in (1.0, -1.0):
                vals += [f(s) * x] * reps
                codes += [cx] * reps
    vals = np.array(vals, np.float32)
    codes = np.array(codes)
    # pad with small exact values so that the exact sum of |v| is 2^20 (all terms are multiples of 2^-20)
    from fractions import Fraction
    rest = Fraction(2 ** 20) - sum(Fraction(float(abs(x))) for x in vals)
    assert rest > 0
    filler = []
    unit = Fraction(2 ** (20 - tau - 2))               # a quarter of the threshold 2^(20-tau): dropped
    while rest > 0:
        take = min(rest, unit)
        # take is a multiple of 2^-33 at worst: split into exactly representable powers of two
        num, den = take.numerator, take.denominator
        bit = 1
        while num:
            if num & 1:
                filler.append(float(Fraction(bit, den)))
            num >>= 1
            bit <<= 1
        rest -= take
    filler = np.array(filler, np.float32)
    assert all(Fraction(float(x)) == Fraction(float(np.float64(x))) for x in filler[:4])
    rng = np.random.default_rng(3)
    allv = np.concatenate([vals, filler])
    allc = np.concatenate([codes, np.full(filler.size, tau + 5)])
    perm = rng.permutation(allv.size)
    allv, allc = allv[perm], allc[perm]
    return np.arange(allv.size, dtype=np.uint32) * 3, allv, allc, allc <= tau


def test_values_exactly_on_below_and_above_bucket_boundaries():
    """Closed form: with b = 2 and sum = 2^20 the boundary of code c is 2^(20-c) exactly, so the code of
    |v| = 2^(20-c) is c, one ulp above it still c, one ulp below it c + 1; the filter keeps c <= tau."""
    tau = 10
    keys, vals, codes, kept = boundary_gradient(tau)
    bad, S = ref.abs_sum(vals)
    assert not bad and S == 2.0 ** 20
    rc, st = ref.compress(keys, vals, ref.params(2.0, tau, 2, 256))
    assert rc == ref.OK
    d = int(st[40:48].view("<u8")[0])
    assert d == int(kept.sum())
    plane = np.array(parse(st)["codes"], np.uint8)     # sign << 7 | code-1 (tau = 10: stored in 5 bits each)
    assert np.array_equal((plane & 0x7F) + 1, codes[kept])
    assert np.array_equal(plane >> 7, (vals[kept] < 0).astype(np.uint8))
    rc, k, v = ref.decompress(st)
    assert np.array_equal(k, keys[kept])
    assert np.array_equal(np.abs(v), (2.0 ** (20 - codes[kept])).astype(np.float32))


@pytest.mark.parametrize("tau", [1, 2, 3, 5, 16, 32, 33, 64, 65, 100, 127])
def test_codes_take_one_plus_ceil_log2_tau_bits(tau):
    """Section 3.2: after the filter a code needs ceil(log2 tau) bits, plus the sign.  The code of a value
    does not depend on tau (only the filter does), so the tokens of a tau < 128 stream must spell the
    codes <= tau of the one-byte-per-code stream of tau = 128, in order, in narrower fields."""
    import math
    rng = np.random.default_rng(tau)
    n = {1: 12, 2: 150, 3: 2000}.get(tau, 5000 + tau)       # few values for tiny tau: b <= 16 must reach them
    keys = np.sort(rng.choice(10 * n, n, replace=False)).astype(np.uint32)
    vals = rng.laplace(0.0, 1e-3, n).astype(np.float32)
    S = float(np.abs(vals.astype(np.float64)).sum())
    base = min(16.0, max(1.01, (S / float(np.median(np.abs(vals)))) ** (1.0 / tau)))   # about half survive
    rc, wide = ref.compress(keys, vals, ref.params(base, 128, 2, 256))
    assert rc == ref.OK
    rc, st = ref.compress(keys, vals, ref.params(base, tau, 2, 256))
    assert rc == ref.OK
    a, b = parse(wide), parse(st)
    w = 1 + (0 if tau == 1 else math.ceil(math.log2(tau)))
    assert b["w"] == w and a["w"] == 8
    keep = [i for i, c in enumerate(a["codes"]) if (c & 0x7F) + 1 <= tau]
    assert b["d"] == len(keep) and b["d"] > 0
    assert b["codes"] == [a["codes"][i] for i in keep]
    assert b["keys"] == [a["keys"][i] for i in keep]
    # size: header, d tokens of w bits padded to 8 bytes, directory, key blocks
    plane = 8 * math.ceil(b["d"] * w / 64)
    key_bytes = sum(8 * (math.ceil(min(256, b["d"] - 256 * i) * 2 / 64)) for i in range(b["nb"]))
    pay = st.size - 64 - plane - 16 * b["nb"] - key_bytes
    assert pay >= 0 and pay % 8 == 0
    # decoding gives the values of the wide stream at the kept positions
    rc, k1, v1 = ref.decompress(wide)
    rc2, k2, v2 = ref.decompress(st)
    assert rc == ref.OK and rc2 == ref.OK
    assert np.array_equal(k2, k1[keep]) and np.array_equal(v2.view(np.uint32), v1[keep].view(np.uint32))


def test_packed_codes_beyond_tau_are_rejected():
    # tau = 5: 4-bit tokens, code-1 in 3 bits can say 5..7, which no encoder writes
    rng = np.random.default_rng(1)
    n = 3000
    keys = np.arange(n, dtype=np.uint32)
    vals = rng.laplace(0.0, 1e-3, n).astype(np.float32)
    rc, st = ref.compress(keys, vals, ref.params(4.0, 5, 2, 256))
    assert rc == ref.OK and parse(st)["d"] > 10
    bad = st.copy()
    bad[64] = (bad[64] & 0xF0) | 0x07          # token 0: sign 0, code-1 = 7
    assert ref.decompress(bad)[0] == ref.ERR_CORRUPT_STREAM
    bad[64] = (st[64] & 0xF0) | 0x04           # code-1 = 4 is code 5 = tau: fine
    rc, k, v = ref.decompress(bad)
    assert rc == ref.OK


# ----------------------------------------------------------------------------- tau above 128 (9-bit tokens)
def test_tables_for_256_codes_in_closed_form_down_to_the_smallest_binary32():
    """b = 2 and sum = 2^100: the boundary of code c is 2^(100-c) exactly while that is a binary32 number
    (normal to 2^-126, denormal to 2^-149).  Below it the two roundings part: the boundary rounds UP to the
    smallest positive binary32, the decoded magnitude rounds to NEAREST, which is zero (2^-150 is a tie
    between 0 and 2^-149 and goes to the even one)."""
    B, V = ref.tables(2.0 ** 100, 2.0, 256)
    for c in range(1, 250):
        x = np.float32(2.0 ** (100 - c))
        assert float(x) == 2.0 ** (100 - c)
        assert B[c] == x.view(np.uint32) and V[c] == x.view(np.uint32), c
    assert list(B[250:257]) == [1] * 7                      # bit pattern 1 = 2^-149
    assert list(V[250:257]) == [0] * 7
    # the tables of a smaller tau are a prefix of these (the chain does not depend on tau)
    B2, V2 = ref.tables(2.0 ** 100, 2.0, 128)
    assert np.array_equal(B2[:129], B[:129]) and np.array_equal(V2[:129], V[:129])
    assert not B2[129:].any()


@pytest.mark.parametrize("seed,b,tau,spread,top", [(20, 1.1, 200, 30, 1.0), (21, 1.05, 256, 30, 1.0),
                                                   (22, 1.3, 129, 45, 1.0), (23, 4.0, 130, 185, 1e37)])
def test_codes_above_128_match_exact_rational_log(seed, b, tau, spread, top):
    """Brute force as above for thresholds past 128: the code is the least c with |v| b^c >= sum, the token
    is nine bits wide (eight for the code-1, one for the sign)."""
    rng = np.random.default_rng(seed)
    n = 400
    v = (np.clip(rng.laplace(0, 1, n), -3, 3) * top * np.exp(rng.uniform(-spread, 0, n))).astype(np.float32)
    S = ref.abs_sum(v)[1]                 # (with b = 4 the codes past 128 need the whole binary32 range)
    info = codes_of(v, ref.params(b, tau, 2, 1024))
    assert info["w"] == 9 and info["tau"] == tau
    got = {k: (c, neg) for k, c, neg in zip(info["keys"], info["code"], info["negative"])}
    checked = above = 0
    for j, x in enumerate(v):
        if x == 0:
            assert j not in got
            continue
        c, margin = exact_code(abs(float(x)), S, b, limit=tau + 2)
        if c is not None and margin < 1e-9:
            continue
        if c is None or c > tau:
            assert j not in got, (j, x, c)
        else:
            assert got[j] == (max(c, 1), bool(x < 0)), (j, x, c, got[j])
            checked += 1
            above += c > 128
    assert checked > 50 and above > (5 if tau >= 200 else 0)


@pytest.mark.parametrize("tau", [129, 200, 256])
def test_a_threshold_above_128_only_adds_survivors(tau):
    """The code of a value does not depend on tau: the stream of tau = 128 must be what is left of the
    stream of a bigger tau once the codes above 128 are struck out, and every survivor it adds has a code
    in 129..tau; decoded values agree on the common part."""
    rng = np.random.default_rng(tau)
    n = 6000
    keys = np.sort(rng.choice(10 * n, n, replace=False)).astype(np.uint32)
    vals = (rng.laplace(0.0, 1e-3, n) * np.exp(rng.uniform(-8, 0, n))).astype(np.float32)
    S = float(np.abs(vals.astype(np.float64)).sum())
    base = (S / float(np.quantile(np.abs(vals), 0.3))) ** (1.0 / tau)       # about 70 % survive at tau
    rc, st8 = ref.compress(keys, vals, ref.params(base, 128, 2, 256))
    rc9, st9 = ref.compress(keys, vals, ref.params(base, tau, 2, 256))
    assert rc == ref.OK and rc9 == ref.OK
    a, b = parse(st8), parse(st9)
    assert a["w"] == 8 and b["w"] == 9 and b["d"] > a["d"] > 100
    common = [i for i, c in enumerate(b["code"]) if c <= 128]
    assert [b["code"][i] for i in common] == a["code"] and [b["negative"][i] for i in common] == a["negative"]
    assert [b["keys"][i] for i in common] == a["keys"]
    assert max(b["code"]) <= tau and min(c for c in b["code"] if c > 128) == 129
    # value plane: d tokens of 9 bits, padded to 8 bytes
    plane = 8 * math.ceil(b["d"] * 9 / 64)
    assert st9.size >= 64 + plane + 16 * b["nb"]
    rc, k8, v8 = ref.decompress(st8)
    rc9, k9, v9 = ref.decompress(st9)
    assert rc == ref.OK and rc9 == ref.OK
    assert np.array_equal(k9[common], k8) and np.array_equal(v9[common].view(np.uint32), v8.view(np.uint32))
    # the under-estimate of Section 3.2 holds for the new codes too: |v|/b < |decoded| <= |v|
    src = dict(zip(keys.tolist(), vals.tolist()))
    for k, x in zip(k9.tolist(), v9.tolist()):
        o = src[k]
        assert (x < 0) == (o < 0) and abs(x) <= abs(o) and abs(o) / base < abs(x) * (1 + 2.0 ** -22)


def test_parameter_limits_above_128():
    k, v = np.arange(10), np.full(10, 1.0, np.float32)
    assert ref.compress(k, v, ref.params(1.1, 256))[0] == ref.OK
    assert ref.compress(k, v, ref.params(1.1, 257))[0] == ref.ERR_INVALID_ARG
    # past 128 the base stops at 4: b^tau must stay a finite binary64 well inside the normal range
    assert ref.compress(k, v, ref.params(4.0, 129))[0] == ref.OK
    assert ref.compress(k, v, ref.params(4.0 + 1e-9, 129))[0] == ref.ERR_INVALID_ARG
    assert ref.compress(k, v, ref.params(16.0, 128))[0] == ref.OK
    # header: tau in 16 bits; a stream that claims 257 is corrupt, and so is a 9-bit code beyond tau
    rc, st = ref.compress(k, v, ref.params(1.1, 200))
    assert rc == ref.OK and parse(st)["d"] == 10 and int(st[6]) == 200 and int(st[7]) == 0
    rc, st2 = ref.compress(k, v, ref.params(1.1, 256))
    assert int(st2[6]) == 0 and int(st2[7]) == 1
    rc, k2, v2 = ref.decompress(st2)
    assert rc == ref.OK and k2.tolist() == list(range(10))
    bad = st2.copy(); bad[6] = 1
    assert ref.decompress(bad)[0] == ref.ERR_CORRUPT_STREAM
    bad = st.copy(); bad[64] = 200                                  # token 0: code-1 = 200 -> code 201 > tau
    assert ref.decompress(bad)[0] == ref.ERR_CORRUPT_STREAM
    bad[64] = 199
    assert ref.decompress(bad)[0] == ref.OK
