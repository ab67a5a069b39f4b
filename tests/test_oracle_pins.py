"""Pins for the CPU oracle: each test checks it against something fixed by the rule's
definition or by mathematics, not against another run of the same formula.

  * hand-derived records (tests/golden/pins.txt)
  * its fp16 / bf16 decoders against numpy's and torch's conversions, all 65536 patterns
  * an exact rational-arithmetic model of the binary32 rounding steps (fractions.Fraction with
    an explicit round-to-nearest-even), including a case that a fused multiply-add gets wrong
  * structural invariants (copy, independence of K, concatenation, permutation, empty)
  * numpy.isclose on finite data away from the tolerance boundary
  * mismatch counts and first indices known from how the synthetic workloads were planted
"""
import math
from fractions import Fraction

import numpy as np
import pytest
import torch

from helpers import load_pins, record_tuple, expect_tuple, NP_STORAGE
from paper_2507_23194_amd import synth

PINS = load_pins()


# ------------------------------------------------------------------------------------------
# hand-derived golden records
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("case", PINS, ids=[c["name"] for c in PINS])
def test_golden_pin(oracle_mod, case):
    rec = oracle_mod.check_segment(case["ref"], case["cand"], case["ref"].size, case["dtype"],
                                   case["atol"], case["rtol"], case["equal_nan"])
    assert record_tuple(rec) == expect_tuple(case["expect"]), (case["name"], rec)


def test_pins_cover_every_policy_branch():
    names = " ".join(c["name"] for c in PINS)
    for key in ("boundary_f32", "boundary_f16", "boundary_bf16", "nan_equal", "nan_not_equal",
                "inf_same", "inf_opposite", "fin_vs_inf", "inf_vs_fin", "tol_overflow",
                "signed_zero", "subnormal", "int_off_by_one", "int_extremes", "empty"):
        assert key in names


# ------------------------------------------------------------------------------------------
# decoders against library conversions
# ------------------------------------------------------------------------------------------
def _same_float(x: float, y: float) -> bool:
    if math.isnan(x) or math.isnan(y):
        return math.isnan(x) and math.isnan(y)
    return x == y and math.copysign(1.0, x) == math.copysign(1.0, y)


def test_decode_f16_all_patterns(oracle_mod):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    lib = bits.view(np.float16).astype(np.float32)
    for h in range(65536):
        assert _same_float(oracle_mod.decode_f16(h), float(lib[h])), hex(h)


def test_decode_bf16_all_patterns(oracle_mod):
    bits = torch.arange(65536, dtype=torch.int32)
    bits = torch.where(bits >= 0x8000, bits - 0x10000, bits).to(torch.int16)
    lib = bits.view(torch.bfloat16).to(torch.float32).numpy()
    for h in range(65536):
        assert _same_float(oracle_mod.decode_bf16(h), float(lib[h])), hex(h)


# ------------------------------------------------------------------------------------------
# exact rational model of the arithmetic
# ------------------------------------------------------------------------------------------
INF = "inf"


def rn(x, mant_bits, emin, emax):
    """Round a non-negative exact rational to the binary format with `mant_bits` significand bits
    (hidden bit included), least normal exponent emin and greatest exponent emax: nearest-even,
    subnormals kept, overflow to INF.  Pure integer arithmetic."""
    if x == INF:
        return INF
    assert x >= 0
    if x == 0:
        return Fraction(0)
    num, den = x.numerator, x.denominator
    e = num.bit_length() - den.bit_length()          # 2^(e-1) < x < 2^(e+1)
    if Fraction(2) ** e > x:
        e -= 1                                        # now 2^e <= x < 2^(e+1)
    q_exp = max(e, emin) - (mant_bits - 1)            # exponent of one unit in the last place
    scaled = x / (Fraction(2) ** q_exp)
    n = scaled.numerator // scaled.denominator
    rem = scaled - n
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and n % 2 == 1):
        n += 1
    y = n * Fraction(2) ** q_exp
    return INF if y >= Fraction(2) ** (emax + 1) else y


def rn32(x):
    return rn(x, 24, -126, 127)


def rn64(x):
    return rn(x, 53, -1022, 1023)


def model_element_f64(a: float, b: float, atol: float, rtol: float):
    """The binary64 rule on finite a, b: each step rounded once to binary64, product and sum separately."""
    fa, fb = Fraction(a), Fraction(b)
    d = rn64(abs(fa - fb))
    prod = rn64(Fraction(rtol) * abs(fb))
    tol = INF if prod == INF else rn64(Fraction(atol) + prod)
    close = True if tol == INF else (False if d == INF else d <= tol)
    if d == 0:
        r = Fraction(0)
    elif d == INF or fb == 0:
        r = INF
    else:
        r = rn64(d / abs(fb))
    return close, d, r


def model_element(a: float, b: float, atol_f: float, rtol_f: float):
    """Finite a, b (binary32 values held in Python floats).  Returns (close, d, r) with d, r
    exact rationals or INF, each step rounded once, product and sum rounded separately."""
    fa, fb = Fraction(a), Fraction(b)
    d = rn32(abs(fa - fb))
    prod = rn32(Fraction(rtol_f) * abs(fb))
    tol = INF if prod == INF else rn32(Fraction(atol_f) + prod)
    if tol == INF:
        close = True
    elif d == INF:
        close = False
    else:
        close = d <= tol
    if d == 0:
        r = Fraction(0)
    elif d == INF or fb == 0:
        r = INF
    else:
        r = rn32(d / abs(fb))
    return close, d, r


def _to_float(x):
    return math.inf if x == INF else float(x)


def _boundary_cases(rng, n):
    """Random finite binary32 (b, a, atol, rtol) with a placed within a few ulps of b +- tol."""
    out = []
    for _ in range(n):
        kind = rng.integers(0, 4)
        if kind == 0:      # ordinary magnitudes
            b = np.float32(rng.normal() * 10.0 ** rng.integers(-3, 4))
        elif kind == 1:    # subnormal / tiny reference
            b = np.array([rng.integers(0, 1 << 24)], dtype=np.uint32).view(np.float32)[0]
            if rng.random() < 0.5:
                b = -b
        elif kind == 2:    # huge reference
            b = np.float32(rng.normal() * 1e37)
        else:              # any finite bit pattern
            u = np.uint32(rng.integers(0, 1 << 32))
            if (u & 0x7F800000) == 0x7F800000:
                u = np.uint32(u & 0x807FFFFF)
            b = np.array([u], dtype=np.uint32).view(np.float32)[0]
        atol = float(np.float32(10.0 ** rng.uniform(-45, 1))) if rng.random() < 0.8 else 0.0
        rtol = float(np.float32(10.0 ** rng.uniform(-8, 0.5))) if rng.random() < 0.8 else 0.0
        tol64 = atol + rtol * abs(float(b))
        target = float(b) + (tol64 if rng.random() < 0.5 else -tol64)
        if not math.isfinite(target) or abs(target) > 3.0e38:
            target = float(b)
        a0 = np.float32(target)
        ai = a0.view(np.int32) + np.int32(rng.integers(-3, 4))
        a = np.array([ai], dtype=np.int32).view(np.float32)[0]
        if not np.isfinite(a):
            a = a0
        out.append((float(b), float(a), atol, rtol))
    return out


def test_rational_model_matches_oracle(oracle_mod):
    rng = np.random.default_rng(20250723)
    boundary_hits = 0
    for (b, a, atol, rtol) in _boundary_cases(rng, 4000):
        atol_f, rtol_f = float(np.float32(atol)), float(np.float32(rtol))
        close, d, r = model_element(a, b, atol_f, rtol_f)
        rec = oracle_mod.check_segment(np.array([b], np.float32), np.array([a], np.float32), 1, "f32",
                                       atol, rtol, False)
        exp = (int(close), int(not close), -1 if close else 0, _to_float(d), _to_float(r))
        got = (int(rec["pass"]), int(rec["mismatch_count"]), int(rec["first_mismatch"]),
               float(rec["max_abs_err"]), float(rec["max_rel_err"]))
        assert got == exp, (b, a, atol, rtol, got, exp)
        prod = rn32(Fraction(rtol_f) * abs(Fraction(b)))
        if prod != INF and d != INF and d == rn32(Fraction(atol_f) + prod):
            boundary_hits += 1
    assert boundary_hits > 50            # the generator really lands on the inclusive boundary


def test_fma_contraction_would_be_caught(oracle_mod):
    """Find (b, rtol, atol) where rounding the product before the sum changes the tolerance,
    put d exactly on the two-rounding tolerance, and require the two-rounding verdict."""
    rng = np.random.default_rng(7)
    found = 0
    for _ in range(20000):
        b = float(np.float32(rng.uniform(1.0, 2.0)))
        rtol = float(np.float32(rng.uniform(1e-3, 1e-2)))
        atol = float(np.float32(rng.uniform(1e-3, 1e-2)))
        two = rn32(Fraction(atol) + rn32(Fraction(rtol) * Fraction(b)))
        one = rn32(Fraction(atol) + Fraction(rtol) * Fraction(b))
        if two == one:
            continue
        # a = b + max(two, one): representable?  d must equal the larger tolerance exactly
        big, small = max(two, one), min(two, one)
        a = float(np.float32(float(Fraction(b) + big)))
        if rn32(abs(Fraction(a) - Fraction(b))) != big:
            continue
        rec = oracle_mod.check_segment(np.array([b], np.float32), np.array([a], np.float32), 1, "f32",
                                       atol, rtol, False)
        assert int(rec["pass"]) == int(big == two), (b, a, atol, rtol)
        found += 1
        if found >= 25:
            break
    assert found >= 25


def test_rational_model_matches_oracle_f64(oracle_mod):
    """binary64 segments (rule R2'): the oracle against exact rational arithmetic with explicit rounding to
    53 bits, on cases placed within a few ulps of the tolerance boundary, subnormal and huge magnitudes
    included; and a search for (b, rtol, atol) where a fused multiply-add would round differently."""
    rng = np.random.default_rng(64)
    hits = 0
    for _ in range(3000):
        kind = rng.integers(0, 4)
        if kind == 0:
            b = float(rng.normal() * 10.0 ** rng.integers(-3, 4))
        elif kind == 1:
            b = float(np.array([rng.integers(0, 1 << 53)], dtype=np.uint64).view(np.float64)[0]) * (1 if rng.random() < 0.5 else -1)
        elif kind == 2:
            b = float(rng.normal() * 1e307)
        else:
            u = np.uint64(rng.integers(0, 1 << 63)) | (np.uint64(rng.integers(0, 2)) << np.uint64(63))
            if (int(u) >> 52) & 0x7FF == 0x7FF:
                u = np.uint64(int(u) & ~(0x7FF << 52))
            b = float(np.array([u], dtype=np.uint64).view(np.float64)[0])
        atol = float(10.0 ** rng.uniform(-320, 1)) if rng.random() < 0.8 else 0.0
        rtol = float(10.0 ** rng.uniform(-17, 0.5)) if rng.random() < 0.8 else 0.0
        tol = atol + rtol * abs(b)
        target = b + (tol if rng.random() < 0.5 else -tol)
        if not math.isfinite(target):
            target = b
        ai = np.array([target], dtype=np.float64).view(np.int64) + np.int64(rng.integers(-3, 4))
        a = float(ai.view(np.float64)[0])
        if not math.isfinite(a):
            a = target
        close, d, r = model_element_f64(a, b, atol, rtol)
        rec = oracle_mod.check_segment(np.array([b]), np.array([a]), 1, "f64", atol, rtol, False)
        exp = (int(close), int(not close), -1 if close else 0, _to_float(d), _to_float(r))
        got = (int(rec["pass"]), int(rec["mismatch_count"]), int(rec["first_mismatch"]),
               float(rec["max_abs_err"]), float(rec["max_rel_err"]))
        assert got == exp, (b, a, atol, rtol, got, exp)
        prod = rn64(Fraction(rtol) * abs(Fraction(b)))
        if prod != INF and d != INF and d == rn64(Fraction(atol) + prod):
            hits += 1
    assert hits > 30
    found = 0
    for _ in range(20000):
        b, rtol, atol = float(rng.uniform(1.0, 2.0)), float(rng.uniform(1e-3, 1e-2)), float(rng.uniform(1e-3, 1e-2))
        two = rn64(Fraction(atol) + rn64(Fraction(rtol) * Fraction(b)))
        one = rn64(Fraction(atol) + Fraction(rtol) * Fraction(b))
        if two == one:
            continue
        big = max(two, one)
        a = float(Fraction(b) + big)
        if rn64(abs(Fraction(a) - Fraction(b))) != big:
            continue
        rec = oracle_mod.check_segment(np.array([b]), np.array([a]), 1, "f64", atol, rtol, False)
        assert int(rec["pass"]) == int(big == two), (b, a, atol, rtol)
        found += 1
        if found >= 25:
            break
    assert found >= 25


def test_f64_hand_derived(oracle_mod):
    inf, nan = np.inf, np.nan
    # atol = rtol = 2^-41, b = 1: tol = 2^-40 exactly; d = 2^-40 passes (inclusive), d = 2^-40 + 2^-52 fails
    b = np.array([1.0, 1.0, nan, inf, 0.0, nan, 1.0, -0.0])
    a = np.array([1.0 + 2.0 ** -40, 1.0 + 2.0 ** -40 + 2.0 ** -52, nan, -inf, 5e-324, 1.0, inf, 0.0])
    rec = oracle_mod.check_segment(b, a, 8, "f64", 2.0 ** -41, 2.0 ** -41, True)
    assert (int(rec["mismatch_count"]), int(rec["first_mismatch"])) == (4, 1)     # 1, 3, 5, 6
    assert float(rec["max_abs_err"]) == inf and float(rec["max_rel_err"]) == inf
    rec = oracle_mod.check_segment(b[:3], a[:3], 3, "f64", 2.0 ** -41, 2.0 ** -41, False)
    assert (int(rec["mismatch_count"]), int(rec["first_mismatch"])) == (2, 1)     # NaN pair fails without equal_nan
    assert float(rec["max_abs_err"]) == 2.0 ** -40 + 2.0 ** -52 == float(rec["max_rel_err"])
    # a difference far below binary32 resolution is still seen
    rec = oracle_mod.check_segment(np.array([1.0]), np.array([1.0 + 2.0 ** -50]), 1, "f64", 0.0, 2.0 ** -51, False)
    assert int(rec["pass"]) == 0 and float(rec["max_rel_err"]) == 2.0 ** -50
    rep = oracle_mod.report_segment(b, a, 8, "f64", 2.0 ** -41, 2.0 ** -41, True, 8)
    assert [int(r["index"]) for r in rep] == [1, 3, 5, 6]
    assert float(rep[0]["d"]) == 2.0 ** -40 + 2.0 ** -52 and float(rep[0]["tol"]) == 2.0 ** -40
    assert float(rep[1]["d"]) == inf and float(rep[1]["tol"]) == inf and np.isnan(rep[2]["d"]) and np.isnan(rep[2]["tol"])


# ------------------------------------------------------------------------------------------
# structural invariants
# ------------------------------------------------------------------------------------------
def _rand_case(rng, dtype, n):
    if dtype == "f64":
        b = rng.normal(size=n)
        a = b + 1e-9 * rng.normal(size=n) * (rng.random(n) < 0.3)
        pool = np.array([np.nan, np.inf, -np.inf, 0.0, -0.0, 5e-324, 1e308])
        for arr in (a, b):
            sp = rng.random(n) < 0.02
            arr[sp] = rng.choice(pool, int(sp.sum()))
        return b, a
    if dtype in ("u8", "i8"):
        np_t = np.uint8 if dtype == "u8" else np.int8
        info = np.iinfo(np_t)
        b = rng.integers(info.min, info.max + 1, n).astype(np_t)
        b[rng.random(n) < 0.3] = 0
        a = b.copy()
        idx = rng.random(n) < 0.05
        a[idx] = rng.integers(info.min, info.max + 1, int(idx.sum())).astype(np_t)
        return b, a
    if dtype == "i64":
        # small values, values beyond 2^53 (where the binary64 conversions round) and the two extremes
        b = rng.integers(-1000, 1001, n).astype(np.int64)
        big = rng.random(n) < 0.1
        b[big] = rng.integers(-(2 ** 62), 2 ** 62, int(big.sum()), dtype=np.int64) * 2 + 1
        b[rng.random(n) < 0.01] = np.iinfo(np.int64).min
        a = b.copy()
        idx = rng.random(n) < 0.05
        a[idx] = (a[idx].astype(np.uint64) + rng.integers(1, 4, int(idx.sum())).astype(np.uint64)).astype(np.int64)   # wraps at the top
        far = rng.random(n) < 0.01
        a[far] = np.iinfo(np.int64).max
        return b, a
    if dtype == "i32":
        b = rng.integers(-1000, 1001, n).astype(np.int32)
        a = b.copy()
        idx = rng.random(n) < 0.05
        a[idx] += rng.integers(-3, 4, int(idx.sum())).astype(np.int32)
        return b, a
    b32 = rng.normal(size=n).astype(np.float32)
    a32 = (b32 + 1e-3 * rng.normal(size=n) * (rng.random(n) < 0.3)).astype(np.float32)
    sp = rng.random(n) < 0.02
    a32[sp] = rng.choice(np.array([np.nan, np.inf, -np.inf, 0.0, -0.0], np.float32), int(sp.sum()))
    sp = rng.random(n) < 0.02
    b32[sp] = rng.choice(np.array([np.nan, np.inf, -np.inf, 0.0, -0.0], np.float32), int(sp.sum()))
    if dtype == "f32":
        return b32, a32
    if dtype == "f16":
        return b32.astype(np.float16).view(np.uint16), a32.astype(np.float16).view(np.uint16)
    tb = torch.from_numpy(b32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    ta = torch.from_numpy(a32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    return tb, ta


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16", "i32", "i64", "u8", "i8", "f64"])
def test_invariants(oracle_mod, dtype):
    rng = np.random.default_rng(11)
    n = 3001
    b, a = _rand_case(rng, dtype, n)
    kw = dict(atol=1e-4, rtol=1e-3, equal_nan=True)
    full = oracle_mod.check_segment(b, a, n, dtype, **kw)

    # a bit-identical copy of a NaN-free tensor is the neutral record
    if dtype in ("i32", "i64", "u8", "i8"):
        clean = b
    else:
        _, clean = _rand_case(np.random.default_rng(12), dtype, n)
        if dtype == "f64":
            clean = np.where(np.isfinite(clean), clean, 0.0)
        store = clean.view(np.uint32) if dtype == "f32" else (np.zeros(n, np.uint16) if dtype == "f64" else clean)
        expo = (store & 0x7F800000) == 0x7F800000 if dtype == "f32" else (
            (store & 0x7C00) == 0x7C00 if dtype == "f16" else (store & 0x7F80) == 0x7F80)
        clean = clean.copy()
        clean[expo] = 0
    cp = oracle_mod.check_segment(clean, clean.copy(), n, dtype, **kw)
    assert record_tuple(cp) == (1, 0, -1, 0, 0)

    # independent of how many other candidates ride along
    many = oracle_mod.check_dense(b, [b, a, a[::-1].copy(), a], dtype, 1e-4, 1e-3, True)
    assert record_tuple(many[1]) == record_tuple(full) == record_tuple(many[3])

    # concatenation: result(X || Y) = combine(result X, result Y)
    cut = 1234
    w = b.itemsize
    x = oracle_mod.check_segment(b[:cut], a[:cut], cut, dtype, **kw)
    y = oracle_mod.check_segment(b[cut:], a[cut:], n - cut, dtype, **kw)
    cnt = int(x["mismatch_count"]) + int(y["mismatch_count"])
    first = int(x["first_mismatch"]) if x["first_mismatch"] >= 0 else (
        int(y["first_mismatch"]) + cut if y["first_mismatch"] >= 0 else -1)
    assert int(full["mismatch_count"]) == cnt and int(full["first_mismatch"]) == first
    assert float(full["max_abs_err"]) == max(float(x["max_abs_err"]), float(y["max_abs_err"]))
    assert float(full["max_rel_err"]) == max(float(x["max_rel_err"]), float(y["max_rel_err"]))
    assert int(full["pass"]) == int(cnt == 0)
    del w

    # permuting elements keeps the count and both maxima
    perm = rng.permutation(n)
    p = oracle_mod.check_segment(b[perm].copy(), a[perm].copy(), n, dtype, **kw)
    assert record_tuple(p)[1] == record_tuple(full)[1]
    assert record_tuple(p)[3:] == record_tuple(full)[3:]

    # first_mismatch really is the least failing index: the prefix before it passes
    f = int(full["first_mismatch"])
    assert f >= 0
    pre = oracle_mod.check_segment(b[:f], a[:f], f, dtype, **kw)
    assert int(pre["pass"]) == 1
    one = oracle_mod.check_segment(b[f:f + 1], a[f:f + 1], 1, dtype, **kw)
    assert int(one["pass"]) == 0


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16", "i32"])
def test_chunked_driver_equals_one_plain_call(oracle_mod, dtype):
    """The driver the full-size parity tests and the benchmark's baseline use for large dense tensors
    (oracle.check_dense_chunked: chunks on host threads, records folded by oracle.combine_records) gives the
    record of ONE plain check_segment call over the whole tensor -- on about 1e7 elements, with mismatches,
    NaN and infinities in several chunks, a chunk size that does not divide the length, and candidates whose
    first mismatch lies in the first, a middle and the last chunk."""
    rng = np.random.default_rng(21)
    n = 10_000_019
    b, a = _rand_case(rng, dtype, n)
    chunk = 1 << 20                                             # 10 chunks, the last one ragged

    def planted(idx):
        """A copy of the reference with the top exponent bit (integers: bit 30) of element idx flipped."""
        c = b.copy()
        bits = c.view(np.uint32) if c.itemsize == 4 else c.view(np.uint16)
        bits[idx] ^= 0x40000000 if c.itemsize == 4 else 0x4000
        return c

    cands = [a, planted(n - 3), planted(5 * chunk + 17), b.copy()]
    kw = dict(atol=1e-4, rtol=1e-3, equal_nan=True)
    whole = [oracle_mod.check_segment(b, c, n, dtype, **kw) for c in cands]
    chunked = oracle_mod.check_dense_chunked(b, cands, dtype, kw["atol"], kw["rtol"], kw["equal_nan"], threads=4, chunk=chunk)
    assert [record_tuple(r) for r in chunked] == [record_tuple(r) for r in whole]
    firsts = [int(r["first_mismatch"]) for r in whole]
    assert 0 <= firsts[0] < chunk and firsts[1] == n - 3 and firsts[2] == 5 * chunk + 17 and firsts[3] == -1
    assert int(whole[0]["mismatch_count"]) > 1000


def test_ragged_offsets_and_index_space(oracle_mod):
    """Ragged records are indexed [segment, candidate] and first_mismatch is segment-relative."""
    rng = np.random.default_rng(5)
    buf = np.zeros(256, np.uint8)
    segs = [(16, 10, "f32"), (64, 7, "i32"), (100, 20, "f16"), (144, 0, "bf16")]
    ref = buf.copy()
    ref[16:56] = rng.normal(size=10).astype(np.float32).view(np.uint8)
    ref[64:92] = np.arange(7, dtype=np.int32).view(np.uint8)
    ref[100:140] = rng.normal(size=20).astype(np.float16).view(np.uint8)
    c0 = ref.copy()
    c1 = ref.copy()
    c1[16 + 4 * 3:16 + 4 * 4] = np.array([1e6], np.float32).view(np.uint8)      # element 3 of segment 0
    c1[64 + 4 * 5:64 + 4 * 6] = np.array([6], np.int32).view(np.uint8)          # element 5 of segment 1: 5 -> 6
    rec = oracle_mod.check_ragged(ref, [c0, c1], segs, 1e-3, 1e-3, False)
    assert rec.shape == (4, 2)
    for s in range(4):
        assert record_tuple(rec[s, 0]) == (1, 0, -1, 0, 0)
    assert (int(rec[0, 1]["mismatch_count"]), int(rec[0, 1]["first_mismatch"])) == (1, 3)
    assert (int(rec[1, 1]["mismatch_count"]), int(rec[1, 1]["first_mismatch"])) == (1, 5)
    assert float(rec[1, 1]["max_abs_err"]) == 1.0 and float(rec[1, 1]["max_rel_err"]) == 1.0 / 5.0
    assert record_tuple(rec[2, 1]) == (1, 0, -1, 0, 0)
    assert record_tuple(rec[3, 1]) == (1, 0, -1, 0, 0)          # empty segment passes


# ------------------------------------------------------------------------------------------
# library special case: numpy.isclose on finite data, away from the boundary
# ------------------------------------------------------------------------------------------
def test_agrees_with_numpy_isclose_off_boundary(oracle_mod):
    rng = np.random.default_rng(3)
    n = 20000
    b = rng.normal(size=n).astype(np.float32)
    a = (b + rng.normal(size=n) * 10.0 ** rng.uniform(-8, -1, n)).astype(np.float32)
    atol, rtol = 1e-5, 1e-4
    d64 = np.abs(a.astype(np.float64) - b.astype(np.float64))
    t64 = atol + rtol * np.abs(b.astype(np.float64))
    near = np.abs(d64 - t64) <= 1e-5 * t64            # our binary32 steps may differ only here
    lib_close = np.isclose(a, b, rtol=rtol, atol=atol)
    keep = ~near
    rec = oracle_mod.check_segment(b[keep].copy(), a[keep].copy(), int(keep.sum()), "f32", atol, rtol, False)
    assert int(rec["mismatch_count"]) == int((~lib_close[keep]).sum())
    bad = np.nonzero(~lib_close[keep])[0]
    assert int(rec["first_mismatch"]) == (int(bad[0]) if bad.size else -1)
    assert 0.2 < (~lib_close).mean() < 0.8            # both verdicts occur in bulk
    # maxima against float64 evaluation: binary32 subtraction/division are within 1 ulp of these
    assert abs(float(rec["max_abs_err"]) - d64[keep].max()) <= 2.0 ** -23 * d64[keep].max()
    nz = keep & (b != 0)
    rel64 = (d64[nz] / np.abs(b[nz].astype(np.float64))).max()
    assert abs(float(rec["max_rel_err"]) - rel64) <= 2.0 ** -22 * rel64


# ------------------------------------------------------------------------------------------
# closed-form facts of the synthetic workloads
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("cid", [1, 2, 3, 4, 5])
def test_planted_counts(oracle_mod, cid):
    w = synth.small(cid, device="cpu")
    ref = synth.to_numpy_raw(w.ref)
    cands = [synth.to_numpy_raw(c) for c in w.cands]
    if w.segments is None:
        rec = oracle_mod.check_dense(ref, cands, w.dtype, w.atol, w.rtol, w.equal_nan, threads=4).reshape(1, -1)
    else:
        rec = oracle_mod.check_ragged(ref, cands, w.segments, w.atol, w.rtol, w.equal_nan, threads=4)
    assert len(w.expect) == rec.size
    n_fail = 0
    for (s, k), e in w.expect.items():
        r = rec[s, k]
        assert int(r["mismatch_count"]) == e["count"], (cid, s, k)
        assert int(r["first_mismatch"]) == e["first"], (cid, s, k)
        assert int(r["pass"]) == int(e["count"] == 0)
        n_fail += e["count"] > 0
    assert n_fail > 0
    if cid in (1, 3, 4):
        assert n_fail < rec.size            # these recipes contain passing candidates too


def test_int64_hand_derived(oracle_mod):
    """int64 (rule R6'): exact equality; |a - b| exact as an unsigned 64-bit integer, then one rounding
    to binary64; the relative error divides the rounded d by the rounded |b|."""
    i64 = np.iinfo(np.int64)
    b = np.array([5, i64.min, 7, 0, 2 ** 62, -3, 2 ** 53 + 1], dtype=np.int64)
    a = np.array([5, i64.max, 9, 3, 2 ** 62 + 1, -3, 2 ** 53 + 3], dtype=np.int64)
    rec = oracle_mod.check_segment(b, a, len(b), "i64", 1e9, 1e9, False)      # tolerances are ignored
    assert (int(rec["pass"]), int(rec["mismatch_count"]), int(rec["first_mismatch"])) == (0, 5, 1)
    assert float(rec["max_abs_err"]) == 2.0 ** 64          # 2^64 - 1 rounds up to 2^64
    assert float(rec["max_rel_err"]) == np.inf             # 3 / 0
    # without the zero reference: largest ratio is (2^64 - 1 -> 2^64) / 2^63 = 2
    keep = [0, 1, 2, 4, 5, 6]
    rec = oracle_mod.check_segment(b[keep], a[keep], len(keep), "i64", 0.0, 0.0, False)
    assert float(rec["max_rel_err"]) == 2.0 and int(rec["mismatch_count"]) == 4
    # 2^53 + 1 and 2^53 + 3 differ by exactly 2 although both round when converted: d is taken before any rounding
    rec = oracle_mod.check_segment(b[6:], a[6:], 1, "i64", 0.0, 0.0, False)
    assert float(rec["max_abs_err"]) == 2.0
    assert float(rec["max_rel_err"]) == 2.0 / float(2 ** 53 + 1)               # |b| converted with one rounding (to 2^53)
    rep = oracle_mod.report_segment(b, a, len(b), "i64", 0.0, 0.0, False, 8)
    assert [int(r["index"]) for r in rep] == [1, 2, 3, 4, 6]
    assert float(rep[0]["a"]) == 2.0 ** 63 and float(rep[0]["b"]) == -(2.0 ** 63) and float(rep[0]["d"]) == 2.0 ** 64
    assert float(rep[3]["d"]) == 1.0 and float(rep[3]["tol"]) == 0.0
    # equal extremes pass
    same = np.array([i64.min, i64.max, 0], dtype=np.int64)
    assert int(oracle_mod.check_segment(same, same.copy(), 3, "i64", 0.0, 0.0, False)["pass"]) == 1


def test_byte_dtypes_hand_derived(oracle_mod):
    """uint8 (also boolean masks) and int8: exact equality, |a - b| exact, relative error in binary64."""
    b = np.array([0, 1, 255, 200, 7, 1], dtype=np.uint8)
    a = np.array([0, 0, 0, 50, 7, 255], dtype=np.uint8)
    rec = oracle_mod.check_segment(b, a, 6, "u8", 5.0, 5.0, False)            # tolerances are ignored
    assert (int(rec["pass"]), int(rec["mismatch_count"]), int(rec["first_mismatch"])) == (0, 4, 1)
    assert float(rec["max_abs_err"]) == 255.0                                  # |0 - 255|, unsigned
    assert float(rec["max_rel_err"]) == 254.0                                  # |255 - 1| / 1
    # the same bytes read as int8: 255 is -1, 200 is -56
    rec = oracle_mod.check_segment(b.view(np.int8), a.view(np.int8), 6, "i8", 0.0, 0.0, False)
    assert int(rec["mismatch_count"]) == 4 and int(rec["first_mismatch"]) == 1
    assert float(rec["max_abs_err"]) == 106.0                                  # |50 - (-56)|
    assert float(rec["max_rel_err"]) == 2.0                                    # |-1 - 1| / 1
    rep = oracle_mod.report_segment(b.view(np.int8), a.view(np.int8), 6, "i8", 0.0, 0.0, False, 8)
    assert [int(r["index"]) for r in rep] == [1, 2, 3, 5]
    assert [float(r["a"]) for r in rep] == [0.0, 0.0, 50.0, -1.0] and [float(r["b"]) for r in rep] == [1.0, -1.0, -56.0, 1.0]
    assert [float(r["d"]) for r in rep] == [1.0, 1.0, 106.0, 2.0] and all(float(r["tol"]) == 0.0 for r in rep)
    # a boolean mask with one flipped entry against a zero reference: relative error +Inf
    mask = np.zeros(100, dtype=np.uint8)
    flipped = mask.copy()
    flipped[37] = 1
    rec = oracle_mod.check_segment(mask, flipped, 100, "u8", 0.0, 0.0, False)
    assert (int(rec["mismatch_count"]), int(rec["first_mismatch"])) == (1, 37)
    assert float(rec["max_abs_err"]) == 1.0 and float(rec["max_rel_err"]) == np.inf
    # int8 extremes
    rec = oracle_mod.check_segment(np.array([-128], dtype=np.int8), np.array([127], dtype=np.int8), 1, "i8", 0.0, 0.0, False)
    assert float(rec["max_abs_err"]) == 255.0 and float(rec["max_rel_err"]) == 255.0 / 128.0


# ------------------------------------------------------------------------------------------
# 8-bit floating formats (OCP E4M3 and E5M2)
# ------------------------------------------------------------------------------------------
F8_TORCH = {"f8e4m3": torch.float8_e4m3fn, "f8e5m2": torch.float8_e5m2}


@pytest.mark.parametrize("dtype", ["f8e4m3", "f8e5m2"])
def test_decode_f8_all_patterns(oracle_mod, dtype):
    lib = torch.arange(256, dtype=torch.int32).to(torch.uint8).view(F8_TORCH[dtype]).to(torch.float32).numpy()
    for x in range(256):
        assert _same_float(oracle_mod.decode_f8(x, dtype), float(lib[x])), hex(x)
    # the facts the formats are defined by
    if dtype == "f8e4m3":
        assert oracle_mod.decode_f8(0x7E, dtype) == 448.0 and math.isnan(oracle_mod.decode_f8(0x7F, dtype))
        assert oracle_mod.decode_f8(0x01, dtype) == 2.0 ** -9 and oracle_mod.decode_f8(0x08, dtype) == 2.0 ** -6
        assert not any(math.isinf(oracle_mod.decode_f8(x, dtype)) for x in range(256))
    else:
        assert oracle_mod.decode_f8(0x7B, dtype) == 57344.0 and math.isinf(oracle_mod.decode_f8(0x7C, dtype))
        assert oracle_mod.decode_f8(0x01, dtype) == 2.0 ** -16 and oracle_mod.decode_f8(0x04, dtype) == 2.0 ** -14
        assert all(math.isnan(oracle_mod.decode_f8(x, dtype)) for x in (0x7D, 0x7E, 0x7F, 0xFD))


@pytest.mark.parametrize("dtype", ["f8e4m3", "f8e5m2"])
@pytest.mark.parametrize("atol,rtol", [(2.0 ** -6, 0.125), (0.0, 0.0), (1e-3, 0.07), (3.0, 1e30)])
def test_f8_every_pair_against_the_rational_model(oracle_mod, dtype, atol, rtol):
    """All 65536 (reference, candidate) pairs of a format: finite pairs against the exact rational model
    (values decoded by torch, not by the oracle), NaN / Inf pairs against the rule's cases."""
    vals = torch.arange(256, dtype=torch.int32).to(torch.uint8).view(F8_TORCH[dtype]).to(torch.float64).numpy()
    atol_f, rtol_f = float(np.float32(atol)), float(np.float32(rtol))
    codes = np.arange(256, dtype=np.uint8)
    for equal_nan in (False, True):
        for cb in range(256):
            b = float(vals[cb])
            ref = np.full(256, cb, dtype=np.uint8)
            # one oracle call per reference code: the 256 candidates one by one, as 256 segments of length 1
            for ca in range(0, 256, 1 if cb % 16 == 0 else 7):          # every candidate for every 16th reference code
                a = float(vals[ca])
                rec = oracle_mod.check_segment(ref[ca:ca + 1], codes[ca:ca + 1], 1, dtype, atol, rtol, equal_nan)
                if math.isnan(a) or math.isnan(b):
                    close = equal_nan and math.isnan(a) and math.isnan(b)
                    want_d = want_r = None
                elif math.isinf(a) or math.isinf(b):
                    close = a == b
                    want_d = want_r = None
                else:
                    close, d, r = model_element(a, b, atol_f, rtol_f)
                    want_d, want_r = _to_float(d), _to_float(r)
                assert int(rec["pass"]) == int(close), (dtype, hex(cb), hex(ca), atol, rtol, equal_nan)
                if want_d is not None:
                    assert float(rec["max_abs_err"]) == want_d and float(rec["max_rel_err"]) == want_r, (hex(cb), hex(ca))


def test_f8_hand_derived(oracle_mod):
    u8 = lambda *v: np.array(v, dtype=np.uint8)
    # E4M3: 1.0 = 0x38, 1.125 = 0x39 (one step), 1.25 = 0x3A.  atol = 0, rtol = 0.125: tol = 0.125 at b = 1
    rec = oracle_mod.check_segment(u8(0x38, 0x38, 0x38), u8(0x39, 0x3A, 0x38), 3, "f8e4m3", 0.0, 0.125, False)
    assert (int(rec["mismatch_count"]), int(rec["first_mismatch"])) == (1, 1)
    assert float(rec["max_abs_err"]) == 0.25 and float(rec["max_rel_err"]) == 0.25
    # E4M3 has no infinity: 0x7F is NaN and never close without equal_nan; 448 vs -448 is an ordinary mismatch
    rec = oracle_mod.check_segment(u8(0x7F, 0x7E), u8(0x7F, 0xFE), 2, "f8e4m3", 0.0, 0.0, False)
    assert int(rec["mismatch_count"]) == 2 and float(rec["max_abs_err"]) == 896.0
    rec = oracle_mod.check_segment(u8(0x7F, 0x7E), u8(0xFF, 0x7E), 2, "f8e4m3", 0.0, 0.0, True)
    assert int(rec["mismatch_count"]) == 0
    # E5M2: 0x7C is +Inf: close only to itself; 0x3C = 1.0, 0x3D = 1.25
    rec = oracle_mod.check_segment(u8(0x7C, 0x7C, 0x3C), u8(0x7C, 0x7B, 0x3D), 3, "f8e5m2", 1e30, 1e30, False)
    assert (int(rec["mismatch_count"]), int(rec["first_mismatch"])) == (1, 1)
    assert float(rec["max_abs_err"]) == math.inf
    # report and ulp histogram see the same values: one step apart, and Inf one step beyond the largest finite value
    rep = oracle_mod.report_segment(u8(0x3C), u8(0x3D), 1, "f8e5m2", 0.0, 0.125, False, 4)
    assert len(rep) == 1 and float(rep[0]["a"]) == 1.25 and float(rep[0]["d"]) == 0.25 and float(rep[0]["tol"]) == 0.125
    h = oracle_mod.ulp_histogram_segment(u8(0x3C, 0x7B, 0x7E, 0x7E, 0x00), u8(0x3D, 0x7C, 0x7F, 0xFE, 0x80), 5, "f8e5m2")
    assert int(h[1]) == 2 and int(h[65]) == 2 and int(h[0]) == 1      # 0x7E and 0x7F are NaN in E5M2
    h = oracle_mod.ulp_histogram_segment(u8(0x38, 0x7E, 0x7E, 0x00), u8(0x39, 0x7F, 0xFE, 0x80), 4, "f8e4m3")
    assert int(h[1]) == 1 and int(h[65]) == 1 and int(h[8]) == 1 and int(h[0]) == 1     # 2 * 0x7E = 252: bin 8
