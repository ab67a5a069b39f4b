"""Pins of the oracle's block-scaled (MX) front end: the element tables against what the OCP Microscaling
Formats specification v1.0 states and against the C oracle's own 8-bit decoders, the scale, hand-derived
records, the cases the scale must not touch (NaN, infinities), the overflow reading, and the tie to the plain
checks that the same numbers must give."""
import math

import numpy as np
import pytest

from oracle import mx


def test_e2m1_codes_are_the_sixteen_listed_values():
    # the specification's table of FP4 (E2M1) encodings: magnitudes 0, 0.5, 1, 1.5, 2, 3, 4, 6; bit 3 is the sign
    want = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]
    t = mx.element_table("mxfp4e2m1")
    assert list(t[:8]) == want
    assert list(t[8:]) == [-v for v in want]
    assert math.copysign(1.0, t[8]) == -1.0                       # code 8 is -0


def test_fp8_tables_have_the_stated_extremes_and_specials():
    e4, e5 = mx.element_table("mxfp8e4m3"), mx.element_table("mxfp8e5m2")
    # E4M3: bias 7, no infinities, NaN only at S.1111.111, largest normal 448, least normal 2^-6, least subnormal 2^-9
    assert e4[0x7E] == 448.0 and e4[0xFE] == -448.0
    assert math.isnan(e4[0x7F]) and math.isnan(e4[0xFF]) and np.isnan(e4).sum() == 2 and not np.isinf(e4).any()
    assert e4[0x08] == 2.0 ** -6 and e4[0x01] == 2.0 ** -9 and e4[0x07] == 7 * 2.0 ** -9
    assert e4[0x38] == 1.0 and e4[0x3C] == 1.5 and e4[0x40] == 2.0
    # E5M2: bias 15, infinities at S.11111.00, NaN at S.11111.{01,10,11}, largest normal 57344, least normal 2^-14,
    # least subnormal 2^-16
    assert e5[0x7B] == 57344.0 and e5[0x7C] == math.inf and e5[0xFC] == -math.inf
    assert all(math.isnan(e5[c]) for c in (0x7D, 0x7E, 0x7F, 0xFD, 0xFE, 0xFF)) and np.isnan(e5).sum() == 6
    assert e5[0x04] == 2.0 ** -14 and e5[0x01] == 2.0 ** -16 and e5[0x3C] == 1.0 and e5[0x3E] == 1.5
    # positive codes ascend with the code, in both
    for t, top in ((e4, 0x7E), (e5, 0x7C)):
        assert all(t[c] < t[c + 1] for c in range(top))


def test_fp8_tables_agree_with_the_c_oracles_decoders(oracle_mod):
    """Two decoders written apart (the C oracle's, pinned on its own, and this one) give the same value for
    every code."""
    for fmt, name in (("mxfp8e4m3", "f8e4m3"), ("mxfp8e5m2", "f8e5m2")):
        t = mx.element_table(fmt)
        for c in range(256):
            v = oracle_mod.decode_f8(c, name)
            assert (math.isnan(v) and math.isnan(t[c])) or (v == t[c] and math.copysign(1, v) == math.copysign(1, t[c])), (fmt, c)


def test_int8_elements_are_sixty_fourths():
    t = mx.element_table("mxint8")
    assert t[0] == 0 and t[1] == 1 / 64 and t[64] == 1.0 and t[127] == 127 / 64 and t[128] == -2.0 and t[255] == -1 / 64


def test_scale_byte():
    assert mx.scale_value(127) == 1.0 and mx.scale_value(128) == 2.0 and mx.scale_value(126) == 0.5
    assert mx.scale_value(0) == 2.0 ** -127 and mx.scale_value(254) == 2.0 ** 127 and math.isnan(mx.scale_value(255))


def test_dequantize_by_hand():
    # two blocks of E4M3: 40 elements, the second block ragged (8 elements) with its own scale
    payload = np.zeros(40, np.uint8)
    payload[0], payload[1], payload[2], payload[31] = 0x38, 0xBC, 0x01, 0x7E        # 1, -1.5, 2^-9, 448
    payload[32], payload[39] = 0x40, 0x7F                                           # 2, NaN
    scales = np.array([130, 120], np.uint8)                                          # 8, 2^-7
    v = mx.dequantize(payload, scales, 40, "mxfp8e4m3")
    assert v.dtype == np.float32
    assert v[0] == 8.0 and v[1] == -12.0 and v[2] == 2.0 ** -6 and v[31] == 3584.0 and v[3] == 0.0
    assert v[32] == 2.0 ** -6 and math.isnan(v[39]) and (v[33:39] == 0).all()
    # FP4: element 2j in the low nibble of byte j
    p4 = np.array([0x21, 0xF7], np.uint8)                                            # codes 1, 2, 7, 15
    v4 = mx.dequantize(p4, np.array([128], np.uint8), 4, "mxfp4e2m1")
    assert list(v4) == [1.0, 2.0, 12.0, -12.0]
    # int8
    vi = mx.dequantize(np.array([64, 0x80, 0xFF], np.uint8), np.array([126], np.uint8), 3, "mxint8")
    assert list(vi) == [0.5, -1.0, -1 / 128]


def test_scale_nan_makes_the_whole_block_nan_and_leaves_the_next_alone():
    payload = np.full(64, 0x38, np.uint8)
    payload[5] = 0x00                                             # also a zero becomes NaN
    v = mx.dequantize(payload, np.array([0xFF, 127], np.uint8), 64, "mxfp8e4m3")
    assert np.isnan(v[:32]).all() and (v[32:] == 1.0).all()


def test_specials_of_the_elements_survive_any_scale():
    payload = np.array([0x7C, 0xFC, 0x7D, 0x00, 0x80], np.uint8)     # E5M2: +Inf, -Inf, NaN, +0, -0
    for s in (0, 127, 254):
        v = mx.dequantize(payload, np.array([s], np.uint8), 5, "mxfp8e5m2")
        assert v[0] == math.inf and v[1] == -math.inf and math.isnan(v[2]) and v[3] == 0 and v[4] == 0
        assert math.copysign(1, v[4]) == -1


def test_least_and_greatest_products():
    # the least product 2^-9 * 2^-127 = 2^-136 and E5M2's 2^-16 * 2^-127 = 2^-143 are binary32 subnormals, held exactly;
    # 448 * 2^127 and 57344 * 2^127 exceed binary32 and become infinities of the product's sign
    v = mx.dequantize(np.array([0x01, 0x7E, 0xFE, 0x30], np.uint8), np.array([0], np.uint8), 4, "mxfp8e4m3")
    assert float(v[0]) == 2.0 ** -136 and float(v[1]) == 448 * 2.0 ** -127 and float(v[3]) == 0.5 * 2.0 ** -127
    v = mx.dequantize(np.array([0x01], np.uint8), np.array([0], np.uint8), 1, "mxfp8e5m2")
    assert float(v[0]) == 2.0 ** -143
    v = mx.dequantize(np.array([0x7E, 0xFE, 0x08, 0x3F], np.uint8), np.array([254], np.uint8), 4, "mxfp8e4m3")
    assert v[0] == math.inf and v[1] == -math.inf and float(v[2]) == 2.0 ** 121
    assert float(v[3]) == 1.875 * 2.0 ** 127                      # the largest product that still fits


@pytest.mark.parametrize("fmt", mx.MX_FORMATS)
def test_dequantize_equals_ldexp_in_binary32(fmt):
    """Another route to the same numbers: the element value held as binary32 (every element value is one), scaled
    by the library's ldexp in binary32, for every code and a spread of scales."""
    t = mx.element_table(fmt)
    ncodes = len(t)
    for s in (0, 1, 60, 126, 127, 128, 200, 253, 254):
        n = ncodes
        if mx.MX_BITS[fmt] == 8:
            payload = np.arange(256, dtype=np.uint8)
        elif mx.MX_BITS[fmt] == 6:                                   # codes 0 .. 63 in element order, 48 bytes
            payload = np.frombuffer(sum(c << (6 * c) for c in range(64)).to_bytes(48, "little"), np.uint8)
        else:
            payload = np.array([(2 * j) | ((2 * j + 1) << 4) for j in range(8)], np.uint8)
        scales = np.full((n + 31) // 32, s, np.uint8)
        got = mx.dequantize(payload, scales, n, fmt)
        with np.errstate(over="ignore"):
            want = np.ldexp(t.astype(np.float32), s - 127).astype(np.float32)
        assert np.array_equal(got, want, equal_nan=True), (fmt, s)
        assert (np.signbit(got) == np.signbit(want)).all()


def test_records_by_hand():
    # reference: 1, 2, 3, 4 (E2M1 codes 2, 4, 5, 6) at scale 1; first candidate: the same numbers at scale 2 (the
    # codes of 0.5, 1, 1.5, 2); second candidate: its last element is 3 * 2 = 6 instead of 4
    ref = np.array([0x42, 0x65], np.uint8)
    ref_s = np.array([127], np.uint8)
    same = np.array([0x21, 0x43], np.uint8)
    same_s = np.array([128], np.uint8)
    r = mx.check_segment_mx(ref, ref_s, same, same_s, 4, "mxfp4e2m1", 0.0, 0.0, False)
    assert (int(r["pass"]), int(r["mismatch_count"]), int(r["first_mismatch"]), float(r["max_abs_err"])) == (1, 0, -1, 0.0)
    off = np.array([0x21, 0x53], np.uint8)                         # 1, 2, 3, 6
    r = mx.check_segment_mx(ref, ref_s, off, same_s, 4, "mxfp4e2m1", 0.5, 0.25, False)
    # |6 - 4| = 2 > 0.5 + 0.25 * 4 = 1.5: one mismatch at index 3, relative error 2 / 4
    assert (int(r["pass"]), int(r["mismatch_count"]), int(r["first_mismatch"])) == (0, 1, 3)
    assert float(r["max_abs_err"]) == 2.0 and float(r["max_rel_err"]) == 0.5
    r = mx.check_segment_mx(ref, ref_s, off, same_s, 4, "mxfp4e2m1", 1.0, 0.25, False)        # 2 <= 1 + 1: inclusive
    assert int(r["pass"]) == 1 and float(r["max_abs_err"]) == 2.0
    # the candidate's scale alone doubles everything: |2b - b| = b, at indices 0..3 -> 1, 2, 3, 4
    r = mx.check_segment_mx(ref, ref_s, ref, same_s, 4, "mxfp4e2m1", 2.5, 0.0, False)
    assert (int(r["mismatch_count"]), int(r["first_mismatch"]), float(r["max_abs_err"]), float(r["max_rel_err"])) == (2, 2, 4.0, 1.0)


def test_nan_scale_in_records():
    payload = np.full(64, 0x38, np.uint8)
    ok_s, nan_s = np.array([127, 127], np.uint8), np.array([127, 0xFF], np.uint8)
    r = mx.check_segment_mx(payload, ok_s, payload, nan_s, 64, "mxfp8e4m3", 1.0, 1.0, False)
    assert (int(r["mismatch_count"]), int(r["first_mismatch"])) == (32, 32)
    r = mx.check_segment_mx(payload, nan_s, payload, nan_s, 64, "mxfp8e4m3", 1.0, 1.0, False)
    assert int(r["mismatch_count"]) == 32                          # NaN against NaN is no match unless asked for
    r = mx.check_segment_mx(payload, nan_s, payload, nan_s, 64, "mxfp8e4m3", 0.0, 0.0, True)
    assert int(r["pass"]) == 1
    r = mx.check_segment_mx(payload, nan_s, payload, ok_s, 64, "mxfp8e4m3", 0.0, 0.0, True)
    assert int(r["mismatch_count"]) == 32


def test_overflowed_products_compare_as_infinities():
    big = np.array([0x7E, 0x7E], np.uint8)
    s = np.array([254], np.uint8)
    r = mx.check_segment_mx(big, s, big, s, 2, "mxfp8e4m3", 0.0, 0.0, False)
    assert int(r["pass"]) == 1                                     # equal infinities are close
    r = mx.check_segment_mx(big, s, np.array([0x7E, 0x08], np.uint8), s, 2, "mxfp8e4m3", 1e30, 1e-3, False)
    assert (int(r["mismatch_count"]), int(r["first_mismatch"])) == (1, 1)      # Inf against 2^121: no tolerance spans that


@pytest.mark.parametrize("fmt,name", [("mxfp8e4m3", "f8e4m3"), ("mxfp8e5m2", "f8e5m2")])
def test_unit_scales_give_the_plain_fp8_record(oracle_mod, fmt, name):
    """With every scale 2^0 the block-scaled check is the plain 8-bit check of the payload."""
    rng = np.random.default_rng(17)
    n = 5000
    b = rng.integers(0, 256, n).astype(np.uint8)
    a = b.copy()
    idx = rng.random(n) < 0.3
    a[idx] = (b[idx].astype(np.int64) + rng.integers(-2, 3, int(idx.sum()))).astype(np.uint8)
    s = np.full((n + 31) // 32, 127, np.uint8)
    for equal_nan in (False, True):
        r = mx.check_segment_mx(b, s, a, s, n, fmt, 1e-2, 1e-1, equal_nan)
        p = oracle_mod.check_segment(b, a, n, name, 1e-2, 1e-1, equal_nan)
        assert all(r[f] == p[f] or (np.isnan(r[f]) and np.isnan(p[f])) for f in r.dtype.names)


def test_a_common_power_of_two_scales_the_absolute_error_only():
    """Multiplying both tensors' scales by 2^j multiplies every difference and every |b| by 2^j exactly (as long as
    nothing leaves binary32's normal range): max_abs_err scales, max_rel_err and the count under a purely relative
    tolerance stay."""
    rng = np.random.default_rng(23)
    n = 2048
    b = rng.integers(0x20, 0x70, n).astype(np.uint8)              # normal, finite E4M3 magnitudes
    a = (b.astype(np.int64) + rng.integers(-1, 2, n)).astype(np.uint8)
    sb = rng.integers(120, 134, n // 32).astype(np.uint8)
    sa = sb.copy()
    sa[::7] += 1                                                   # some blocks of the candidate are off by 2x
    r0 = mx.check_segment_mx(b, sb, a, sa, n, "mxfp8e4m3", 0.0, 0.125, False)
    r1 = mx.check_segment_mx(b, sb + 20, a, sa + 20, n, "mxfp8e4m3", 0.0, 0.125, False)
    assert int(r0["mismatch_count"]) == int(r1["mismatch_count"]) > 0 and int(r0["first_mismatch"]) == int(r1["first_mismatch"])
    assert float(r1["max_abs_err"]) == float(r0["max_abs_err"]) * 2.0 ** 20
    assert float(r1["max_rel_err"]) == float(r0["max_rel_err"])


def test_fp6_tables_have_the_stated_extremes():
    # the specification's table of FP6 encodings.  E2M3: bias 1, largest normal 7.5, least normal 1, largest subnormal
    # 0.875, least subnormal 0.125.  E3M2: bias 3, largest normal 28, least normal 0.25, largest subnormal 0.1875, least
    # subnormal 0.0625.  Neither has infinities or NaN; bit 5 is the sign.
    a, b = mx.element_table("mxfp6e2m3"), mx.element_table("mxfp6e3m2")
    assert len(a) == 64 and len(b) == 64 and np.isfinite(a).all() and np.isfinite(b).all()
    assert a[0x1F] == 7.5 and a[0x08] == 1.0 and a[0x07] == 0.875 and a[0x01] == 0.125 and a[0x00] == 0.0
    assert b[0x1F] == 28.0 and b[0x04] == 0.25 and b[0x03] == 0.1875 and b[0x01] == 0.0625 and b[0x00] == 0.0
    for t in (a, b):
        assert all(t[c] < t[c + 1] for c in range(31))                       # positive codes ascend with the code
        assert all(t[c + 32] == -t[c] for c in range(32)) and math.copysign(1.0, t[32]) == -1.0
    # every FP6 value is an E4M3 value too (three mantissa bits at most, exponents inside E4M3's range)
    e4 = set(mx.element_table("mxfp8e4m3")[:0x7F].tolist())
    assert set(a[:32].tolist()) <= e4 and set(b[:32].tolist()) <= e4


def test_fp6_codes_are_packed_without_gaps():
    # four codes in three bytes: 0x01, 0x02, 0x03, 0x3F -> bits 000001 | 000010 | 000011 | 111111 from the low end:
    # byte 0 = 01 + low two bits of 0x02 (10) on top = 0x81, byte 1 = high four bits of 0x02 (0000) + low four of 0x03
    # (0011) on top = 0x30, byte 2 = high two bits of 0x03 (00) + 0x3F on top = 0xFC
    payload = np.array([0x81, 0x30, 0xFC], np.uint8)
    assert list(mx.payload_codes(payload, 4, "mxfp6e2m3")) == [0x01, 0x02, 0x03, 0x3F]
    v = mx.dequantize(payload, np.array([128], np.uint8), 4, "mxfp6e2m3")           # scale 2
    assert list(v) == [0.25, 0.5, 0.75, -15.0]
    v = mx.dequantize(payload, np.array([126], np.uint8), 4, "mxfp6e3m2")           # scale 1/2
    assert list(v) == [0.03125, 0.0625, 0.09375, -14.0]
    # a whole block: code i in element i, read back in order
    codes = np.arange(32, dtype=np.int64) * 2 + 1                                   # 1, 3, ..., 63
    number = sum(int(c) << (6 * i) for i, c in enumerate(codes))
    block = np.frombuffer(number.to_bytes(24, "little"), np.uint8)
    assert list(mx.payload_codes(block, 32, "mxfp6e3m2")) == list(codes)


def test_fp6_records_equal_those_of_the_same_numbers_in_e4m3():
    """The same numbers written as FP6 codes and as E4M3 codes must give the same records: the FP6 path against the
    8-bit one, whose decoder is pinned on its own."""
    rng = np.random.default_rng(77)
    for fmt in ("mxfp6e2m3", "mxfp6e3m2"):
        t6, t8 = mx.element_table(fmt), mx.element_table("mxfp8e4m3")
        to8 = {}
        for c8 in range(256):
            if not math.isnan(t8[c8]):
                to8[(float(t8[c8]), math.copysign(1.0, t8[c8]))] = c8
        n = 96
        def pack(codes):
            number = sum(int(c) << (6 * i) for i, c in enumerate(codes))
            return np.frombuffer(number.to_bytes(n * 6 // 8, "little"), np.uint8).copy()
        ref6 = rng.integers(0, 64, n); cand6 = ref6.copy()
        step = rng.random(n) < 0.4
        cand6[step] = (cand6[step] + rng.integers(-2, 3, int(step.sum()))) % 64
        scales_b = rng.integers(120, 135, n // 32).astype(np.uint8); scales_a = scales_b.copy(); scales_a[1] += 1
        ref8 = np.array([to8[(float(t6[c]), math.copysign(1.0, t6[c]))] for c in ref6], np.uint8)
        cand8 = np.array([to8[(float(t6[c]), math.copysign(1.0, t6[c]))] for c in cand6], np.uint8)
        for atol, rtol in ((0.0, 0.0), (0.05, 0.1)):
            r6 = mx.check_segment_mx(pack(ref6), scales_b, pack(cand6), scales_a, n, fmt, atol, rtol, False)
            r8 = mx.check_segment_mx(ref8, scales_b, cand8, scales_a, n, "mxfp8e4m3", atol, rtol, False)
            assert r6 == r8 and r6["mismatch_count"] > 0
