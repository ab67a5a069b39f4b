"""Pins of the oracle's ulp-distance histogram (oracle_ulp_histogram_segment), CPU only.

The histogram is the second half of the numeric error trace for the Reflector (GEAK sections 4.1 and
4.2); the paper does not define it, the reading (rules U1-U4) is in oracle/geak_oracle.c.  None of
the pins looks at a bit pattern the way the oracle does:
  * binary16 / bfloat16: the ladder is built by decoding all 65536 patterns with torch, sorting the
    values and merging the two zeros; the distance is a difference of positions on it;
  * binary32 / binary64: small distances are counted by walking numpy.nextafter; any distance comes
    from a closed form on the value (math.frexp and exact fractions, no bit casts);
  * hand-derived cases, and the invariants (bins sum to numel, symmetry, a copy sits in bin 0)."""
import math
from fractions import Fraction

import numpy as np
import pytest
import torch


def _bins_of(distances, nan_count=0):
    out = np.zeros(66, dtype=np.uint64)
    for d in distances:
        out[int(d).bit_length()] += 1
    out[65] += nan_count
    return out


# ---- 16-bit formats: the ladder by sorting -------------------------------------------------------
def _ladder(torch_dtype):
    bits = np.arange(65536, dtype=np.int64)
    vals = torch.from_numpy(bits.astype(np.uint16).view(np.int16)).view(torch_dtype).to(torch.float64).numpy()
    finite_or_inf = ~np.isnan(vals)
    rungs = np.unique(vals[finite_or_inf])              # sorted; -0 and +0 compare equal and merge
    pos = np.full(65536, -1, dtype=np.int64)
    pos[finite_or_inf] = np.searchsorted(rungs, vals[finite_or_inf])
    return pos                                          # position of every pattern on the ladder, -1 for NaN


@pytest.mark.parametrize("dtype,torch_dtype", [("f16", torch.float16), ("bf16", torch.bfloat16)])
def test_16bit_against_sorted_ladder(oracle_mod, dtype, torch_dtype):
    pos = _ladder(torch_dtype)
    rng = np.random.default_rng(1)
    n = 200000
    b = rng.integers(0, 65536, n).astype(np.uint16)
    a = rng.integers(0, 65536, n).astype(np.uint16)
    near = rng.random(n) < 0.5                          # half of the pairs a few patterns apart
    a[near] = (b[near].astype(np.int64) + rng.integers(-5, 6, int(near.sum()))).astype(np.uint16)
    # every pattern against its neighbours and against the two zeros, so that all rungs appear
    allp = np.arange(65536, dtype=np.int64).astype(np.uint16)
    b = np.concatenate([b, allp, allp, allp])
    a = np.concatenate([a, np.roll(allp, 1), np.zeros(65536, np.uint16), np.full(65536, 0x8000, np.uint16)])
    pa, pb = pos[a], pos[b]
    isnan = (pa < 0) | (pb < 0)
    want = _bins_of(np.abs(pa[~isnan] - pb[~isnan]), int(isnan.sum()))
    got = oracle_mod.ulp_histogram_segment(b, a, b.size, dtype)
    assert (got == want).all(), (got, want)
    assert int(got.sum()) == b.size


# ---- 32- and 64-bit formats ----------------------------------------------------------------------
def _walk(x, y, np_t, limit=400):
    """Number of numpy.nextafter steps from x to y (both of type np_t); None beyond `limit`."""
    steps = 0
    x, y = np_t(x), np_t(y)
    while x != y:
        x = np.nextafter(x, y)
        steps += 1
        if steps > limit:
            return None
    return steps


def _count(x, p, emin):
    """Number of values of the format (precision p, least normal exponent emin) in (0, |x|]:
    subnormals and the least normal are k * 2^(emin - p + 1), k = 1 .. 2^(p-1); binade E holds
    2^E * (1 + j / 2^(p-1)), j = 0 .. 2^(p-1) - 1; infinity is one past the largest finite value."""
    x = abs(x)
    if x == 0:
        return 0
    if math.isinf(x):
        emax = -emin + 1
        return (emax - emin + 1) * 2 ** (p - 1) + 2 ** (p - 1)
    m, e = math.frexp(x)                                # x = m * 2^e, 0.5 <= m < 1
    E = e - 1
    if E < emin:
        k = Fraction(x) / Fraction(2) ** (emin - p + 1)
        assert k.denominator == 1
        return int(k)
    j = (Fraction(x) / Fraction(2) ** E - 1) * 2 ** (p - 1)
    assert j.denominator == 1
    return 2 ** (p - 1) + (E - emin) * 2 ** (p - 1) + int(j)


def _distance_closed_form(a, b, p, emin):
    if (math.copysign(1.0, a) < 0) == (math.copysign(1.0, b) < 0) or a == 0 or b == 0:
        same = (math.copysign(1.0, a) < 0) == (math.copysign(1.0, b) < 0)
        return abs(_count(a, p, emin) - _count(b, p, emin)) if same else _count(a, p, emin) + _count(b, p, emin)
    return _count(a, p, emin) + _count(b, p, emin)


FORMATS = {"f32": (np.float32, 24, -126), "f64": (np.float64, 53, -1022)}


@pytest.mark.parametrize("dtype", ["f32", "f64"])
def test_closed_form_agrees_with_nextafter_walk(dtype):
    """The closed form used below is itself checked against counting steps."""
    np_t, p, emin = FORMATS[dtype]
    tiny = float(np.nextafter(np_t(0), np_t(1)))
    fmax = float(np.finfo(np_t).max)
    rng = np.random.default_rng(2)
    bases = [0.0, -0.0, tiny, -tiny, float(np.finfo(np_t).tiny), 1.0, 2.0, -1.0, fmax, -fmax, 3 * tiny, 0.75]
    bases += [float(np_t(rng.normal() * 10.0 ** rng.integers(-30, 30))) for _ in range(30)]
    for x in bases:
        for steps in (0, 1, 2, 3, 7, 100):
            for direction in (np.inf, -np.inf):
                y = np_t(x)
                for _ in range(steps):
                    y = np.nextafter(y, np_t(direction))
                assert _walk(x, y, np_t) == _distance_closed_form(float(x), float(y), p, emin), (x, float(y))


@pytest.mark.parametrize("dtype", ["f32", "f64"])
def test_wide_formats_against_closed_form(oracle_mod, dtype):
    np_t, p, emin = FORMATS[dtype]
    rng = np.random.default_rng(3)
    n = 4000
    info = np.finfo(np_t)
    b = (rng.normal(size=n) * 10.0 ** rng.integers(-40 if dtype == "f32" else -300, 38 if dtype == "f32" else 300, n)).astype(np_t)
    a = (b * (1 + rng.normal(size=n) * 10.0 ** rng.integers(-17, 1, n))).astype(np_t)
    far = rng.random(n) < 0.2
    a[far] = (rng.normal(size=int(far.sum())) * 10.0 ** rng.integers(-30, 30, int(far.sum()))).astype(np_t)
    pool = np.array([0.0, -0.0, np.inf, -np.inf, info.max, -info.max, info.tiny, -info.tiny,
                     np.nextafter(np_t(0), np_t(1)), -np.nextafter(np_t(0), np_t(1)), np.nan], dtype=np_t)
    for arr in (a, b):
        sp = rng.random(n) < 0.1
        arr[sp] = rng.choice(pool, int(sp.sum()))
    steps = rng.random(n) < 0.3                         # a few steps apart, by nextafter
    a[steps] = np.nextafter(b[steps], np_t(np.inf))
    isnan = np.isnan(a) | np.isnan(b)
    dist = [_distance_closed_form(float(x), float(y), p, emin) for x, y in zip(a[~isnan], b[~isnan])]
    want = _bins_of(dist, int(isnan.sum()))
    got = oracle_mod.ulp_histogram_segment(b, a, n, dtype)
    assert (got == want).all(), (got, want)
    # element by element as well, so that two errors cannot cancel inside a bin count
    for x, y in list(zip(a, b))[:600]:
        one = oracle_mod.ulp_histogram_segment(np.array([y], np_t), np.array([x], np_t), 1, dtype)
        if math.isnan(float(x)) or math.isnan(float(y)):
            assert int(one[65]) == 1
        else:
            assert int(one[_distance_closed_form(float(x), float(y), p, emin).bit_length()]) == 1


# ---- hand-derived cases --------------------------------------------------------------------------
def _only_bin(h):
    nz = np.nonzero(h)[0]
    assert len(nz) == 1 and int(h[nz[0]]) == 1
    return int(nz[0])


def test_hand_derived(oracle_mod):
    H = oracle_mod.ulp_histogram_segment
    f32 = lambda v: np.array([v], dtype=np.float32)
    f64 = lambda v: np.array([v], dtype=np.float64)
    u16 = lambda v: np.array([v], dtype=np.uint16)
    # binary32: 2^23 values per binade; one step; the zeros coincide; the least subnormals straddle zero
    assert _only_bin(H(f32(1.0), f32(2.0), 1, "f32")) == 24
    assert _only_bin(H(f32(1.0), f32(1.0 + 2.0 ** -23), 1, "f32")) == 1
    assert _only_bin(H(f32(1.0), f32(1.0 + 3 * 2.0 ** -23), 1, "f32")) == 2       # 3 steps: bin [2, 4)
    assert _only_bin(H(f32(1.0), f32(1.0 + 4 * 2.0 ** -23), 1, "f32")) == 3       # 4 steps: bin [4, 8)
    assert _only_bin(H(f32(0.0), f32(-0.0), 1, "f32")) == 0
    assert _only_bin(H(f32(2.0 ** -149), f32(-2.0 ** -149), 1, "f32")) == 2       # 2 steps
    assert _only_bin(H(f32(np.finfo(np.float32).max), f32(np.inf), 1, "f32")) == 1
    assert _only_bin(H(f32(-np.inf), f32(np.inf), 1, "f32")) == 32               # 2 * 0x7F800000 = 0xFF000000
    assert _only_bin(H(f32(np.inf), f32(np.inf), 1, "f32")) == 0
    for v in (1.0, np.inf, np.nan):
        assert _only_bin(H(f32(np.nan), f32(v), 1, "f32")) == 65
        assert _only_bin(H(f32(v), f32(np.nan), 1, "f32")) == 65
    # binary16: 1024 values per binade; bfloat16: 128; binary64: 2^52
    assert _only_bin(H(u16(0x3C00), u16(0x4000), 1, "f16")) == 11
    assert _only_bin(H(u16(0x3F80), u16(0x4000), 1, "bf16")) == 8
    assert _only_bin(H(u16(0x7C00), u16(0xFC00), 1, "f16")) == 16                # 2 * 0x7C00 = 0xF800
    assert _only_bin(H(u16(0x7F80), u16(0x7F81), 1, "bf16")) == 65               # a NaN next to +Inf
    assert _only_bin(H(u16(0x7BFF), u16(0x7C00), 1, "f16")) == 1                 # largest finite to +Inf
    assert _only_bin(H(f64(1.0), f64(2.0), 1, "f64")) == 53
    assert _only_bin(H(f64(-np.inf), f64(np.inf), 1, "f64")) == 64               # 2 * 0x7FF0000000000000
    assert _only_bin(H(f64(5e-324), f64(-5e-324), 1, "f64")) == 2
    # integers: |a - b| exact
    i = lambda v, t: np.array([v], dtype=t)
    assert _only_bin(H(i(-2 ** 31, np.int32), i(2 ** 31 - 1, np.int32), 1, "i32")) == 32
    assert _only_bin(H(i(-2 ** 63, np.int64), i(2 ** 63 - 1, np.int64), 1, "i64")) == 64
    assert _only_bin(H(i(2 ** 62, np.int64), i(2 ** 62 + 1, np.int64), 1, "i64")) == 1
    assert _only_bin(H(i(7, np.int64), i(7, np.int64), 1, "i64")) == 0
    assert _only_bin(H(i(0, np.uint8), i(255, np.uint8), 1, "u8")) == 8
    assert _only_bin(H(i(-128, np.int8), i(127, np.int8), 1, "i8")) == 8
    assert _only_bin(H(i(-1, np.int8), i(1, np.int8), 1, "i8")) == 2
    assert int(H(f32(1.0), f32(1.0), 0, "f32").sum()) == 0                       # empty segment


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16", "i32", "i64", "u8", "i8", "f64"])
def test_invariants(oracle_mod, dtype):
    rng = np.random.default_rng(4)
    n = 5000
    np_t = {"f32": np.uint32, "f16": np.uint16, "bf16": np.uint16, "i32": np.int32, "i64": np.int64,
            "u8": np.uint8, "i8": np.int8, "f64": np.uint64}[dtype]
    info = np.iinfo(np_t)
    b = rng.integers(info.min, info.max, n, dtype=np_t, endpoint=True)
    a = rng.integers(info.min, info.max, n, dtype=np_t, endpoint=True)
    h_ab = oracle_mod.ulp_histogram_segment(b, a, n, dtype)
    h_ba = oracle_mod.ulp_histogram_segment(a, b, n, dtype)
    assert int(h_ab.sum()) == n and (h_ab == h_ba).all()                          # U4, symmetry
    h_bb = oracle_mod.ulp_histogram_segment(b, b, n, dtype)
    assert int(h_bb[0]) + int(h_bb[65]) == n                                      # a copy: distance 0, or NaN
    if dtype in ("i32", "i64", "u8", "i8"):
        assert int(h_bb[65]) == 0 and int(h_ab[65]) == 0
    # concatenation: the histogram of two halves adds up
    w = b.itemsize
    h1 = oracle_mod.ulp_histogram_segment(b, a, n // 2, dtype)
    h2 = oracle_mod.ulp_histogram_segment(b, a, n - n // 2, dtype, ref_byte_offset=(n // 2) * w)
    assert (h1 + h2 == h_ab).all()


@pytest.mark.parametrize("dtype,torch_dtype", [("f8e4m3", torch.float8_e4m3fn), ("f8e5m2", torch.float8_e5m2)])
def test_8bit_every_pair_against_sorted_ladder(oracle_mod, dtype, torch_dtype):
    vals = torch.arange(256, dtype=torch.int32).to(torch.uint8).view(torch_dtype).to(torch.float64).numpy()
    ok = ~np.isnan(vals)
    rungs = np.unique(vals[ok])                          # sorted; the two zeros merge
    pos = np.full(256, -1, dtype=np.int64)
    pos[ok] = np.searchsorted(rungs, vals[ok])
    b = np.repeat(np.arange(256, dtype=np.uint8), 256)
    a = np.tile(np.arange(256, dtype=np.uint8), 256)
    pa, pb = pos[a], pos[b]
    isnan = (pa < 0) | (pb < 0)
    want = _bins_of(np.abs(pa[~isnan] - pb[~isnan]), int(isnan.sum()))
    got = oracle_mod.ulp_histogram_segment(b, a, b.size, dtype)
    assert (got == want).all(), (got, want)
    for cb, ca in [(0x00, 0x80), (0x01, 0x81), (0x38, 0x39), (0x7B, 0x7C), (0x7E, 0xFE)]:
        one = oracle_mod.ulp_histogram_segment(np.array([cb], np.uint8), np.array([ca], np.uint8), 1, dtype)
        if pos[cb] < 0 or pos[ca] < 0:
            assert int(one[65]) == 1
        else:
            assert int(one[int(abs(pos[cb] - pos[ca])).bit_length()]) == 1
