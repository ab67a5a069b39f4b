"""Block-scaled (MX) segments on the GPU against the oracle's front end (oracle/mx.py: every element written
out as the binary32 value it encodes, then the unchanged rule): records and mismatch reports for the three
one-byte element formats, the four-bit one and the two six-bit ones, all payload codes and scale bytes (2^-127, 2^127, NaN among them), candidates whose
payload, scales or both differ, sizes from one block to several work items with every tail shape."""
import numpy as np
import pytest
import torch

from oracle import mx
from paper_2507_23194_amd import binding as B
from test_gpu_parity import _assert_same

pytestmark = pytest.mark.gpu

FORMATS = ["mxfp8e4m3", "mxfp8e5m2", "mxint8", "mxfp4e2m1", "mxfp6e2m3", "mxfp6e3m2"]


def _tensors(rng, fmt, n, K):
    """(payload, scales) of the reference and of K candidates; n elements (the four-bit format: n / 2 payload bytes,
    every byte two codes, so what follows perturbs codes of either half)."""
    nb = n // 32
    n = n * mx.MX_BITS[fmt] // 8                          # payload bytes from here on
    payload = rng.integers(0, 256, n).astype(np.uint8)
    scales = rng.integers(110, 140, nb).astype(np.uint8)
    pick = rng.random(nb)
    scales[pick < 0.04] = 0
    scales[(pick >= 0.04) & (pick < 0.08)] = 254
    scales[(pick >= 0.08) & (pick < 0.11)] = 255
    scales[(pick >= 0.11) & (pick < 0.14)] = rng.integers(0, 255)
    out = [(payload, scales)]
    for k in range(K):
        p, s = payload.copy(), scales.copy()
        if k % 5 == 0:                                     # codes moved by a step or two, some replaced, some signs flipped
            step = rng.random(n) < 0.3
            p[step] = (p[step].astype(np.int64) + rng.integers(-2, 3, int(step.sum()))).astype(np.uint8)
            repl = rng.random(n) < 0.02
            p[repl] = rng.integers(0, 256, int(repl.sum())).astype(np.uint8)
            flip = rng.random(n) < 0.01
            p[flip] ^= 0x80
        elif k % 5 == 1:                                   # the reference itself
            pass
        elif k % 5 == 2:                                   # other scales: off by a factor of two, NaN, NaN removed
            blk = rng.random(nb) < 0.2
            s[blk] = np.clip(s[blk].astype(np.int64) + rng.choice([-1, 1], int(blk.sum())), 0, 254).astype(np.uint8)
            s[rng.random(nb) < 0.03] = 255
            s[(scales == 255) & (rng.random(nb) < 0.5)] = 127
        elif k % 5 == 3:                                   # both
            step = rng.random(n) < 0.1
            p[step] = (p[step].astype(np.int64) + rng.integers(-1, 2, int(step.sum()))).astype(np.uint8)
            blk = rng.random(nb) < 0.1
            s[blk] = rng.integers(0, 256, int(blk.sum())).astype(np.uint8)
        else:                                              # one element, the last
            p[n - 1] ^= 0x10                               # (the high nibble: the four-bit format's last element too)
        out.append((p, s))
    return out


def _pack(tensors_per_segment):
    """One buffer per tensor: for every segment its payload on the 16-byte grid, then its scales right behind.
    Returns (buffers, table entries (payload offset, numel, scale offset))."""
    ntens = len(tensors_per_segment[0])
    parts = [[] for _ in range(ntens)]
    table, off = [], 0
    for seg in tensors_per_segment:
        n, nb = seg[0][0].size, seg[0][1].size            # payload bytes, blocks
        pad = (-(n + nb + 3)) % 16
        table.append((off, nb * 32, off + n + 3))
        for t, (p, s) in enumerate(seg):
            parts[t].append(np.concatenate([p, np.full(3, 0xEE, np.uint8), s, np.full(pad, 0xDD, np.uint8)]))
        off += n + 3 + nb + pad
    return [np.concatenate(p) for p in parts], table


def _gpu(bufs, table, fmts, K, atol, rtol, equal_nan, max_records=6):
    dev = [torch.from_numpy(b.copy()).cuda() for b in bufs]
    ck = B.Checker(mx=[(o, n, so, f) for (o, n, so), f in zip(table, fmts)], num_candidates=K, atol=atol, rtol=rtol,
                   equal_nan=equal_nan, device=0)
    try:
        ck.run(dev[0], dev[1:])
        rec = ck.read().copy()
        rep, cnt = ck.report(dev[0], dev[1:], max_records)
        return rec, rep, cnt
    finally:
        ck.close()


def _compare(oracle_mod, segs, fmts, K, atol, rtol, equal_nan, what):
    bufs, table = _pack(segs)
    rec, rep, cnt = _gpu(bufs, table, fmts, K, atol, rtol, equal_nan)
    cpu = np.zeros((len(segs), K), dtype=rec.dtype)
    for s, seg in enumerate(segs):
        n = seg[0][1].size * 32
        b = mx.dequantize(seg[0][0], seg[0][1], n, fmts[s])
        for k in range(K):
            a = mx.dequantize(seg[k + 1][0], seg[k + 1][1], n, fmts[s])
            r = oracle_mod.check_segment(b, a, n, "f32", atol, rtol, equal_nan)
            for f in cpu.dtype.names:
                cpu[s, k][f] = r[f]
            want = oracle_mod.report_segment(b, a, n, "f32", atol, rtol, equal_nan, 6)
            assert int(cnt[s, k]) == len(want), (what, s, k)
            got = rep[s, k][:len(want)]
            assert (got["index"] == want["index"]).all(), (what, s, k)
            assert all(np.array_equal(got[f], want[f], equal_nan=True) for f in ("a", "b", "d", "tol")), (what, s, k)
    _assert_same(rec, cpu, what)
    return rec


@pytest.mark.parametrize("fmt", FORMATS)
@pytest.mark.parametrize("n", [32, 5 * 32, 1024 + 32, 4096 + 64, 3 * 4096 + 31 * 32, 6 * 4096, 2 * 8192 + 96])
def test_one_segment(oracle_mod, fmt, n):
    print("mx", fmt, n, flush=True)
    rng = np.random.default_rng(8800 + n + FORMATS.index(fmt))
    K = 5
    seg = _tensors(rng, fmt, n, K)
    for equal_nan, atol, rtol in ((False, 1e-2, 0.07), (True, 0.0, 0.0)):
        rec = _compare(oracle_mod, [seg], [fmt], K, atol, rtol, equal_nan, f"{fmt} n={n} equal_nan={equal_nan}")
    assert rec[0, 1]["pass"] == 1                          # equal_nan, zero tolerance: the reference passes against itself


def test_several_segments_of_all_formats(oracle_mod):
    """Formats mixed in one plan, segments of uneven length (a wave's run crosses segments and formats), K = 7
    (tails need batches of four, two and one candidate), per-segment tolerances."""
    print("mx mixed", flush=True)
    rng = np.random.default_rng(8900)
    K = 7
    sizes = [64, 2048, 4096 * 2 + 512, 32, 4096, 1024 + 64, 4096 * 3]
    fmts = [FORMATS[i % len(FORMATS)] for i in range(len(sizes))]
    segs = [_tensors(rng, f, n, K) for f, n in zip(fmts, sizes)]
    bufs, table = _pack(segs)
    tols = [(10.0 ** -(i % 3), 0.05 * (i % 4)) for i in range(len(sizes))]
    dev = [torch.from_numpy(b.copy()).cuda() for b in bufs]
    ck = B.Checker(mx=[(o, n, so, f) for (o, n, so), f in zip(table, fmts)], num_candidates=K, equal_nan=False, device=0, tolerances=tols)
    try:
        ck.run(dev[0], dev[1:])
        rec = ck.read().copy()
        with pytest.raises(B.GeakError) as err:
            ck.ulp_histogram(dev[0], dev[1:])
        assert err.value.status == B.GEAK_EDTYPE
    finally:
        ck.close()
    cpu = np.zeros((len(segs), K), dtype=rec.dtype)
    for s, seg in enumerate(segs):
        for k in range(K):
            r = mx.check_segment_mx(seg[0][0], seg[0][1], seg[k + 1][0], seg[k + 1][1], sizes[s], fmts[s], tols[s][0], tols[s][1], False)
            for f in cpu.dtype.names:
                cpu[s, k][f] = r[f]
    _assert_same(rec, cpu, "mixed formats")


@pytest.mark.parametrize("seed", range(8))
def test_random_block_scaled_plan(oracle_mod, seed):
    """Seeded random plans: a few segments of random format and length (whole blocks, from one block to several
    work items), random candidate count and per-segment tolerances; records and reports against the oracle."""
    rng = np.random.default_rng(9500 + seed)
    nsegs, K = int(rng.integers(1, 7)), int(rng.integers(1, 10))
    fmts = [FORMATS[int(rng.integers(0, len(FORMATS)))] for _ in range(nsegs)]
    sizes = [32 * int(rng.choice([1, int(rng.integers(2, 33)), int(rng.integers(33, 129)), int(rng.integers(129, 400))])) for _ in range(nsegs)]
    print("random block-scaled plan", seed, list(zip(fmts, sizes)), "K", K, flush=True)
    segs = [_tensors(rng, f, n, K) for f, n in zip(fmts, sizes)]
    tols = [(float(rng.choice([0.0, 1e-3, 0.25, 1e30])), float(rng.choice([0.0, 1e-2, 0.125, 3.0]))) for _ in range(nsegs)]
    equal_nan = bool(rng.integers(0, 2))
    bufs, table = _pack(segs)
    dev = [torch.from_numpy(b.copy()).cuda() for b in bufs]
    ck = B.Checker(mx=[(o, n, so, f) for (o, n, so), f in zip(table, fmts)], num_candidates=K, equal_nan=equal_nan, device=0, tolerances=tols)
    try:
        ck.run(dev[0], dev[1:])
        rec = ck.read().copy()
        rep, cnt = ck.report(dev[0], dev[1:], 4)
    finally:
        ck.close()
    cpu = np.zeros((nsegs, K), dtype=rec.dtype)
    for s, seg in enumerate(segs):
        b = mx.dequantize(seg[0][0], seg[0][1], sizes[s], fmts[s])
        for k in range(K):
            a = mx.dequantize(seg[k + 1][0], seg[k + 1][1], sizes[s], fmts[s])
            r = oracle_mod.check_segment(b, a, sizes[s], "f32", tols[s][0], tols[s][1], equal_nan)
            for f in cpu.dtype.names:
                cpu[s, k][f] = r[f]
            want = oracle_mod.report_segment(b, a, sizes[s], "f32", tols[s][0], tols[s][1], equal_nan, 4)
            assert int(cnt[s, k]) == len(want), (seed, s, k)
            got = rep[s, k][:len(want)]
            assert (got["index"] == want["index"]).all(), (seed, s, k)
            assert all(np.array_equal(got[f], want[f], equal_nan=True) for f in ("a", "b", "d", "tol")), (seed, s, k)
    _assert_same(rec, cpu, f"random block-scaled plan {seed}")


@pytest.mark.parametrize("fmt", ["mxfp8e4m3", "mxfp8e5m2"])
def test_the_same_numbers_under_other_scales_pass(oracle_mod, fmt):
    """A candidate that stores every block one binade lower in the payload and one higher in the scale encodes
    the same numbers: it passes with zero tolerance.  (Normal codes only: the payload's exponent field is
    lowered by one.)"""
    print("mx re-encoded", fmt, flush=True)
    rng = np.random.default_rng(9000)
    n = 4096 * 2 + 320
    mbits = 3 if fmt == "mxfp8e4m3" else 2
    exp = rng.integers(2, 14 if fmt == "mxfp8e4m3" else 29, n)
    code = ((rng.integers(0, 2, n) << 7) | (exp << mbits) | rng.integers(0, 1 << mbits, n)).astype(np.uint8)
    scales = rng.integers(90, 160, n // 32).astype(np.uint8)
    lower = (code - (1 << mbits)).astype(np.uint8)
    segs = [[(code, scales), (lower, (scales + 1).astype(np.uint8)), (lower, scales)]]
    rec = _compare(oracle_mod, segs, [fmt], 2, 0.0, 0.0, False, f"{fmt} re-encoded")
    assert rec[0, 0]["pass"] == 1 and rec[0, 0]["max_abs_err"] == 0.0
    assert rec[0, 1]["pass"] == 0 and rec[0, 1]["mismatch_count"] == n and rec[0, 1]["max_rel_err"] == 0.5


def test_extreme_products(oracle_mod):
    """The least products (binary32 subnormals: 2^-9 * 2^-127, int8's 1/64 * 2^-127) and the ones beyond binary32
    (448 * 2^127, -128/64 * 2^127): exact where they fit, infinities where they do not."""
    print("mx extremes", flush=True)
    n = 64
    for fmt in FORMATS:
        nbytes = n * mx.MX_BITS[fmt] // 8
        codes = np.tile(np.array([0x01, 0x7E, 0xFE, 0x00, 0x80, 0x7B, 0x81, 0x08], np.uint8), nbytes // 8)
        cand = codes.copy()
        cand[[1, 9, nbytes - 7]] = [0x7D, 0x02, 0x7D]
        for lo, hi in ((0, 254), (1, 253)):
            s = np.array([lo, hi], np.uint8)
            segs = [[(codes, s), (cand, s), (codes, s[::-1].copy())]]
            _compare(oracle_mod, segs, [fmt], 2, 0.0, 0.25, False, f"{fmt} extremes {lo} {hi}")


def test_mx_plan_argument_errors():
    ok = (0, 64, 100, "mxfp8e4m3")
    st, plan = B.geak_check_plan_mx([ok], None, 2, 0.0, 0.0, False, 0)
    assert st == B.GEAK_OK
    B.geak_check_destroy(plan)
    for bad, code in (((8, 64, 100, "mxfp8e4m3"), B.GEAK_EALIGN),           # payload off the 16-byte grid
                      ((0, 40, 100, "mxfp8e4m3"), B.GEAK_EINVAL),           # ragged last block
                      ((0, 64, 63, "mxfp8e4m3"), B.GEAK_EBOUNDS),           # scales inside the payload
                      ((0, 64, 100, "f8e4m3"), B.GEAK_EDTYPE),              # not a block-scaled element format
                      ((0, 64, 2 ** 64 - 1, "mxint8"), B.GEAK_EBOUNDS)):
        st, plan = B.geak_check_plan_mx([bad], None, 2, 0.0, 0.0, False, 0)
        assert st == code and plan is None, (bad, st)
    st, plan = B.geak_check_plan([(0, 64, B.GEAK_MXINT8)], 2, 0.0, 0.0, False, 0)      # and not in a plain plan
    assert st == B.GEAK_EDTYPE
    # two segments whose scale regions collide
    st, plan = B.geak_check_plan_mx([(0, 64, 1000, "mxint8"), (64, 64, 1001, "mxint8")], None, 1, 0.0, 0.0, False, 0)
    assert st == B.GEAK_EBOUNDS


def test_read_probe_over_a_block_scaled_plan(oracle_mod):
    """The read-only probe reads what a run reads, the scale bytes behind the last payload included, and leaves the
    plan's next run alone."""
    print("mx probe", flush=True)
    rng = np.random.default_rng(8899)
    K = 3
    segs = [_tensors(rng, f, n, K) for f, n in (("mxfp8e4m3", 4096 + 64), ("mxfp4e2m1", 8192))]
    bufs, table = _pack(segs)
    fmts = ["mxfp8e4m3", "mxfp4e2m1"]
    dev = [torch.from_numpy(b.copy()).cuda() for b in bufs]
    ck = B.Checker(mx=[(o, n, so, f) for (o, n, so), f in zip(table, fmts)], num_candidates=K, atol=1e-2, rtol=0.05, equal_nan=False, device=0)
    try:
        ck.run(dev[0], dev[1:])
        first = ck.read().copy()
        ck.read_probe(dev[0], dev[1:])
        torch.cuda.synchronize()
        ck.run(dev[0], dev[1:])
        _assert_same(ck.read().copy(), first, "run after a probe")
    finally:
        ck.close()


@pytest.mark.parametrize("fmt", ["mxfp6e2m3", "mxfp6e3m2"])
def test_every_six_bit_code_at_every_position(oracle_mod, fmt):
    """Each of the 64 codes in each of a lane's sixteen positions (the codes straddle bytes and words differently at
    each), against candidates holding the next code, the negated one and the same one under another scale."""
    print("mx six-bit codes", fmt, flush=True)
    n = 4096 + 1024                                           # a full item and a tail
    i = np.arange(n)
    codes = (i // 16 + i % 16 * 5) % 64                        # position p of slot s holds code (s + 5 p) mod 64: every pair occurs

    def pack(c):
        out = np.zeros(n * 3 // 4, np.uint8)
        for j in range(0, n, 4):                               # four codes in three bytes
            v = int(c[j]) | int(c[j + 1]) << 6 | int(c[j + 2]) << 12 | int(c[j + 3]) << 18
            out[j * 3 // 4: j * 3 // 4 + 3] = [v & 0xFF, (v >> 8) & 0xFF, v >> 16]
        return out
    assert {(int(c), int(p)) for c, p in zip(codes, i % 16)} == {(c, p) for c in range(64) for p in range(16)}
    scales = np.full(n // 32, 127, np.uint8)
    other = scales.copy(); other[::3] = 129
    segs = [[(pack(codes), scales), (pack((codes + 1) % 64), scales), (pack(codes ^ 0x20), scales), (pack(codes), other)]]
    _compare(oracle_mod, segs, [fmt], 3, 0.01, 0.1, False, f"{fmt} all codes")
    rec = _compare(oracle_mod, [[(pack(codes), scales), (pack(codes), scales), (pack(codes ^ 0x20), scales)]], [fmt], 2, 0.0, 0.0, False,
                   f"{fmt} all codes, zero tolerance")
    assert rec[0, 0]["pass"] == 1 and rec[0, 1]["mismatch_count"] == n - (codes % 32 == 0).sum()      # only +0 against -0 passes
