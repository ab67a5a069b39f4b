"""Seeded random plans: segment tables of random length, dtypes, sizes, alignments and tolerances,
checked, reported and histogrammed on the GPU and compared with the oracle segment by segment."""
import numpy as np
import pytest
import torch

from helpers import record_tuple
from paper_2507_23194_amd import binding as B
from paper_2507_23194_amd import synth
from test_gpu_parity import _special_case

pytestmark = pytest.mark.gpu

DTYPES = ["f32", "f16", "bf16", "i32", "i64", "u8", "i8", "f64", "f8e4m3", "f8e5m2"]


def _random_case(seed):
    rng = np.random.default_rng(seed)
    nsegs = int(rng.integers(1, 40))
    K = int(rng.integers(1, 10))
    align = int(rng.choice([1, 2, 4, 8, 16]))
    segs, tols, parts, off = [], [], [], 0
    for _ in range(nsegs):
        dt = DTYPES[int(rng.integers(0, len(DTYPES)))]
        w = synth.ELEM_SIZE[dt]
        n = int(rng.choice([0, 1, int(rng.integers(2, 70)), int(rng.integers(70, 5000)), int(rng.integers(5000, 40000))]))
        a = max(align, w)
        off = (off + a - 1) // a * a + w * int(rng.integers(0, 3)) * (align < 16)
        off = (off + w - 1) // w * w
        segs.append((off, n, dt))
        tols.append((float(rng.choice([0.0, 1e-6, 1e-3, 0.25, 1e30])), float(rng.choice([0.0, 1e-5, 1e-2, 0.125, 3.0]))))
        if n:
            b, _ = _special_case(rng, dt, n)
            cands = [(_special_case(rng, dt, n)[1] if rng.random() < 0.7 else b.copy()) for _ in range(K)]
            parts.append((off, b, cands))
        off += n * w
    total = (off + 15) // 16 * 16 + 16
    ref = np.zeros(total, dtype=np.uint8)
    cbufs = [np.zeros(total, dtype=np.uint8) for _ in range(K)]
    for off, b, cands in parts:
        ref[off:off + b.nbytes] = b.view(np.uint8)
        for k in range(K):
            cbufs[k][off:off + b.nbytes] = cands[k].view(np.uint8)
    return segs, tols, K, bool(rng.integers(0, 2)), ref, cbufs


@pytest.mark.parametrize("seed", range(24))
def test_random_plan(oracle_mod, seed):
    segs, tols, K, equal_nan, ref, cbufs = _random_case(seed)
    print("random plan", seed, len(segs), "segments", K, "candidates", flush=True)
    dref = torch.from_numpy(ref).cuda()
    dc = [torch.from_numpy(c).cuda() for c in cbufs]
    ck = B.Checker(segs, num_candidates=K, equal_nan=equal_nan, device=0, tolerances=tols)
    try:
        ck.run(dref, dc)
        gpu = ck.read().copy()
        rec, cnt = ck.report(dref, dc, 5)
        verdict, failed = ck.verdicts()
        hist = ck.ulp_histogram(dref, dc)
    finally:
        ck.close()
    for s, (off, n, dt) in enumerate(segs):
        atol, rtol = tols[s]
        for k in range(K):
            cpu = oracle_mod.check_segment(ref, cbufs[k], n, dt, atol, rtol, equal_nan, ref_byte_offset=off)
            assert record_tuple(gpu[s, k]) == record_tuple(cpu), (seed, s, k, dt, n, off, atol, rtol, equal_nan)
            rep = oracle_mod.report_segment(ref, cbufs[k], n, dt, atol, rtol, equal_nan, 5, ref_byte_offset=off)
            assert int(cnt[s, k]) == len(rep), (seed, s, k, dt)
            got = rec[s, k][:len(rep)]
            assert (got["index"] == rep["index"]).all(), (seed, s, k, dt)
            for f in ("a", "b", "d", "tol"):
                assert np.array_equal(got[f], rep[f], equal_nan=True), (seed, s, k, dt, f)
            want = oracle_mod.ulp_histogram_segment(ref, cbufs[k], n, dt, ref_byte_offset=off)
            assert (hist[s, k] == want).all(), (seed, s, k, dt, n, hist[s, k], want)
    assert verdict.tolist() == [bool((gpu[:, k]["pass"] == 1).all()) for k in range(K)]
    assert failed.tolist() == [int((gpu[:, k]["pass"] == 0).sum()) for k in range(K)]


def _random_pitched_case(seed):
    """Pitched segments of random geometry: rows from a few bytes to several items long, pitches that are
    row-tight, 16-byte multiples (short rows then travel as row groups) or only element-aligned, starts on
    16-byte boundaries or anywhere, padding filled with different garbage in every tensor."""
    rng = np.random.default_rng(1000 + seed)
    nsegs = int(rng.integers(1, 12))
    K = int(rng.integers(1, 6))
    layouts, tols, flat, off = [], [], [], 0
    for _ in range(nsegs):
        dt = DTYPES[int(rng.integers(0, len(DTYPES)))]
        w = synth.ELEM_SIZE[dt]
        rows = int(rng.choice([0, 1, 2, int(rng.integers(3, 40)), int(rng.integers(40, 700))]))
        row_elems = int(rng.choice([1, int(rng.integers(2, 40)), int(rng.integers(40, 2048 // w + 1)), int(rng.integers(2048 // w, 3 * 4096 // w))]))
        if rows * row_elems > 300000:
            rows = max(1, 300000 // row_elems)
        row_bytes = row_elems * w
        kind = int(rng.integers(0, 3))
        if kind == 0:                                   # rows on 16-byte boundaries
            pitch = (row_bytes + 15) // 16 * 16 + 16 * int(rng.integers(0, 4))
            off = (off + 15) // 16 * 16
        elif kind == 1:                                 # element-aligned only
            pitch = row_bytes + w * int(rng.integers(0, 9))
            off = (off + w - 1) // w * w + w * int(rng.integers(0, 5))
        else:                                           # 16-byte pitch, start anywhere
            pitch = (row_bytes + 15) // 16 * 16
            off = (off + w - 1) // w * w + w * int(rng.integers(0, 3))
        layouts.append((off, rows, row_elems, pitch, dt))
        tols.append((float(rng.choice([0.0, 1e-3, 0.25])), float(rng.choice([0.0, 1e-2, 0.125]))))
        n = rows * row_elems
        if n:
            b, _ = _special_case(rng, dt, n)
            cands = [(_special_case(rng, dt, n)[1] if rng.random() < 0.7 else b.copy()) for _ in range(K)]
            if K > 1:
                cands[1][: n // 2] = b[: n // 2]        # a first mismatch somewhere inside
        else:
            b, cands = np.zeros(0, np.uint8), [np.zeros(0, np.uint8)] * K
        flat.append((b, cands, n, dt))
        off += (rows - 1) * pitch + row_bytes if rows else 0
    total = (off + 31) // 16 * 16
    ref = rng.integers(0, 256, total, dtype=np.uint8)
    cbufs = [rng.integers(0, 256, total, dtype=np.uint8) for _ in range(K)]
    for (off, rows, row_elems, pitch, dt), (b, cands, n, _) in zip(layouts, flat):
        w = synth.ELEM_SIZE[dt]
        for r in range(rows):
            lo = off + r * pitch
            ref[lo:lo + row_elems * w] = b[r * row_elems:(r + 1) * row_elems].view(np.uint8)
            for k in range(K):
                cbufs[k][lo:lo + row_elems * w] = cands[k][r * row_elems:(r + 1) * row_elems].view(np.uint8)
    return layouts, tols, K, bool(rng.integers(0, 2)), ref, cbufs, flat


@pytest.mark.parametrize("seed", range(12))
def test_random_pitched_plan(oracle_mod, seed):
    layouts, tols, K, equal_nan, ref, cbufs, flat = _random_pitched_case(seed)
    print("random pitched plan", seed, layouts, K, "candidates", flush=True)
    dref = torch.from_numpy(ref).cuda()
    dc = [torch.from_numpy(c).cuda() for c in cbufs]
    ck = B.Checker(pitched=layouts, num_candidates=K, equal_nan=equal_nan, device=0, tolerances=tols)
    try:
        ck.run(dref, dc)
        gpu = ck.read().copy()
        rec, cnt = ck.report(dref, dc, 5)
        hist = ck.ulp_histogram(dref, dc)
    finally:
        ck.close()
    for s, (b, cands, n, dt) in enumerate(flat):
        atol, rtol = tols[s]
        for k in range(K):
            cpu = oracle_mod.check_segment(b, cands[k], n, dt, atol, rtol, equal_nan)
            assert record_tuple(gpu[s, k]) == record_tuple(cpu), (seed, s, k, layouts[s], atol, rtol, equal_nan)
            rep = oracle_mod.report_segment(b, cands[k], n, dt, atol, rtol, equal_nan, 5)
            assert int(cnt[s, k]) == len(rep), (seed, s, k, layouts[s])
            got = rec[s, k][:len(rep)]
            assert (got["index"] == rep["index"]).all(), (seed, s, k, layouts[s])
            for f in ("a", "b", "d", "tol"):
                assert np.array_equal(got[f], rep[f], equal_nan=True), (seed, s, k, layouts[s], f)
            want = oracle_mod.ulp_histogram_segment(b, cands[k], n, dt)
            assert (hist[s, k] == want).all(), (seed, s, k, layouts[s], hist[s, k], want)


def test_many_short_pitched_segments(oracle_mod):
    """Several hundred small pitched segments (row groups, tails, rows off the 16-byte grid) with four
    candidates: more than a thousand pairs, so one wave reduces each, rescans of row groups included."""
    rng = np.random.default_rng(4242)
    K, layouts, flat, off = 4, [], [], 0
    for s in range(300):
        dt = DTYPES[s % len(DTYPES)]
        w = synth.ELEM_SIZE[dt]
        rows, row_elems = int(rng.integers(1, 30)), int(rng.integers(1, 600 // w + 2))
        if s % 3:
            pitch = (row_elems * w + 15) // 16 * 16 + 16 * int(rng.integers(0, 2))
            off = (off + 15) // 16 * 16
        else:
            pitch = row_elems * w + w * int(rng.integers(1, 4))
            off = (off + w - 1) // w * w + w
        layouts.append((off, rows, row_elems, pitch, dt))
        n = rows * row_elems
        b, _ = _special_case(rng, dt, n)
        cands = [b.copy(), _special_case(rng, dt, n)[1], b.copy(), b.copy()]
        cands[1][: n // 2] = b[: n // 2]
        cands[3][n - 1:] = _special_case(rng, dt, n)[1][n - 1:]              # at most the last element differs
        flat.append((b, cands, n, dt))
        off += (rows - 1) * pitch + row_elems * w
    total = (off + 31) // 16 * 16
    ref = rng.integers(0, 256, total, dtype=np.uint8)
    cbufs = [rng.integers(0, 256, total, dtype=np.uint8) for _ in range(K)]
    for (off, rows, row_elems, pitch, dt), (b, cands, n, _) in zip(layouts, flat):
        w = synth.ELEM_SIZE[dt]
        for r in range(rows):
            lo = off + r * pitch
            ref[lo:lo + row_elems * w] = b[r * row_elems:(r + 1) * row_elems].view(np.uint8)
            for k in range(K):
                cbufs[k][lo:lo + row_elems * w] = cands[k][r * row_elems:(r + 1) * row_elems].view(np.uint8)
    dref = torch.from_numpy(ref).cuda()
    dc = [torch.from_numpy(c).cuda() for c in cbufs]
    ck = B.Checker(pitched=layouts, num_candidates=K, atol=1e-3, rtol=1e-2, equal_nan=True, device=0)
    try:
        ck.run(dref, dc)
        gpu = ck.read().copy()
    finally:
        ck.close()
    for s, (b, cands, n, dt) in enumerate(flat):
        for k in range(K):
            cpu = oracle_mod.check_segment(b, cands[k], n, dt, 1e-3, 1e-2, True)
            assert record_tuple(gpu[s, k]) == record_tuple(cpu), (s, k, layouts[s])
