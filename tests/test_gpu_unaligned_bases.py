"""Base pointers that are only element-aligned: slices of larger tensors as reference and candidates, each
tensor at its own offset from the 16-byte grid.  Records, mismatch report and ulp histogram equal the oracle's
on the same elements -- dense tensors of every dtype, a ragged batch whose segments start on any byte, and
short pitched rows that are grouped into work items."""
import numpy as np
import pytest
import torch

from helpers import record_tuple
from paper_2507_23194_amd import binding as B
from paper_2507_23194_amd import synth
from test_gpu_parity import _special_case, _assert_same, _stacked

pytestmark = pytest.mark.gpu


def _placed(raw_bytes: np.ndarray, shift: int) -> torch.Tensor:
    """The bytes on the device, `shift` bytes behind a 256-byte aligned address, other garbage around them."""
    n = raw_bytes.size
    buf = torch.randint(0, 256, (n + 64 + 256,), dtype=torch.uint8, device="cuda")
    base = (-buf.data_ptr()) % 256 + shift
    view = buf[base:base + n]
    view.copy_(torch.from_numpy(raw_bytes.copy()))
    assert view.data_ptr() % 256 == shift % 256
    return view


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16", "i32", "i64", "u8", "i8", "f64", "f8e4m3", "f8e5m2"])
@pytest.mark.parametrize("n", [1, 37, 4096 + 5, 3 * 4096 + 1000])
def test_dense_tensors_at_odd_addresses(oracle_mod, dtype, n):
    print("odd bases", dtype, n, flush=True)
    w = synth.ELEM_SIZE[dtype]
    rng = np.random.default_rng(7000 + n + w)
    b, a0 = _special_case(rng, dtype, n)
    _, a1 = _special_case(rng, dtype, n, special=0.0)
    cands = [a0, b.copy(), a1, a0.copy()]
    # shifts in bytes: multiples of the element size, different for every tensor, 0 and the largest among them
    steps = 16 // w
    shifts = [((3 + 5 * t) % steps) * w for t in range(5)]
    shifts[2] = 0
    shifts[4] = (steps - 1) * w
    ref = _placed(b.view(np.uint8), shifts[0])
    dcs = [_placed(c.view(np.uint8), s) for c, s in zip(cands, shifts[1:])]
    for equal_nan, atol, rtol in ((False, 1e-3, 1e-3), (True, 0.0, 0.0)):
        ck = B.Checker(dense=(dtype, (n,)), num_candidates=len(cands), atol=atol, rtol=rtol, equal_nan=equal_nan, device=0)
        try:
            ck.run(ref, dcs)
            gpu = ck.read().copy()
            rec, cnt = ck.report(ref, dcs, 5)
            hist = ck.ulp_histogram(ref, dcs)
        finally:
            ck.close()
        cpu = oracle_mod.check_dense(b, cands, dtype, atol, rtol, equal_nan, threads=2).reshape(1, -1)
        _assert_same(gpu, cpu, f"{dtype} n={n} shifts={shifts}")
        for k, c in enumerate(cands):
            rep = oracle_mod.report_segment(b, c, n, dtype, atol, rtol, equal_nan, 5)
            assert int(cnt[0, k]) == len(rep)
            got = rec[0, k][:len(rep)]
            assert (got["index"] == rep["index"]).all()
            assert all(np.array_equal(got[f], rep[f], equal_nan=True) for f in ("a", "b", "d", "tol"))
            assert (hist[0, k] == oracle_mod.ulp_histogram_segment(b, c, n, dtype)).all(), (dtype, n, k)


@pytest.mark.parametrize("dtypes,base_align", [(("u8", "i8", "f8e4m3", "f8e5m2"), 1), (("f16", "bf16", "u8"), 2),
                                               (("f32", "i32", "f16", "u8"), 4), (("f64", "i64", "f32", "bf16"), 8)])
def test_ragged_batch_at_odd_addresses(oracle_mod, dtypes, base_align):
    """Packed buffers whose bases sit off the grid by different amounts; the segments inside start on any
    multiple of their element size, so first items, tails and full items all occur at odd addresses."""
    print("ragged odd bases", dtypes, base_align, flush=True)
    w = synth.config4(num_segments=120, log2_max=14.0, num_candidates=3, device="cpu", align=base_align, seed=500 + base_align, dtypes=dtypes)
    raw = [synth.to_numpy_raw(t).view(np.uint8) for t in [w.ref] + w.cands]
    steps = 16 // base_align
    shifts = [((1 + 3 * t) % steps) * base_align for t in range(len(raw))]
    dev = [_placed(r, s) for r, s in zip(raw, shifts)]
    ck = B.Checker(w.segments, num_candidates=len(w.cands), atol=w.atol, rtol=w.rtol, equal_nan=w.equal_nan, device=0)
    try:
        ck.run(dev[0], dev[1:])
        gpu = ck.read().copy()
        hist = ck.ulp_histogram(dev[0], dev[1:])
    finally:
        ck.close()
    cpu = oracle_mod.check_ragged(raw[0], raw[1:], w.segments, w.atol, w.rtol, w.equal_nan, threads=4)
    _assert_same(gpu, cpu, f"ragged at shifts {shifts}")
    for (s, k), e in w.expect.items():
        assert int(gpu[s, k]["mismatch_count"]) == e["count"] and int(gpu[s, k]["first_mismatch"]) == e["first"]
    for s, (off, numel, dt) in enumerate(w.segments):
        for k in range(len(w.cands)):
            assert (hist[s, k] == oracle_mod.ulp_histogram_segment(raw[0], raw[1 + k], numel, dt, ref_byte_offset=off)).all(), (s, k)


def test_row_groups_at_odd_addresses(oracle_mod):
    """Short pitched rows grouped into items (their offsets and pitch are multiples of 16), in tensors whose
    bases are not: every row then starts off the grid, and every row's last vector is read byte by byte."""
    rng = np.random.default_rng(77)
    layouts = _stacked([(300, 100, 112, "u8"), (77, 33, 80, "bf16"), (130, 50, 64, "f8e4m3"), (64, 1000, 1008, "i8"), (333, 7, 16, "f16")], start=32)
    K = 3
    total = max(off + (rows - 1) * pitch + re * synth.ELEM_SIZE[dt] for off, rows, re, pitch, dt in layouts)
    total = (total + 31) // 16 * 16
    bufs = [rng.integers(0, 256, total, dtype=np.uint8) for _ in range(K + 1)]
    flat = []
    for off, rows, re, pitch, dt in layouts:
        n, w = rows * re, synth.ELEM_SIZE[dt]
        b, _ = _special_case(rng, dt, n)
        cs = [(_special_case(rng, dt, n)[1] if k else b.copy()) for k in range(K)]
        for r in range(rows):
            lo = off + r * pitch
            bufs[0][lo:lo + re * w] = b[r * re:(r + 1) * re].view(np.uint8)
            for k in range(K):
                bufs[1 + k][lo:lo + re * w] = cs[k][r * re:(r + 1) * re].view(np.uint8)
        flat.append((b, cs, n, dt))
    dev = [_placed(x, s) for x, s in zip(bufs, (6, 0, 14, 2))]
    ck = B.Checker(pitched=layouts, num_candidates=K, atol=1e-3, rtol=1e-2, equal_nan=True, device=0)
    try:
        ck.run(dev[0], dev[1:])
        gpu = ck.read().copy()
    finally:
        ck.close()
    for s, (b, cs, n, dt) in enumerate(flat):
        for k in range(K):
            cpu = oracle_mod.check_segment(b, cs[k], n, dt, 1e-3, 1e-2, True)
            assert record_tuple(gpu[s, k]) == record_tuple(cpu), (s, k, dt)
