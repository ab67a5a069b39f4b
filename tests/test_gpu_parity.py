"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same bytes.
All five result fields must agree bit for bit (doubles compared by bit pattern): every field is an
order-independent reduction (sum, min, NaN-free max), so no tolerance applies."""
import numpy as np
import pytest
import torch

from helpers import load_pins, record_tuple, expect_tuple, workload_oracle, host_threads, oracle_dense_chunked
from paper_2507_23194_amd import binding as B
from paper_2507_23194_amd import synth

pytestmark = pytest.mark.gpu

TORCH_STORAGE = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16, "i32": torch.int32,
                 "i64": torch.int64, "u8": torch.uint8, "i8": torch.int8, "f64": torch.float64,
                 "f8e4m3": torch.uint8, "f8e5m2": torch.uint8}


def _to_device(arr: np.ndarray, dtype: str) -> torch.Tensor:
    """numpy storage (float32 / uint16 bit patterns / int32) -> device tensor with 16-byte aligned base
    (bases off the grid: test_gpu_unaligned_bases.py)."""
    if dtype in ("f16", "bf16"):
        t = torch.from_numpy(arr.view(np.int16).copy()).view(TORCH_STORAGE[dtype])
    else:
        t = torch.from_numpy(arr.copy())
    out = torch.empty(max(1, t.numel()), dtype=t.dtype, device="cuda")
    out[:t.numel()].copy_(t)
    return out[:t.numel()] if t.numel() else out[:0]


def _assert_same(gpu, cpu, what):
    assert gpu.shape == cpu.shape, what
    bad = [(idx, record_tuple(gpu[idx]), record_tuple(cpu[idx]))
           for idx in np.ndindex(gpu.shape) if record_tuple(gpu[idx]) != record_tuple(cpu[idx])]
    assert not bad, f"{what}: {len(bad)} of {gpu.size} records differ; first (index, gpu, oracle): {bad[0]}"


def _dense_gpu(ref_np, cand_nps, dtype, atol, rtol, equal_nan):
    ref = _to_device(ref_np, dtype)
    cands = [_to_device(c, dtype) for c in cand_nps]
    ck = B.Checker(dense=(dtype, (ref_np.size,)), num_candidates=len(cands), atol=atol, rtol=rtol,
                   equal_nan=equal_nan, device=0)
    try:
        ck.run(ref, cands)
        return ck.read().copy()
    finally:
        ck.close()


PINS = load_pins()


@pytest.mark.parametrize("case", PINS, ids=[c["name"] for c in PINS])
def test_golden_pins_on_gpu(case):
    print("pin", case["name"], flush=True)
    rec = _dense_gpu(case["ref"], [case["cand"]], case["dtype"], case["atol"], case["rtol"], case["equal_nan"])
    assert rec.shape == (1, 1)
    assert record_tuple(rec[0, 0]) == expect_tuple(case["expect"]), case["name"]


def _special_case(rng, dtype, n, special=0.02):
    """Random tensors rich in NaN, +-Inf, signed zeros, subnormals, huge values and near-boundary pairs."""
    if dtype in ("f8e4m3", "f8e5m2"):
        # byte codes: every pattern occurs (NaN, and for E5M2 the infinities, among them); candidates are
        # copies with some codes moved by a step or two, some replaced, some sign-flipped
        b = rng.integers(0, 256, n).astype(np.uint8)
        b[rng.random(n) < 0.2] = rng.choice(np.array([0x00, 0x80, 0x01, 0x7B, 0x7C, 0x7E, 0x7F, 0xFC, 0xFF], np.uint8))
        a = b.copy()
        step = rng.random(n) < 0.3
        a[step] = (b[step].astype(np.int64) + rng.integers(-2, 3, int(step.sum()))).astype(np.uint8)
        repl = rng.random(n) < 0.05
        a[repl] = rng.integers(0, 256, int(repl.sum())).astype(np.uint8)
        flip = rng.random(n) < 0.02
        a[flip] ^= 0x80
        if special > 0:
            sp = rng.random(n) < special
            a[sp] = rng.choice(np.array([0x7C, 0x7F, 0xFC, 0xFF, 0x7E, 0x00], np.uint8), int(sp.sum()))
        return b, a
    if dtype in ("u8", "i8"):
        np_t = np.uint8 if dtype == "u8" else np.int8
        info = np.iinfo(np_t)
        b = rng.integers(info.min, info.max + 1, n).astype(np_t)
        b[rng.random(n) < 0.3] = 0
        a = b.copy()
        idx = rng.random(n) < 0.01
        a[idx] = rng.integers(info.min, info.max + 1, int(idx.sum())).astype(np_t)
        return b, a
    if dtype == "i64":
        b = rng.integers(-2 ** 63, 2 ** 63, n, dtype=np.int64)
        b[rng.random(n) < 0.3] = 0
        b[rng.random(n) < 0.2] = rng.integers(-1000, 1000)
        b[rng.random(n) < 0.01] = np.iinfo(np.int64).min
        a = b.copy()
        idx = rng.random(n) < 0.01
        a[idx] = rng.integers(-2 ** 63, 2 ** 63, int(idx.sum()), dtype=np.int64)
        near = rng.random(n) < 0.01
        a[near] = (b[near].astype(np.uint64) + np.uint64(1)).astype(np.int64)
        a[rng.random(n) < 0.005] = np.iinfo(np.int64).max
        return b, a
    if dtype == "i32":
        b = rng.integers(-2 ** 31, 2 ** 31, n).astype(np.int32)
        b[rng.random(n) < 0.3] = 0
        a = b.copy()
        idx = rng.random(n) < 0.01
        a[idx] = rng.integers(-2 ** 31, 2 ** 31, int(idx.sum())).astype(np.int32)
        return b, a
    if dtype == "f64":
        b = rng.normal(size=n) * 10.0 ** rng.integers(-3, 3, n)
        a = b * (1 + 1e-3 * rng.normal(size=n)) + 1e-4 * rng.normal(size=n) * (rng.random(n) < 0.5)
        # pairs within a few units in the last place of the 1e-3 / 1e-3 boundary
        edge = rng.random(n) < 0.2
        tol = 1e-3 + 1e-3 * np.abs(b)
        a[edge] = b[edge] + tol[edge] * (1.0 + rng.integers(-4, 5, int(edge.sum())) * 2.0 ** -52) * rng.choice([-1.0, 1.0], int(edge.sum()))
        pool = np.array([np.nan, np.inf, -np.inf, 0.0, -0.0, 5e-324, -5e-324, 1.7e308, -1.7e308, 1e-310, 3e38, 1e-45, 0.9e308])
        for arr in (a, b):
            sp = rng.random(n) < special
            arr[sp] = rng.choice(pool, int(sp.sum()))
        same = rng.random(n) < 0.3
        a[same] = b[same]
        return b, a
    b32 = (rng.normal(size=n) * 10.0 ** rng.integers(-3, 3, n)).astype(np.float32)
    a32 = (b32 * (1 + 1e-3 * rng.normal(size=n)) + 1e-4 * rng.normal(size=n) * (rng.random(n) < 0.5)).astype(np.float32)
    pool = np.array([np.nan, np.inf, -np.inf, 0.0, -0.0, 1e-45, -1e-45, 3e38, -3e38, 1e-40, 65504.0, 6e-8], np.float32)
    for arr in (a32, b32):
        sp = rng.random(n) < special
        arr[sp] = rng.choice(pool, int(sp.sum()))
    same = rng.random(n) < 0.3
    a32[same] = b32[same]
    if dtype == "f32":
        return b32, a32
    if dtype == "f16":
        with np.errstate(over="ignore"):
            return b32.astype(np.float16).view(np.uint16), a32.astype(np.float16).view(np.uint16)
    tb = torch.from_numpy(b32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    ta = torch.from_numpy(a32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    return tb, ta


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16", "i32", "i64", "u8", "i8", "f64", "f8e4m3", "f8e5m2"])
@pytest.mark.parametrize("n", [1, 63, 2048, 4097, 70001, 1 << 20])
def test_special_values_dense(oracle_mod, dtype, n):
    print("special", dtype, n, flush=True)
    rng = np.random.default_rng(1000 + n)
    b, a0 = _special_case(rng, dtype, n)
    _, a1 = _special_case(rng, dtype, n, special=0.0)
    cands = [a0, b.copy(), a1]
    for equal_nan in (False, True):
        for (atol, rtol) in ((1e-3, 1e-3), (0.0, 0.0), (1e30, 3.0)):
            gpu = _dense_gpu(b, cands, dtype, atol, rtol, equal_nan)
            cpu = oracle_mod.check_dense(b, cands, dtype, atol, rtol, equal_nan, threads=3).reshape(1, -1)
            _assert_same(gpu, cpu, f"{dtype} n={n} atol={atol} rtol={rtol} equal_nan={equal_nan}")


def test_increasing_errors_keep_raising_the_maxima(oracle_mod):
    """Errors that grow along the tensor make every item raise both maxima (the slow path every time)."""
    n = 300000
    b = np.linspace(1.0, 2.0, n, dtype=np.float32)
    a = (b + np.linspace(0, 1e-2, n, dtype=np.float32)).astype(np.float32)
    gpu = _dense_gpu(b, [a, a[::-1].copy()], "f32", 1e-5, 1e-5, False)
    cpu = oracle_mod.check_dense(b, [a, a[::-1].copy()], "f32", 1e-5, 1e-5, False).reshape(1, -1)
    _assert_same(gpu, cpu, "increasing errors")


@pytest.mark.parametrize("second", [1, 300, 4096, 5000])
def test_relative_error_margin_that_underflows(oracle_mod, second):
    """max_rel_err is 0.75 after the first element (|7 - 4| / 4).  A later element b = 2^-149, a = 2^-148 has
    relative error exactly 1, but 0.75 * |b| - |a - b| = -2^-151 is below half the least subnormal: a filter
    that computes that margin gets -0 and must still count it as "may raise".  The later element sits in the
    same vector, the same item, or the same wave's next item (4096: the wave has then read 0.75 back)."""
    n = 1 << 23                                          # two items per wave
    b = np.ones(n, dtype=np.float32)
    a = b.copy()
    b[0], a[0] = 4.0, 7.0
    b[second] = np.float32(2.0 ** -149)
    a[second] = np.float32(2.0 ** -148)
    cpu = oracle_dense_chunked(oracle_mod, b, [a], "f32", 0.0, 0.0, False, host_threads()).reshape(1, -1)
    # the oracle's own answer is fixed by hand: two mismatches, first at 0, maxima 3 and exactly 1
    assert record_tuple(cpu[0, 0])[:3] == (0, 2, 0)
    assert float(cpu[0, 0]["max_abs_err"]) == 3.0 and float(cpu[0, 0]["max_rel_err"]) == 1.0
    gpu = _dense_gpu(b, [a], "f32", 0.0, 0.0, False)
    _assert_same(gpu, cpu, f"underflowing margin, second element at {second}")


@pytest.mark.parametrize("K", [1, 2, 5, 64, 65, 256])
def test_candidate_counts(oracle_mod, K):
    print("K", K, flush=True)
    rng = np.random.default_rng(K)
    n = 9000
    b, _ = _special_case(rng, "f16", n)
    cands = [_special_case(rng, "f16", n)[1] if k % 3 else b.copy() for k in range(K)]
    gpu = _dense_gpu(b, cands, "f16", 1e-2, 1e-2, True)
    cpu = oracle_mod.check_dense(b, cands, "f16", 1e-2, 1e-2, True, threads=4).reshape(1, -1)
    _assert_same(gpu, cpu, f"K={K}")


@pytest.mark.parametrize("cid", [1, 2, 3, 4, 5])
def test_small_configs(oracle_mod, cid):
    print("small config", cid, flush=True)
    w = synth.small(cid, device="cuda")
    gpu = B.check_workload(w)
    cpu = workload_oracle(oracle_mod, w)
    _assert_same(gpu, cpu, w.name)
    for (s, k), e in w.expect.items():
        assert int(gpu[s, k]["mismatch_count"]) == e["count"] and int(gpu[s, k]["first_mismatch"]) == e["first"]


@pytest.mark.parametrize("align", [2, 4, 16])
def test_ragged_unaligned_starts(oracle_mod, align):
    print("ragged align", align, flush=True)
    w = synth.config4(num_segments=160, log2_max=14.0, num_candidates=3, device="cuda", align=align, seed=align)
    gpu = B.check_workload(w)
    cpu = workload_oracle(oracle_mod, w)
    _assert_same(gpu, cpu, f"ragged align={align}")


@pytest.mark.parametrize("align,dtypes", [(1, ("u8", "f32", "i8", "f16", "i64", "f64", "f8e4m3", "bf16", "f8e5m2", "i32")),
                                          (16, ("f32", "f16", "bf16", "i32"))])
def test_ragged_many_pairs(oracle_mod, align, dtypes):
    """Plans with more than a thousand (segment, candidate) pairs are reduced by one wave per pair: every
    dtype, segment starts on any byte, mismatches in first items off the 16-byte grid, full items and tails."""
    print("ragged, many pairs", align, flush=True)
    w = synth.config4(num_segments=420, log2_max=13.0, num_candidates=3, device="cuda", align=align, seed=300 + align, dtypes=dtypes)
    assert len(w.segments) * len(w.cands) >= 1024
    gpu = B.check_workload(w)
    cpu = workload_oracle(oracle_mod, w)
    _assert_same(gpu, cpu, f"ragged, many pairs, align={align}")
    for (s, k), e in w.expect.items():
        assert int(gpu[s, k]["mismatch_count"]) == e["count"] and int(gpu[s, k]["first_mismatch"]) == e["first"]


def test_per_segment_tolerances(oracle_mod):
    """Every segment judged with its own atol / rtol (tight, loose, zero): records equal the oracle's,
    called segment by segment with that segment's pair; int32 segments ignore theirs."""
    rng = np.random.default_rng(77)
    w = synth.small(4, device="cuda")
    tols = [(float(10.0 ** rng.uniform(-7, -1)), float(10.0 ** rng.uniform(-7, -1))) if s % 5 else (0.0, 0.0)
            for s in range(len(w.segments))]
    ck = B.Checker(w.segments, num_candidates=len(w.cands), equal_nan=w.equal_nan, device=0, tolerances=tols)
    try:
        ck.run(w.ref, w.cands)
        gpu = ck.read().copy()
        rec, cnt = ck.report(w.ref, w.cands, 3)
    finally:
        ck.close()
    ref = synth.to_numpy_raw(w.ref)
    cands = [synth.to_numpy_raw(c) for c in w.cands]
    differs = 0
    for s, (off, numel, dt) in enumerate(w.segments):
        atol, rtol = tols[s]
        for k, c in enumerate(cands):
            cpu = oracle_mod.check_segment(ref, c, numel, dt, atol, rtol, w.equal_nan, ref_byte_offset=off)
            assert record_tuple(gpu[s, k]) == record_tuple(cpu), (s, k, dt, numel, atol, rtol)
            plain = oracle_mod.check_segment(ref, c, numel, dt, w.atol, w.rtol, w.equal_nan, ref_byte_offset=off)
            differs += int(cpu["mismatch_count"]) != int(plain["mismatch_count"])
            rep = oracle_mod.report_segment(ref, c, numel, dt, atol, rtol, w.equal_nan, 3, ref_byte_offset=off)
            assert int(cnt[s, k]) == len(rep)
            got = rec[s, k][:len(rep)]
            assert (got["index"] == rep["index"]).all()
            assert all(np.array_equal(got[f], rep[f], equal_nan=True) for f in ("a", "b", "d", "tol"))
    assert differs > 20          # the per-segment pairs really change verdicts relative to one plan-wide pair


@pytest.mark.parametrize("align", [8, 16])
def test_ragged_batch_with_int64_segments(oracle_mod, align):
    """The ragged recipe with int64 segments among the others (index outputs next to value outputs),
    with segment starts on 16-byte and on bare 8-byte boundaries."""
    w = synth.config4(num_segments=96, log2_max=15.0, num_candidates=4, device="cuda", align=align, seed=21,
                      dtypes=("f32", "i64", "bf16", "i64", "i32", "f16"))
    assert sum(dt == "i64" for _, _, dt in w.segments) > 20
    gpu = B.check_workload(w)
    cpu = workload_oracle(oracle_mod, w)
    _assert_same(gpu, cpu, f"ragged with int64, align {align}")
    for (s, k), e in w.expect.items():
        assert int(gpu[s, k]["mismatch_count"]) == e["count"] and int(gpu[s, k]["first_mismatch"]) == e["first"]


@pytest.mark.parametrize("align", [8, 16])
def test_ragged_batch_with_f64_segments(oracle_mod, align):
    """binary64 segments (reference outputs computed in double precision) among the others, with
    segment starts on 16-byte and on bare 8-byte boundaries."""
    w = synth.config4(num_segments=96, log2_max=15.0, num_candidates=4, device="cuda", align=align, seed=23,
                      dtypes=("f64", "f32", "f64", "bf16", "i64", "f16"))
    assert sum(dt == "f64" for _, _, dt in w.segments) > 20
    gpu = B.check_workload(w)
    cpu = workload_oracle(oracle_mod, w)
    _assert_same(gpu, cpu, f"ragged with binary64, align {align}")
    for (s, k), e in w.expect.items():
        assert int(gpu[s, k]["mismatch_count"]) == e["count"] and int(gpu[s, k]["first_mismatch"]) == e["first"]


@pytest.mark.parametrize("atol,rtol", [(1e300, 0.0), (0.0, 1e200), (5e-324, 1e-320), (1e-12, 1e-12), (1.7e308, 1.7e308)])
def test_f64_tolerances_outside_binary32(oracle_mod, atol, rtol):
    """binary64 segments take atol / rtol as given: values that overflow, underflow or round in binary32."""
    rng = np.random.default_rng(31)
    n = 50000
    b, a0 = _special_case(rng, "f64", n)
    _, a1 = _special_case(rng, "f64", n, special=0.0)
    a2 = b + rng.choice([-1.0, 1.0], n) * (atol + rtol * np.abs(b)) * (1.0 + rng.integers(-2, 3, n) * 2.0 ** -52) \
        if np.isfinite(atol + rtol * 1e3) else a1.copy()
    for equal_nan in (False, True):
        gpu = _dense_gpu(b, [a0, a1, a2], "f64", atol, rtol, equal_nan)
        cpu = oracle_mod.check_dense(b, [a0, a1, a2], "f64", atol, rtol, equal_nan, threads=3).reshape(1, -1)
        _assert_same(gpu, cpu, f"f64 atol={atol} rtol={rtol} equal_nan={equal_nan}")


@pytest.mark.parametrize("second", [1, 300, 512, 5000])
def test_relative_error_margin_that_underflows_f64(oracle_mod, second):
    """The binary64 form of the underflowing margin: after max_rel_err = 0.75, an element b = 2^-1074,
    a = 2^-1073 has relative error exactly 1 while 0.75 * |b| - |a - b| rounds to -0."""
    n = 1 << 21
    b = np.ones(n, dtype=np.float64)
    a = b.copy()
    b[0], a[0] = 4.0, 7.0
    b[second] = 2.0 ** -1074
    a[second] = 2.0 ** -1073
    cpu = oracle_dense_chunked(oracle_mod, b, [a], "f64", 0.0, 0.0, False, host_threads()).reshape(1, -1)
    assert record_tuple(cpu[0, 0])[:3] == (0, 2, 0)
    assert float(cpu[0, 0]["max_abs_err"]) == 3.0 and float(cpu[0, 0]["max_rel_err"]) == 1.0
    gpu = _dense_gpu(b, [a], "f64", 0.0, 0.0, False)
    _assert_same(gpu, cpu, f"underflowing margin in binary64, second element at {second}")


@pytest.mark.parametrize("align", [1, 16])
def test_ragged_batch_with_f8_segments(oracle_mod, align):
    """Segments in the 8-bit floating formats (outputs of quantising kernels) among the others, starting on
    any byte.  (The recipe's planted counts are not asserted here: where the format's spacing reaches 1,
    the planted +0.5 is a tie that may round back to the reference.)"""
    w = synth.config4(num_segments=96, log2_max=15.0, num_candidates=3, device="cuda", align=align, seed=24,
                      dtypes=("f8e4m3", "f32", "f8e5m2", "f16", "f8e4m3", "u8"))
    assert sum(dt.startswith("f8") for _, _, dt in w.segments) > 30
    gpu = B.check_workload(w)
    cpu = workload_oracle(oracle_mod, w)
    _assert_same(gpu, cpu, f"ragged with 8-bit floats, align {align}")
    assert sum(int(gpu[s, k]["mismatch_count"]) > 0 for s in range(gpu.shape[0]) for k in range(gpu.shape[1])) > 30


@pytest.mark.parametrize("dtype", ["f8e4m3", "f8e5m2"])
@pytest.mark.parametrize("atol,rtol", [(0.0, 0.0), (2.0 ** -6, 0.125), (1.0, 3e38), (0.3, 0.0)])
def test_f8_tolerance_sweep(oracle_mod, dtype, atol, rtol):
    """Coarse formats make exact boundaries common (d = tol with both exactly representable)."""
    rng = np.random.default_rng(41)
    n = 300000
    b, a0 = _special_case(rng, dtype, n)
    _, a1 = _special_case(rng, dtype, n, special=0.0)
    for equal_nan in (False, True):
        gpu = _dense_gpu(b, [a0, b.copy(), a1], dtype, atol, rtol, equal_nan)
        cpu = oracle_mod.check_dense(b, [a0, b.copy(), a1], dtype, atol, rtol, equal_nan, threads=3).reshape(1, -1)
        _assert_same(gpu, cpu, f"{dtype} atol={atol} rtol={rtol} equal_nan={equal_nan}")


@pytest.mark.parametrize("align", [1, 16])
def test_ragged_batch_with_byte_segments(oracle_mod, align):
    """Boolean-mask-like uint8 and int8 segments among the others, with segment starts on any byte."""
    w = synth.config4(num_segments=96, log2_max=15.0, num_candidates=3, device="cuda", align=align, seed=22,
                      dtypes=("u8", "f32", "i8", "u8", "f16", "i64"))
    assert sum(dt in ("u8", "i8") for _, _, dt in w.segments) > 30
    gpu = B.check_workload(w)
    cpu = workload_oracle(oracle_mod, w)
    _assert_same(gpu, cpu, f"ragged with byte dtypes, align {align}")
    for (s, k), e in w.expect.items():
        assert int(gpu[s, k]["mismatch_count"]) == e["count"] and int(gpu[s, k]["first_mismatch"]) == e["first"]


def test_dense_mask_with_many_flips(oracle_mod):
    """A large boolean mask whose candidates differ in many places: every vector of some items trips."""
    rng = np.random.default_rng(5)
    n = (1 << 21) + 77
    b = (rng.random(n) < 0.5).astype(np.uint8)
    cands = [b.copy(), b ^ (rng.random(n) < 0.2).astype(np.uint8), 1 - b]
    gpu = _dense_gpu(b, cands, "u8", 0.0, 0.0, False)
    cpu = oracle_dense_chunked(oracle_mod, b, cands, "u8", 0.0, 0.0, False, host_threads()).reshape(1, -1)
    _assert_same(gpu, cpu, "dense mask")
    assert int(gpu[0, 2]["mismatch_count"]) == n and int(gpu[0, 0]["pass"]) == 1


def test_empty_and_tiny_segments(oracle_mod):
    segs = [(0, 0, "f32"), (16, 1, "bf16"), (32, 0, "i32"), (48, 3, "i32"), (64, 2049, "f16"), (4176, 0, "f16")]
    total = 4176 + 16
    rng = np.random.default_rng(9)
    ref = torch.from_numpy(rng.integers(0, 256, total, dtype=np.uint8))
    # keep the fp16 segment finite and the bf16 element ordinary
    ref[64:64 + 4098] = torch.from_numpy(rng.normal(size=2049).astype(np.float16).view(np.uint8))
    ref[16:18] = torch.tensor([0x80, 0x3F], dtype=torch.uint8)
    c0 = ref.clone()
    c1 = ref.clone()
    c1[48 + 8] ^= 1                       # third int of segment 3
    c1[64 + 2 * 2048 + 1] ^= 0x40         # last fp16 element of segment 4
    w = synth.Workload("tiny", 1e-3, 1e-3, False, ref.cuda(), [c0.cuda(), c1.cuda()], None, None, segs, {})
    gpu = B.check_workload(w)
    cpu = workload_oracle(oracle_mod, w)
    _assert_same(gpu, cpu, "tiny segments")
    assert record_tuple(gpu[0, 1]) == (1, 0, -1, 0, 0) and record_tuple(gpu[5, 0]) == (1, 0, -1, 0, 0)
    assert int(gpu[3, 1]["first_mismatch"]) == 2 and int(gpu[4, 1]["first_mismatch"]) == 2048


def test_rerun_and_grid_independence(oracle_mod):
    """Same plan run twice, and the same data under a different segment cut, give identical records."""
    w = synth.small(2, device="cuda")
    ck = B.Checker(dense=(w.dtype, (w.ref.numel(),)), num_candidates=len(w.cands), atol=w.atol, rtol=w.rtol,
                   equal_nan=w.equal_nan, device=0)
    ck.run(w.ref, w.cands)
    r1 = ck.read().copy()
    ck.run(w.ref, w.cands)
    r2 = ck.read().copy()
    ck.close()
    _assert_same(r1, r2, "rerun")
    # cut the same tensor into 3 segments; combine and compare counts / maxima
    n = w.ref.numel()
    cuts = [0, 1000, n // 2 + 3, n]
    segs = [(2 * cuts[i], cuts[i + 1] - cuts[i], "f16") for i in range(3)]
    ref8 = w.ref.view(torch.uint8)
    c8 = [c.view(torch.uint8) for c in w.cands]
    w2 = synth.Workload("cut", w.atol, w.rtol, w.equal_nan, ref8, c8, None, None, segs, {})
    parts = B.check_workload(w2)
    for k in range(len(w.cands)):
        assert int(r1[0, k]["mismatch_count"]) == sum(int(parts[s, k]["mismatch_count"]) for s in range(3))
        assert float(r1[0, k]["max_abs_err"]) == max(float(parts[s, k]["max_abs_err"]) for s in range(3))
        assert float(r1[0, k]["max_rel_err"]) == max(float(parts[s, k]["max_rel_err"]) for s in range(3))


def test_run_argument_errors():
    ck = B.Checker(dense=("f32", (1024,)), num_candidates=2, atol=0, rtol=0, equal_nan=False, device=0)
    x = torch.zeros(1024 + 4, device="cuda")
    ok = x[:1024].data_ptr()
    assert ok % 16 == 0
    ws, res = ck.workspace.data_ptr(), ck.results.data_ptr()
    assert B.geak_check_run(ck.plan, 0, [ok, ok], ws, res, 0) == B.GEAK_EINVAL
    assert B.geak_check_run(ck.plan, ok, [ok, 0], ws, res, 0) == B.GEAK_EINVAL
    assert B.geak_check_run(ck.plan, ok + 2, [ok, ok], ws, res, 0) == B.GEAK_EALIGN      # not a multiple of the element size
    assert B.geak_check_run(ck.plan, ok, [ok, ok + 1], ws, res, 0) == B.GEAK_EALIGN
    assert B.geak_check_run(ck.plan, ok + 4, [ok, ok + 8], ws, res, 0) == B.GEAK_OK        # element-aligned bases will do
    assert B.geak_check_run(ck.plan, ok, [ok, ok], 0, res, 0) == B.GEAK_EWORKSPACE
    assert B.geak_check_run(ck.plan, ok, [ok, ok], ws, 0, 0) == B.GEAK_EINVAL
    assert B.geak_check_run(ck.plan, ok, [ok, ok], ws, res, 0) == B.GEAK_OK
    assert [record_tuple(r) for r in ck.read()[0]] == [(1, 0, -1, 0, 0)] * 2
    ck.close()
    st, plan = B.geak_check_plan([(0, 4, "f32")], 1, 0, 0, 0, 99)       # no such device
    assert st == B.GEAK_EHIP and plan is None


def test_argument_errors_of_the_other_entry_points():
    """Report, ulp histogram and verdicts reject null and misaligned pointers before anything is launched."""
    ck = B.Checker(dense=("f16", (4096,)), num_candidates=2, atol=0, rtol=0, equal_nan=False, device=0)
    x = torch.zeros(4096 + 16, dtype=torch.float16, device="cuda")
    ok = x[:4096].data_ptr()
    ws, res = ck.workspace.data_ptr(), ck.results.data_ptr()
    assert B.geak_check_run(ck.plan, ok, [ok, ok], ws, res, 0) == B.GEAK_OK
    scratch = torch.zeros(B.geak_check_ulp_workspace_bytes(ck.plan) + 16, dtype=torch.uint8, device="cuda")
    hist = torch.zeros(2 * B.GEAK_ULP_BINS + 2, dtype=torch.int64, device="cuda")
    sp, hp = scratch.data_ptr(), hist.data_ptr()
    assert B.geak_check_ulp_histogram(ck.plan, ok, [ok, ok], 0, hp, 0) == B.GEAK_EINVAL
    assert B.geak_check_ulp_histogram(ck.plan, ok, [ok, ok], sp, 0, 0) == B.GEAK_EINVAL
    assert B.geak_check_ulp_histogram(ck.plan, 0, [ok, ok], sp, hp, 0) == B.GEAK_EINVAL
    assert B.geak_check_ulp_histogram(ck.plan, ok, [ok, 0], sp, hp, 0) == B.GEAK_EINVAL
    assert B.geak_check_ulp_histogram(ck.plan, ok + 1, [ok, ok], sp, hp, 0) == B.GEAK_EALIGN
    assert B.geak_check_ulp_histogram(ck.plan, ok, [ok, ok], sp + 4, hp, 0) == B.GEAK_EALIGN
    assert B.geak_check_ulp_histogram(ck.plan, ok, [ok, ok], sp, hp + 4, 0) == B.GEAK_EALIGN
    assert B.geak_check_ulp_histogram(ck.plan, ok, [ok, ok], sp, hp, 0) == B.GEAK_OK
    torch.cuda.synchronize()
    assert hist[:2 * B.GEAK_ULP_BINS].view(2, -1)[:, 0].tolist() == [4096, 4096]       # identical tensors: all at distance 0
    verdict = torch.zeros(4, dtype=torch.int32, device="cuda")
    assert B.geak_check_verdicts(ck.plan, 0, verdict.data_ptr(), 0, 0) == B.GEAK_EINVAL
    assert B.geak_check_verdicts(ck.plan, res, 0, 0, 0) == B.GEAK_EINVAL
    assert B.geak_check_verdicts(ck.plan, res, verdict.data_ptr() + 2, 0, 0) == B.GEAK_EALIGN
    assert B.geak_check_verdicts(ck.plan, res, verdict.data_ptr(), 0, 0) == B.GEAK_OK
    torch.cuda.synchronize()
    assert verdict[:2].tolist() == [1, 1]
    rec = torch.zeros(2 * 4 * 40, dtype=torch.uint8, device="cuda")
    cnt = torch.zeros(2, dtype=torch.int32, device="cuda")
    assert B.geak_check_report(ck.plan, ok, [ok, ok], ws, res, 0, rec.data_ptr(), cnt.data_ptr(), 0) == B.GEAK_EINVAL   # M = 0
    assert B.geak_check_report(ck.plan, ok, [ok, ok], ws, res, 4, 0, cnt.data_ptr(), 0) == B.GEAK_EINVAL
    assert B.geak_check_report(ck.plan, ok, [ok, ok], ws, res, 4, rec.data_ptr(), cnt.data_ptr(), 0) == B.GEAK_OK
    torch.cuda.synchronize()
    assert cnt.tolist() == [0, 0]
    ck.close()
    # host-only plans run nothing
    st, plan = B.geak_check_plan([(0, 4, "f32")], 1, 0, 0, 0, -1)
    assert st == B.GEAK_OK
    assert B.geak_check_ulp_histogram(plan, ok, [ok], sp, hp, 0) == B.GEAK_EINVAL
    assert B.geak_check_verdicts(plan, res, verdict.data_ptr(), 0, 0) == B.GEAK_EINVAL
    B.geak_check_destroy(plan)


def test_non_default_stream(oracle_mod):
    w = synth.small(1, device="cuda")
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        gpu = B.check_workload(w)
    cpu = workload_oracle(oracle_mod, w)
    _assert_same(gpu, cpu, "side stream")


# ---- full-size configurations, in the launch configuration the benchmark times -------------------
def _full(oracle_mod, cid, oracle_candidates=None):
    print("full config", cid, flush=True)
    w = synth.CONFIGS[cid](device="cuda")
    print("  generated", w.name, w.algorithmic_bytes() / 1e9, "GB", flush=True)
    gpu = B.check_workload(w)
    print("  gpu done", flush=True)
    for (s, k), e in w.expect.items():                       # closed-form facts, every candidate
        assert int(gpu[s, k]["mismatch_count"]) == e["count"], (cid, s, k)
        assert int(gpu[s, k]["first_mismatch"]) == e["first"], (cid, s, k)
        assert int(gpu[s, k]["pass"]) == int(e["count"] == 0)
    ks = list(range(len(w.cands))) if oracle_candidates is None else oracle_candidates
    cpu = workload_oracle(oracle_mod, w, cand_subset=ks)
    print("  oracle done on candidates", ks, "threads", host_threads(), flush=True)
    _assert_same(gpu[:, ks], cpu, f"{w.name} candidates {ks}")


def test_full_config1(oracle_mod):
    _full(oracle_mod, 1)


def test_full_config2(oracle_mod):
    _full(oracle_mod, 2)            # all 64 candidates, all five fields, element by element through the oracle


def test_full_config3(oracle_mod):
    _full(oracle_mod, 3)            # all 16 candidates


def test_full_config4(oracle_mod):
    _full(oracle_mod, 4)


def test_full_config4_runs_the_layout_by_compute_unit():
    """The ragged workload is the one whose block table is cut by compute unit (test_full_config4 and the full-size
    histogram test then prove that layout against the oracle); the dense ones keep the plain table."""
    w = synth.CONFIGS[4](device="cuda")
    ck = B.Checker(w.segments, num_candidates=len(w.cands), atol=w.atol, rtol=w.rtol, equal_nan=w.equal_nan, device=0)
    try:
        info = ck.info()
        assert info.block_map == B.GEAK_MAP_BY_UNIT and info.unit_groups == torch.cuda.get_device_properties(0).multi_processor_count
        assert info.grid_blocks % info.unit_groups == 0 and info.grid_blocks // info.unit_groups >= 2
    finally:
        ck.close()
    ck = B.Checker(dense=("f16", (1 << 24,)), num_candidates=4, atol=0.0, rtol=0.0, equal_nan=False, device=0)
    try:
        assert ck.info().block_map == B.GEAK_MAP_ROTATED          # 8192 items fill the grid: plain table, XCDs taking turns
    finally:
        ck.close()


def test_layout_by_compute_unit_with_three_blocks_per_unit(oracle_mod):
    """180 candidates: the blocks' LDS leaves room for three per compute unit, so a unit's group of ranges has three."""
    print("by unit, three per unit", flush=True)
    K = 180
    w = synth.config4(device="cuda", seed=41, num_candidates=K, log2_max=16.5, dtypes=("f32", "f16", "bf16", "i32", "u8"))
    ck = B.Checker(w.segments, num_candidates=K, atol=w.atol, rtol=w.rtol, equal_nan=w.equal_nan, device=0)
    try:
        info = ck.info()
        assert info.block_map == B.GEAK_MAP_BY_UNIT and info.grid_blocks == 3 * info.unit_groups
        ck.run(w.ref, w.cands)
        gpu = ck.read().copy()
    finally:
        ck.close()
    ks = [0, 1, 59, 90, 178, 179]
    _assert_same(gpu[:, ks], workload_oracle(oracle_mod, w, cand_subset=ks), "three blocks per unit")
    for (s, k), e in w.expect.items():
        assert int(gpu[s, k]["mismatch_count"]) == e["count"] and int(gpu[s, k]["first_mismatch"]) == e["first"], (s, k)


def test_full_config5(oracle_mod):
    # every third candidate element by element through the oracle (11 x 2^30 elements: what the time limit
    # allows), all 32 by the planted counts and first indices
    _full(oracle_mod, 5, oracle_candidates=list(range(0, 32, 3)))


def test_verdicts_over_all_unit_tests(oracle_mod):
    """A candidate is correct only if every segment passes: the device verdicts against the oracle's
    AND over its own records, with the count of failing segments."""
    from oracle import metrics as M
    w = synth.small(4, device="cuda")
    ck = B.Checker(w.segments, num_candidates=len(w.cands), atol=w.atol, rtol=w.rtol, equal_nan=w.equal_nan, device=0)
    try:
        ck.run(w.ref, w.cands)
        gpu = ck.read().copy()
        verdict, failed = ck.verdicts()
    finally:
        ck.close()
    cpu = workload_oracle(oracle_mod, w)
    _assert_same(gpu, cpu, "records under the verdicts")
    assert verdict.tolist() == M.verdicts(cpu).tolist()
    assert failed.tolist() == [(cpu[:, k]["pass"] == 0).sum() for k in range(len(w.cands))]
    # a dense plan with a clean copy among the candidates: exactly that one is correct
    rng = np.random.default_rng(3)
    b, a = _special_case(rng, "f32", 5000, special=0.0)
    ref = _to_device(b, "f32")
    cands = [_to_device(a, "f32"), _to_device(b.copy(), "f32"), _to_device(a, "f32")]
    ck = B.Checker(dense=("f32", (b.size,)), num_candidates=3, atol=0.0, rtol=0.0, equal_nan=False, device=0)
    try:
        ck.run(ref, cands)
        verdict, failed = ck.verdicts()
    finally:
        ck.close()
    assert verdict.tolist() == [False, True, False] and failed.tolist() == [1, 0, 1]


def _stacked(rows_specs, start=0):
    """Pitched segments one after the other, each starting on the next 16-byte boundary."""
    out, off = [], start
    for rows, row_elems, pitch, dt in rows_specs:
        out.append((off, rows, row_elems, pitch, dt))
        off = (off + rows * pitch + 15) // 16 * 16
    return out


@pytest.mark.parametrize("case", ["long_rows", "short_rows", "odd_bytes", "mixed", "row_groups"])
def test_pitched_segments(oracle_mod, case):
    """Outputs in padded buffers: rows `pitch_bytes` apart, the padding between them filled with different
    garbage in every tensor.  Records, report, verdicts and ulp histograms equal the oracle's on contiguous
    copies of the same elements (indices flat and row-major, padding not counted)."""
    rng = np.random.default_rng(sum(map(ord, case)))
    layouts = {
        "long_rows": [(0, 5, 9000, 9000 * 2 + 64, "f16")],                       # rows of more than two items, 16-byte aligned
        "short_rows": [(16, 300, 100, 416, "f32")],                              # every row a tail item
        "odd_bytes": [(3, 40, 1000, 1003, "u8"), (50000, 9, 700, 712, "f8e4m3")],  # rows start on any byte
        "mixed": [(0, 6, 5000, 20480, "f32"), (131072, 3, 3000, 24064, "f64"), (204800, 17, 33, 80, "bf16"), (208000, 0, 5, 64, "i32"),
                  (208000, 2, 4097, 16400, "i32")],
        # short rows on 16-byte boundaries, grouped into items: every dtype, rows of one vector up to 128 vectors,
        # partial last vectors, row counts that leave a short last group
        "row_groups": _stacked([(1000, 64, 256, "bf16"), (77, 33, 80, "bf16"), (300, 100, 112, "u8"), (9, 3, 32, "f64"),
                                (130, 50, 64, "f8e4m3"), (200, 17, 80, "f32"), (40, 100, 816, "i64"), (333, 7, 16, "f16"),
                                (50, 500, 2016, "i32"), (64, 1000, 1008, "i8"), (20, 2048, 2064, "f8e5m2"), (3, 5, 48, "f32"),
                                (515, 31, 128, "f32")], start=64),
    }[case]
    K = 3
    total = max(off + (rows - 1) * pitch + re * synth.ELEM_SIZE[dt] if rows else off for off, rows, re, pitch, dt in layouts)
    total = (total + 31) // 16 * 16
    ref = rng.integers(0, 256, total, dtype=np.uint8)                            # garbage everywhere, also in the padding
    cbufs = [rng.integers(0, 256, total, dtype=np.uint8) for _ in range(K)]
    flat = []                                                                     # contiguous copies for the oracle
    for off, rows, re, pitch, dt in layouts:
        n = rows * re
        w = synth.ELEM_SIZE[dt]
        if n:
            b, _ = _special_case(rng, dt, n)
            cs = [(_special_case(rng, dt, n)[1] if k else b.copy()) for k in range(K)]
            cs[1][: n // 2] = b[: n // 2]                                         # a first mismatch somewhere inside
            for r in range(rows):
                lo = off + r * pitch
                ref[lo:lo + re * w] = b[r * re:(r + 1) * re].view(np.uint8)
                for k in range(K):
                    cbufs[k][lo:lo + re * w] = cs[k][r * re:(r + 1) * re].view(np.uint8)
        else:
            b, cs = np.zeros(0, np.uint8), [np.zeros(0, np.uint8)] * K
        flat.append((b, cs, n, dt))
    dref = torch.from_numpy(ref).cuda()
    dc = [torch.from_numpy(c).cuda() for c in cbufs]
    ck = B.Checker(pitched=layouts, num_candidates=K, atol=1e-3, rtol=1e-2, equal_nan=True, device=0)
    try:
        ck.run(dref, dc)
        gpu = ck.read().copy()
        rec, cnt = ck.report(dref, dc, 6)
        verdict, _ = ck.verdicts()
        hist = ck.ulp_histogram(dref, dc)
    finally:
        ck.close()
    for s, (b, cs, n, dt) in enumerate(flat):
        for k in range(K):
            cpu = oracle_mod.check_segment(b, cs[k], n, dt, 1e-3, 1e-2, True)
            assert record_tuple(gpu[s, k]) == record_tuple(cpu), (case, s, k, dt)
            rep = oracle_mod.report_segment(b, cs[k], n, dt, 1e-3, 1e-2, True, 6)
            assert int(cnt[s, k]) == len(rep)
            got = rec[s, k][:len(rep)]
            assert (got["index"] == rep["index"]).all(), (case, s, k)
            assert all(np.array_equal(got[f], rep[f], equal_nan=True) for f in ("a", "b", "d", "tol"))
            assert (hist[s, k] == oracle_mod.ulp_histogram_segment(b, cs[k], n, dt)).all(), (case, s, k)
    assert verdict.tolist() == [bool((gpu[:, k]["pass"] == 1).all()) for k in range(K)]
    assert verdict[0]                                                             # candidate 0 is a copy (NaN equal to NaN)
