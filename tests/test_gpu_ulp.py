"""GPU parity of the ulp-distance histogram (geak_check_ulp_histogram, through the C ABI) against the
oracle's histogram of the same bytes: every one of the 66 counts of every (segment, candidate) pair
must be equal."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

from helpers import host_threads
from paper_2507_23194_amd import binding as B
from paper_2507_23194_amd import synth
from test_gpu_parity import _to_device, _special_case

pytestmark = pytest.mark.gpu


def _dense_hist(b, cands, dtype):
    ref = _to_device(b, dtype)
    cs = [_to_device(c, dtype) for c in cands]
    ck = B.Checker(dense=(dtype, (b.size,)), num_candidates=len(cs), atol=0.0, rtol=0.0, equal_nan=False, device=0)
    try:
        return ck.ulp_histogram(ref, cs)[0].copy()
    finally:
        ck.close()


def _assert_hist(gpu, cpu, what):
    assert gpu.shape == cpu.shape, what
    if not (gpu == cpu).all():
        bad = np.argwhere(gpu != cpu)[0]
        raise AssertionError(f"{what}: first difference at {tuple(bad)}: gpu {gpu[tuple(bad)]} oracle {cpu[tuple(bad)]}\n"
                             f"gpu row {gpu[tuple(bad[:-1])]}\noracle row {cpu[tuple(bad[:-1])]}")


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16", "i32", "i64", "u8", "i8", "f64", "f8e4m3", "f8e5m2"])
@pytest.mark.parametrize("n", [1, 63, 2049, 70001, (1 << 20) + 5])
def test_histogram_special_values(oracle_mod, dtype, n):
    print("ulp", dtype, n, flush=True)
    rng = np.random.default_rng(2000 + n)
    b, a0 = _special_case(rng, dtype, n)
    _, a1 = _special_case(rng, dtype, n, special=0.0)
    # a candidate of unrelated values: distances of every size, every lane in a different bin
    a2 = rng.integers(0, 256, b.nbytes, dtype=np.uint8).view(b.dtype)[:n].copy()
    cands = [a0, b.copy(), a1, a2]
    gpu = _dense_hist(b, cands, dtype)
    cpu = np.stack([oracle_mod.ulp_histogram_segment(b, c, n, dtype) for c in cands])
    _assert_hist(gpu, cpu, f"{dtype} n={n}")
    assert (gpu.sum(axis=1) == n).all()
    assert int(gpu[1, 0]) + int(gpu[1, 65]) == n             # the copy: distance 0, or NaN


@pytest.mark.parametrize("dtype,K", [("f64", 100), ("f32", 80), ("f16", 150), ("u8", 256)])
def test_histogram_candidate_passes(oracle_mod, dtype, K):
    """More candidates than one pass holds (38 rows of binary64, 75 of binary32, 142 of the 16-bit dtypes)."""
    print("ulp passes", dtype, K, flush=True)
    rng = np.random.default_rng(K)
    n = 9001
    b, _ = _special_case(rng, dtype, n)
    cands = [_special_case(rng, dtype, n)[1] if k % 3 else b.copy() for k in range(K)]
    gpu = _dense_hist(b, cands, dtype)
    cpu = np.stack([oracle_mod.ulp_histogram_segment(b, c, n, dtype) for c in cands])
    _assert_hist(gpu, cpu, f"{dtype} K={K}")


@pytest.mark.parametrize("align,dtypes", [(16, ("f32", "f16", "bf16", "i32")), (1, ("u8", "f32", "i8", "f16", "i64", "f64")), (1, ("f8e4m3", "f16", "f8e5m2", "u8")),
                                          (8, ("f64", "i64", "bf16"))])
def test_histogram_ragged(oracle_mod, align, dtypes):
    print("ulp ragged", align, dtypes, flush=True)
    w = synth.config4(num_segments=120, log2_max=14.5, num_candidates=3, device="cuda", align=align, seed=40 + align,
                      dtypes=dtypes)
    ck = B.Checker(w.segments, num_candidates=len(w.cands), atol=w.atol, rtol=w.rtol, equal_nan=w.equal_nan, device=0)
    try:
        gpu = ck.ulp_histogram(w.ref, w.cands).copy()
        again = ck.ulp_histogram(w.ref, w.cands).copy()      # the scratch is reused as it was left
    finally:
        ck.close()
    ref = synth.to_numpy_raw(w.ref)
    cands = [synth.to_numpy_raw(c) for c in w.cands]
    cpu = np.zeros_like(gpu)
    for s, (off, numel, dt) in enumerate(w.segments):
        for k, c in enumerate(cands):
            cpu[s, k] = oracle_mod.ulp_histogram_segment(ref, c, numel, dt, ref_byte_offset=off)
    _assert_hist(gpu, cpu, f"ragged align={align}")
    _assert_hist(again, cpu, f"ragged align={align}, second call")


def test_histogram_empty_segments(oracle_mod):
    segs = [(0, 0, "f32"), (16, 5, "f16"), (32, 0, "i64")]
    ref = torch.zeros(48, dtype=torch.uint8, device="cuda")
    cand = ref.clone()
    cand[16] = 3                                             # first fp16 element: pattern 3, three steps from zero
    ck = B.Checker(segs, num_candidates=1, atol=0.0, rtol=0.0, equal_nan=False, device=0)
    try:
        h = ck.ulp_histogram(ref, [cand])
    finally:
        ck.close()
    assert h.shape == (3, 1, 66)
    assert int(h[0].sum()) == 0 and int(h[2].sum()) == 0
    assert int(h[1, 0, 0]) == 4 and int(h[1, 0, 2]) == 1 and int(h[1].sum()) == 5


def _oracle_hist_chunked(oracle_mod, ref, cand, numel, dtype, off, chunk=1 << 22):
    w = synth.ELEM_SIZE[dtype]
    bounds = list(range(0, numel, chunk))
    with ThreadPoolExecutor(max_workers=host_threads()) as ex:
        parts = list(ex.map(lambda lo: oracle_mod.ulp_histogram_segment(ref, cand, min(chunk, numel - lo), dtype,
                                                                        ref_byte_offset=off + lo * w), bounds))
    return np.sum(parts, axis=0, dtype=np.uint64)


@pytest.mark.parametrize("cid,ks", [(2, [0, 40]), (3, [1, 9]), (4, None), (5, [3])])
def test_histogram_full_configs(oracle_mod, cid, ks):
    """The benchmark's workloads at full size: all 66 counts of the sampled candidates against the oracle,
    and the sum of every pair's bins against the segment length."""
    print("ulp full config", cid, flush=True)
    w = synth.CONFIGS[cid](device="cuda")
    if w.segments is None:
        ck = B.Checker(dense=(w.dtype, (w.ref.numel(),)), num_candidates=len(w.cands), atol=w.atol, rtol=w.rtol,
                       equal_nan=w.equal_nan, device=0)
        segments = [(0, w.ref.numel(), w.dtype)]
    else:
        ck = B.Checker(w.segments, num_candidates=len(w.cands), atol=w.atol, rtol=w.rtol, equal_nan=w.equal_nan, device=0)
        segments = w.segments
    try:
        gpu = ck.ulp_histogram(w.ref, w.cands).copy()
    finally:
        ck.close()
    print("  gpu done", flush=True)
    numels = np.array([n for _, n, _ in segments], dtype=np.uint64)
    assert (gpu.sum(axis=2) == numels[:, None]).all()
    ref = synth.to_numpy_raw(w.ref)
    for k in (range(len(w.cands)) if ks is None else ks):
        c = synth.to_numpy_raw(w.cands[k])
        for s, (off, numel, dt) in enumerate(segments):
            cpu = _oracle_hist_chunked(oracle_mod, ref, c, numel, dt, off) if numel > (1 << 22) else \
                oracle_mod.ulp_histogram_segment(ref, c, numel, dt, ref_byte_offset=off)
            assert (gpu[s, k] == cpu).all(), (cid, s, k, gpu[s, k], cpu)
    print("  oracle done", flush=True)
