"""GPU parity of the mismatch report (geak_check_report, through the C ABI) against the oracle's
report on the same bytes: counts, indices and the four values of every reported element must agree
exactly (NaN compared as NaN: payloads are not specified)."""
import numpy as np
import pytest
import torch

from helpers import host_threads
from paper_2507_23194_amd import binding as B
from paper_2507_23194_amd import synth
from test_gpu_parity import _to_device, _special_case

pytestmark = pytest.mark.gpu


def _same_values(x, y):
    return bool(np.all((x == y) | (np.isnan(x) & np.isnan(y))))


def _assert_reports_equal(gpu_rec, gpu_cnt, cpu_list, what):
    for k, cpu in enumerate(cpu_list):
        n = int(gpu_cnt[k])
        assert n == len(cpu), f"{what}: candidate {k}: count {n} vs oracle {len(cpu)}"
        got = gpu_rec[k][:n]
        assert (got["index"] == cpu["index"]).all(), f"{what}: candidate {k}: indices differ"
        for f in ("a", "b", "d", "tol"):
            assert _same_values(got[f], cpu[f]), f"{what}: candidate {k}: field {f} differs"


def _dense_report(b, cands, dtype, atol, rtol, equal_nan, M):
    ref = _to_device(b, dtype)
    cs = [_to_device(c, dtype) for c in cands]
    ck = B.Checker(dense=(dtype, (b.size,)), num_candidates=len(cs), atol=atol, rtol=rtol, equal_nan=equal_nan, device=0)
    try:
        ck.run(ref, cs)
        rec, cnt = ck.report(ref, cs, M)
        res = ck.read().copy()
        return rec[0], cnt[0], res[0]
    finally:
        ck.close()


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16", "i32", "i64", "u8", "i8", "f64", "f8e4m3", "f8e5m2"])
@pytest.mark.parametrize("n", [1, 300, 2049, 70001])
def test_report_special_values(oracle_mod, dtype, n):
    print("report", dtype, n, flush=True)
    rng = np.random.default_rng(1000 + n)
    b, _ = _special_case(rng, dtype, n)
    cands = [_special_case(rng, dtype, n)[1], b.copy(), _special_case(rng, dtype, n)[1]]
    for M in (1, 5, 64):
        for equal_nan in (False, True):
            rec, cnt, res = _dense_report(b, cands, dtype, 1e-2, 1e-2, equal_nan, M)
            cpu = [oracle_mod.report_segment(b, c, n, dtype, 1e-2, 1e-2, equal_nan, M) for c in cands]
            _assert_reports_equal(rec, cnt, cpu, f"{dtype} n={n} M={M} equal_nan={equal_nan}")
            assert int(cnt[1]) == 0 or dtype not in ("i32", "i64", "u8", "i8")    # an integer copy has nothing to report
            for k in range(3):
                assert int(cnt[k]) == min(M, int(res[k]["mismatch_count"]))


def test_report_sparse_mismatches_across_tiles(oracle_mod):
    """Fewer mismatches than asked for, far apart: the scan runs to the end of the tensor and the
    ranks carry over from tile to tile."""
    n = 1 << 20
    b = np.linspace(-1, 1, n, dtype=np.float32)
    a = b.copy()
    where = [5, 2047, 2048, 4100, 300000, 300001, n - 1]
    a[where] += 1.0
    a2 = b.copy()
    a2[n // 2:] += 1.0                                           # dense mismatches: early exit
    rec, cnt, res = _dense_report(b, [a, a2, b.copy()], "f32", 1e-3, 1e-3, False, 16)
    cpu = [oracle_mod.report_segment(b, c, n, "f32", 1e-3, 1e-3, False, 16) for c in (a, a2, b)]
    _assert_reports_equal(rec, cnt, cpu, "sparse")
    assert [int(i) for i in rec[0]["index"][:7]] == where and int(cnt[0]) == 7
    assert int(cnt[1]) == 16 and int(rec[1]["index"][0]) == n // 2 and int(cnt[2]) == 0


def test_report_ragged_batch(oracle_mod):
    w = synth.small(4, device="cuda")
    ck = B.Checker(w.segments, num_candidates=len(w.cands), atol=w.atol, rtol=w.rtol, equal_nan=w.equal_nan, device=0)
    try:
        ck.run(w.ref, w.cands)
        M = 6
        rec, cnt = ck.report(w.ref, w.cands, M)
        res = ck.read().copy()
    finally:
        ck.close()
    ref = synth.to_numpy_raw(w.ref)
    cands = [synth.to_numpy_raw(c) for c in w.cands]
    for s, (off, numel, dt) in enumerate(w.segments):
        cpu = [oracle_mod.report_segment(ref, c, numel, dt, w.atol, w.rtol, w.equal_nan, M, ref_byte_offset=off)
               for c in cands]
        _assert_reports_equal(rec[s], cnt[s], cpu, f"segment {s} ({dt}, {numel} elements)")
        for k in range(len(cands)):
            assert int(cnt[s, k]) == min(M, int(res[s, k]["mismatch_count"]))


def test_report_argument_errors():
    st, plan = B.geak_check_plan_dense("f32", [1024], 2, 1e-3, 1e-3, 0, 0)
    assert st == B.GEAK_OK
    t = torch.zeros(1024, device="cuda")
    ws = torch.zeros(max(16, B.geak_check_workspace_bytes(plan)), dtype=torch.uint8, device="cuda")
    res = torch.zeros(2 * 40, dtype=torch.uint8, device="cuda")
    recs = torch.zeros(2 * 4 * 40, dtype=torch.uint8, device="cuda")
    cnt = torch.zeros(2, dtype=torch.int32, device="cuda")
    ptrs = [t.data_ptr(), t.data_ptr()]
    assert B.geak_check_report(plan, t.data_ptr(), ptrs, ws.data_ptr(), res.data_ptr(), 0, recs.data_ptr(), cnt.data_ptr(), 0) == B.GEAK_EINVAL
    assert B.geak_check_report(plan, t.data_ptr(), ptrs, ws.data_ptr(), 0, 4, recs.data_ptr(), cnt.data_ptr(), 0) == B.GEAK_EINVAL
    assert B.geak_check_report(plan, t.data_ptr(), ptrs, 0, res.data_ptr(), 4, recs.data_ptr(), cnt.data_ptr(), 0) == B.GEAK_EWORKSPACE
    assert B.geak_check_report(plan, t.data_ptr() + 2, ptrs, ws.data_ptr(), res.data_ptr(), 4, recs.data_ptr(), cnt.data_ptr(), 0) == B.GEAK_EALIGN      # off the element grid
    torch.cuda.synchronize()
    B.geak_check_destroy(plan)
