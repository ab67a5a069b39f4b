"""geak_check_run_static -- the entry point for callers that cannot allocate -- gives the records of
geak_check_run: through the C ABI, on two calls in a row, the second on a smaller input (all calls on
a GPU share one scratch array, which keeps the previous call's contents), and it refuses plans whose
workspace exceeds the array."""
import numpy as np
import pytest
import torch

from helpers import record_tuple
from paper_2507_23194_amd import binding as B
from paper_2507_23194_amd import synth

pytestmark = pytest.mark.gpu


def _both(w):
    """Records of geak_check_run (caller's workspace) and of geak_check_run_static for one workload."""
    if w.segments is None:
        ck = B.Checker(dense=(w.dtype, (w.ref.numel(),)), num_candidates=len(w.cands), atol=w.atol, rtol=w.rtol,
                       equal_nan=w.equal_nan, device=0)
    else:
        ck = B.Checker(w.segments, num_candidates=len(w.cands), atol=w.atol, rtol=w.rtol, equal_nan=w.equal_nan, device=0)
    try:
        assert B.geak_check_workspace_bytes(ck.plan) <= B.GEAK_STATIC_SCRATCH_BYTES
        ck.run(w.ref, w.cands)
        plain = ck.read().copy()
        ck.results.fill_(0xAB)                                  # the static run must write every record itself
        torch.cuda.synchronize()
        stream = torch.cuda.current_stream(0).cuda_stream
        st = B.geak_check_run_static(ck.plan, w.ref.data_ptr(), [c.data_ptr() for c in w.cands], ck.results.data_ptr(), stream)
        assert st == B.GEAK_OK, B.geak_status_string(st)
        static = ck.read().copy()
    finally:
        ck.close()
    return plain, static


def test_static_scratch_run_equals_plain_run_twice_second_smaller():
    big = synth.config2(rows=1024, cols=1500, num_candidates=6, device="cuda")      # dense fp16 with NaN / Inf, ragged tail
    small = synth.small(4, device="cuda")                                           # ragged mixed batch, fewer bytes
    assert small.algorithmic_bytes() < big.algorithmic_bytes()
    for w in (big, small):
        plain, static = _both(w)
        assert plain.shape == static.shape
        assert [record_tuple(r) for r in plain.reshape(-1)] == [record_tuple(r) for r in static.reshape(-1)], w.name
        for (s, k), e in w.expect.items():                      # and both agree with what the generator planted
            assert int(static[s, k]["mismatch_count"]) == e["count"] and int(static[s, k]["first_mismatch"]) == e["first"]


def test_static_scratch_run_refuses_what_does_not_fit():
    # 2^28 fp32 elements, 256 candidates: 4096 slots x 256 x 16 bytes of partials alone exceed the array
    st, plan = B.geak_check_plan_dense("f32", [1 << 28], 256, 1e-5, 1e-5, False, 0)
    assert st == B.GEAK_OK
    try:
        assert B.geak_check_workspace_bytes(plan) > B.GEAK_STATIC_SCRATCH_BYTES
        x = torch.zeros(64, dtype=torch.float32, device="cuda")
        res = torch.zeros(256 * B.RESULT_DTYPE.itemsize, dtype=torch.uint8, device="cuda")
        st = B.geak_check_run_static(plan, x.data_ptr(), [x.data_ptr()] * 256, res.data_ptr(), 0)
        assert st == B.GEAK_EWORKSPACE
        torch.cuda.synchronize()
        assert int(res.sum()) == 0                              # nothing was enqueued
    finally:
        B.geak_check_destroy(plan)
