"""geak_check_run neither allocates nor synchronises, so a caller may capture it into a HIP graph and
replay it.  Every replay must give the records of the eager run, also after the data has changed
between replays and with eager work of the same plan in between."""
import numpy as np
import pytest
import torch

from helpers import record_tuple, workload_oracle
from paper_2507_23194_amd import binding as B
from paper_2507_23194_amd import synth

pytestmark = pytest.mark.gpu


def _records(ck):
    return [record_tuple(r) for r in ck.read().reshape(-1)]


@pytest.mark.parametrize("cid", [1, 4])
def test_captured_run_replays_like_the_eager_run(oracle_mod, cid):
    w = synth.small(cid, device="cuda")
    if w.segments is None:
        ck = B.Checker(dense=(w.dtype, (w.ref.numel(),)), num_candidates=len(w.cands), atol=w.atol, rtol=w.rtol,
                       equal_nan=w.equal_nan, device=0)
    else:
        ck = B.Checker(w.segments, num_candidates=len(w.cands), atol=w.atol, rtol=w.rtol, equal_nan=w.equal_nan, device=0)
    try:
        ck.run(w.ref, w.cands)
        eager = _records(ck)
        cpu = workload_oracle(oracle_mod, w)
        assert eager == [record_tuple(r) for r in cpu.reshape(-1)]

        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            ck.run(w.ref, w.cands)
        for replay in range(3):
            ck.results.zero_()
            torch.cuda.synchronize()
            graph.replay()
            assert _records(ck) == eager, f"replay {replay}"
            ck.run(w.ref, w.cands)                          # eager work of the same plan between the replays
            assert _records(ck) == eager

        # the graph holds pointers, not data: change one candidate in place and replay
        saved = w.cands[0].clone()
        w.cands[0].copy_(w.ref)                             # candidate 0 becomes a copy of the reference
        torch.cuda.synchronize()
        graph.replay()
        changed = ck.read().copy()
        ck.run(w.ref, w.cands)
        assert [record_tuple(r) for r in changed.reshape(-1)] == _records(ck)
        assert all(int(changed[s, 0]["mismatch_count"]) == 0 or w.equal_nan is False for s in range(changed.shape[0]))
        w.cands[0].copy_(saved)
        torch.cuda.synchronize()
        graph.replay()
        assert _records(ck) == eager
    finally:
        ck.close()
