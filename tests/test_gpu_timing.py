"""The latency harness of the performance test: repetitions bracketed by events on the caller's stream, each
from cold caches when a flush buffer is given.  A kernel under test whose 128 MiB of input stay in the
last-level cache between runs (a library reduction, standing in for a generated kernel) is much slower cold
than warm; the check itself reads with non-temporal loads and takes the same time either way.  The latency
tables fed through geak_metrics_speedup give the oracle's speedup bit for bit."""
import numpy as np
import pytest
import torch

from paper_2507_23194_amd import binding as B
from paper_2507_23194_amd import synth
from oracle import metrics as M

pytestmark = pytest.mark.gpu


def _checker(w):
    return B.Checker(dense=(w.dtype, (w.ref.numel(),)), num_candidates=len(w.cands), atol=w.atol, rtol=w.rtol,
                     equal_nan=w.equal_nan, device=0)


def test_cold_latency_exceeds_warm_latency_and_feeds_the_speedup():
    flush = torch.empty(512 << 20, dtype=torch.uint8, device="cuda")          # twice the last-level cache
    w = synth.config1(device="cuda")                                          # 36 MiB in all: stays in the caches between runs
    ck = _checker(w)
    half = B.Checker(dense=(w.dtype, (w.ref.numel(),)), num_candidates=4, atol=w.atol, rtol=w.rtol, equal_nan=False, device=0)
    stream = torch.cuda.current_stream(0).cuda_stream
    try:
        def all_candidates(hip_stream):
            assert B.geak_check_run(ck.plan, w.ref.data_ptr(), [c.data_ptr() for c in w.cands], ck.workspace.data_ptr(),
                                    ck.results.data_ptr(), hip_stream) == B.GEAK_OK

        def four_candidates(hip_stream):
            assert B.geak_check_run(half.plan, w.ref.data_ptr(), [c.data_ptr() for c in w.cands[:4]], half.workspace.data_ptr(),
                                    half.results.data_ptr(), hip_stream) == B.GEAK_OK

        st, warm = B.geak_timing_measure(all_candidates, 5, 25, 0, 0, stream)
        assert st == B.GEAK_OK and warm.shape == (25,) and (warm > 0).all()
        st, cold = B.geak_timing_measure(all_candidates, 5, 25, flush.data_ptr(), flush.numel(), stream)
        assert st == B.GEAK_OK and (cold > 0).all()
        print(f"check on config 1: warm median {np.median(warm) * 1e3:.1f} us, cold median {np.median(cold) * 1e3:.1f} us", flush=True)
        # a kernel under test that reads through the caches: 128 MiB summed by the library, resident between warm runs
        x = torch.randn(32 << 20, device="cuda")
        out = torch.empty((), device="cuda")
        st, warm_sum = B.geak_timing_measure(lambda s: torch.sum(x, dim=0, out=out), 5, 25, 0, 0, stream)
        st2, cold_sum = B.geak_timing_measure(lambda s: torch.sum(x, dim=0, out=out), 5, 25, flush.data_ptr(), flush.numel(), stream)
        assert st == st2 == B.GEAK_OK
        print(f"sum of 128 MiB: warm median {np.median(warm_sum) * 1e3:.1f} us, cold median {np.median(cold_sum) * 1e3:.1f} us", flush=True)
        assert np.median(cold_sum) > 1.3 * np.median(warm_sum)                # what was cached had to come from memory again
        # the records are those of an ordinary run
        torch.cuda.synchronize()
        rec = ck.read()
        for (s, k), e in w.expect.items():
            assert int(rec[s, k]["mismatch_count"]) == e["count"]

        # two "unit tests" (cold and warm), a "reference kernel" (eight candidates) and a "generated" one (four):
        # the latency tables through the library's speedup and through the oracle's
        st, cold4 = B.geak_timing_measure(four_candidates, 3, 25, flush.data_ptr(), flush.numel(), stream)
        st2, warm4 = B.geak_timing_measure(four_candidates, 3, 24, 0, 0, stream)
        assert st == st2 == B.GEAK_OK
        ref_table = np.stack([cold, warm])
        gen_table = np.stack([cold4[:24], warm4])
        st, sp = B.geak_metrics_speedup(ref_table, gen_table)
        assert st == B.GEAK_OK
        want = M.speedup([list(r) for r in ref_table], [list(g) for g in gen_table])
        assert np.float64(sp).view(np.uint64) == np.float64(want).view(np.uint64)
        assert sp > 1.0                                                        # half the candidates take less time
    finally:
        ck.close()
        half.close()


def test_flush_overwrites_the_scratch_buffer_and_rejects_bad_arguments():
    buf = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream(0).cuda_stream
    assert B.geak_timing_flush(buf.data_ptr(), buf.numel(), stream) == B.GEAK_OK
    torch.cuda.synchronize()
    first = buf.clone()
    assert B.geak_timing_flush(buf.data_ptr(), buf.numel(), stream) == B.GEAK_OK
    torch.cuda.synchronize()
    assert not torch.equal(first, buf)                                         # a new value every time: the stores are not silent
    assert len(torch.unique(buf.view(torch.int32))) == 1                       # every 16-byte vector was written
    assert B.geak_timing_flush(0, 1024, stream) == B.GEAK_EINVAL
    assert B.geak_timing_flush(buf.data_ptr(), 8, stream) == B.GEAK_EINVAL
    assert B.geak_timing_flush(buf.data_ptr() + 4, 1024, stream) == B.GEAK_EALIGN
    st, _ = B.geak_timing_measure(lambda s: None, 0, 0, 0, 0, stream)
    assert st == B.GEAK_EINVAL                                                 # no repetitions
    def failing(_stream):
        raise RuntimeError("the kernel under test could not be launched")
    st, _ = B.geak_timing_measure(failing, 0, 3, 0, 0, stream)
    assert st == B.GEAK_EINVAL
    st, lat = B.geak_timing_measure(lambda s: None, 1, 4, 0, 0, stream)         # an empty launch: event pairs only
    assert st == B.GEAK_OK and lat.shape == (4,) and (lat >= 0).all()
