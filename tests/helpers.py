"""Shared test plumbing: fixture parsing and record comparison.  No arithmetic of the rule."""
import math
import os
import struct

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")

NP_STORAGE = {"f32": np.float32, "f16": np.uint16, "bf16": np.uint16, "i32": np.int32}
FIELDS = ("pass", "mismatch_count", "first_mismatch", "max_abs_err", "max_rel_err")


def _scalar(expr: str) -> float:
    return float(eval(expr, {"__builtins__": {}}, {"inf": math.inf}))


def _tensor(text: str, dtype: str) -> np.ndarray:
    toks = text.split()
    if dtype == "i32":
        return np.array([int(t, 0) for t in toks], dtype=np.int32)
    if dtype == "f32":
        out = np.zeros(len(toks), dtype=np.float32)
        bits = out.view(np.uint32)
        for i, t in enumerate(toks):
            if t.lower().startswith("0x"):
                bits[i] = int(t, 16)
            else:
                v = _scalar(t)
                out[i] = np.float32(v)
                assert math.isinf(v) or float(out[i]) == v, f"{t} is not a binary32 value"
        return out
    # f16 / bf16: raw bit patterns only
    return np.array([int(t, 16) for t in toks], dtype=np.uint16)


def load_pins(path=None):
    """Yield dicts for every case of tests/golden/pins.txt."""
    path = path or os.path.join(GOLDEN, "pins.txt")
    cases = []
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, dtype, atol, rtol, eq, ref, cand, exp = [p.strip() for p in line.split("|")]
            e = exp.split()
            cases.append(dict(
                name=name, dtype=dtype, atol=_scalar(atol), rtol=_scalar(rtol), equal_nan=bool(int(eq)),
                ref=_tensor(ref, dtype), cand=_tensor(cand, dtype),
                expect=dict(zip(FIELDS, (int(e[0]), int(e[1]), int(e[2]), _scalar(e[3]), _scalar(e[4])))),
            ))
    return cases


def f64_bits(x) -> int:
    return struct.unpack("<Q", struct.pack("<d", float(x)))[0]


def record_tuple(rec):
    """(pass, count, first, bits(max_abs), bits(max_rel)) -- doubles compared by bit pattern."""
    return (int(rec["pass"]), int(rec["mismatch_count"]), int(rec["first_mismatch"]),
            f64_bits(rec["max_abs_err"]), f64_bits(rec["max_rel_err"]))


def expect_tuple(e):
    return (e["pass"], e["mismatch_count"], e["first_mismatch"], f64_bits(e["max_abs_err"]), f64_bits(e["max_rel_err"]))


# ---- oracle drivers used by the GPU parity tests and the benchmark's baseline leg --------------
def combine_records(parts, offsets):
    """Fold the records of consecutive chunks of one tensor (chunk i starts at flat index
    offsets[i]) into the record of the whole tensor: counts add, first index is the least,
    both maxima are maxima.  (Pinned by the concatenation invariant in test_oracle_pins.)"""
    out = np.zeros(1, dtype=parts[0].dtype)[0]
    count, first, ma, mr = 0, -1, 0.0, 0.0
    for rec, off in zip(parts, offsets):
        count += int(rec["mismatch_count"])
        if first < 0 and int(rec["first_mismatch"]) >= 0:
            first = int(rec["first_mismatch"]) + off
        ma = max(ma, float(rec["max_abs_err"]))
        mr = max(mr, float(rec["max_rel_err"]))
    out["pass"] = int(count == 0)
    out["mismatch_count"] = count
    out["first_mismatch"] = first
    out["max_abs_err"] = ma
    out["max_rel_err"] = mr
    return out


def oracle_dense_chunked(oracle_mod, ref_np, cand_nps, dtype, atol, rtol, equal_nan, threads, chunk=1 << 22):
    """Oracle records of a large dense tensor, with the element range cut into chunks so that the
    plain C loop can run on several host threads."""
    from concurrent.futures import ThreadPoolExecutor
    n = ref_np.size
    bounds = list(range(0, n, chunk)) or [0]
    jobs = [(k, lo) for k in range(len(cand_nps)) for lo in bounds]

    def run(job):
        k, lo = job
        hi = min(n, lo + chunk)
        return oracle_mod.check_segment(ref_np[lo:hi], cand_nps[k][lo:hi], hi - lo, dtype, atol, rtol, equal_nan)

    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        recs = list(ex.map(run, jobs))
    out = []
    for k in range(len(cand_nps)):
        out.append(combine_records(recs[k * len(bounds):(k + 1) * len(bounds)], bounds))
    return np.array(out, dtype=recs[0].dtype)


def host_threads() -> int:
    import os
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:
        n = os.cpu_count() or 1
    return max(1, min(16, n))


def workload_oracle(oracle_mod, w, threads=None, cand_subset=None):
    """Oracle records (segments, candidates) of a synth.Workload whose tensors may live on the GPU."""
    from paper_2507_23194_amd import synth
    threads = threads or host_threads()
    ks = list(range(len(w.cands))) if cand_subset is None else list(cand_subset)
    ref = synth.to_numpy_raw(w.ref)
    if w.segments is None:
        out = []
        for k in ks:                                   # one candidate on the host at a time
            c = synth.to_numpy_raw(w.cands[k])
            out.append(oracle_dense_chunked(oracle_mod, ref, [c], w.dtype, w.atol, w.rtol, w.equal_nan, threads)[0])
        return np.array(out, dtype=out[0].dtype).reshape(1, -1)
    cands = [synth.to_numpy_raw(w.cands[k]) for k in ks]
    return oracle_mod.check_ragged(ref, cands, w.segments, w.atol, w.rtol, w.equal_nan, threads=threads)
