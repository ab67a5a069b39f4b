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


# ---- oracle drivers used by the GPU parity tests -------------------------------------------------
def combine_records(parts, offsets):
    import oracle
    return oracle.combine_records(parts, offsets)


def oracle_dense_chunked(oracle_mod, ref_np, cand_nps, dtype, atol, rtol, equal_nan, threads, chunk=1 << 22):
    """Oracle records of a large dense tensor: oracle.check_dense_chunked (pinned against one plain
    check_segment call in test_oracle_pins.py::test_chunked_driver_equals_one_plain_call)."""
    return oracle_mod.check_dense_chunked(ref_np, cand_nps, dtype, atol, rtol, equal_nan, threads=threads, chunk=chunk)


def host_threads() -> int:
    """Worker threads for the oracle: the host cores this process may use, at most the 16 that are a
    one-GPU machine's share."""
    import oracle
    return max(1, min(16, oracle.host_cores()))


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
