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
