"""ctypes front end of the plain-C oracle (geak_oracle.c).  TEST INFRASTRUCTURE ONLY.

The rule it applies is the reading of GEAK section 3.1 (tolerance-based comparison of
output tensors) and section 3.3 (every unit test must pass; the reference is ground
truth) written out in geak_oracle.c.  Nothing here is shared with the HIP path.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "geak_oracle.c")
_LIB = os.path.join(_HERE, "libgeak_oracle.so")

DTYPE_CODES = {"f32": 0, "f16": 1, "bf16": 2, "i32": 3, "i64": 4, "u8": 5, "i8": 6, "f64": 7,
               "f8e4m3": 8, "f8e5m2": 9}
ELEM_SIZE = {"f32": 4, "f16": 2, "bf16": 2, "i32": 4, "i64": 8, "u8": 1, "i8": 1, "f64": 8, "f8e4m3": 1, "f8e5m2": 1}

# One record per (segment, candidate); field meaning as in geak_oracle.c (R7-R9).
RECORD_DTYPE = np.dtype(
    [
        ("pass", "<i4"),
        ("reserved", "<i4"),
        ("mismatch_count", "<u8"),
        ("first_mismatch", "<i8"),
        ("max_abs_err", "<f8"),
        ("max_rel_err", "<f8"),
    ]
)

# One reported mismatch; field meaning as in geak_oracle.c (oracle_report_segment).
MISMATCH_DTYPE = np.dtype([("index", "<i8"), ("a", "<f8"), ("b", "<f8"), ("d", "<f8"), ("tol", "<f8")])

_lock = threading.Lock()
_lib = None


def build(force: bool = False) -> str:
    """Compile geak_oracle.c with gcc (no FMA contraction, no fast-math)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = [
            "gcc", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
            "-o", _LIB, _SRC, "-lm",
        ]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = ctypes.CDLL(build())
            lib.oracle_check_segment.restype = ctypes.c_int
            lib.oracle_check_segment.argtypes = [
                ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int,
                ctypes.c_double, ctypes.c_double, ctypes.c_int, ctypes.c_void_p,
            ]
            lib.oracle_report_segment.restype = ctypes.c_int64
            lib.oracle_report_segment.argtypes = [
                ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int,
                ctypes.c_double, ctypes.c_double, ctypes.c_int, ctypes.c_uint64, ctypes.c_void_p,
            ]
            lib.oracle_ulp_histogram_segment.restype = ctypes.c_int
            lib.oracle_ulp_histogram_segment.argtypes = [
                ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int, ctypes.c_void_p,
            ]
            lib.oracle_decode_f16.restype = ctypes.c_float
            lib.oracle_decode_f16.argtypes = [ctypes.c_uint16]
            lib.oracle_decode_bf16.restype = ctypes.c_float
            lib.oracle_decode_bf16.argtypes = [ctypes.c_uint16]
            lib.oracle_decode_f8e4m3.restype = ctypes.c_float
            lib.oracle_decode_f8e4m3.argtypes = [ctypes.c_uint8]
            lib.oracle_decode_f8e5m2.restype = ctypes.c_float
            lib.oracle_decode_f8e5m2.argtypes = [ctypes.c_uint8]
            _lib = lib
    return _lib


def decode_f8(bits: int, dtype: str) -> float:
    lib = _load()
    return float((lib.oracle_decode_f8e4m3 if dtype == "f8e4m3" else lib.oracle_decode_f8e5m2)(int(bits) & 0xFF))


def decode_f16(bits: int) -> float:
    return float(_load().oracle_decode_f16(int(bits) & 0xFFFF))


def decode_bf16(bits: int) -> float:
    return float(_load().oracle_decode_bf16(int(bits) & 0xFFFF))


def _as_bytes(x) -> np.ndarray:
    """Raw little-endian bytes of a contiguous numpy array, no copy when possible."""
    a = np.ascontiguousarray(x)
    return a.reshape(-1).view(np.uint8)


def check_segment(ref, cand, numel: int, dtype: str, atol: float, rtol: float,
                  equal_nan: bool, ref_byte_offset: int = 0, cand_byte_offset: int | None = None):
    """One (segment, candidate) pair.  ref/cand: numpy arrays holding the raw storage
    (f16/bf16 as uint16 bit patterns or any array whose bytes are the tensor's bytes)."""
    lib = _load()
    if cand_byte_offset is None:
        cand_byte_offset = ref_byte_offset
    rb, cb = _as_bytes(ref), _as_bytes(cand)
    need = numel * ELEM_SIZE[dtype]
    if ref_byte_offset + need > rb.size or cand_byte_offset + need > cb.size:
        raise ValueError("segment exceeds buffer")
    out = np.zeros(1, dtype=RECORD_DTYPE)
    rc = lib.oracle_check_segment(
        rb.ctypes.data + ref_byte_offset, cb.ctypes.data + cand_byte_offset,
        numel, DTYPE_CODES[dtype], float(atol), float(rtol), int(bool(equal_nan)),
        out.ctypes.data,
    )
    if rc != 0:
        raise RuntimeError("oracle_check_segment failed")
    return out[0]


def report_segment(ref, cand, numel: int, dtype: str, atol: float, rtol: float, equal_nan: bool,
                   max_records: int, ref_byte_offset: int = 0, cand_byte_offset: int | None = None) -> np.ndarray:
    """The first max_records mismatches of one (segment, candidate) pair, as a MISMATCH_DTYPE array
    (its length is min(max_records, mismatch count))."""
    lib = _load()
    if cand_byte_offset is None:
        cand_byte_offset = ref_byte_offset
    rb, cb = _as_bytes(ref), _as_bytes(cand)
    need = numel * ELEM_SIZE[dtype]
    if ref_byte_offset + need > rb.size or cand_byte_offset + need > cb.size:
        raise ValueError("segment exceeds buffer")
    out = np.zeros(max(1, max_records), dtype=MISMATCH_DTYPE)
    n = lib.oracle_report_segment(
        rb.ctypes.data + ref_byte_offset, cb.ctypes.data + cand_byte_offset,
        numel, DTYPE_CODES[dtype], float(atol), float(rtol), int(bool(equal_nan)),
        int(max_records), out.ctypes.data,
    )
    if n < 0:
        raise RuntimeError("oracle_report_segment failed")
    return out[:n].copy()


ULP_BINS = 66


def ulp_histogram_segment(ref, cand, numel: int, dtype: str, ref_byte_offset: int = 0,
                          cand_byte_offset: int | None = None) -> np.ndarray:
    """Counts of the elements of one (segment, candidate) pair by ulp distance (rules U1-U4 of
    geak_oracle.c): uint64 array of ULP_BINS entries."""
    lib = _load()
    if cand_byte_offset is None:
        cand_byte_offset = ref_byte_offset
    rb, cb = _as_bytes(ref), _as_bytes(cand)
    need = numel * ELEM_SIZE[dtype]
    if ref_byte_offset + need > rb.size or cand_byte_offset + need > cb.size:
        raise ValueError("segment exceeds buffer")
    out = np.zeros(ULP_BINS, dtype=np.uint64)
    rc = lib.oracle_ulp_histogram_segment(rb.ctypes.data + ref_byte_offset, cb.ctypes.data + cand_byte_offset,
                                          numel, DTYPE_CODES[dtype], out.ctypes.data)
    if rc != 0:
        raise RuntimeError("oracle_ulp_histogram_segment failed")
    return out


def _run_pairs(jobs, threads: int):
    """jobs: list of zero-argument callables; ctypes releases the GIL during the C loop."""
    if threads <= 1 or len(jobs) <= 1:
        return [j() for j in jobs]
    with ThreadPoolExecutor(max_workers=threads) as ex:
        return list(ex.map(lambda j: j(), jobs))


def check_dense(ref, cands, dtype: str, atol: float, rtol: float, equal_nan: bool,
                threads: int = 1) -> np.ndarray:
    """Dense case: one segment.  Returns RECORD_DTYPE array of shape (K,)."""
    rb = _as_bytes(ref)
    numel = rb.size // ELEM_SIZE[dtype]
    jobs = [
        (lambda c=c: check_segment(rb, c, numel, dtype, atol, rtol, equal_nan))
        for c in cands
    ]
    return np.array(_run_pairs(jobs, threads), dtype=RECORD_DTYPE)


def gather_rows(buf, rows: int, row_elems: int, dtype: str, byte_offset: int, pitch_bytes: int, elem_stride: int = 1) -> np.ndarray:
    """The rows * row_elems elements of a 2-D layout, gathered into one contiguous array of raw storage
    (row-major): element (r, c) is read at byte_offset + r * pitch_bytes + c * elem_stride * (element size).
    pitch_bytes == 0 repeats one row for every r, elem_stride == 0 repeats one element along a row -- how a
    reference that is broadcast against the candidates is laid out.  Plain index arithmetic, nothing else."""
    w = ELEM_SIZE[dtype]
    raw = _as_bytes(buf)
    if byte_offset % w or pitch_bytes % w:
        raise ValueError("offsets must be multiples of the element size")
    store = {1: np.uint8, 2: np.uint16, 4: np.uint32, 8: np.uint64}[w]
    elems = raw[: raw.size // w * w].view(store)
    out = np.zeros(rows * row_elems, dtype=store)
    for r in range(rows):
        for c in range(row_elems):
            out[r * row_elems + c] = elems[(byte_offset + r * pitch_bytes) // w + c * elem_stride]
    return out


def check_segment_mapped(ref, cand, rows: int, row_elems: int, dtype: str, atol: float, rtol: float, equal_nan: bool,
                         cand_byte_offset: int, cand_pitch_bytes: int, ref_byte_offset: int, ref_pitch_bytes: int,
                         ref_elem_stride: int = 1):
    """One (segment, candidate) pair whose reference has a layout of its own: the candidate's element (r, c)
    is judged against the reference element that gather_rows finds for (r, c); indices are flat and row-major
    over rows * row_elems.  The rule itself is check_segment's, unchanged."""
    b = gather_rows(ref, rows, row_elems, dtype, ref_byte_offset, ref_pitch_bytes, ref_elem_stride)
    a = gather_rows(cand, rows, row_elems, dtype, cand_byte_offset, cand_pitch_bytes, 1)
    return check_segment(b, a, rows * row_elems, dtype, atol, rtol, equal_nan)


def gather_nd(buf, shape, stride_bytes, dtype: str, byte_offset: int) -> np.ndarray:
    """The elements of an N-d layout gathered into one contiguous array of raw storage, row-major over `shape`:
    element (i0, i1, ...) is read at byte_offset + i0 * stride_bytes[0] + i1 * stride_bytes[1] + ...  A stride of 0
    repeats the dimension (a broadcast operand).  Plain index arithmetic, nothing else."""
    w = ELEM_SIZE[dtype]
    raw = _as_bytes(buf)
    if byte_offset % w or any(int(t) % w for t in stride_bytes) or len(shape) != len(stride_bytes):
        raise ValueError("offsets and strides must be multiples of the element size, one stride per dimension")
    store = {1: np.uint8, 2: np.uint16, 4: np.uint32, 8: np.uint64}[w]
    elems = raw[: raw.size // w * w].view(store)
    total = 1
    for e in shape:
        total *= int(e)
    out = np.zeros(total, dtype=store)
    index = [0] * len(shape)
    for flat in range(total):
        at = byte_offset
        for d in range(len(shape)):
            at += index[d] * int(stride_bytes[d])
        out[flat] = elems[at // w]
        for d in range(len(shape) - 1, -1, -1):              # the next index in row-major order
            index[d] += 1
            if index[d] < int(shape[d]):
                break
            index[d] = 0
    return out


def check_segment_nd(ref, cand, shape, dtype: str, atol: float, rtol: float, equal_nan: bool, cand_byte_offset: int,
                     cand_stride_bytes, ref_byte_offset: int, ref_stride_bytes):
    """One (segment, candidate) pair of N-d tensors, each with its own strides (the reference's may be 0 where it is
    broadcast): element by element in row-major order of `shape`, the rule itself check_segment's, unchanged."""
    b = gather_nd(ref, shape, ref_stride_bytes, dtype, ref_byte_offset)
    a = gather_nd(cand, shape, cand_stride_bytes, dtype, cand_byte_offset)
    return check_segment(b, a, b.size, dtype, atol, rtol, equal_nan)


def combine_records(parts, offsets):
    """Fold the records of consecutive chunks of one tensor (chunk i starts at flat index offsets[i]) into the
    record of the whole tensor.  Every field of the record is a sum, a least index or a maximum over the
    elements (R7-R9 of geak_oracle.c), so the fold is: counts add, the first index is that of the first chunk
    that has one, shifted by the chunk's start, and each maximum is the maximum of the chunks' maxima."""
    out = np.zeros(1, dtype=RECORD_DTYPE)[0]
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


def check_dense_chunked(ref, cands, dtype: str, atol: float, rtol: float, equal_nan: bool, threads: int = 1,
                        chunk: int = 1 << 22) -> np.ndarray:
    """check_dense for large tensors: the element range is cut into chunks, each chunk is one plain
    check_segment call (so that the C loop can run on several host threads), and the chunks' records are
    folded with combine_records.  ref / cands: numpy arrays of the raw storage, one element per entry."""
    n = ref.size
    bounds = list(range(0, n, chunk)) or [0]
    jobs = [(lambda k=k, lo=lo: check_segment(ref[lo:min(n, lo + chunk)], cands[k][lo:min(n, lo + chunk)],
                                              min(n, lo + chunk) - lo, dtype, atol, rtol, equal_nan))
            for k in range(len(cands)) for lo in bounds]
    recs = _run_pairs(jobs, threads)
    out = [combine_records(recs[k * len(bounds):(k + 1) * len(bounds)], bounds) for k in range(len(cands))]
    return np.array(out, dtype=RECORD_DTYPE)


def host_cores() -> int:
    """Host cores this process may run on."""
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:
        return os.cpu_count() or 1


def check_ragged(ref_buf, cand_bufs, segments, atol: float, rtol: float, equal_nan: bool,
                 threads: int = 1) -> np.ndarray:
    """Ragged case.  segments: iterable of (byte_offset, numel, dtype_name); every candidate
    buffer is packed with the same table as the reference.  Returns records of shape (S, K),
    index [s, k]."""
    rb = _as_bytes(ref_buf)
    cbs = [_as_bytes(c) for c in cand_bufs]
    segments = list(segments)
    jobs = []
    for (off, numel, dt) in segments:
        for cb in cbs:
            jobs.append(
                lambda off=off, numel=numel, dt=dt, cb=cb: check_segment(
                    rb, cb, numel, dt, atol, rtol, equal_nan, ref_byte_offset=off)
            )
    flat = _run_pairs(jobs, threads)
    return np.array(flat, dtype=RECORD_DTYPE).reshape(len(segments), len(cbs))
