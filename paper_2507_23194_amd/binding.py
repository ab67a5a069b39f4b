"""ctypes binding of libgeakcheck.so -- argument marshalling only.

Every function named ``geak_check_*`` below is the C entry point of the same name declared in
``include/geak_check.h``; all computation happens in the HIP kernels behind it.  PyTorch is used
for device memory and streams and nowhere else.  There is no CPU fallback: if the library has not
been built, the first call raises.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgeakcheck.so")
BUILD_SCRIPT = os.path.join(_HERE, "csrc", "build.sh")

GEAK_OK = 0
GEAK_EINVAL, GEAK_EDTYPE, GEAK_EALIGN, GEAK_EBOUNDS, GEAK_ENOMEM, GEAK_EWORKSPACE, GEAK_EHIP = 1, 2, 3, 4, 5, 6, 7
GEAK_F32, GEAK_F16, GEAK_BF16, GEAK_I32, GEAK_I64, GEAK_U8, GEAK_I8, GEAK_F64 = 0, 1, 2, 3, 4, 5, 6, 7
GEAK_F8E4M3, GEAK_F8E5M2 = 8, 9
GEAK_MXFP8_E4M3, GEAK_MXFP8_E5M2, GEAK_MXINT8, GEAK_MXFP4_E2M1, GEAK_MXFP6_E2M3, GEAK_MXFP6_E3M2 = 10, 11, 12, 13, 14, 15        # element formats of block-scaled segments
GEAK_MAX_CANDIDATES = 256
GEAK_ITEM_FULL, GEAK_ITEM_FIRST, GEAK_ITEM_LAST, GEAK_ITEM_ALIGNED, GEAK_ITEM_ROWS, GEAK_ITEM_REFMAP, GEAK_ITEM_STREAM = 1, 2, 4, 8, 16, 32, 64
GEAK_ULP_BINS = 66
GEAK_STATIC_SCRATCH_BYTES = 8 << 20

DTYPE_CODE = {"f32": GEAK_F32, "f16": GEAK_F16, "bf16": GEAK_BF16, "i32": GEAK_I32, "i64": GEAK_I64,
              "u8": GEAK_U8, "i8": GEAK_I8, "f64": GEAK_F64, "f8e4m3": GEAK_F8E4M3, "f8e5m2": GEAK_F8E5M2}
ELEM_SIZE = {GEAK_F32: 4, GEAK_F16: 2, GEAK_BF16: 2, GEAK_I32: 4, GEAK_I64: 8, GEAK_U8: 1, GEAK_I8: 1, GEAK_F64: 8, GEAK_F8E4M3: 1, GEAK_F8E5M2: 1}

SEGMENT_DTYPE = np.dtype([("byte_offset", "<u8"), ("numel", "<u8"), ("dtype", "<i4"), ("reserved", "<i4")])
SEGMENT2D_DTYPE = np.dtype([("byte_offset", "<u8"), ("rows", "<u8"), ("row_elems", "<u8"), ("pitch_bytes", "<u8"),
                            ("dtype", "<i4"), ("reserved", "<i4")])
SEGMENT_MAPPED_DTYPE = np.dtype([("byte_offset", "<u8"), ("rows", "<u8"), ("row_elems", "<u8"), ("pitch_bytes", "<u8"),
                                 ("ref_byte_offset", "<u8"), ("ref_pitch_bytes", "<u8"), ("ref_elem_stride", "<i4"), ("dtype", "<i4")])
SEGMENT_MX_DTYPE = np.dtype([("byte_offset", "<u8"), ("numel", "<u8"), ("scale_byte_offset", "<u8"), ("dtype", "<i4"), ("reserved", "<i4")])
MX_DTYPE_CODE = {"mxfp8e4m3": GEAK_MXFP8_E4M3, "mxfp8e5m2": GEAK_MXFP8_E5M2, "mxint8": GEAK_MXINT8, "mxfp4e2m1": GEAK_MXFP4_E2M1,
                 "mxfp6e2m3": GEAK_MXFP6_E2M3, "mxfp6e3m2": GEAK_MXFP6_E3M2}
SEGMENT_ANY_DTYPE = np.dtype([("byte_offset", "<u8"), ("rows", "<u8"), ("row_elems", "<u8"), ("pitch_bytes", "<u8"),
                              ("aux_byte_offset", "<u8"), ("aux_pitch_bytes", "<u8"), ("ref_elem_stride", "<i4"), ("dtype", "<i4"),
                              ("kind", "<i4"), ("reserved", "<i4")])
GEAK_KIND_PITCHED, GEAK_KIND_MAPPED, GEAK_KIND_MX = 0, 1, 2
GEAK_MAX_DIMS = 4
SEGMENT_ND_DTYPE = np.dtype([("byte_offset", "<u8"), ("ref_byte_offset", "<u8"), ("shape", "<u8", (GEAK_MAX_DIMS,)),
                             ("stride_bytes", "<u8", (GEAK_MAX_DIMS,)), ("ref_stride_bytes", "<u8", (GEAK_MAX_DIMS,)), ("ndim", "<i4"), ("dtype", "<i4")])
RESULT_DTYPE = np.dtype([("pass", "<i4"), ("reserved", "<i4"), ("mismatch_count", "<u8"),
                         ("first_mismatch", "<i8"), ("max_abs_err", "<f8"), ("max_rel_err", "<f8")])
MISMATCH_DTYPE = np.dtype([("index", "<i8"), ("a", "<f8"), ("b", "<f8"), ("d", "<f8"), ("tol", "<f8")])
ITEM_DTYPE = np.dtype([("byte_offset", "<u8"), ("elem_start", "<u8"), ("segment", "<u4"), ("slot", "<u4"),
                       ("numel", "<u2"), ("dtype", "u1"), ("flags", "u1"), ("next", "<u4")])
GEAK_NO_ITEM = 0xFFFFFFFF
GEAK_MAP_PLAIN, GEAK_MAP_ROTATED, GEAK_MAP_BY_UNIT = 0, 1, 2


class PlanInfo(ctypes.Structure):
    _fields_ = [("num_segments", ctypes.c_uint64), ("num_items", ctypes.c_uint64), ("num_slots", ctypes.c_uint64),
                ("algorithmic_bytes", ctypes.c_uint64), ("num_candidates", ctypes.c_uint32),
                ("grid_blocks", ctypes.c_uint32), ("block_threads", ctypes.c_uint32), ("lds_bytes", ctypes.c_uint32),
                ("item_bytes", ctypes.c_uint32), ("device", ctypes.c_int32),
                ("unit_groups", ctypes.c_uint32), ("block_map", ctypes.c_uint32)]


LAUNCH_FN = ctypes.CFUNCTYPE(ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p)     # geak_launch_fn(user, hip_stream)


class GeakError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {geak_status_string(status)} (status {status})")


_lib = None


def build_library(verbose: bool = False) -> str:
    """Compile csrc/ for gfx950 with hipcc into libgeakcheck.so next to this file."""
    proc = subprocess.run(["bash", BUILD_SCRIPT], capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError("building libgeakcheck.so failed:\n" + proc.stdout + proc.stderr)
    if verbose:
        print(proc.stdout.strip())
    return LIB_PATH


def ensure_library() -> str:
    """Build the library only when none is there; what is built is loaded as it is -- and must have been
    built from the sources beside it (check_build_id raises otherwise)."""
    if not os.path.exists(LIB_PATH):
        build_library()
    check_build_id()
    return LIB_PATH


def source_digest() -> str:
    """Digest of the sources the library is built from, computed as csrc/build.sh does: the header and every
    file of csrc/, concatenated in bytewise path order; 16 hex digits of the SHA-256."""
    import glob
    import hashlib
    root = os.path.dirname(_HERE)
    paths = glob.glob(os.path.join(root, "include", "*.h")) + glob.glob(os.path.join(_HERE, "csrc", "*"))
    rel = sorted(os.path.relpath(p, root).encode() for p in paths if os.path.isfile(p))
    h = hashlib.sha256()
    for r in rel:
        with open(os.path.join(root, r.decode()), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def geak_check_build_id() -> str:
    return library().geak_check_build_id().decode()


def check_build_id() -> str:
    """Raises unless the loaded library was built from the sources in this tree; returns the id."""
    built, here = geak_check_build_id(), source_digest()
    if built != here:
        raise RuntimeError(f"{LIB_PATH} was built from other sources (build id {built}, sources here {here}): "
                           "run paper_2507_23194_amd/csrc/build.sh (or __graft_entry__.build()) again")
    return built


def library() -> ctypes.CDLL:
    """The loaded C library; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run paper_2507_23194_amd/csrc/build.sh "
                               "(or __graft_entry__.build()) first; there is no CPU fallback")
        lib = ctypes.CDLL(LIB_PATH)
        vp, u64, i32, dbl = ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int32, ctypes.c_double
        lib.geak_check_plan.restype = ctypes.c_int
        lib.geak_check_plan.argtypes = [ctypes.POINTER(vp), vp, u64, i32, dbl, dbl, i32, i32]
        lib.geak_check_plan_tolerances.restype = ctypes.c_int
        lib.geak_check_plan_tolerances.argtypes = [ctypes.POINTER(vp), vp, vp, u64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32]
        lib.geak_check_plan_pitched.restype = ctypes.c_int
        lib.geak_check_plan_pitched.argtypes = [ctypes.POINTER(vp), vp, vp, u64, ctypes.c_int32, ctypes.c_double, ctypes.c_double,
                                                ctypes.c_int32, ctypes.c_int32]
        lib.geak_check_plan_mapped.restype = ctypes.c_int
        lib.geak_check_plan_mapped.argtypes = [ctypes.POINTER(vp), vp, vp, u64, ctypes.c_int32, ctypes.c_double, ctypes.c_double,
                                               ctypes.c_int32, ctypes.c_int32]
        lib.geak_check_plan_mx.restype = ctypes.c_int
        lib.geak_check_plan_mx.argtypes = [ctypes.POINTER(vp), vp, vp, u64, ctypes.c_int32, ctypes.c_double, ctypes.c_double,
                                           ctypes.c_int32, ctypes.c_int32]
        lib.geak_check_plan_nd.restype = ctypes.c_int
        lib.geak_check_plan_nd.argtypes = [ctypes.POINTER(vp), vp, vp, u64, ctypes.c_int32, ctypes.c_double, ctypes.c_double,
                                           ctypes.c_int32, ctypes.c_int32]
        lib.geak_check_plan_table.restype = ctypes.c_int
        lib.geak_check_plan_table.argtypes = [ctypes.POINTER(vp), vp, vp, u64, ctypes.c_int32, ctypes.c_double, ctypes.c_double,
                                              ctypes.c_int32, ctypes.c_int32]
        lib.geak_check_plan_dense.restype = ctypes.c_int
        lib.geak_check_plan_dense.argtypes = [ctypes.POINTER(vp), i32, ctypes.POINTER(ctypes.c_int64), i32, i32, dbl, dbl, i32, i32]
        lib.geak_check_workspace_bytes.restype = u64
        lib.geak_check_workspace_bytes.argtypes = [vp]
        lib.geak_check_result_count.restype = u64
        lib.geak_check_result_count.argtypes = [vp]
        lib.geak_check_run.restype = ctypes.c_int
        lib.geak_check_run.argtypes = [vp, vp, ctypes.POINTER(vp), vp, vp, vp]
        lib.geak_check_run_static.restype = ctypes.c_int
        lib.geak_check_run_static.argtypes = [vp, vp, ctypes.POINTER(vp), vp, vp]
        lib.geak_check_destroy.restype = None
        lib.geak_check_destroy.argtypes = [vp]
        lib.geak_check_build_id.restype = ctypes.c_char_p
        lib.geak_check_build_id.argtypes = []
        lib.geak_status_string.restype = ctypes.c_char_p
        lib.geak_status_string.argtypes = [ctypes.c_int]
        lib.geak_check_plan_info.restype = ctypes.c_int
        lib.geak_check_plan_info.argtypes = [vp, ctypes.POINTER(PlanInfo)]
        lib.geak_check_plan_blocks.restype = u64
        lib.geak_check_plan_blocks.argtypes = [vp, vp, u64]
        lib.geak_check_plan_waves.restype = u64
        lib.geak_check_plan_waves.argtypes = [vp, vp, u64]
        lib.geak_check_plan_items.restype = u64
        lib.geak_check_plan_items.argtypes = [vp, vp, u64]
        lib.geak_check_plan_ref_offsets.restype = u64
        lib.geak_check_plan_ref_offsets.argtypes = [vp, vp, u64]
        lib.geak_check_report.restype = ctypes.c_int
        lib.geak_check_report.argtypes = [vp, vp, ctypes.POINTER(vp), vp, vp, ctypes.c_uint32, vp, vp, vp]
        lib.geak_check_ulp_workspace_bytes.restype = u64
        lib.geak_check_ulp_workspace_bytes.argtypes = [vp]
        lib.geak_check_ulp_histogram.restype = ctypes.c_int
        lib.geak_check_ulp_histogram.argtypes = [vp, vp, ctypes.POINTER(vp), vp, vp, vp]
        lib.geak_check_verdicts.restype = ctypes.c_int
        lib.geak_check_verdicts.argtypes = [vp, vp, vp, vp, vp]
        dp = ctypes.POINTER(ctypes.c_double)
        lib.geak_metrics_accuracy.restype = ctypes.c_int
        lib.geak_metrics_accuracy.argtypes = [vp, vp, u64, dp, dp]
        lib.geak_metrics_speedup.restype = ctypes.c_int
        lib.geak_metrics_speedup.argtypes = [vp, u64, vp, u64, u64, dp]
        lib.geak_metrics_pass_at_k.restype = ctypes.c_int
        lib.geak_metrics_pass_at_k.argtypes = [u64, u64, u64, dp]
        lib.geak_timing_flush.restype = ctypes.c_int
        lib.geak_timing_flush.argtypes = [vp, u64, vp]
        lib.geak_timing_measure.restype = ctypes.c_int
        lib.geak_timing_measure.argtypes = [LAUNCH_FN, vp, ctypes.c_uint32, ctypes.c_uint32, vp, u64, vp, dp]
        lib.geak_check_read_probe.restype = ctypes.c_int
        lib.geak_check_read_probe.argtypes = [vp, vp, ctypes.POINTER(vp), vp, vp]
        lib.geak_check_profile_enable.restype = ctypes.c_int
        lib.geak_check_profile_enable.argtypes = [vp, ctypes.c_uint32]
        lib.geak_check_profile_read.restype = u64
        lib.geak_check_profile_read.argtypes = [vp, ctypes.POINTER(ctypes.c_float), u64]
        _lib = lib
    return _lib


EXPORTED = ["geak_check_plan", "geak_check_plan_tolerances", "geak_check_plan_pitched", "geak_check_plan_mapped", "geak_check_plan_mx", "geak_check_plan_nd", "geak_check_plan_table", "geak_check_plan_dense", "geak_check_workspace_bytes", "geak_check_result_count",
            "geak_check_run", "geak_check_run_static", "geak_check_destroy", "geak_status_string", "geak_check_build_id", "geak_check_plan_info",
            "geak_check_plan_items", "geak_check_plan_ref_offsets", "geak_check_plan_blocks", "geak_check_plan_waves", "geak_check_profile_enable", "geak_check_profile_read", "geak_check_read_probe", "geak_check_report",
            "geak_check_ulp_workspace_bytes", "geak_check_ulp_histogram", "geak_check_verdicts",
            "geak_metrics_accuracy", "geak_metrics_speedup", "geak_metrics_pass_at_k", "geak_timing_flush", "geak_timing_measure"]


# ---- one Python function per C entry point -------------------------------------------------------
def geak_status_string(status: int) -> str:
    return library().geak_status_string(int(status)).decode()


def geak_check_plan(segments, num_candidates: int, atol: float, rtol: float, equal_nan, device: int):
    """segments: iterable of (byte_offset, numel, dtype code or name).  Returns (status, plan handle or None)."""
    segs = list(segments)
    arr = np.zeros(len(segs), dtype=SEGMENT_DTYPE)
    for i, (off, n, dt) in enumerate(segs):
        arr[i] = (off, n, DTYPE_CODE.get(dt, dt), 0)
    return geak_check_plan_raw(arr, len(segs), num_candidates, atol, rtol, int(equal_nan), device)


def geak_check_plan_tolerances(segments, tolerances, num_candidates: int, equal_nan, device: int):
    """segments as for geak_check_plan; tolerances: one (atol, rtol) pair per segment, or None (null pointer).
    Returns (status, plan handle or None)."""
    segs = list(segments)
    arr = np.zeros(len(segs), dtype=SEGMENT_DTYPE)
    for i, (off, n, dt) in enumerate(segs):
        arr[i] = (off, n, DTYPE_CODE.get(dt, dt), 0)
    tol = None if tolerances is None else np.ascontiguousarray(np.asarray(list(tolerances), dtype=np.float64).reshape(-1, 2))
    out = ctypes.c_void_p(None)
    st = library().geak_check_plan_tolerances(ctypes.byref(out), arr.ctypes.data, None if tol is None else tol.ctypes.data,
                                              len(segs), num_candidates, int(equal_nan), int(device))
    return st, (out.value if st == GEAK_OK else None)


def geak_check_plan_pitched(segments, tolerances, num_candidates: int, atol: float, rtol: float, equal_nan, device: int):
    """segments: iterable of (byte_offset, rows, row_elems, pitch_bytes, dtype name); tolerances: one (atol, rtol)
    pair per segment or None, then atol / rtol apply to all.  Returns (status, plan handle or None)."""
    segs = list(segments)
    arr = np.zeros(len(segs), dtype=SEGMENT2D_DTYPE)
    for i, (off, rows, row_elems, pitch, dt) in enumerate(segs):
        arr[i] = (off, rows, row_elems, pitch, DTYPE_CODE.get(dt, dt), 0)
    tol = None if tolerances is None else np.ascontiguousarray(np.asarray(list(tolerances), dtype=np.float64).reshape(-1, 2))
    out = ctypes.c_void_p(None)
    st = library().geak_check_plan_pitched(ctypes.byref(out), arr.ctypes.data, None if tol is None else tol.ctypes.data,
                                           len(segs), num_candidates, float(atol), float(rtol), int(equal_nan), int(device))
    return st, (out.value if st == GEAK_OK else None)


def geak_check_plan_mapped(segments, tolerances, num_candidates: int, atol: float, rtol: float, equal_nan, device: int):
    """segments: iterable of (byte_offset, rows, row_elems, pitch_bytes, ref_byte_offset, ref_pitch_bytes,
    ref_elem_stride, dtype name); tolerances: one (atol, rtol) pair per segment or None, then atol / rtol apply to
    all.  Returns (status, plan handle or None)."""
    segs = list(segments)
    arr = np.zeros(len(segs), dtype=SEGMENT_MAPPED_DTYPE)
    for i, (off, rows, row_elems, pitch, ref_off, ref_pitch, ref_stride, dt) in enumerate(segs):
        arr[i] = (off, rows, row_elems, pitch, ref_off, ref_pitch, ref_stride, DTYPE_CODE.get(dt, dt))
    tol = None if tolerances is None else np.ascontiguousarray(np.asarray(list(tolerances), dtype=np.float64).reshape(-1, 2))
    out = ctypes.c_void_p(None)
    st = library().geak_check_plan_mapped(ctypes.byref(out), arr.ctypes.data if len(segs) else None,
                                          None if tol is None else tol.ctypes.data,
                                          len(segs), num_candidates, float(atol), float(rtol), int(equal_nan), int(device))
    return st, (out.value if st == GEAK_OK else None)


def geak_check_plan_mx(segments, tolerances, num_candidates: int, atol: float, rtol: float, equal_nan, device: int):
    """segments: iterable of (payload byte_offset, numel, scale_byte_offset, element format name or code); tolerances:
    one (atol, rtol) pair per segment or None, then atol / rtol apply to all.  Returns (status, plan handle or None)."""
    segs = list(segments)
    arr = np.zeros(len(segs), dtype=SEGMENT_MX_DTYPE)
    for i, (off, n, scale_off, dt) in enumerate(segs):
        arr[i] = (off, n, scale_off, MX_DTYPE_CODE.get(dt, DTYPE_CODE.get(dt, dt)), 0)
    tol = None if tolerances is None else np.ascontiguousarray(np.asarray(list(tolerances), dtype=np.float64).reshape(-1, 2))
    out = ctypes.c_void_p(None)
    st = library().geak_check_plan_mx(ctypes.byref(out), arr.ctypes.data if len(segs) else None,
                                      None if tol is None else tol.ctypes.data,
                                      len(segs), num_candidates, float(atol), float(rtol), int(equal_nan), int(device))
    return st, (out.value if st == GEAK_OK else None)


def geak_check_plan_nd(segments, tolerances, num_candidates: int, atol: float, rtol: float, equal_nan, device: int):
    """segments: iterable of (byte_offset, ref_byte_offset, shape, stride_bytes, ref_stride_bytes, dtype code or name), the
    three sequences of equal length <= GEAK_MAX_DIMS; tolerances: one (atol, rtol) pair per segment or None.
    Returns (status, plan handle or None)."""
    segs = list(segments)
    arr = np.zeros(len(segs), dtype=SEGMENT_ND_DTYPE)
    for i, (off, ref_off, shape, strides, ref_strides, dt) in enumerate(segs):
        nd = len(shape)
        arr[i]["byte_offset"], arr[i]["ref_byte_offset"], arr[i]["ndim"], arr[i]["dtype"] = off, ref_off, nd, DTYPE_CODE.get(dt, dt)
        if nd <= GEAK_MAX_DIMS:                                  # more dimensions than the record holds: the library refuses ndim
            arr[i]["shape"][:nd], arr[i]["stride_bytes"][:nd], arr[i]["ref_stride_bytes"][:nd] = shape, strides, ref_strides
    tol = None if tolerances is None else np.ascontiguousarray(np.asarray(list(tolerances), dtype=np.float64).reshape(-1, 2))
    out = ctypes.c_void_p(None)
    st = library().geak_check_plan_nd(ctypes.byref(out), arr.ctypes.data if len(segs) else None, None if tol is None else tol.ctypes.data,
                                      len(segs), num_candidates, float(atol), float(rtol), int(equal_nan), int(device))
    return st, (out.value if st == GEAK_OK else None)


def geak_check_plan_table(segments, tolerances, num_candidates: int, atol: float, rtol: float, equal_nan, device: int):
    """segments: iterable of ("pitched", byte_offset, rows, row_elems, pitch_bytes, dtype),
    ("mapped", byte_offset, rows, row_elems, pitch_bytes, ref_byte_offset, ref_pitch_bytes, ref_elem_stride, dtype) or
    ("mx", byte_offset, numel, scale_byte_offset, format); tolerances: one (atol, rtol) pair per segment or None.
    Returns (status, plan handle or None)."""
    segs = list(segments)
    arr = np.zeros(len(segs), dtype=SEGMENT_ANY_DTYPE)
    for i, sg in enumerate(segs):
        if sg[0] == "pitched":
            _, off, rows, row_elems, pitch, dt = sg
            arr[i] = (off, rows, row_elems, pitch, 0, 0, 0, DTYPE_CODE.get(dt, dt), GEAK_KIND_PITCHED, 0)
        elif sg[0] == "mapped":
            _, off, rows, row_elems, pitch, ref_off, ref_pitch, ref_stride, dt = sg
            arr[i] = (off, rows, row_elems, pitch, ref_off, ref_pitch, ref_stride, DTYPE_CODE.get(dt, dt), GEAK_KIND_MAPPED, 0)
        else:
            _, off, n, scale_off, dt = sg
            arr[i] = (off, 1, n, 0, scale_off, 0, 0, MX_DTYPE_CODE.get(dt, DTYPE_CODE.get(dt, dt)), GEAK_KIND_MX, 0)
    tol = None if tolerances is None else np.ascontiguousarray(np.asarray(list(tolerances), dtype=np.float64).reshape(-1, 2))
    out = ctypes.c_void_p(None)
    st = library().geak_check_plan_table(ctypes.byref(out), arr.ctypes.data if len(segs) else None,
                                         None if tol is None else tol.ctypes.data,
                                         len(segs), num_candidates, float(atol), float(rtol), int(equal_nan), int(device))
    return st, (out.value if st == GEAK_OK else None)


def geak_check_plan_raw(seg_array, nsegs: int, num_candidates: int, atol: float, rtol: float, equal_nan: int, device: int):
    """As the C call: seg_array is a numpy SEGMENT_DTYPE array or None (null pointer)."""
    out = ctypes.c_void_p(None)
    ptr = None if seg_array is None else seg_array.ctypes.data
    st = library().geak_check_plan(ctypes.byref(out), ptr, nsegs, num_candidates, float(atol), float(rtol),
                                   int(equal_nan), int(device))
    return st, (out.value if st == GEAK_OK else None)


def geak_check_plan_dense(dtype, shape: Sequence[int], num_candidates: int, atol: float, rtol: float, equal_nan, device: int):
    out = ctypes.c_void_p(None)
    shp = (ctypes.c_int64 * max(1, len(shape)))(*shape)
    st = library().geak_check_plan_dense(ctypes.byref(out), DTYPE_CODE.get(dtype, dtype), shp, len(shape), num_candidates,
                                         float(atol), float(rtol), int(equal_nan), int(device))
    return st, (out.value if st == GEAK_OK else None)


def geak_check_workspace_bytes(plan) -> int:
    return int(library().geak_check_workspace_bytes(plan))


def geak_check_result_count(plan) -> int:
    return int(library().geak_check_result_count(plan))


def geak_check_run(plan, ref_ptr: int, cand_ptrs: Sequence[int], workspace_ptr: int, results_ptr: int, stream: int) -> int:
    """All pointers are device addresses as integers; stream is a hipStream_t as integer (0 = default)."""
    arr = (ctypes.c_void_p * max(1, len(cand_ptrs)))(*cand_ptrs)
    return int(library().geak_check_run(plan, ref_ptr, arr, workspace_ptr, results_ptr, stream))


def geak_check_run_static(plan, ref_ptr: int, cand_ptrs: Sequence[int], results_ptr: int, stream: int) -> int:
    """geak_check_run on the library's static scratch array: no workspace argument, no allocation."""
    arr = (ctypes.c_void_p * max(1, len(cand_ptrs)))(*cand_ptrs)
    return int(library().geak_check_run_static(plan, ref_ptr, arr, results_ptr, stream))


def geak_check_report(plan, ref_ptr: int, cand_ptrs: Sequence[int], workspace_ptr: int, results_ptr: int,
                      max_records: int, records_ptr: int, counts_ptr: int, stream: int) -> int:
    """Enqueue the mismatch report of a completed run; all pointers are device addresses."""
    arr = (ctypes.c_void_p * max(1, len(cand_ptrs)))(*cand_ptrs)
    return int(library().geak_check_report(plan, ref_ptr, arr, workspace_ptr, results_ptr, max_records,
                                           records_ptr, counts_ptr, stream))


def geak_check_ulp_workspace_bytes(plan) -> int:
    return int(library().geak_check_ulp_workspace_bytes(plan))


def geak_check_ulp_histogram(plan, ref_ptr: int, cand_ptrs: Sequence[int], ulp_workspace_ptr: int, hist_ptr: int, stream: int) -> int:
    """Enqueue the ulp-distance histogram; all pointers are device addresses."""
    arr = (ctypes.c_void_p * max(1, len(cand_ptrs)))(*cand_ptrs)
    return int(library().geak_check_ulp_histogram(plan, ref_ptr, arr, ulp_workspace_ptr, hist_ptr, stream))


def geak_check_verdicts(plan, results_ptr: int, verdicts_ptr: int, failed_tests_ptr: int, stream: int) -> int:
    """Enqueue the per-candidate verdicts (all unit tests pass) of a completed run; device addresses."""
    return int(library().geak_check_verdicts(plan, results_ptr, verdicts_ptr, failed_tests_ptr or None, stream))


def geak_metrics_accuracy(compiled, correct):
    """(status, call accuracy, execution accuracy) of flag sequences of equal length (host arithmetic)."""
    a = np.ascontiguousarray(np.asarray(compiled, dtype=np.int32))
    b = np.ascontiguousarray(np.asarray(correct, dtype=np.int32))
    if a.shape != b.shape:
        raise ValueError("compiled and correct must have the same length")
    call, execution = ctypes.c_double(), ctypes.c_double()
    st = int(library().geak_metrics_accuracy(a.ctypes.data, b.ctypes.data, a.size, ctypes.byref(call), ctypes.byref(execution)))
    return st, call.value, execution.value


def geak_metrics_speedup(ref_latencies, gen_latencies):
    """(status, speedup) of two [test][repetition] latency tables (host arithmetic)."""
    r = np.ascontiguousarray(np.asarray(ref_latencies, dtype=np.float64))
    g = np.ascontiguousarray(np.asarray(gen_latencies, dtype=np.float64))
    if r.ndim != 2 or g.ndim != 2 or r.shape[0] != g.shape[0]:
        raise ValueError("latency tables must be [test][repetition] with the same number of tests")
    out = ctypes.c_double()
    st = int(library().geak_metrics_speedup(r.ctypes.data, r.shape[1], g.ctypes.data, g.shape[1], r.shape[0], ctypes.byref(out)))
    return st, out.value


def geak_metrics_pass_at_k(n: int, c: int, k: int):
    """(status, pass@k)."""
    out = ctypes.c_double()
    st = int(library().geak_metrics_pass_at_k(n, c, k, ctypes.byref(out)))
    return st, out.value


def geak_timing_flush(scratch_ptr: int, scratch_bytes: int, stream: int) -> int:
    """Enqueue the cache flush (an overwrite of the caller's scratch buffer) on the stream."""
    return int(library().geak_timing_flush(scratch_ptr, scratch_bytes, stream))


def geak_timing_measure(launch, warmup: int, repetitions: int, flush_scratch_ptr: int, flush_bytes: int, stream: int):
    """(status, latencies in ms) of `repetitions` timed calls of launch(stream), each after a cache flush when a
    flush buffer is given.  `launch` is a Python callable taking the stream (an integer) and enqueuing the kernel
    under test on it."""
    def trampoline(_user, hip_stream):
        try:
            launch(hip_stream or 0)
            return 0
        except Exception:
            return 1
    cb = LAUNCH_FN(trampoline)
    out = (ctypes.c_double * max(1, repetitions))()
    st = int(library().geak_timing_measure(cb, None, warmup, repetitions, flush_scratch_ptr or None, flush_bytes, stream or None, out))
    return st, np.array(out[:repetitions], dtype=np.float64)


def geak_check_read_probe(plan, ref_ptr: int, cand_ptrs: Sequence[int], workspace_ptr: int, stream: int) -> int:
    """Enqueue the read-only probe over the bytes a run of the plan reads (measurement aid)."""
    arr = (ctypes.c_void_p * max(1, len(cand_ptrs)))(*cand_ptrs)
    return int(library().geak_check_read_probe(plan, ref_ptr, arr, workspace_ptr, stream))


def geak_check_destroy(plan) -> None:
    library().geak_check_destroy(plan)


def geak_check_plan_info(plan) -> PlanInfo:
    info = PlanInfo()
    st = library().geak_check_plan_info(plan, ctypes.byref(info))
    if st != GEAK_OK:
        raise GeakError(st, "geak_check_plan_info")
    return info


def geak_check_plan_items(plan) -> np.ndarray:
    n = int(library().geak_check_plan_items(plan, None, 0))
    out = np.zeros(n, dtype=ITEM_DTYPE)
    if n:
        library().geak_check_plan_items(plan, out.ctypes.data, n)
    return out


def geak_check_plan_ref_offsets(plan) -> np.ndarray:
    n = int(library().geak_check_plan_ref_offsets(plan, None, 0))
    out = np.zeros(n, dtype=np.uint64)
    if n:
        library().geak_check_plan_ref_offsets(plan, out.ctypes.data, n)
    return out


def geak_check_plan_blocks(plan) -> np.ndarray:
    n = int(library().geak_check_plan_blocks(plan, None, 0))
    out = np.zeros(n, dtype=np.uint32)
    if n:
        library().geak_check_plan_blocks(plan, out.ctypes.data, n)
    return out


def geak_check_plan_waves(plan) -> np.ndarray:
    n = int(library().geak_check_plan_waves(plan, None, 0))
    out = np.zeros(n, dtype=np.uint32)
    if n:
        library().geak_check_plan_waves(plan, out.ctypes.data, n)
    return out


def geak_check_profile_enable(plan, num_pairs: int) -> int:
    return int(library().geak_check_profile_enable(plan, num_pairs))


def geak_check_profile_read(plan, capacity: int) -> np.ndarray:
    buf = (ctypes.c_float * max(1, capacity))()
    n = int(library().geak_check_profile_read(plan, buf, capacity))
    return np.array(buf[:n], dtype=np.float32)


# ---- torch plumbing: device buffers and the current stream ----------------------------------------
class Checker:
    """A plan plus its workspace and results buffers (torch tensors on the plan's device)."""

    def __init__(self, segments=None, *, dense=None, pitched=None, mapped=None, mx=None, table=None, nd=None, num_candidates: int, atol: float = 0.0, rtol: float = 0.0,
                 equal_nan: bool, device: int = 0, tolerances=None):
        import torch
        if table is not None:
            st, plan = geak_check_plan_table(table, tolerances, num_candidates, atol, rtol, equal_nan, device)
        elif nd is not None:
            st, plan = geak_check_plan_nd(nd, tolerances, num_candidates, atol, rtol, equal_nan, device)
        elif mx is not None:
            st, plan = geak_check_plan_mx(mx, tolerances, num_candidates, atol, rtol, equal_nan, device)
        elif mapped is not None:
            st, plan = geak_check_plan_mapped(mapped, tolerances, num_candidates, atol, rtol, equal_nan, device)
        elif pitched is not None:
            st, plan = geak_check_plan_pitched(pitched, tolerances, num_candidates, atol, rtol, equal_nan, device)
        elif tolerances is not None:
            st, plan = geak_check_plan_tolerances(segments, tolerances, num_candidates, equal_nan, device)
        elif dense is not None:
            dtype, shape = dense
            st, plan = geak_check_plan_dense(dtype, list(shape), num_candidates, atol, rtol, equal_nan, device)
        else:
            st, plan = geak_check_plan(segments, num_candidates, atol, rtol, equal_nan, device)
        if st != GEAK_OK:
            raise GeakError(st, "geak_check_plan")
        self.plan = plan
        self.device = device
        self.num_candidates = num_candidates
        dev = torch.device("cuda", device)
        self.workspace = torch.empty(max(16, geak_check_workspace_bytes(plan)), dtype=torch.uint8, device=dev)
        self.n_results = geak_check_result_count(plan)
        self.results = torch.empty(self.n_results * RESULT_DTYPE.itemsize, dtype=torch.uint8, device=dev)

    def info(self) -> PlanInfo:
        return geak_check_plan_info(self.plan)

    def run(self, ref, cands) -> None:
        """Enqueue on torch's current stream of the plan's device; asynchronous."""
        import torch
        assert len(cands) == self.num_candidates
        stream = torch.cuda.current_stream(self.device).cuda_stream
        st = geak_check_run(self.plan, ref.data_ptr(), [c.data_ptr() for c in cands],
                            self.workspace.data_ptr(), self.results.data_ptr(), stream)
        if st != GEAK_OK:
            raise GeakError(st, "geak_check_run")

    def report(self, ref, cands, max_records: int):
        """Mismatch report of the last run on the same tensors: (records, counts), records a
        MISMATCH_DTYPE array of shape (segments, candidates, max_records) of which the first
        counts[s, k] entries of each pair are valid.  Synchronises."""
        import torch
        pairs = self.results.numel() * self.results.element_size() // RESULT_DTYPE.itemsize
        records = torch.zeros(max(1, pairs * max_records * MISMATCH_DTYPE.itemsize), dtype=torch.uint8, device=self.results.device)
        counts = torch.zeros(max(1, pairs), dtype=torch.int32, device=self.results.device)
        stream = torch.cuda.current_stream(self.device).cuda_stream
        st = geak_check_report(self.plan, ref.data_ptr(), [c.data_ptr() for c in cands], self.workspace.data_ptr(),
                               self.results.data_ptr(), max_records, records.data_ptr(), counts.data_ptr(), stream)
        if st != GEAK_OK:
            raise GeakError(st, "geak_check_report")
        torch.cuda.current_stream(self.device).synchronize()
        rec = records.cpu().numpy()[:pairs * max_records * MISMATCH_DTYPE.itemsize].view(MISMATCH_DTYPE)
        return (rec.reshape(-1, self.num_candidates, max_records),
                counts.cpu().numpy()[:pairs].astype(np.int64).reshape(-1, self.num_candidates))

    def ulp_histogram_enqueue(self, ref, cands):
        """Enqueue the ulp-distance histogram on torch's current stream; returns the device tensor
        (segments * candidates * GEAK_ULP_BINS int64 counts) that it fills.  Asynchronous."""
        import torch
        if getattr(self, "ulp_workspace", None) is None:
            dev = self.results.device
            self.ulp_workspace = torch.empty(max(16, geak_check_ulp_workspace_bytes(self.plan)), dtype=torch.uint8, device=dev)
            self.ulp_hist = torch.empty(max(1, self.n_results * GEAK_ULP_BINS), dtype=torch.int64, device=dev)
        stream = torch.cuda.current_stream(self.device).cuda_stream
        st = geak_check_ulp_histogram(self.plan, ref.data_ptr(), [c.data_ptr() for c in cands],
                                      self.ulp_workspace.data_ptr(), self.ulp_hist.data_ptr(), stream)
        if st != GEAK_OK:
            raise GeakError(st, "geak_check_ulp_histogram")
        return self.ulp_hist

    def ulp_histogram(self, ref, cands) -> np.ndarray:
        """Counts by ulp distance, uint64 array of shape (segments, candidates, GEAK_ULP_BINS).  Synchronises."""
        import torch
        hist = self.ulp_histogram_enqueue(ref, cands)
        torch.cuda.current_stream(self.device).synchronize()
        host = hist.cpu().numpy()[:self.n_results * GEAK_ULP_BINS].view(np.uint64)
        return host.reshape(-1, self.num_candidates, GEAK_ULP_BINS)

    def verdicts(self):
        """Per candidate: (all unit tests pass, number of failing tests) of the last run.  Synchronises."""
        import torch
        v = torch.empty(max(1, self.num_candidates), dtype=torch.int32, device=self.results.device)
        f = torch.empty(max(1, self.num_candidates), dtype=torch.int32, device=self.results.device)
        stream = torch.cuda.current_stream(self.device).cuda_stream
        st = geak_check_verdicts(self.plan, self.results.data_ptr(), v.data_ptr(), f.data_ptr(), stream)
        if st != GEAK_OK:
            raise GeakError(st, "geak_check_verdicts")
        torch.cuda.current_stream(self.device).synchronize()
        return v.cpu().numpy()[:self.num_candidates].astype(bool), f.cpu().numpy()[:self.num_candidates].astype(np.int64)

    def read_probe(self, ref, cands) -> None:
        """Enqueue the read-only probe over the same tensors on torch's current stream."""
        import torch
        stream = torch.cuda.current_stream(self.device).cuda_stream
        st = geak_check_read_probe(self.plan, ref.data_ptr(), [c.data_ptr() for c in cands],
                                   self.workspace.data_ptr(), stream)
        if st != GEAK_OK:
            raise GeakError(st, "geak_check_read_probe")

    def read(self) -> np.ndarray:
        """Synchronise and return the records as a RESULT_DTYPE array of shape (segments, candidates)."""
        import torch
        torch.cuda.current_stream(self.device).synchronize()
        host = self.results.cpu().numpy().view(RESULT_DTYPE)
        return host.reshape(-1, self.num_candidates)

    def close(self) -> None:
        if self.plan is not None:
            geak_check_destroy(self.plan)
            self.plan = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def check_workload(w, device: int = 0) -> np.ndarray:
    """Run a synth.Workload (tensors already on the device) and return its records (segments, candidates)."""
    if w.segments is None:
        ck = Checker(dense=(w.dtype, (w.ref.numel(),)), num_candidates=len(w.cands), atol=w.atol, rtol=w.rtol,
                     equal_nan=w.equal_nan, device=device)
    else:
        ck = Checker(w.segments, num_candidates=len(w.cands), atol=w.atol, rtol=w.rtol, equal_nan=w.equal_nan,
                     device=device)
    try:
        ck.run(w.ref, w.cands)
        return ck.read().copy()
    finally:
        ck.close()
