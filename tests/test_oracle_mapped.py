"""Pins of the oracle's reference-with-its-own-layout front end (oracle.gather_rows / check_segment_mapped):
hand-derived records for the four layouts -- own pitch, one row for all rows, one element per row, one
element for everything -- and the tie to the plain check on the same elements."""
import numpy as np
import pytest

from helpers import record_tuple


def test_gather_is_plain_index_arithmetic(oracle_mod):
    buf = np.arange(40, dtype=np.float32)                     # element i holds the value i
    g = lambda **kw: oracle_mod.gather_rows(buf, dtype="f32", **kw).view(np.float32).tolist()
    assert g(rows=2, row_elems=3, byte_offset=8, pitch_bytes=20) == [2, 3, 4, 7, 8, 9]          # rows five elements apart
    assert g(rows=3, row_elems=2, byte_offset=4, pitch_bytes=0) == [1, 2, 1, 2, 1, 2]           # one row for all
    assert g(rows=2, row_elems=3, byte_offset=0, pitch_bytes=16, elem_stride=0) == [0, 0, 0, 4, 4, 4]   # one element per row
    assert g(rows=2, row_elems=2, byte_offset=12, pitch_bytes=0, elem_stride=0) == [3, 3, 3, 3]         # one element in all
    assert g(rows=0, row_elems=5, byte_offset=0, pitch_bytes=0) == []
    with pytest.raises(ValueError):
        oracle_mod.gather_rows(buf, 1, 1, "f32", 2, 0)


def test_hand_derived_records(oracle_mod):
    kw = dict(atol=0.25, rtol=0.0, equal_nan=False)
    # candidates: two rows of three, the second row 16 bytes behind the first (one float of padding)
    cand = np.array([1.0, 2.0, 3.0, 99.0, 1.0, 2.5, 3.0, 99.0], np.float32)
    # one reference row for both rows: [1, 2, 3]; flat index 4 (row 1, column 1) is off by 0.5
    ref_row = np.array([7.0, 1.0, 2.0, 3.0], np.float32)
    rec = oracle_mod.check_segment_mapped(ref_row, cand, 2, 3, "f32", cand_byte_offset=0, cand_pitch_bytes=16,
                                          ref_byte_offset=4, ref_pitch_bytes=0, **kw)
    assert record_tuple(rec) == record_tuple(dict(zip(("pass", "mismatch_count", "first_mismatch", "max_abs_err", "max_rel_err"),
                                                      (0, 1, 4, 0.5, 0.25))))
    # one reference element per row: row 0 against 2, row 1 against 1 -> d = [1,0,1 | 0,1.5,2]
    ref_col = np.array([2.0, 1.0], np.float32)
    rec = oracle_mod.check_segment_mapped(ref_col, cand, 2, 3, "f32", cand_byte_offset=0, cand_pitch_bytes=16,
                                          ref_byte_offset=0, ref_pitch_bytes=4, ref_elem_stride=0, **kw)
    assert (int(rec["mismatch_count"]), int(rec["first_mismatch"]), float(rec["max_abs_err"]), float(rec["max_rel_err"])) == (4, 0, 2.0, 2.0)
    # a reference with rows of its own pitch (three floats of padding) and an offset: equal to the candidates but one element
    ref_own = np.array([5.0, 5.0, 1.0, 2.0, 3.0, 0.0, 0.0, 0.0, 1.0, 2.0, 3.0], np.float32)
    rec = oracle_mod.check_segment_mapped(ref_own, cand, 2, 3, "f32", cand_byte_offset=0, cand_pitch_bytes=16,
                                          ref_byte_offset=8, ref_pitch_bytes=24, **kw)
    assert (int(rec["mismatch_count"]), int(rec["first_mismatch"]), float(rec["max_abs_err"])) == (1, 4, 0.5)
    # one reference element for everything, integer dtype: exact equality
    ci = np.array([7, 7, 8, 7], np.int32)
    rec = oracle_mod.check_segment_mapped(np.array([0, 7], np.int32), ci, 2, 2, "i32", cand_byte_offset=0, cand_pitch_bytes=8,
                                          ref_byte_offset=4, ref_pitch_bytes=0, ref_elem_stride=0, atol=9.0, rtol=9.0, equal_nan=False)
    assert (int(rec["mismatch_count"]), int(rec["first_mismatch"]), float(rec["max_abs_err"]), float(rec["max_rel_err"])) == (1, 2, 1.0, 1.0 / 7.0)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16", "u8", "f64", "i64"])
def test_same_layout_on_both_sides_is_the_plain_check(oracle_mod, dtype):
    rng = np.random.default_rng(3)
    w = oracle_mod.ELEM_SIZE[dtype]
    rows, row_elems, pitch = 7, 33, (33 + 5) * w
    raw_ref = rng.integers(0, 256, rows * pitch + 64, dtype=np.uint8)
    raw_cand = raw_ref.copy()
    raw_cand[rng.integers(0, raw_cand.size, 40)] ^= 0x11
    a = oracle_mod.gather_rows(raw_cand, rows, row_elems, dtype, 16, pitch)
    b = oracle_mod.gather_rows(raw_ref, rows, row_elems, dtype, 16, pitch)
    plain = oracle_mod.check_segment(b, a, rows * row_elems, dtype, 1e-3, 1e-3, True)
    mapped = oracle_mod.check_segment_mapped(raw_ref, raw_cand, rows, row_elems, dtype, 1e-3, 1e-3, True, 16, pitch, 16, pitch)
    assert record_tuple(plain) == record_tuple(mapped)


def test_transposed_reference_equals_plain_check_of_its_transpose(oracle_mod):
    """A reference stored transposed (element (r, c) at c * rows + r: rows one element apart, neighbours of a row
    `rows` apart) judged through the index map gives the record of the plain check against its transpose written
    out by the library's transpose."""
    rng = np.random.default_rng(41)
    rows, cols = 13, 29
    b = rng.normal(size=(rows, cols)).astype(np.float32)
    a = (b * (1 + 2e-3 * rng.normal(size=b.shape))).astype(np.float32)
    stored = np.ascontiguousarray(b.T)                              # cols x rows
    got = oracle_mod.check_segment_mapped(stored.view(np.uint8).reshape(-1), a.view(np.uint8).reshape(-1), rows, cols, "f32",
                                          1e-3, 1e-3, False, 0, cols * 4, 0, 4, rows)
    want = oracle_mod.check_segment(b.reshape(-1), a.reshape(-1), rows * cols, "f32", 1e-3, 1e-3, False)
    assert all(got[f] == want[f] for f in got.dtype.names) and int(got["mismatch_count"]) > 0
    # every third element of a longer row
    wide = rng.integers(0, 100, size=(rows, 3 * cols + 5)).astype(np.int32)
    picked = np.ascontiguousarray(wide[:, 2::3][:, :cols])
    g = oracle_mod.gather_rows(wide.view(np.uint8).reshape(-1), rows, cols, "i32", 8, (3 * cols + 5) * 4, 3)
    assert (g.view(np.int32) == picked.reshape(-1)).all()


def test_gather_nd_equals_numpys_own_strided_views(oracle_mod):
    """The N-d index map against the library's: broadcasting, transposes and slices of a numpy array are strided
    views whose strides numpy computes itself; gathering by those strides must give the view's elements in order."""
    rng = np.random.default_rng(5)
    for dt, np_t in (("f32", np.float32), ("bf16", np.uint16), ("i64", np.int64), ("u8", np.uint8)):
        base = rng.integers(0, 200, (3, 4, 5, 6)).astype(np_t)
        views = [base, base.transpose(2, 0, 3, 1), base[:, 1:3, ::2, 1:], base.transpose(3, 2, 1, 0)[::2],
                 np.broadcast_to(base[:, :1, :, :1], (3, 7, 5, 2)), np.broadcast_to(base[1, 2, 3, 4:5].reshape(()), (2, 3, 4)),
                 np.broadcast_to(base[None, 0, :, 0, :], (4, 4, 6))]
        for v in views:
            off = v.__array_interface__["data"][0] - base.__array_interface__["data"][0]
            got = oracle_mod.gather_nd(base, v.shape, v.strides, dt, off)
            assert np.array_equal(got, np.ascontiguousarray(v).reshape(-1).view(got.dtype)), (dt, v.shape, v.strides)
    # two dimensions: the 2-D map is the special case
    buf = rng.integers(0, 255, 4000).astype(np.uint8)
    assert np.array_equal(oracle_mod.gather_nd(buf, (7, 9), (80, 8), "f32", 12), oracle_mod.gather_rows(buf, 7, 9, "f32", 12, 80, 2))
    with pytest.raises(ValueError):
        oracle_mod.gather_nd(buf, (2, 2), (6, 4), "f32", 0)


def test_nd_records_by_hand_and_against_the_plain_check(oracle_mod):
    # candidate [2, 2, 3] contiguous; reference [2, 1, 3] broadcast over the middle dimension
    ref = np.array([1, 2, 3, 10, 20, 30], np.float32)
    cand = np.array([1, 2, 3, 1, 2, 4, 10, 20, 30, 11, 20, 30], np.float32)        # elements (0,1,2) and (1,1,0) differ by 1
    r = oracle_mod.check_segment_nd(ref, cand, (2, 2, 3), "f32", 0.5, 0.0, False, 0, (24, 12, 4), 0, (12, 0, 4))
    assert (int(r["pass"]), int(r["mismatch_count"]), int(r["first_mismatch"])) == (0, 2, 5)
    assert float(r["max_abs_err"]) == 1.0 and float(r["max_rel_err"]) == float(np.float32(1.0) / np.float32(3.0))
    r = oracle_mod.check_segment_nd(ref, cand, (2, 2, 3), "f32", 1.0, 0.0, False, 0, (24, 12, 4), 0, (12, 0, 4))
    assert int(r["pass"]) == 1 and int(r["first_mismatch"]) == -1                  # inclusive: 1 <= 1
    # the same through numpy's broadcasting and the plain check
    rng = np.random.default_rng(6)
    b = rng.standard_normal((3, 1, 4, 1)).astype(np.float32)
    a = (np.broadcast_to(b, (3, 5, 4, 6)) + (rng.random((3, 5, 4, 6)) < 0.1) * 0.25).astype(np.float32)
    want = oracle_mod.check_segment(np.ascontiguousarray(np.broadcast_to(b, a.shape)), a, a.size, "f32", 1e-3, 1e-3, False)
    got = oracle_mod.check_segment_nd(b, a, a.shape, "f32", 1e-3, 1e-3, False, 0, a.strides, 0, (16, 0, 4, 0))
    assert got == want and got["mismatch_count"] > 0
