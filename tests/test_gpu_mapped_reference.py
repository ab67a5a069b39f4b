"""References with a layout of their own (geak_check_plan_mapped): one reference row for all rows, one
reference element per row, one element for the whole output, a reference with its own pitch and start, strided
reference rows and a reference stored transposed.
Records, mismatch report and ulp histogram equal what the oracle finds when it gathers the reference by plain
index arithmetic (oracle.gather_rows) and applies the unchanged rule -- every dtype, rows that are grouped,
rows that start off the 16-byte grid, rows longer than several work items, several such segments in one plan."""
import numpy as np
import pytest
import torch

from paper_2507_23194_amd import binding as B
from paper_2507_23194_amd import synth
from test_gpu_parity import _special_case, _assert_same

pytestmark = pytest.mark.gpu

DTYPES = ["f32", "f16", "bf16", "i32", "i64", "u8", "i8", "f64", "f8e4m3", "f8e5m2"]
STORE = {1: np.uint8, 2: np.uint16, 4: np.uint32, 8: np.uint64}


def _segment(rng, dtype, rows, cols, kind, cand_pad, cand_shift, ref_pad, ref_shift, cand_base, ref_base, K):
    """Bytes of one segment for the reference buffer and for K candidate buffers, plus its table entry.
    kind: "row" one reference row for all rows, "col" one reference element per row, "scalar" one for all,
    "pitch" a full reference with its own pitch.  Pads and shifts in elements."""
    w = synth.ELEM_SIZE[dtype]
    store = STORE[w]
    if kind in ("strided", "transposed"):
        return _segment_strided(rng, dtype, rows, cols, kind, cand_pad, cand_shift, ref_pad, ref_shift, cand_base, ref_base, K)
    ref_rows, ref_cols = {"row": (1, cols), "col": (rows, 1), "scalar": (1, 1), "pitch": (rows, cols)}[kind]
    n_store = ref_rows * ref_cols
    b_store, a_store = _special_case(rng, dtype, max(1, n_store))
    b_store, a_store = b_store.view(store), a_store.view(store)
    _, other = _special_case(rng, dtype, max(1, rows * cols))
    other = other.view(store)
    # the reference's bytes: its rows ref_cols + ref_pad elements apart (a column's elements 1 + ref_pad apart)
    ref_pitch_elems = 0 if kind in ("row", "scalar") else ref_cols + ref_pad
    ref_len = ref_shift + (ref_rows - 1) * ref_pitch_elems + ref_cols if rows * cols else ref_shift
    ref_bytes = rng.integers(0, 256, ref_len * w + 16, dtype=np.uint8)
    ref_elems = ref_bytes[: (ref_len) * w].view(store)
    for r in range(ref_rows if rows * cols else 0):
        ref_elems[ref_shift + r * ref_pitch_elems: ref_shift + r * ref_pitch_elems + ref_cols] = b_store[r * ref_cols:(r + 1) * ref_cols]
    # what candidate element (r, c) is compared with, and the same gather of the perturbed copy
    rr = np.arange(rows)[:, None] * (ref_cols if ref_rows > 1 else 0)
    cc = np.arange(cols)[None, :] * (1 if ref_cols > 1 else 0)
    idx = (rr + cc).reshape(-1)
    if n_store == 1:
        idx = np.zeros(rows * cols, dtype=np.int64)
    cand_pitch_elems = cols + cand_pad
    cand_len = cand_shift + (rows - 1) * cand_pitch_elems + cols if rows * cols else cand_shift
    cands = []
    for k in range(K):
        full = (b_store[idx] if k == 1 else a_store[idx]).copy()           # candidate 1 equals the reference everywhere
        if k != 1 and full.size:
            same = rng.random(full.size) < 0.3
            full[same] = b_store[idx][same]
            repl = rng.random(full.size) < 0.01
            full[repl] = other[repl]
        cb = rng.integers(0, 256, cand_len * w + 16, dtype=np.uint8)
        ce = cb[: cand_len * w].view(store)
        for r in range(rows if cols else 0):
            ce[cand_shift + r * cand_pitch_elems: cand_shift + r * cand_pitch_elems + cols] = full[r * cols:(r + 1) * cols]
        cands.append(cb)
    entry = (cand_base + cand_shift * w, rows, cols, cand_pitch_elems * w, ref_base + ref_shift * w, ref_pitch_elems * w,
             0 if kind in ("col", "scalar") else 1, dtype)
    return ref_bytes, cands, entry


def _segment_strided(rng, dtype, rows, cols, kind, cand_pad, cand_shift, ref_pad, ref_shift, cand_base, ref_base, K):
    """The reference's rows are strided: "transposed" stores element (r, c) at c * rows + r (rows one element apart,
    neighbours of a row `rows` apart), "strided" keeps every (2 + ref_pad)-th element of rows that lie a full strided
    row apart."""
    w = synth.ELEM_SIZE[dtype]
    store = STORE[w]
    n = rows * cols
    b_full, a_full = _special_case(rng, dtype, max(1, n))
    b_full, a_full = b_full.view(store)[:n], a_full.view(store)[:n]
    _, other = _special_case(rng, dtype, max(1, n))
    other = other.view(store)[:n]
    if kind == "transposed":
        stride, ref_pitch_elems = max(rows, 1), 1
    else:
        stride = 2 + ref_pad
        ref_pitch_elems = (cols - 1) * stride + 1 + ref_pad if cols else 0
    r_idx, c_idx = np.divmod(np.arange(n), max(cols, 1))
    where = ref_shift + r_idx * ref_pitch_elems + c_idx * stride
    ref_len = int(where.max()) + 1 if n else ref_shift
    ref_bytes = rng.integers(0, 256, ref_len * w + 16, dtype=np.uint8)
    ref_bytes[: ref_len * w].view(store)[where] = b_full
    cand_pitch_elems = cols + cand_pad
    cand_len = cand_shift + (rows - 1) * cand_pitch_elems + cols if n else cand_shift
    cands = []
    for k in range(K):
        full = (b_full if k == 1 else a_full).copy()
        if k != 1 and n:
            same = rng.random(n) < 0.3
            full[same] = b_full[same]
            repl = rng.random(n) < 0.01
            full[repl] = other[repl]
        cb = rng.integers(0, 256, cand_len * w + 16, dtype=np.uint8)
        ce = cb[: cand_len * w].view(store)
        for r in range(rows if cols else 0):
            ce[cand_shift + r * cand_pitch_elems: cand_shift + r * cand_pitch_elems + cols] = full[r * cols:(r + 1) * cols]
        cands.append(cb)
    entry = (cand_base + cand_shift * w, rows, cols, cand_pitch_elems * w, ref_base + ref_shift * w, ref_pitch_elems * w, stride, dtype)
    return ref_bytes, cands, entry


def _build(rng, specs, K):
    """Packs the segments one behind the other (each starting 16-byte aligned plus its own shift)."""
    ref_parts, cand_parts, table = [], [[] for _ in range(K)], []
    ref_base = cand_base = 0
    for sp in specs:
        rb, cbs, entry = _segment(rng, K=K, cand_base=cand_base, ref_base=ref_base, **sp)
        pad_r, pad_c = (-rb.size) % 16, (-cbs[0].size) % 16
        ref_parts.append(np.concatenate([rb, np.zeros(pad_r, np.uint8)]))
        for k in range(K):
            cand_parts[k].append(np.concatenate([cbs[k], np.zeros(pad_c, np.uint8)]))
        table.append(entry)
        ref_base += rb.size + pad_r
        cand_base += cbs[0].size + pad_c
    return np.concatenate(ref_parts), [np.concatenate(p) for p in cand_parts], table


def _run_and_compare(oracle_mod, ref_np, cand_nps, table, atol, rtol, equal_nan, what, with_report=True, tolerances=None):
    ref = torch.from_numpy(ref_np.copy()).cuda()
    cands = [torch.from_numpy(c.copy()).cuda() for c in cand_nps]
    K = len(cands)
    ck = B.Checker(mapped=table, num_candidates=K, atol=atol, rtol=rtol, equal_nan=equal_nan, device=0, tolerances=tolerances)
    try:
        ck.run(ref, cands)
        gpu = ck.read().copy()
        rec, cnt = ck.report(ref, cands, 6) if with_report else (None, None)
        hist = ck.ulp_histogram(ref, cands) if with_report else None
    finally:
        ck.close()
    cpu = np.zeros((len(table), K), dtype=gpu.dtype)
    for s, (coff, rows, cols, cpitch, roff, rpitch, stride, dtype) in enumerate(table):
        if tolerances is not None:
            atol, rtol = tolerances[s]
        for k in range(K):
            r = oracle_mod.check_segment_mapped(ref_np, cand_nps[k], rows, cols, dtype, atol, rtol, equal_nan,
                                                coff, cpitch, roff, rpitch, stride)
            for f in cpu.dtype.names:
                cpu[s, k][f] = r[f]
    _assert_same(gpu, cpu, what)
    if not with_report:
        return gpu
    for s, (coff, rows, cols, cpitch, roff, rpitch, stride, dtype) in enumerate(table):
        if tolerances is not None:
            atol, rtol = tolerances[s]
        b = oracle_mod.gather_rows(ref_np, rows, cols, dtype, roff, rpitch, stride)
        for k in range(K):
            a = oracle_mod.gather_rows(cand_nps[k], rows, cols, dtype, coff, cpitch, 1)
            rep = oracle_mod.report_segment(b, a, rows * cols, dtype, atol, rtol, equal_nan, 6)
            assert int(cnt[s, k]) == len(rep), (what, s, k)
            got = rec[s, k][:len(rep)]
            assert (got["index"] == rep["index"]).all(), (what, s, k)
            assert all(np.array_equal(got[f], rep[f], equal_nan=True) for f in ("a", "b", "d", "tol")), (what, s, k)
            assert (hist[s, k] == oracle_mod.ulp_histogram_segment(b, a, rows * cols, dtype)).all(), (what, s, k)
    return gpu


@pytest.mark.parametrize("dtype", DTYPES)
def test_all_layouts_every_dtype(oracle_mod, dtype):
    """Short rows (grouped when the candidates' rows start on the grid, one by one when they do not), all
    reference layouts (one row, one element per row, one element, own pitch, strided rows, stored transposed),
    reference and candidates at their own odd element offsets."""
    print("mapped layouts", dtype, flush=True)
    w = synth.ELEM_SIZE[dtype]
    rng = np.random.default_rng(9100 + DTYPES.index(dtype))
    grid = 16 // w                                   # elements per 16 bytes
    specs = []
    for kind in ("row", "col", "scalar", "pitch", "strided", "transposed"):
        # rows on the grid (pitch a multiple of 16 bytes, no shift): row groups
        specs.append(dict(dtype=dtype, rows=37, cols=3 * grid + 1, kind=kind, cand_pad=grid - 1, cand_shift=0, ref_pad=2, ref_shift=1))
        # rows off the grid: shifted first items and plain tails, row by row
        specs.append(dict(dtype=dtype, rows=9, cols=5 * grid + 3, kind=kind, cand_pad=1 if grid > 1 else 3, cand_shift=grid - 1, ref_pad=0, ref_shift=3))
    specs.append(dict(dtype=dtype, rows=0, cols=7, kind="row", cand_pad=0, cand_shift=0, ref_pad=0, ref_shift=0))     # empty
    specs.append(dict(dtype=dtype, rows=1, cols=1, kind="scalar", cand_pad=0, cand_shift=0, ref_pad=0, ref_shift=0))  # one element
    ref_np, cand_nps, table = _build(rng, specs, K=3)
    for equal_nan, atol, rtol in ((False, 1e-3, 1e-3), (True, 0.0, 0.0)):
        gpu = _run_and_compare(oracle_mod, ref_np, cand_nps, table, atol, rtol, equal_nan, f"{dtype} equal_nan={equal_nan}")
        assert (gpu[-2, :]["pass"] == 1).all() and (gpu[-2, :]["first_mismatch"] == -1).all()     # the empty segment


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("kind", ["row", "col", "pitch", "transposed"])
def test_rows_longer_than_work_items(oracle_mod, dtype, kind):
    """Rows of more than two full work items plus a tail: the items inside a row are as long as full ones but
    take the guarded path, since their reference lies elsewhere; rows start on and off the grid."""
    print("mapped long rows", dtype, kind, flush=True)
    w = synth.ELEM_SIZE[dtype]
    per = 4096 // w
    rng = np.random.default_rng(9200 + 7 * DTYPES.index(dtype) + len(kind))
    specs = [dict(dtype=dtype, rows=3, cols=2 * per + 77, kind=kind, cand_pad=(16 // w) * 3 - (77 % (16 // w)), cand_shift=0, ref_pad=5, ref_shift=2),
             dict(dtype=dtype, rows=2, cols=per + 1, kind=kind, cand_pad=0, cand_shift=1, ref_pad=0, ref_shift=0)]
    ref_np, cand_nps, table = _build(rng, specs, K=5)
    _run_and_compare(oracle_mod, ref_np, cand_nps, table, 1e-3, 1e-3, False, f"{dtype} {kind} long rows")


@pytest.mark.parametrize("seed", range(12))
def test_random_mapped_plan(oracle_mod, seed):
    """Seeded random plans: a few segments of random dtype, geometry (rows from one element to several work items,
    pitches tight, padded to the grid or odd, starts on or off the grid), reference layout and tolerances."""
    rng = np.random.default_rng(9400 + seed)
    nsegs, K = int(rng.integers(1, 9)), int(rng.integers(1, 6))
    specs, tols = [], []
    for _ in range(nsegs):
        dtype = DTYPES[int(rng.integers(0, len(DTYPES)))]
        w = synth.ELEM_SIZE[dtype]
        grid = 16 // w
        rows = int(rng.choice([0, 1, 2, int(rng.integers(3, 40)), int(rng.integers(40, 300))]))
        cols = int(rng.choice([1, int(rng.integers(2, 40)), int(rng.integers(40, 2048 // w + 1)), int(rng.integers(2048 // w, 3 * 4096 // w))]))
        if rows * cols > 30000:
            rows = max(1, 30000 // cols)
        on_grid = bool(rng.integers(0, 2))
        cand_pad = int((-cols) % grid + grid * rng.integers(0, 3)) if on_grid else int(rng.integers(0, 9))
        specs.append(dict(dtype=dtype, rows=rows, cols=cols, kind=str(rng.choice(["row", "col", "scalar", "pitch", "strided", "transposed"])),
                          cand_pad=cand_pad, cand_shift=0 if on_grid else int(rng.integers(0, 2 * grid)),
                          ref_pad=int(rng.integers(0, 5)), ref_shift=int(rng.integers(0, 7))))
        tols.append((float(rng.choice([0.0, 1e-3, 0.25])), float(rng.choice([0.0, 1e-2, 0.125]))))
    print("random mapped plan", seed, [(sp["dtype"], sp["rows"], sp["cols"], sp["kind"]) for sp in specs], "K", K, flush=True)
    ref_np, cand_nps, table = _build(rng, specs, K=K)
    _run_and_compare(oracle_mod, ref_np, cand_nps, table, 0.0, 0.0, bool(rng.integers(0, 2)), f"random mapped plan {seed}", tolerances=tols)


def test_mapped_reference_equals_plain_check_of_the_expanded_reference(oracle_mod):
    """The same candidates checked twice on the GPU: against a reference row through the mapped plan, and
    against that row written out for every row through the plain pitched plan.  Every record agrees."""
    print("mapped vs expanded", flush=True)
    rng = np.random.default_rng(9300)
    rows, cols, K = 129, 1000, 4
    b_row = rng.normal(size=cols).astype(np.float32)
    cands = [(np.tile(b_row, (rows, 1)) * (1 + 1e-3 * rng.normal(size=(rows, cols)))).astype(np.float32) for _ in range(K)]
    cands[2] = np.tile(b_row, (rows, 1))
    cands[0][77, 5] = np.nan
    ref_row = torch.from_numpy(b_row).cuda()
    ref_full = torch.from_numpy(np.tile(b_row, (rows, 1))).cuda()
    dc = [torch.from_numpy(c).cuda() for c in cands]
    recs = []
    for kw, ref in ((dict(mapped=[(0, rows, cols, cols * 4, 0, 0, 1, "f32")]), ref_row), (dict(pitched=[(0, rows, cols, cols * 4, "f32")]), ref_full)):
        ck = B.Checker(num_candidates=K, atol=1e-3, rtol=1e-3, equal_nan=False, device=0, **kw)
        try:
            ck.run(ref, dc)
            recs.append(ck.read().copy())
        finally:
            ck.close()
    _assert_same(recs[0], recs[1], "row reference against its expansion")
    # the read-only probe walks the same span of every buffer: refused where the reference is shorter
    ck = B.Checker(mapped=[(0, rows, cols, cols * 4, 0, 0, 1, "f32")], num_candidates=K, atol=1e-3, rtol=1e-3, equal_nan=False, device=0)
    try:
        with pytest.raises(B.GeakError) as err:
            ck.read_probe(ref_row, dc)
        assert err.value.status == B.GEAK_EINVAL
    finally:
        ck.close()
    assert recs[0][0, 2]["pass"] == 1 and recs[0][0, 0]["first_mismatch"] <= 77 * cols + 5
    cpu = oracle_mod.check_segment_mapped(b_row.view(np.uint8), cands[0].view(np.uint8).reshape(-1), rows, cols, "f32", 1e-3, 1e-3, False,
                                          0, cols * 4, 0, 0, 1)
    assert int(recs[0][0, 0]["mismatch_count"]) == int(cpu["mismatch_count"])


def test_mapped_plan_argument_errors():
    ok = (0, 4, 8, 32, 0, 0, 1, "f32")
    st, plan = B.geak_check_plan_mapped([ok], None, 2, 0.0, 0.0, False, 0)
    assert st == B.GEAK_OK
    B.geak_check_destroy(plan)
    for bad, code in (((0, 4, 8, 32, 0, 0, -1, "f32"), B.GEAK_EINVAL),         # negative stride
                      ((0, 4, 8, 32, 0, 0, 1 << 22, "f32"), B.GEAK_EBOUNDS),   # stride too long
                      ((0, 4, 8, 32, 2, 0, 1, "f32"), B.GEAK_EALIGN),          # reference offset off the element grid
                      ((0, 4, 8, 32, 0, 6, 1, "f32"), B.GEAK_EALIGN),          # reference pitch off the element grid
                      ((0, 4, 8, 30, 0, 0, 1, "f32"), B.GEAK_EALIGN),          # candidates' pitch
                      ((0, 4, 8, 16, 0, 0, 1, "f32"), B.GEAK_EBOUNDS),         # candidates' rows run into each other
                      ((0, 4, 8, 32, 2 ** 64 - 8, 4, 1, "f32"), B.GEAK_EBOUNDS),   # reference leaves the address space
                      ((0, 4, 8, 32, 0, 0, 1, 77), B.GEAK_EDTYPE)):
        st, plan = B.geak_check_plan_mapped([bad], None, 2, 0.0, 0.0, False, 0)
        assert st == code and plan is None, (bad, st)
