"""Host-side checks of the C-ABI boundary (no GPU): the library loads, exports every symbol the
header declares, validates its arguments, and cuts segments into a work table that covers every
element exactly once."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2507_23194_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return B.library()


def test_header_symbols_are_exported(lib):
    text = open(os.path.join(ROOT, "include", "geak_check.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(geak_[a-z_]+)\s*\(", text))
    assert declared == set(B.EXPORTED)
    for name in declared:
        assert getattr(lib, name) is not None


def test_struct_sizes_match_header():
    assert B.SEGMENT_DTYPE.itemsize == 24
    assert B.RESULT_DTYPE.itemsize == 40
    assert B.ITEM_DTYPE.itemsize == 32
    assert B.MISMATCH_DTYPE.itemsize == 40
    assert ctypes.sizeof(B.PlanInfo) == 64
    assert B.SEGMENT2D_DTYPE.itemsize == 40 and B.SEGMENT_MAPPED_DTYPE.itemsize == 56
    assert B.SEGMENT_MX_DTYPE.itemsize == 32 and B.SEGMENT_ANY_DTYPE.itemsize == 64


def _plan(segs, K=2, atol=1e-3, rtol=1e-3, eq=0, device=-1):
    return B.geak_check_plan(segs, K, atol, rtol, eq, device)


def test_status_strings(lib):
    seen = {B.geak_status_string(s) for s in range(8)}
    assert len(seen) == 8 and "ok" in seen


@pytest.mark.parametrize("kwargs,segs,status", [
    (dict(K=0), [(0, 4, "f32")], B.GEAK_EINVAL),
    (dict(K=257), [(0, 4, "f32")], B.GEAK_EINVAL),
    (dict(atol=-1.0), [(0, 4, "f32")], B.GEAK_EINVAL),
    (dict(rtol=float("nan")), [(0, 4, "f32")], B.GEAK_EINVAL),
    (dict(atol=float("inf")), [(0, 4, "f32")], B.GEAK_EINVAL),
    (dict(rtol=1e300), [(0, 4, "f32")], B.GEAK_EINVAL),          # infinite once converted to binary32
    (dict(eq=2), [(0, 4, "f32")], B.GEAK_EINVAL),
    (dict(), [], B.GEAK_EINVAL),
    (dict(), [(0, 4, 10)], B.GEAK_EDTYPE),
    (dict(), [(0, 4, -1)], B.GEAK_EDTYPE),
    (dict(), [(4, 4, "f64")], B.GEAK_EALIGN),
    (dict(), [(2, 4, "f32")], B.GEAK_EALIGN),
    (dict(), [(1, 4, "f16")], B.GEAK_EALIGN),
    (dict(), [(0, 8, "f32"), (16, 4, "f32")], B.GEAK_EBOUNDS),   # overlap
    (dict(), [(2 ** 63, 2 ** 62, "f32")], B.GEAK_EBOUNDS),       # offset + size overflows
    (dict(), [(0, 2 ** 41, "f16")], B.GEAK_EBOUNDS),             # above the per-segment limit
])
def test_plan_rejects(lib, kwargs, segs, status):
    st, plan = _plan(segs, **kwargs)
    assert st == status and plan is None


def test_null_arguments(lib):
    st, plan = B.geak_check_plan_raw(None, 1, 2, 0.0, 0.0, 0, -1)
    assert st == B.GEAK_EINVAL and plan is None
    assert lib.geak_check_plan(None, None, 1, 2, 0.0, 0.0, 0, -1) == B.GEAK_EINVAL
    assert B.geak_check_workspace_bytes(None) == 0
    assert B.geak_check_result_count(None) == 0
    B.geak_check_destroy(None)


def test_host_only_plan_cannot_run(lib):
    st, plan = _plan([(0, 1000, "f32")])
    assert st == B.GEAK_OK
    try:
        assert B.geak_check_run(plan, 16, [16, 16], 16, 16, 0) == B.GEAK_EINVAL
    finally:
        B.geak_check_destroy(plan)


def test_dense_plan_shapes(lib):
    st, plan = B.geak_check_plan_dense("bf16", [16, 32, 4096, 128], 16, 1e-2, 1.6e-2, 0, -1)
    assert st == B.GEAK_OK
    info = B.geak_check_plan_info(plan)
    n = 16 * 32 * 4096 * 128
    assert info.num_segments == 1 and info.num_candidates == 16
    assert info.algorithmic_bytes == 17 * n * 2
    assert info.num_items == n * 2 // info.item_bytes
    assert B.geak_check_result_count(plan) == 16
    B.geak_check_destroy(plan)
    # scalar and empty shapes
    st, plan = B.geak_check_plan_dense("f32", [], 1, 0, 0, 0, -1)
    assert st == B.GEAK_OK and B.geak_check_plan_info(plan).num_items == 1
    B.geak_check_destroy(plan)
    st, plan = B.geak_check_plan_dense("f32", [5, 0, 7], 3, 0, 0, 0, -1)
    assert st == B.GEAK_OK
    assert B.geak_check_plan_info(plan).num_items == 0 and B.geak_check_workspace_bytes(plan) == 0
    assert B.geak_check_result_count(plan) == 3
    B.geak_check_destroy(plan)
    st, plan = B.geak_check_plan_dense("f32", [4, -1], 3, 0, 0, 0, -1)
    assert st == B.GEAK_EINVAL


def _check_table(segs, K):
    st, plan = _plan(segs, K=K)
    assert st == B.GEAK_OK
    try:
        info = B.geak_check_plan_info(plan)
        items = B.geak_check_plan_items(plan)
        assert len(items) == info.num_items
        waves = info.block_threads // 64
        blocks = B.geak_check_plan_blocks(plan).astype(np.int64)
        assert len(blocks) == info.grid_blocks + 1 and blocks[0] == 0 and blocks[-1] == len(items)
        assert (np.diff(blocks) > 0).all() or len(items) == 0          # no empty block, nothing past the table
        esize = {0: 4, 1: 2, 2: 2, 3: 4, 4: 8, 5: 1, 6: 1, 7: 8, 8: 1, 9: 1}
        # every element of every segment is covered exactly once, in order
        cursor = {}
        for j, it in enumerate(items):
            s = int(it["segment"])
            off, n, dt = segs[s]
            code = B.DTYPE_CODE[dt]
            w = esize[code]
            assert it["dtype"] == code
            assert it["elem_start"] == cursor.get(s, 0)
            assert it["byte_offset"] == off + int(it["elem_start"]) * w
            assert 1 <= it["numel"] <= info.item_bytes // w
            if it["flags"] & B.GEAK_ITEM_FULL:
                assert it["byte_offset"] % 16 == 0 and it["numel"] * w == info.item_bytes
            assert bool(it["flags"] & B.GEAK_ITEM_ALIGNED) == (it["byte_offset"] % 16 == 0)
            if not it["flags"] & B.GEAK_ITEM_ALIGNED:
                # a start off the 16-byte grid: the segment's first item, which ends where a full item read
                # from the boundary before it would end (or with the segment), so that the next one is aligned
                skip = int(it["byte_offset"]) % 16
                assert it["elem_start"] == 0 and skip % w == 0
                assert int(it["numel"]) * w == min(n * w, info.item_bytes - skip)
            cursor[s] = cursor.get(s, 0) + int(it["numel"])
        for s, (off, n, dt) in enumerate(segs):
            assert cursor.get(s, 0) == n
        # items of one segment are contiguous in the table and segments appear in order
        seg_ids = items["segment"].astype(np.int64)
        assert (np.diff(seg_ids) >= 0).all()
        # every wave's list (its first item, then along the next links) stays inside its block's
        # range and ascends; together the lists hold every item exactly once
        first = B.geak_check_plan_waves(plan).astype(np.int64)
        assert len(first) == info.grid_blocks * waves
        nxt = items["next"].astype(np.int64)
        sequences, owner = [], np.full(len(items), -1, dtype=np.int64)
        for wv, j in enumerate(first):
            b = wv // waves
            mine = []
            while j != B.GEAK_NO_ITEM:
                assert blocks[b] <= j < blocks[b + 1] and owner[j] == -1
                assert not mine or j > mine[-1]
                owner[j] = wv
                mine.append(int(j))
                j = nxt[j]
            sequences.append(items[mine])
        assert (owner >= 0).all()
        # run structure: following one wave through its list, FIRST opens and LAST closes each
        # (wave, segment) run, the slot is constant inside a run and unique to it
        seen_slots = {}
        for mine in sequences:
            open_slot = None
            for it in mine:
                if it["flags"] & B.GEAK_ITEM_FIRST:
                    assert open_slot is None
                    open_slot = int(it["slot"])
                    assert open_slot not in seen_slots
                    seen_slots[open_slot] = int(it["segment"])
                assert open_slot == int(it["slot"])
                assert seen_slots[open_slot] == int(it["segment"])
                if it["flags"] & B.GEAK_ITEM_LAST:
                    open_slot = None
            assert open_slot is None
        assert len(seen_slots) == info.num_slots
        assert sorted(seen_slots) == list(range(info.num_slots))
        # slots of a segment are contiguous
        by_seg = {}
        for slot, s in seen_slots.items():
            by_seg.setdefault(s, []).append(slot)
        for s, sl in by_seg.items():
            assert max(sl) - min(sl) + 1 == len(sl)
        assert info.algorithmic_bytes == (K + 1) * sum(n * esize[B.DTYPE_CODE[dt]] for _, n, dt in segs)
        ws = B.geak_check_workspace_bytes(plan)
        replicas = 64
        while replicas > 4 and replicas * K > 512:
            replicas //= 2
        while replicas > 1 and len(segs) * K * replicas * 16 > (16 << 20):
            replicas //= 2
        assert ws == (0 if len(items) == 0 else 256 * 8 + len(segs) * K * replicas * 16 + info.num_slots * K * 16)
    finally:
        B.geak_check_destroy(plan)


def test_work_table_dense(lib):
    _check_table([(0, 1 << 22, "f32")], 3)               # more items than workers
    _check_table([(0, 5000, "f16")], 2)                  # ragged tail
    _check_table([(0, 1, "i32")], 1)
    _check_table([(0, 5000, "i64")], 2)                  # 512 elements per item
    _check_table([(3, 10000, "u8"), (10240, 4096, "i8")], 2)   # 4096 elements per item, the first one 3 bytes off the grid
    _check_table([(8, 700, "i64"), (8192, 3, "i64")], 3)  # a start 8 bytes off the grid
    _check_table([(8, 700, "f64"), (8192, 3, "f64"), (16384, 5000, "f64")], 3)
    _check_table([(5, 9000, "f8e4m3"), (16384, 4096, "f8e5m2")], 2)


def test_work_table_ragged_unaligned(lib):
    rng = np.random.default_rng(0)
    segs, off = [], 0
    for s in range(200):
        dt = ["f32", "f16", "bf16", "i32"][rng.integers(0, 4)]
        w = 2 if dt in ("f16", "bf16") else 4
        off = (off + w - 1) // w * w + w * int(rng.integers(0, 9))
        n = int(2 ** rng.uniform(0, 17)) if s % 7 else 0
        segs.append((off, n, dt))
        off += n * w
    _check_table(segs, 4)
    # same table in shuffled order is still legal (segments need not be sorted by offset)
    perm = rng.permutation(len(segs))
    _check_table([segs[i] for i in perm], 4)


def test_work_table_many_segments_uneven_blocks(lib):
    # the ragged benchmark shape: more items than workers, item count not a multiple of the grid
    rng = np.random.default_rng(3)
    segs, off = [], 0
    for s in range(1024):
        dt = ["f32", "f16", "bf16", "i32"][rng.integers(0, 4)]
        w = 2 if dt in ("f16", "bf16") else 4
        n = max(1, int(2 ** (20 * rng.random())))
        off = (off + 15) // 16 * 16
        segs.append((off, n, dt))
        off += n * w
    _check_table(segs, 4)
    st, plan = _plan(segs, K=4)
    info = B.geak_check_plan_info(plan)
    assert info.num_items % info.grid_blocks != 0
    # ranges are cut at equal estimated cost: blocks of tails hold fewer items than blocks of full items
    blocks = B.geak_check_plan_blocks(plan).astype(np.int64)
    sizes = np.diff(blocks)
    assert sizes.min() >= 1 and sizes.max() > sizes.min()
    # inside a block the items are dealt by cost too; a tail weighs about two and a half items and a
    # 16-bit item about one and a half int32 items, so the counts of a block's waves stay close
    items = B.geak_check_plan_items(plan)
    first = B.geak_check_plan_waves(plan).astype(np.int64)
    counts = np.zeros(len(first), dtype=np.int64)
    for wv, j in enumerate(first):
        while j != B.GEAK_NO_ITEM:
            counts[wv] += 1
            j = int(items["next"][j])
    per_block = counts.reshape(info.grid_blocks, 4)
    assert counts.sum() == info.num_items
    assert (per_block.max(axis=1) - per_block.min(axis=1) <= 6).all()         # a block of bfloat16 items, tails and int32 items
    assert (per_block.max(axis=1) - per_block.min(axis=1)).mean() < 1.5
    B.geak_check_destroy(plan)


def _range_of_block(b, grid, units, block_map):
    """Which range of the block table block b runs (the rule in the header's comment on geak_check_plan_blocks)."""
    if block_map == B.GEAK_MAP_PLAIN:
        return b
    u, q = b % units, b // units
    g = u ^ ((u >> 3) & 7)
    return g * (grid // units) + q if block_map == B.GEAK_MAP_BY_UNIT else q * units + g


def test_ragged_batch_is_cut_by_compute_unit(lib):
    """A batch of mixed dtypes and sizes that fills the grid: the table is laid out by compute unit, every unit
    streams nearly the same number of slices, and the blocks' ranges of a unit are equal in what they cost a wave;
    a dense tensor keeps the plain layout."""
    rng = np.random.default_rng(3)
    segs, off = [], 0
    for s in range(1024):
        dt = ["f32", "f16", "bf16", "i32"][rng.integers(0, 4)]
        w = 2 if dt in ("f16", "bf16") else 4
        n = max(1, int(2 ** (20 * rng.random())))
        off = (off + 15) // 16 * 16
        segs.append((off, n, dt))
        off += n * w
    st, plan = _plan(segs, K=4)
    assert st == B.GEAK_OK
    info = B.geak_check_plan_info(plan)
    units, grid = int(info.unit_groups), int(info.grid_blocks)
    assert units == 256 and grid == 1024 and info.block_map == B.GEAK_MAP_BY_UNIT       # host-only plans assume 256 compute units, four blocks each
    _check_lists_and_runs(plan)
    items = B.geak_check_plan_items(plan)
    blocks = B.geak_check_plan_blocks(plan).astype(np.int64)
    per = grid // units
    full = (items["flags"] & B.GEAK_ITEM_FULL) != 0
    cum_full = np.concatenate([[0], np.cumsum(full)])
    unit_full = np.array([cum_full[blocks[(g + 1) * per]] - cum_full[blocks[g * per]] for g in range(units)])
    assert unit_full.min() >= 0.75 * unit_full.max()                          # units of many small segments hold fewer full items
    big = unit_full >= np.median(unit_full)
    assert unit_full[big].max() - unit_full[big].min() <= 0.05 * unit_full.mean()
    # the map from blocks to ranges is one to one, and a unit's blocks run one group of ranges
    ranges = np.array([_range_of_block(b, grid, units, B.GEAK_MAP_BY_UNIT) for b in range(grid)])
    assert sorted(ranges) == list(range(grid))
    for u in (0, 1, 9, 77, 255):
        assert sorted(ranges[u::units] // per) == [ranges[u] // per] * per
    B.geak_check_destroy(plan)
    # segments all binary32 and of one size, a dense tensor: the plain ranges already load the units evenly; a grid
    # that fills the chip still rotates the XCDs, a smaller one does not
    for st_plan in (_plan([(i * (1 << 22), 1 << 20, "f32") for i in range(64)], K=4), B.geak_check_plan_dense("bf16", [1 << 27], 8, 0, 0, 0, -1)):
        info = B.geak_check_plan_info(st_plan[1])
        assert info.block_map == B.GEAK_MAP_ROTATED and info.unit_groups == 256
        ranges = np.array([_range_of_block(b, 1024, 256, B.GEAK_MAP_ROTATED) for b in range(1024)])
        assert sorted(ranges) == list(range(1024)) and (ranges // 8 == np.arange(1024) // 8).all()       # within its stripe of eight
        assert len({int(r) % 8 for r in ranges[0::8]}) == 8                                                # XCD 0 takes every position of a stripe in turn
        B.geak_check_destroy(st_plan[1])
    st, plan = B.geak_check_plan_dense("f32", [1 << 20], 2, 0, 0, 0, -1)
    info = B.geak_check_plan_info(plan)
    assert info.block_map == B.GEAK_MAP_PLAIN and info.unit_groups == 1 and info.grid_blocks < 1024
    B.geak_check_destroy(plan)


def test_work_table_persistent_grid(lib):
    # a tensor large enough that every worker gets several items: the grid is capped
    st, plan = B.geak_check_plan_dense("f32", [1 << 26], 2, 0, 0, 0, -1)
    info = B.geak_check_plan_info(plan)
    assert info.num_items == (1 << 28) // info.item_bytes
    assert info.grid_blocks == 256 * 4                   # host-only plans assume 256 compute units
    assert info.num_slots == info.grid_blocks * 4
    sizes = np.diff(B.geak_check_plan_blocks(plan).astype(np.int64))
    assert sizes.max() - sizes.min() <= 1                # a dense tensor splits evenly
    B.geak_check_destroy(plan)


def test_per_segment_tolerances_are_validated(lib):
    segs = [(0, 100, "f32"), (400, 50, "f16")]
    st, plan = B.geak_check_plan_tolerances(segs, [(1e-3, 1e-2), (0.0, 0.5)], 2, 0, -1)
    assert st == B.GEAK_OK
    assert B.geak_check_result_count(plan) == 4
    B.geak_check_destroy(plan)
    for bad in ([(1e-3, 1e-2), (-1.0, 0.0)], [(float("nan"), 0.0), (0.0, 0.0)], [(0.0, float("inf")), (0.0, 0.0)],
                [(1e300, 0.0), (0.0, 0.0)]):                       # the last: finite in binary64, infinite in binary32
        st, plan = B.geak_check_plan_tolerances(segs, bad, 2, 0, -1)
        assert st == B.GEAK_EINVAL and plan is None
    st, plan = B.geak_check_plan_tolerances(segs, None, 2, 0, -1)
    assert st == B.GEAK_EINVAL and plan is None
    # binary64 segments take their pair as given: it only has to be finite in binary64
    segs = [(0, 100, "f64"), (800, 50, "f32")]
    st, plan = B.geak_check_plan_tolerances(segs, [(1e300, 1e-320), (1e-3, 0.0)], 2, 0, -1)
    assert st == B.GEAK_OK
    B.geak_check_destroy(plan)
    st, plan = B.geak_check_plan_tolerances(segs, [(1e-3, 0.0), (1e300, 0.0)], 2, 0, -1)
    assert st == B.GEAK_EINVAL and plan is None
    st, plan = B.geak_check_plan(segs[:1], 2, 1e300, 1e300, 0, -1)
    assert st == B.GEAK_OK
    B.geak_check_destroy(plan)
    st, plan = B.geak_check_plan(segs, 2, 1e300, 0.0, 0, -1)
    assert st == B.GEAK_EINVAL and plan is None


def test_ulp_histogram_workspace(lib):
    """Scratch of the ulp histogram: the pointer table plus one 32-bit row per (slot, candidate),
    as long as the widest dtype of the plan needs (18 slots for the 16-bit dtypes, 66 for the 64-bit ones)."""
    st, plan = B.geak_check_plan_dense("f16", [1 << 20], 3, 0, 0, 0, -1)
    info = B.geak_check_plan_info(plan)
    assert B.geak_check_ulp_workspace_bytes(plan) == 2048 + info.num_slots * 3 * 18 * 4
    B.geak_check_destroy(plan)
    st, plan = _plan([(0, 100, "u8"), (128, 10, "f64")], K=2)
    info = B.geak_check_plan_info(plan)
    assert B.geak_check_ulp_workspace_bytes(plan) == 2048 + info.num_slots * 2 * 66 * 4
    B.geak_check_destroy(plan)
    assert B.geak_check_ulp_workspace_bytes(None) == 0


def test_pitched_segments_table(lib):
    """Rows of a pitched segment are cut like segments of their own, with flat row-major element indices;
    rows that lie back to back collapse into the contiguous layout."""
    esize = {"f32": 4, "f16": 2, "u8": 1, "f64": 8}
    segs = [(0, 3, 5000, 5000 * 2 + 32, "f16"), (40000, 7, 100, 416, "f32"), (50003, 4, 1000, 1003, "u8"), (60000, 0, 9, 72, "f64")]
    st, plan = B.geak_check_plan_pitched(segs, None, 2, 1e-3, 1e-3, 0, -1)
    assert st == B.GEAK_OK
    items = B.geak_check_plan_items(plan)
    info = B.geak_check_plan_info(plan)
    assert info.num_segments == 4 and B.geak_check_result_count(plan) == 8
    assert info.algorithmic_bytes == 3 * (3 * 5000 * 2 + 7 * 100 * 4 + 4 * 1000)
    covered = {}
    for it in items:
        s = int(it["segment"])
        off, rows, row_elems, pitch, dt = segs[s]
        w = esize[dt]
        e0, n = int(it["elem_start"]), int(it["numel"])
        r, c = divmod(e0, row_elems)
        if it["flags"] & B.GEAK_ITEM_ROWS:                              # whole short rows, grouped
            assert c == 0 and n % row_elems == 0 and n // row_elems >= 1
            assert off % 16 == 0 and pitch % 16 == 0
            assert (n // row_elems) * -(-row_elems * w // 16) <= 256   # the rows' vectors fit the item's 256 slots
            assert not it["flags"] & B.GEAK_ITEM_FULL
        else:
            assert c + n <= row_elems                                   # otherwise an item never crosses a row
        assert int(it["byte_offset"]) == off + r * pitch + c * w
        assert bool(it["flags"] & B.GEAK_ITEM_ALIGNED) == (int(it["byte_offset"]) % 16 == 0)
        assert e0 == covered.get(s, 0)                                  # in order, no gaps
        covered[s] = e0 + n
    assert covered == {0: 15000, 1: 700, 2: 4000}
    assert [int(i["numel"]) for i in items if i["segment"] == 1] == [700]      # seven rows of 400 bytes: one group
    assert not any(i["flags"] & B.GEAK_ITEM_ROWS for i in items if i["segment"] != 1)   # long rows, or rows on odd bytes
    B.geak_check_destroy(plan)
    # rows back to back are the contiguous layout
    st, p1 = B.geak_check_plan_pitched([(64, 10, 3000, 12000, "f32")], None, 2, 0, 0, 0, -1)
    st2, p2 = B.geak_check_plan([(64, 30000, "f32")], 2, 0, 0, 0, -1)
    assert st == st2 == B.GEAK_OK
    assert (B.geak_check_plan_items(p1) == B.geak_check_plan_items(p2)).all()
    B.geak_check_destroy(p1)
    B.geak_check_destroy(p2)


@pytest.mark.parametrize("rows,row_elems,pitch,dt,group", [
    (1000, 64, 256, "bf16", 32),          # 128-byte rows: 8 vectors each, 32 rows per item
    (77, 33, 80, "bf16", 51),             # 66 bytes: 5 vectors (the last partial), 51 rows per item
    (10, 512, 2064, "f32", 2),            # 2048 bytes: the longest rows that are grouped
    (10, 513, 2064, "f32", 0),            # one element more: row by row, each a tail
    (300, 100, 112, "u8", 36),            # 100 bytes: 7 vectors
    (9, 3, 32, "f64", 128),               # 24 bytes: 2 vectors
    (5, 64, 264, "bf16", 0),              # pitch no multiple of 16: rows start off the boundary, row by row
])
def test_row_group_items(lib, rows, row_elems, pitch, dt, group):
    """Short rows that start on 16-byte boundaries are grouped, as many whole rows as 256 vector slots hold."""
    st, plan = B.geak_check_plan_pitched([(32, rows, row_elems, pitch, dt)], None, 2, 0, 0, 0, -1)
    assert st == B.GEAK_OK
    items = B.geak_check_plan_items(plan)
    grouped = [bool(i["flags"] & B.GEAK_ITEM_ROWS) for i in items]
    if not group:
        assert not any(grouped)
    else:
        assert all(grouped)
        counts = [int(i["numel"]) // row_elems for i in items]
        assert counts == [group] * (rows // group) + ([rows % group] if rows % group else [])
        assert [int(i["elem_start"]) for i in items] == [g * group * row_elems for g in range(len(items))]
        assert [int(i["byte_offset"]) for i in items] == [32 + g * group * pitch for g in range(len(items))]
    assert sum(int(i["numel"]) for i in items) == rows * row_elems
    B.geak_check_destroy(plan)


@pytest.mark.parametrize("segs,status", [
    ([(0, 4, 100, 396, "f32")], B.GEAK_EBOUNDS),                       # rows overlap: pitch shorter than a row
    ([(0, 4, 100, 402, "f32")], B.GEAK_EALIGN),                        # pitch not a multiple of the element size
    ([(2, 4, 100, 400, "f32")], B.GEAK_EALIGN),
    ([(0, 4, 100, 800, "f32"), (400, 4, 100, 800, "f32")], B.GEAK_EBOUNDS),   # interleaved: spans overlap
    ([(0, 2 ** 30, 2 ** 30, 2 ** 32, "f32")], B.GEAK_EBOUNDS),         # too many elements
    ([(0, 2 ** 20, 16, 2 ** 62, "f32")], B.GEAK_EBOUNDS),              # the last row lies beyond the address space
    ([(0, 4, 100, 400, 12)], B.GEAK_EDTYPE),
])
def test_pitched_plan_rejects(lib, segs, status):
    st, plan = B.geak_check_plan_pitched(segs, None, 2, 0, 0, 0, -1)
    assert st == status and plan is None


def test_item_count_in_closed_form(lib):
    """The planner sizes its table before it builds it, without walking the rows: the count must equal the
    number of items it then makes (a smaller count would overflow the reservation unnoticed, a larger one
    would refuse plans that fit), for rows on and off the 16-byte grid, grouped and not."""
    rng = np.random.default_rng(9)
    esize = {"f32": 4, "f16": 2, "u8": 1, "f64": 8}
    for _ in range(60):
        dt = ["f32", "f16", "u8", "f64"][int(rng.integers(0, 4))]
        w = esize[dt]
        rows = int(rng.integers(1, 40))
        row_elems = int(rng.integers(1, 6000))
        pitch = (row_elems + int(rng.integers(0, 40))) * w
        off = int(rng.integers(0, 64)) * w
        st, plan = B.geak_check_plan_pitched([(off, rows, row_elems, pitch, dt)], None, 2, 0.0, 0.0, False, -1)
        assert st == B.GEAK_OK
        try:
            items = B.geak_check_plan_items(plan)
            assert len(items) == B.geak_check_plan_info(plan).num_items
            assert int(items["numel"].astype(np.int64).sum()) == rows * row_elems
        finally:
            B.geak_check_destroy(plan)
    # 2^31 short rows that start on 16-byte boundaries are 2^23 row groups: planned, not refused
    st, plan = B.geak_check_plan_pitched([(0, 1 << 31, 16, 32, "u8")], None, 1, 0.0, 0.0, False, -1)
    assert st == B.GEAK_OK
    assert B.geak_check_plan_info(plan).num_items == (1 << 31) // 256
    B.geak_check_destroy(plan)


def test_mapped_reference_table(lib):
    """Segments whose reference has a layout of its own: the candidates' side is cut like a pitched segment
    (rows never collapse), every item carries the mapped flag, and the table of reference offsets says for each
    item where the element lies that its first element is compared with."""
    esize = {"f32": 4, "f16": 2, "u8": 1, "f64": 8}
    #        cand off, rows, cols, pitch, ref off, ref pitch, stride
    segs = [(0, 3, 5000, 5000 * 2 + 32, 6, 0, 1, "f16"),               # one reference row for all rows; long rows
            (40000, 7, 100, 416, 100, 400, 1, "f32"),                  # own pitch; short rows on the grid: grouped
            (50003, 4, 1000, 1003, 77, 3, 0, "u8"),                    # one element per row, 3 bytes apart; rows off the grid
            (60000, 5, 9, 80, 4096, 0, 0, "f64"),                      # one element for all
            (70000, 0, 9, 72, 0, 0, 1, "f64"),                         # empty
            (80000, 2, 2048, 2048 * 4, 0, 2048 * 4, 1, "f32"),         # rows back to back, each two full-length items
            (100000, 3, 1500, 6000, 8, 4, 3, "f32")]                   # stored transposed: rows 4 bytes apart, elements 3 apart
    st, plan = B.geak_check_plan_mapped(segs, None, 3, 1e-3, 1e-3, 0, -1)
    assert st == B.GEAK_OK
    items = B.geak_check_plan_items(plan)
    ref_off = B.geak_check_plan_ref_offsets(plan)
    info = B.geak_check_plan_info(plan)
    assert len(ref_off) == len(items) == info.num_items
    # candidates' elements K times, the reference's distinct elements once
    cand_bytes = 3 * 5000 * 2 + 7 * 100 * 4 + 4 * 1000 + 5 * 9 * 8 + 2 * 2048 * 4 + 3 * 1500 * 4
    ref_bytes = 5000 * 2 + 7 * 100 * 4 + 4 * 1 + 8 + 2 * 2048 * 4 + 3 * 1500 * 4
    assert info.algorithmic_bytes == 3 * cand_bytes + ref_bytes
    covered = {}
    for it, ro in zip(items, ref_off):
        s = int(it["segment"])
        off, rows, cols, pitch, roff, rpitch, stride, dt = segs[s]
        w = esize[dt]
        e0, n = int(it["elem_start"]), int(it["numel"])
        r, c = divmod(e0, cols)
        assert it["flags"] & B.GEAK_ITEM_REFMAP
        # full items where the candidates' side allows it and the reference is contiguous along the row
        assert bool(it["flags"] & B.GEAK_ITEM_FULL) == (n * w == 4096 and int(it["byte_offset"]) % 16 == 0 and stride == 1)
        assert int(it["byte_offset"]) == off + r * pitch + c * w
        assert int(ro) == roff + r * rpitch + c * w * stride
        if it["flags"] & B.GEAK_ITEM_ROWS:
            assert c == 0 and n % cols == 0
        else:
            assert c + n <= cols
        assert e0 == covered.get(s, 0)
        covered[s] = e0 + n
    assert covered == {0: 15000, 1: 700, 2: 4000, 3: 45, 5: 4096, 6: 4500}
    assert all(i["flags"] & B.GEAK_ITEM_ROWS for i in items if i["segment"] in (1, 3))
    assert [int(i["numel"]) for i in items if i["segment"] == 5] == [1024, 1024, 1024, 1024]
    B.geak_check_destroy(plan)
    # plans without such a segment have no table, and no item of theirs carries the flag
    st, plan = B.geak_check_plan_pitched([(0, 3, 5000, 5000 * 2 + 32, "f16")], None, 2, 0, 0, 0, -1)
    assert len(B.geak_check_plan_ref_offsets(plan)) == 0
    assert not any(i["flags"] & B.GEAK_ITEM_REFMAP for i in B.geak_check_plan_items(plan))
    B.geak_check_destroy(plan)


@pytest.mark.parametrize("seg,status", [
    ((0, 4, 8, 32, 0, 0, -1, "f32"), B.GEAK_EINVAL),              # negative stride
    ((0, 4, 8, 32, 0, 0, 1 << 22, "f32"), B.GEAK_EBOUNDS),        # stride too long
    ((0, 4, 2 ** 39, 2 ** 41, 0, 0, (1 << 22) - 1, "f32"), B.GEAK_EBOUNDS),   # the strided row leaves the address space
    ((0, 4, 8, 32, 2, 0, 1, "f32"), B.GEAK_EALIGN),               # reference offset off the element grid
    ((0, 4, 8, 32, 0, 6, 1, "f32"), B.GEAK_EALIGN),               # reference pitch off the element grid
    ((0, 4, 8, 30, 0, 0, 1, "f32"), B.GEAK_EALIGN),               # the candidates' pitch
    ((0, 4, 8, 16, 0, 0, 1, "f32"), B.GEAK_EBOUNDS),              # the candidates' rows run into each other
    ((0, 4, 8, 32, 2 ** 64 - 8, 4, 1, "f32"), B.GEAK_EBOUNDS),    # the reference leaves the address space
    ((0, 4, 8, 32, 0, 2 ** 63, 1, "f32"), B.GEAK_EBOUNDS),
    ((0, 4, 8, 32, 0, 0, 1, 77), B.GEAK_EDTYPE),
])
def test_mapped_plan_rejects(lib, seg, status):
    st, plan = B.geak_check_plan_mapped([seg], None, 2, 0.0, 0.0, False, -1)
    assert st == status and plan is None
    # overlapping reference rows and a reference region shared by two segments are fine
    st, plan = B.geak_check_plan_mapped([(0, 4, 8, 32, 0, 4, 1, "f32"), (128, 4, 8, 32, 0, 4, 1, "f32")], None, 2, 0.0, 0.0, False, -1)
    assert st == B.GEAK_OK
    B.geak_check_destroy(plan)


def test_block_scaled_plan_table(lib):
    """Block-scaled segments: contiguous one-byte payloads on the 16-byte grid, cut into full items and plain
    tails on block boundaries; payload and scale bytes of every tensor count once."""
    segs = [(0, 4096 * 3 + 64, 20000, "mxfp8e4m3"), (32768, 32, 40000, "mxint8"), (40960, 0, 50000, "mxfp8e5m2")]
    st, plan = B.geak_check_plan_mx(segs, None, 3, 1e-3, 1e-3, 0, -1)
    assert st == B.GEAK_OK
    items = B.geak_check_plan_items(plan)
    info = B.geak_check_plan_info(plan)
    assert info.algorithmic_bytes == 4 * ((4096 * 3 + 64) * 33 // 32 + 33)
    assert [(int(i["byte_offset"]), int(i["elem_start"]), int(i["numel"]), int(i["dtype"])) for i in items] == \
        [(0, 0, 4096, 10), (4096, 4096, 4096, 10), (8192, 8192, 4096, 10), (12288, 12288, 64, 10), (32768, 0, 32, 12)]
    assert [bool(i["flags"] & B.GEAK_ITEM_FULL) for i in items] == [True, True, True, False, False]
    assert all(i["flags"] & B.GEAK_ITEM_ALIGNED and not i["flags"] & (B.GEAK_ITEM_REFMAP | B.GEAK_ITEM_ROWS) for i in items)
    assert all(int(i["elem_start"]) % 32 == 0 for i in items)           # an item starts with a block
    assert len(B.geak_check_plan_ref_offsets(plan)) == 0
    B.geak_check_destroy(plan)
    # the four-bit format: two elements per byte, a full item is 4096 elements = 2 KiB of payload
    st, plan = B.geak_check_plan_mx([(64, 4096 * 2 + 96, 9000, "mxfp4e2m1")], None, 2, 0, 0, 0, -1)
    assert st == B.GEAK_OK
    items = B.geak_check_plan_items(plan)
    assert [(int(i["byte_offset"]), int(i["elem_start"]), int(i["numel"]), bool(i["flags"] & B.GEAK_ITEM_FULL)) for i in items] == \
        [(64, 0, 4096, True), (64 + 2048, 4096, 4096, True), (64 + 4096, 8192, 96, False)]
    assert B.geak_check_plan_info(plan).algorithmic_bytes == 3 * ((8192 + 96) // 2 + (8192 + 96) // 32)
    B.geak_check_destroy(plan)
    # the six-bit formats: four elements in three bytes, a full item is 4096 elements = 3 KiB of payload
    for fmt in ("mxfp6e2m3", "mxfp6e3m2"):
        st, plan = B.geak_check_plan_mx([(64, 4096 * 2 + 96, 9000, fmt)], None, 2, 0, 0, 0, -1)
        assert st == B.GEAK_OK
        items = B.geak_check_plan_items(plan)
        assert [(int(i["byte_offset"]), int(i["elem_start"]), int(i["numel"]), bool(i["flags"] & B.GEAK_ITEM_FULL)) for i in items] == \
            [(64, 0, 4096, True), (64 + 3072, 4096, 4096, True), (64 + 6144, 8192, 96, False)]
        assert all(int(i["dtype"]) == B.MX_DTYPE_CODE[fmt] for i in items)
        assert B.geak_check_plan_info(plan).algorithmic_bytes == 3 * ((8192 + 96) * 3 // 4 + (8192 + 96) // 32)
        B.geak_check_destroy(plan)
    assert B.geak_check_plan_mx([(0, 64, 48, "mxfp6e2m3")], None, 1, 0, 0, 0, -1)[0] == B.GEAK_OK         # 64 elements: 48 bytes
    assert B.geak_check_plan_mx([(0, 64, 47, "mxfp6e2m3")], None, 1, 0, 0, 0, -1)[0] == B.GEAK_EBOUNDS
    # its payload is half as long: scales may sit where a one-byte format's payload would still run
    assert B.geak_check_plan_mx([(0, 64, 32, "mxfp4e2m1")], None, 1, 0, 0, 0, -1)[0] == B.GEAK_OK
    assert B.geak_check_plan_mx([(0, 64, 31, "mxfp4e2m1")], None, 1, 0, 0, 0, -1)[0] == B.GEAK_EBOUNDS


@pytest.mark.parametrize("seg,status", [
    ((8, 64, 100, "mxfp8e4m3"), B.GEAK_EALIGN),                # payload off the 16-byte grid
    ((0, 40, 100, "mxfp8e4m3"), B.GEAK_EINVAL),                # ragged last block
    ((0, 64, 63, "mxfp8e4m3"), B.GEAK_EBOUNDS),                # scales inside the payload
    ((0, 64, 100, "f8e4m3"), B.GEAK_EDTYPE),                   # not a block-scaled element format
    ((0, 64, 100, 16), B.GEAK_EDTYPE),
    ((0, 64, 2 ** 64 - 1, "mxint8"), B.GEAK_EBOUNDS),
])
def test_block_scaled_plan_rejects(lib, seg, status):
    st, plan = B.geak_check_plan_mx([seg], None, 2, 0.0, 0.0, False, -1)
    assert st == status and plan is None
    for code in (B.GEAK_MXFP8_E4M3, B.GEAK_MXFP8_E5M2, B.GEAK_MXINT8, B.GEAK_MXFP4_E2M1, B.GEAK_MXFP6_E2M3, B.GEAK_MXFP6_E3M2):    # these codes are not for the other plan calls
        assert B.geak_check_plan([(0, 64, code)], 2, 0.0, 0.0, False, -1)[0] == B.GEAK_EDTYPE
        assert B.geak_check_plan_pitched([(0, 2, 32, 32, code)], None, 2, 0.0, 0.0, False, -1)[0] == B.GEAK_EDTYPE
        assert B.geak_check_plan_mapped([(0, 2, 32, 32, 0, 0, 1, code)], None, 2, 0.0, 0.0, False, -1)[0] == B.GEAK_EDTYPE
    st, plan = B.geak_check_plan_mx([(0, 64, 1000, "mxint8"), (64, 64, 1001, "mxint8")], None, 1, 0.0, 0.0, False, -1)
    assert st == B.GEAK_EBOUNDS                                            # scale regions collide


def _check_lists_and_runs(plan):
    """The part of a plan that does not depend on how its segments are laid out: the block ranges partition the table, the
    waves' lists hold every item exactly once and ascend, FIRST / LAST bracket the (wave, segment) runs, slots are unique to
    their run and contiguous per segment."""
    info = B.geak_check_plan_info(plan)
    items = B.geak_check_plan_items(plan)
    waves = info.block_threads // 64
    blocks = B.geak_check_plan_blocks(plan).astype(np.int64)
    assert len(blocks) == info.grid_blocks + 1 and blocks[0] == 0 and blocks[-1] == len(items)
    assert (np.diff(blocks) > 0).all() or len(items) == 0
    assert (np.diff(items["segment"].astype(np.int64)) >= 0).all()
    first = B.geak_check_plan_waves(plan).astype(np.int64)
    nxt = items["next"].astype(np.int64)
    owner = np.full(len(items), -1, dtype=np.int64)
    seen_slots = {}
    for wv, j in enumerate(first):
        b, last_j, open_slot = wv // waves, -1, None
        while j != B.GEAK_NO_ITEM:
            assert blocks[b] <= j < blocks[b + 1] and owner[j] == -1 and j > last_j
            owner[j], last_j = wv, j
            it = items[j]
            if it["flags"] & B.GEAK_ITEM_FIRST:
                assert open_slot is None and int(it["slot"]) not in seen_slots
                open_slot = int(it["slot"])
                seen_slots[open_slot] = int(it["segment"])
            assert open_slot == int(it["slot"]) and seen_slots[open_slot] == int(it["segment"])
            if it["flags"] & B.GEAK_ITEM_LAST:
                open_slot = None
            j = nxt[j]
        assert open_slot is None
    assert (owner >= 0).all() and sorted(seen_slots) == list(range(info.num_slots))
    by_seg = {}
    for slot, sg in seen_slots.items():
        by_seg.setdefault(sg, []).append(slot)
    assert all(max(sl) - min(sl) + 1 == len(sl) for sl in by_seg.values())
    return info, items


@pytest.mark.parametrize("seed", range(10))
def test_random_mapped_and_block_scaled_tables(lib, seed):
    """Seeded random plans of the two newer kinds: every element covered exactly once and in order, candidate and
    reference offsets as the layout says, flags as documented, and the same list / run structure as every plan."""
    rng = np.random.default_rng(700 + seed)
    esize = {"f32": 4, "f16": 2, "bf16": 2, "i32": 4, "i64": 8, "u8": 1, "i8": 1, "f64": 8, "f8e4m3": 1, "f8e5m2": 1}
    K = int(rng.integers(1, 9))
    # --- mapped references
    segs, off = [], 0
    for _ in range(int(rng.integers(1, 30))):
        dt = list(esize)[int(rng.integers(0, len(esize)))]
        w = esize[dt]
        rows = int(rng.choice([0, 1, 2, int(rng.integers(3, 50)), int(rng.integers(50, 3000))]))
        cols = int(rng.choice([1, int(rng.integers(2, 40)), int(rng.integers(40, 2048 // w + 1)), int(rng.integers(2048 // w, 5 * 4096 // w))]))
        tight = cols * w
        pitch = int(rng.choice([tight, (tight + 15) // 16 * 16, tight + w * int(rng.integers(1, 9))]))
        off = (off + 15) // 16 * 16 if rng.random() < 0.5 else (off + w - 1) // w * w + w * int(rng.integers(0, 5))
        stride = int(rng.choice([0, 1, 1, 1, 2, 7, max(rows, 1)]))
        rpitch = w * int(rng.choice([0, 1, cols, cols + 3, (cols - 1) * max(stride, 1) + 1]))
        segs.append((off, rows, cols, pitch, w * int(rng.integers(0, 100)), rpitch, stride, dt))
        off += (rows - 1) * pitch + tight if rows else 0
    st, plan = B.geak_check_plan_mapped(segs, None, K, 1e-3, 1e-3, 0, -1)
    assert st == B.GEAK_OK, st
    info, items = _check_lists_and_runs(plan)
    ref_off = B.geak_check_plan_ref_offsets(plan)
    assert len(ref_off) == len(items)
    cursor = {}
    for it, ro in zip(items, ref_off):
        sg = int(it["segment"])
        coff, rows, cols, pitch, roff, rpitch, stride, dt = segs[sg]
        w = esize[dt]
        e0, n = int(it["elem_start"]), int(it["numel"])
        r, c = divmod(e0, cols)
        assert e0 == cursor.get(sg, 0) and it["flags"] & B.GEAK_ITEM_REFMAP
        assert int(it["byte_offset"]) == coff + r * pitch + c * w and int(ro) == roff + r * rpitch + c * w * stride
        assert bool(it["flags"] & B.GEAK_ITEM_ALIGNED) == (int(it["byte_offset"]) % 16 == 0)
        if it["flags"] & B.GEAK_ITEM_ROWS:
            assert c == 0 and n % cols == 0 and coff % 16 == 0 and pitch % 16 == 0 and cols * w <= 2048 and rows > 1
            assert not it["flags"] & B.GEAK_ITEM_FULL
        else:
            assert c + n <= cols
            assert bool(it["flags"] & B.GEAK_ITEM_FULL) == (n * w == 4096 and int(it["byte_offset"]) % 16 == 0 and stride == 1)
        cursor[sg] = e0 + n
    assert all(cursor.get(sg, 0) == segs[sg][1] * segs[sg][2] for sg in range(len(segs)))
    B.geak_check_destroy(plan)
    # --- block-scaled segments
    bits = {"mxfp8e4m3": 8, "mxfp8e5m2": 8, "mxint8": 8, "mxfp4e2m1": 4, "mxfp6e2m3": 6, "mxfp6e3m2": 6}
    segs, off = [], 0
    for _ in range(int(rng.integers(1, 30))):
        fmt = list(bits)[int(rng.integers(0, len(bits)))]
        n = 32 * int(rng.choice([0, 1, int(rng.integers(2, 200)), int(rng.integers(200, 3000))]))
        off = (off + 15) // 16 * 16
        pb = n * bits[fmt] // 8
        segs.append((off, n, off + pb + int(rng.integers(0, 7)), fmt))
        off = segs[-1][2] + n // 32
    st, plan = B.geak_check_plan_mx(segs, None, K, 1e-3, 1e-3, 0, -1)
    assert st == B.GEAK_OK, st
    info, items = _check_lists_and_runs(plan)
    cursor = {}
    for it in items:
        sg = int(it["segment"])
        poff, n_seg, soff, fmt = segs[sg]
        e0, n = int(it["elem_start"]), int(it["numel"])
        assert e0 == cursor.get(sg, 0) and e0 % 32 == 0 and n % 32 == 0 and 0 < n <= 4096
        assert int(it["byte_offset"]) == poff + e0 * bits[fmt] // 8 and int(it["byte_offset"]) % 16 == 0
        assert bool(it["flags"] & B.GEAK_ITEM_FULL) == (n == 4096)
        assert it["flags"] & B.GEAK_ITEM_ALIGNED and not it["flags"] & (B.GEAK_ITEM_ROWS | B.GEAK_ITEM_REFMAP)
        cursor[sg] = e0 + n
    assert all(cursor.get(sg, 0) == segs[sg][1] for sg in range(len(segs)))
    assert info.algorithmic_bytes == (K + 1) * sum(n * bits[f] // 8 + n // 32 for _, n, _, f in segs)
    B.geak_check_destroy(plan)


def test_table_of_mixed_kinds_builds_what_each_entry_point_builds(lib):
    """geak_check_plan_table with one kind of entry gives the items of that kind's own entry point; a mixed table
    gives the concatenation, with the table of reference offsets covering every item."""
    pitched = [(0, 3, 5000, 5000 * 2 + 32, "f16"), (40000, 7, 100, 416, "f32"), (50003, 4, 1000, 1003, "u8"), (60000, 1, 700, 2800, "f32")]
    mapped = [(0, 37, 301, 304 * 4, 8, 0, 1, "f32"), (80000, 5, 9, 80, 4096, 8, 5, "f64")]
    mxs = [(0, 4096 * 2 + 64, 20000, "mxfp8e4m3"), (32768, 8192 + 96, 40000, "mxfp4e2m1")]
    def items_of(st_plan):
        st, plan = st_plan
        assert st == B.GEAK_OK
        out = B.geak_check_plan_items(plan), B.geak_check_plan_ref_offsets(plan), B.geak_check_plan_info(plan).algorithmic_bytes
        B.geak_check_destroy(plan)
        return out
    for own, table in ((B.geak_check_plan_pitched(pitched, None, 2, 0, 0, 0, -1), [("pitched",) + p for p in pitched]),
                       (B.geak_check_plan_mapped(mapped, None, 2, 0, 0, 0, -1), [("mapped",) + m for m in mapped]),
                       (B.geak_check_plan_mx(mxs, None, 2, 0, 0, 0, -1), [("mx",) + m for m in mxs])):
        a, b = items_of(own), items_of(B.geak_check_plan_table(table, None, 2, 0, 0, 0, -1))
        assert (a[0] == b[0]).all() and (a[1] == b[1]).all() and a[2] == b[2]
    # mixed: the kinds one behind the other in one buffer layout
    shift = 200000
    table = [("pitched",) + pitched[1], ("mapped", shift) + mapped[0][1:], ("mx", 2 * shift, mxs[1][1], 2 * shift + 50000, mxs[1][3]),
             ("pitched", 3 * shift, 0, 7, 28, "i32"), ("mapped", 3 * shift + 64) + mapped[1][1:]]
    items, ref_off, alg = items_of(B.geak_check_plan_table(table, None, 3, 0, 0, 0, -1))
    assert sorted(set(int(i["segment"]) for i in items)) == [0, 1, 2, 4] and len(ref_off) == len(items)
    for it, ro in zip(items, ref_off):
        if it["flags"] & B.GEAK_ITEM_REFMAP:
            assert int(it["segment"]) in (1, 4)
        else:
            assert int(ro) == int(it["byte_offset"])
    assert alg == 4 * 7 * 100 * 4 + (3 * 37 * 301 * 4 + 301 * 4) + 4 * ((8192 + 96) // 2 + (8192 + 96) // 32) + (3 * 45 * 8 + 45 * 8)
    # a kind's unused fields must be 0, the kind known
    arr_bad = [("mx", 0, 64, 100, "f32")]
    assert B.geak_check_plan_table(arr_bad, None, 1, 0, 0, 0, -1)[0] == B.GEAK_EDTYPE
    assert B.geak_check_plan_table([("pitched", 0, 1, 64, 64, B.GEAK_MXINT8)], None, 1, 0, 0, 0, -1)[0] == B.GEAK_EDTYPE


def _nd_offsets(off, shape, strides):
    """Byte offset of every element of an N-d layout, row-major over shape (numpy's own index arithmetic)."""
    out = np.full(tuple(shape), off, dtype=np.int64)
    for d, (n, t) in enumerate(zip(shape, strides)):
        idx = np.arange(n, dtype=np.int64) * int(t)
        out = out + idx.reshape([-1 if e == d else 1 for e in range(len(shape))])
    return out.reshape(-1)


def _check_nd_plan(segs, K=2):
    """Every element of every N-d segment is covered exactly once, at the candidates' and the reference's right bytes."""
    st, plan = B.geak_check_plan_nd(segs, None, K, 1e-3, 1e-3, False, -1)
    assert st == B.GEAK_OK, st
    try:
        _check_lists_and_runs(plan)
        items = B.geak_check_plan_items(plan)
        ref_off = B.geak_check_plan_ref_offsets(plan).astype(np.int64)
        assert len(ref_off) == len(items)
        for sg, (off, roff, shape, strides, rstrides, dt) in enumerate(segs):
            w = {"f32": 4, "f16": 2, "bf16": 2, "i32": 4, "i64": 8, "u8": 1, "f64": 8, "i8": 1}[dt]
            want_c, want_r = _nd_offsets(off, shape, strides), _nd_offsets(roff, shape, rstrides)
            got_c, got_r = np.full(want_c.size, -1, np.int64), np.full(want_c.size, -1, np.int64)
            mine = [j for j in range(len(items)) if int(items[j]["segment"]) == sg]
            # the 2-D geometry of the segment as the plan holds it: from two neighbouring elements / rows of the items
            for j in mine:
                it = items[j]
                e0, n, base = int(it["elem_start"]), int(it["numel"]), int(it["byte_offset"])
                assert (got_c[e0:e0 + n] == -1).all()
                if it["flags"] & B.GEAK_ITEM_ROWS:
                    cols = shape[-1]
                    rows_here = n // cols
                    # rows of one 2-D block: pitch = the second-to-last stride on both sides
                    for r in range(rows_here):
                        got_c[e0 + r * cols: e0 + (r + 1) * cols] = base + r * strides[-2] + np.arange(cols) * w
                        got_r[e0 + r * cols: e0 + (r + 1) * cols] = ref_off[j] + r * rstrides[-2] + np.arange(cols) * rstrides[-1]
                else:
                    got_c[e0:e0 + n] = base + np.arange(n) * w
                    got_r[e0:e0 + n] = ref_off[j] + np.arange(n) * rstrides_inner(shape, strides, rstrides)
                    assert bool(it["flags"] & B.GEAK_ITEM_FULL) <= (rstrides_inner(shape, strides, rstrides) == w)
            assert np.array_equal(got_c, want_c), sg
            assert np.array_equal(got_r, want_r), sg
    finally:
        B.geak_check_destroy(plan)


def rstrides_inner(shape, strides, rstrides):
    """The reference's byte stride along what the planner treats as a row: the innermost dimension with extent > 1 (the
    dimensions merged into it share that stride by construction); the element size's worth for a single element."""
    for d in range(len(shape) - 1, -1, -1):
        if shape[d] > 1:
            return int(rstrides[d])
    return 0


def test_nd_segments_cover_every_element_at_the_right_bytes(lib):
    segs = [
        # [B, H, S, D] contiguous against a reference [1, H, 1, D] (broadcast over batch and sequence)
        (0, 0, (2, 3, 5, 8), (480, 160, 32, 4), (0, 32, 0, 4), "f32"),
        # a slice of a larger bf16 array (padded rows and planes) against a transposed view of a compact one
        (4096, 512, (3, 4, 6), (400, 80, 2), (2, 6, 24), "bf16"),
        # four dimensions that do not merge: every stride padded; reference permuted and strided
        (8192, 2048, (2, 3, 4, 5), (2000, 600, 120, 8), (8, 16, 1920, 48), "i64"),
        # long rows: full items inside N-d blocks; reference row contiguous, planes broadcast
        (65536, 16384, (2, 2, 3, 3000), (80000, 38000, 12032, 4), (0, 36000, 12000, 4), "i32"),
        # one element, and an empty tensor
        (400000, 0, (1, 1), (4, 4), (0, 0), "f32"),
        (400016, 0, (3, 0, 2), (0, 8, 4), (0, 0, 4), "f32"),
        # a column of a wider array: the innermost extent is 1 and the rows are a padded stride apart
        (500000, 200, (5, 6, 1), (96, 16, 4), (24, 4, 4), "f32"),
        (501000, 300, (7, 1), (12, 4), (4, 4), "f32"),
        # bytes, short rows on the 16-byte grid (row groups inside the blocks), reference one element per row
        (400064, 100, (3, 5, 7, 16), (2048, 256, 32, 1), (35, 7, 1, 0), "u8"),
    ]
    _check_nd_plan(segs)


def test_nd_segments_that_fold_give_the_two_dimensional_plan(lib):
    """Dimensions that both tensors step through in one stride are merged, extents of 1 dropped: a contiguous [2, 3, 4, 8]
    tensor against a [1, 1, 1, 8] reference is 24 rows of 8 with one reference row; against a reference of the same
    layout it is one row."""
    pairs = [
        ((0, 64, (2, 3, 4, 8), (384, 128, 32, 4), (0, 0, 0, 4), "f32"), (0, 24, 8, 32, 64, 0, 1, "f32")),
        ((0, 64, (2, 3, 4, 8), (384, 128, 32, 4), (384, 128, 32, 4), "f32"), (0, 1, 192, 768, 64, 0, 1, "f32")),
        ((16, 0, (5, 1, 7), (56, 999, 8), (0, 0, 16), "i64"), (16, 5, 7, 56, 0, 0, 2, "i64")),
        ((0, 0, (6, 10), (64, 4), (4, 24), "f32"), (0, 6, 10, 64, 0, 4, 6, "f32")),                      # transposed: stays two-dimensional
        ((0, 32, (4, 2, 16), (128, 64, 2), (0, 0, 0), "f16"), (0, 4 * 2, 16, 64, 32, 0, 0, "f16")),       # splat over everything
    ]
    for nd, mapped in pairs:
        st, a = B.geak_check_plan_nd([nd], None, 3, 0.0, 0.0, False, -1)
        st2, b = B.geak_check_plan_mapped([mapped], None, 3, 0.0, 0.0, False, -1)
        assert st == B.GEAK_OK and st2 == B.GEAK_OK, (nd, st, st2)
        ia, ib = B.geak_check_plan_items(a), B.geak_check_plan_items(b)
        assert ia.tobytes() == ib.tobytes(), nd
        assert np.array_equal(B.geak_check_plan_ref_offsets(a), B.geak_check_plan_ref_offsets(b))
        assert B.geak_check_plan_info(a).algorithmic_bytes == B.geak_check_plan_info(b).algorithmic_bytes
        B.geak_check_destroy(a); B.geak_check_destroy(b)


@pytest.mark.parametrize("seg,status", [
    ((0, 0, (2, 3, 4, 5, 6), (1, 1, 1, 1, 1), (1, 1, 1, 1, 1), "u8"), B.GEAK_EINVAL),                 # five dimensions
    ((0, 0, (4, 8), (64, 8), (32, 4), "f32"), B.GEAK_EINVAL),                                        # candidates' innermost not contiguous
    ((0, 0, (4, 8), (30, 4), (32, 4), "f32"), B.GEAK_EALIGN),                                        # stride off the element grid
    ((0, 0, (4, 8), (32, 4), (34, 4), "f32"), B.GEAK_EALIGN),
    ((2, 0, (4, 8), (32, 4), (32, 4), "f32"), B.GEAK_EALIGN),                                        # offset off the element grid
    ((0, 0, (4, 8), (16, 4), (32, 4), "f32"), B.GEAK_EBOUNDS),                                       # rows run into each other
    ((0, 0, (3, 4, 8), (100, 32, 4), (0, 0, 4), "f32"), B.GEAK_EBOUNDS),                             # planes run into each other
    ((0, 0, (2, 3, 4, 8), (300, 128, 32, 4), (0, 0, 0, 4), "f32"), B.GEAK_EBOUNDS),
    ((0, 0, (1 << 21, 1 << 21), (1 << 23, 4), (0, 4), "f32"), B.GEAK_EBOUNDS),                       # more than 2^40 elements
    ((0, 0, (4, 8), (32, 4), (0, 4 << 22), "f32"), B.GEAK_EBOUNDS),                                  # reference stride too large
    ((0, 0, (1 << 17, 1 << 16, 2, 2), (1 << 23, 64, 16, 4), (0, 0, 0, 4), "f32"), B.GEAK_EBOUNDS),     # more 2-D blocks than the item table holds
    ((0, 0, (4, 8), (32, 4), (0, 4), "mxint8"), B.GEAK_EDTYPE),
    ((2 ** 64 - 64, 0, (4, 8), (32, 4), (0, 4), "f32"), B.GEAK_EBOUNDS),                             # beyond the address space
])
def test_nd_plan_rejects(lib, seg, status):
    dt = seg[5]
    seg = seg[:5] + (B.MX_DTYPE_CODE.get(dt, dt),)
    st, plan = B.geak_check_plan_nd([seg], None, 2, 0.0, 0.0, False, -1)
    assert st == status and plan is None, (seg, st)


def test_row_groups_of_whole_vectors_are_marked_for_streaming(lib):
    """Row groups whose rows are whole 16-byte vectors carry GEAK_ITEM_STREAM (the compare kernel streams them like full
    items, slots that a group leaves idle reading as 0); rows that end in a partial vector, a reference with strided
    rows and pitches whose group does not fit 32 bits do not."""
    def flags_of(st_plan):
        st, plan = st_plan
        assert st == B.GEAK_OK
        items = B.geak_check_plan_items(plan)
        B.geak_check_destroy(plan)
        return [int(f) for f in items["flags"]]
    S, R = B.GEAK_ITEM_STREAM, B.GEAK_ITEM_ROWS
    # 40 rows of 64 binary32 (16 vectors each): groups of 16 rows, the last one of 8 rows
    f = flags_of(B.geak_check_plan_pitched([(0, 40, 64, 320, "f32")], None, 2, 0, 0, 0, -1))
    assert len(f) == 3 and all(x & S and x & R for x in f)
    # rows of 48 binary32 (12 vectors: 21 rows leave 4 slots idle) stream, rows of 62 (the last vector partial) do not
    assert all(x & S for x in flags_of(B.geak_check_plan_pitched([(0, 64, 48, 256, "f32")], None, 2, 0, 0, 0, -1)))
    assert not any(x & S for x in flags_of(B.geak_check_plan_pitched([(0, 64, 62, 256, "f32")], None, 2, 0, 0, 0, -1)))
    # a reference of its own: contiguous rows (any pitch, also one row for all) and one element per row stream, strided rows do not
    f = flags_of(B.geak_check_plan_mapped([(0, 32, 128, 512, 0, 0, 1, "bf16")], None, 2, 0, 0, 0, -1))
    assert all(x & S and x & B.GEAK_ITEM_REFMAP for x in f) and len(f) == 2
    assert all(x & S for x in flags_of(B.geak_check_plan_mapped([(0, 32, 128, 512, 0, 2, 0, "bf16")], None, 2, 0, 0, 0, -1)))
    assert not any(x & S for x in flags_of(B.geak_check_plan_mapped([(0, 32, 128, 512, 0, 512, 2, "bf16")], None, 2, 0, 0, 0, -1)))
    # a pitch of 2^29 bytes: fifteen of them do not fit 32 bits
    f = flags_of(B.geak_check_plan_pitched([(0, 32, 64, 1 << 29, "f32")], None, 2, 0, 0, 0, -1))
    assert all(x & R for x in f) and not any(x & S for x in f)
    f = flags_of(B.geak_check_plan_pitched([(0, 32, 64, 1 << 28, "f32")], None, 2, 0, 0, 0, -1))
    assert all(x & S for x in f)
    # fifteen pitches plus a vector's offset in the row must fit as well
    f = flags_of(B.geak_check_plan_pitched([(0, 32, 64, ((1 << 32) - 256) // 15 // 16 * 16, "f32")], None, 2, 0, 0, 0, -1))
    assert not any(x & S for x in f)
