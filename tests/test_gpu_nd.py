"""N-d segments (geak_check_plan_nd): candidates that are slices of larger, padded arrays, references that are
broadcast along some dimensions, transposed, strided or permuted views of compact ones.  The arrays are built with
numpy, whose own strides and offsets go into the table; records, mismatch report and ulp histogram equal what the
oracle finds when it gathers both sides by plain index arithmetic (oracle.gather_nd) and applies the unchanged rule."""
import numpy as np
import pytest
import torch

from paper_2507_23194_amd import binding as B
from paper_2507_23194_amd import synth
from test_gpu_parity import _special_case, _assert_same

pytestmark = pytest.mark.gpu

STORE = {1: np.uint8, 2: np.uint16, 4: np.uint32, 8: np.uint64}


def _offset(view, base):
    return view.__array_interface__["data"][0] - base.__array_interface__["data"][0]


def _case(rng, dtype, shape, ref_kind, cand_pad, K):
    """One segment: returns (reference storage, reference view, [candidate storage], [candidate view]) as arrays of the
    dtype's storage type.  ref_kind: "same" | "bcast:<mask>" (1 = the dimension is broadcast) | "perm:<order>" |
    "strided" (every other element of a wider innermost dimension)."""
    w = synth.ELEM_SIZE[dtype]
    store = STORE[w]
    nd = len(shape)
    if ref_kind.startswith("bcast:"):
        mask = [c == "1" for c in ref_kind[6:]]
        small = tuple(1 if m else e for e, m in zip(shape, mask))
    else:
        small = tuple(shape)
    n_small = int(np.prod(small)) if nd else 1
    b, a = _special_case(rng, dtype, max(1, n_small))
    b, a = b.view(store)[:n_small].reshape(small), a.view(store)[:n_small].reshape(small)
    if ref_kind.startswith("perm:"):
        order = [int(c) for c in ref_kind[5:]]
        inv = np.argsort(order)
        ref_store = np.ascontiguousarray(b.transpose(order))                # stored permuted ...
        ref_view = ref_store.transpose(inv)                                 # ... and viewed back in the candidates' order
    elif ref_kind == "strided":
        wide = rng.integers(0, 255, tuple(shape[:-1]) + (2 * shape[-1] + 1,)).astype(store)
        wide[..., 1::2][..., :shape[-1]] = b
        ref_store, ref_view = wide, wide[..., 1::2][..., :shape[-1]]
    else:
        ref_store = b.copy()
        ref_view = np.broadcast_to(ref_store, shape)
    want_b, want_a = np.broadcast_to(b, shape), np.broadcast_to(a, shape)
    cands_store, cands_view = [], []
    padded = tuple(e + p for e, p in zip(shape, cand_pad))
    for k in range(K):
        full = (want_b if k == 1 else want_a).copy()                        # candidate 1 equals the reference everywhere
        if k != 1 and full.size:
            same = rng.random(full.shape) < 0.3
            full[same] = want_b[same]
        if nd == 0:                                                         # a 0-d view of a one-element array
            big = rng.integers(0, 255, (1,)).astype(store)
            view = big.reshape(())
        else:
            big = rng.integers(0, 255, padded).astype(store)
            view = big[tuple(slice(p // 2, p // 2 + e) for e, p in zip(shape, cand_pad))]
        view[...] = full
        cands_store.append(big)
        cands_view.append(view)
    return ref_store, ref_view, cands_store, cands_view


def _run(oracle_mod, cases, K, atol, rtol, equal_nan, what, base_shift=0, ulp=True):
    """cases: list of (dtype, shape, ref_kind, cand_pad).  All segments of a tensor go into one buffer, 16-byte aligned
    one after the other (plus base_shift bytes in front, a multiple of the largest element)."""
    rng = np.random.default_rng(abs(hash(what)) % (2 ** 32))
    ref_parts, cand_parts, segs, meta = [], [[] for _ in range(K)], [], []
    ref_at, cand_at = base_shift, base_shift
    for dtype, shape, ref_kind, cand_pad in cases:
        rs, rv, cs, cv = _case(rng, dtype, shape, ref_kind, cand_pad, K)
        ref_parts.append((ref_at, rs))
        for k in range(K):
            cand_parts[k].append((cand_at, cs[k]))
        segs.append((cand_at + _offset(cv[0], cs[0]), ref_at + _offset(rv, rs), tuple(shape), tuple(cv[0].strides), tuple(rv.strides), dtype))
        meta.append((dtype, shape))
        ref_at = (ref_at + rs.nbytes + 15) // 16 * 16 + base_shift % 16
        cand_at = (cand_at + cs[0].nbytes + 15) // 16 * 16 + base_shift % 16

    def assemble(parts, total):
        buf = np.full(total + 16, 0xA5, np.uint8)
        for at, arr in parts:
            buf[at:at + arr.nbytes] = arr.reshape(-1).view(np.uint8)
        return buf
    ref_np = assemble(ref_parts, ref_at)
    cand_nps = [assemble(cand_parts[k], cand_at) for k in range(K)]
    ref = torch.from_numpy(ref_np.copy()).cuda()
    cands = [torch.from_numpy(c.copy()).cuda() for c in cand_nps]
    ck = B.Checker(nd=segs, num_candidates=K, atol=atol, rtol=rtol, equal_nan=equal_nan, device=0)
    try:
        ck.run(ref, cands)
        gpu = ck.read().copy()
        rep, cnt = ck.report(ref, cands, 5)
        hist = ck.ulp_histogram(ref, cands).copy() if ulp else None
    finally:
        ck.close()
    cpu = np.zeros_like(gpu)
    for s, (off, roff, shape, strides, rstrides, dtype) in enumerate(segs):
        b = oracle_mod.gather_nd(ref_np, shape, rstrides, dtype, roff)
        for k in range(K):
            a = oracle_mod.gather_nd(cand_nps[k], shape, strides, dtype, off)
            r = oracle_mod.check_segment(b, a, b.size, dtype, atol, rtol, equal_nan)
            for f in cpu.dtype.names:
                cpu[s, k][f] = r[f]
            want = oracle_mod.report_segment(b, a, b.size, dtype, atol, rtol, equal_nan, 5)
            assert int(cnt[s, k]) == len(want), (what, s, k)
            got = rep[s, k][:len(want)]
            assert (got["index"] == want["index"]).all(), (what, s, k, got["index"], want["index"])
            assert all(np.array_equal(got[f], want[f], equal_nan=True) for f in ("a", "b", "d", "tol")), (what, s, k)
            if ulp:
                assert (hist[s, k] == oracle_mod.ulp_histogram_segment(b, a, b.size, dtype)).all(), (what, s, k)
    _assert_same(gpu, cpu, what)
    return gpu


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16", "i32", "i64", "u8", "f64", "f8e4m3"])
def test_broadcast_and_permuted_references(oracle_mod, dtype):
    print("nd", dtype, flush=True)
    cases = [
        (dtype, (2, 3, 5, 8), "bcast:1010", (0, 0, 0, 0)),            # [1, H, 1, D] against [B, H, S, D]
        (dtype, (2, 3, 5, 8), "bcast:0101", (1, 0, 2, 4)),            # one element per row, planes of their own; padded candidates
        (dtype, (3, 4, 6), "perm:201", (0, 1, 2)),                    # a permuted (transposed) reference
        (dtype, (2, 3, 4, 5), "perm:3120", (1, 1, 1, 3)),
        (dtype, (4, 3, 40), "strided", (0, 2, 8)),                    # every other element of wider rows
        (dtype, (2, 2, 3, 3000), "bcast:1000", (0, 0, 0, 8)),         # long rows: full work items inside the blocks
        (dtype, (5, 7, 16), "bcast:111", (0, 0, 0)),                  # one reference element for everything
        (dtype, (3, 0, 4), "same", (0, 0, 0)),                        # empty
        (dtype, (), "same", ()),                                      # a single element
        (dtype, (2, 3, 4, 8), "same", (0, 0, 0, 0)),                  # the same layout on both sides: folds to one row
    ]
    gpu = _run(oracle_mod, cases, 3, 1e-2, 1e-2, False, f"nd {dtype}")
    assert (gpu[:, 1]["pass"] == 1).all() or dtype in ("f32", "f16", "bf16", "f64", "f8e4m3")      # floats: NaN against itself fails without equal_nan
    _run(oracle_mod, cases[:5], 2, 0.0, 0.0, True, f"nd {dtype} exact")


def test_bases_off_the_sixteen_byte_grid(oracle_mod):
    cases = [("f32", (3, 4, 10), "bcast:100", (0, 1, 3)), ("f32", (2, 2, 3, 33), "perm:0132", (0, 0, 1, 1)), ("f32", (4, 5, 64), "bcast:010", (0, 0, 0))]
    for shift in (4, 8, 12):
        print("nd shifted", shift, flush=True)
        _run(oracle_mod, cases, 3, 1e-3, 1e-3, False, f"nd shift {shift}", base_shift=shift)


@pytest.mark.parametrize("seed", range(6))
def test_random_nd_plans(oracle_mod, seed):
    print("nd random", seed, flush=True)
    rng = np.random.default_rng(9900 + seed)
    cases = []
    for _ in range(int(rng.integers(2, 7))):
        dtype = str(rng.choice(["f32", "f16", "bf16", "i32", "u8", "i64"]))
        nd = int(rng.integers(1, 5))
        shape = tuple(int(rng.choice([1, 2, 3, 5, 8, 17])) for _ in range(nd - 1)) + (int(rng.choice([1, 7, 16, 100, 700, 2500])),)
        kind = str(rng.choice(["same", "bcast", "perm", "strided"]))
        if kind == "bcast":
            kind = "bcast:" + "".join(str(int(rng.integers(0, 2))) for _ in range(nd))
        elif kind == "perm":
            kind = "perm:" + "".join(str(int(i)) for i in rng.permutation(nd))
        pad = tuple(int(rng.choice([0, 0, 1, 3])) for _ in range(nd - 1)) + (int(rng.choice([0, 0, 4, 12])),)
        cases.append((dtype, shape, kind, pad))
    K = int(rng.integers(1, 5))
    _run(oracle_mod, cases, K, float(rng.choice([0.0, 1e-3, 0.1])), float(rng.choice([0.0, 1e-2])), bool(rng.integers(0, 2)), f"nd random {seed}")


def test_nd_plan_refuses_the_read_probe():
    ck = B.Checker(nd=[(0, 0, (2, 3, 8), (96, 32, 4), (0, 0, 4), "f32")], num_candidates=1, atol=0.0, rtol=0.0, equal_nan=False, device=0)
    try:
        x = torch.zeros(64, dtype=torch.float32, device="cuda")
        with pytest.raises(B.GeakError):
            ck.read_probe(x, [x])
    finally:
        ck.close()


def test_row_groups_that_leave_slots_idle(oracle_mod):
    """Rows of whole vectors whose groups do not fill an item's 256 vector slots (12 or 3 vectors per row), and ragged last
    groups: the compare kernel streams them with the idle slots reading as 0; against a reference that is one row for
    all, one element per row, or compact rows of its own pitch."""
    print("nd idle slots", flush=True)
    cases = [
        ("f32", (45, 48), "bcast:10", (0, 4)), ("f32", (45, 48), "bcast:01", (0, 4)), ("f32", (21 * 3 + 5, 48), "same", (0, 4)),
        ("bf16", (100, 24), "bcast:10", (0, 8)), ("bf16", (3, 37, 24), "bcast:010", (0, 0, 8)), ("bf16", (3, 37, 24), "bcast:101", (0, 1, 8)),
        ("u8", (300, 48), "bcast:01", (0, 16)), ("i64", (50, 6), "same", (0, 2)), ("f16", (2, 2, 90, 40), "bcast:1100", (0, 0, 0, 8)),
    ]
    _run(oracle_mod, cases, 3, 1e-2, 1e-2, False, "nd idle slots")
    _run(oracle_mod, cases, 5, 0.0, 0.0, True, "nd idle slots exact")
