"""One plan for a batch of unit-test outputs of different kinds (geak_check_plan_table): contiguous and padded
segments, segments whose reference has its own layout, block-scaled segments and an empty one in one table, one
launch; every record and the mismatch report against the oracle's function for that kind of segment."""
import numpy as np
import pytest
import torch

from oracle import mx
from paper_2507_23194_amd import binding as B
from paper_2507_23194_amd import synth
from test_gpu_parity import _special_case, _assert_same
from test_gpu_mapped_reference import _segment
from test_gpu_mx import _tensors

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed", range(4))
def test_mixed_table(oracle_mod, seed):
    print("mixed table", seed, flush=True)
    rng = np.random.default_rng(9600 + seed)
    K = int(rng.integers(2, 7))
    cand_parts = [[] for _ in range(K)]            # candidate buffers and the reference buffer share the offsets of
    ref_parts = []                                 # everything but the mapped references, which lie behind the rest
    table, checks, off = [], [], 0

    def place(ref_bytes, cand_bytes_list):
        nonlocal off
        pad = (-ref_bytes.size) % 16
        ref_parts.append(np.concatenate([ref_bytes, rng.integers(0, 256, pad, dtype=np.uint8)]))
        for k in range(K):
            cand_parts[k].append(np.concatenate([cand_bytes_list[k], rng.integers(0, 256, pad, dtype=np.uint8)]))
        start = off
        off += ref_bytes.size + pad
        return start

    mapped_refs = []
    order = list(rng.permutation(["plain", "pitched", "mapped_row", "mapped_t", "mx8", "mx4", "empty", "plain2"]))
    for kind in order:
        if kind in ("plain", "plain2"):
            dt = str(rng.choice(["f32", "f16", "i32", "u8", "f64"]))
            n = int(rng.integers(1, 20000))
            b, _ = _special_case(rng, dt, n)
            cands = [(_special_case(rng, dt, n)[1] if k != 1 else b.copy()) for k in range(K)]
            w = synth.ELEM_SIZE[dt]
            start = place(b.view(np.uint8), [c.view(np.uint8) for c in cands])
            table.append(("pitched", start, 1, n, n * w, dt))
            checks.append(("plain", dt, n, start))
        elif kind == "pitched":
            dt = str(rng.choice(["bf16", "f32", "i8"]))
            w = synth.ELEM_SIZE[dt]
            rows, cols = int(rng.integers(2, 60)), int(rng.integers(1, 700))
            pitch = (cols * w + 15) // 16 * 16 + 16
            b, _ = _special_case(rng, dt, rows * cols)
            cands = [_special_case(rng, dt, rows * cols)[1] for _ in range(K)]
            store = np.dtype({1: np.uint8, 2: np.uint16, 4: np.uint32}[w])
            def padded(x):
                buf = rng.integers(0, 256, rows * pitch, dtype=np.uint8)
                v = buf.view(store).reshape(rows, pitch // w)
                v[:, :cols] = x.view(store).reshape(rows, cols)
                return buf
            start = place(padded(b), [padded(c) for c in cands])
            table.append(("pitched", start, rows, cols, pitch, dt))
            checks.append(("gathered", dt, rows, cols, start, pitch, start, pitch, 1, "same"))
        elif kind in ("mapped_row", "mapped_t"):
            dt = str(rng.choice(["f32", "bf16", "i32"]))
            rows, cols = int(rng.integers(2, 40)), int(rng.integers(1, 1300))
            rb, cbs, entry = _segment(rng, dt, rows, cols, "row" if kind == "mapped_row" else "transposed", cand_pad=int(rng.integers(0, 5)),
                                      cand_shift=0, ref_pad=0, ref_shift=int(rng.integers(0, 4)), cand_base=0, ref_base=0, K=K)
            start = place(rng.integers(0, 256, cbs[0].size, dtype=np.uint8), cbs)          # the reference buffer holds garbage here
            mapped_refs.append((len(table), rb))
            table.append(["mapped", start + entry[0], rows, cols, entry[3], entry[4], entry[5], entry[6], dt])      # reference offset patched below
            checks.append(("mapped", len(table) - 1))
        elif kind in ("mx8", "mx4"):
            fmt = str(rng.choice(["mxfp8e4m3", "mxfp8e5m2", "mxint8"])) if kind == "mx8" else str(rng.choice(["mxfp4e2m1", "mxfp6e2m3", "mxfp6e3m2"]))
            n = 32 * int(rng.integers(1, 400))
            tensors = _tensors(rng, fmt, n, K)
            blob = lambda t: np.concatenate([t[0], np.full(5, 0xEE, np.uint8), t[1]])
            start = place(blob(tensors[0]), [blob(t) for t in tensors[1:]])
            table.append(("mx", start, n, start + tensors[0][0].size + 5, fmt))
            checks.append(("mx", fmt, n, tensors))
        else:
            table.append(("pitched", off, 0, 5, 20, "f32"))
            checks.append(("empty",))
    # the mapped references behind everything else in the reference buffer
    ref_tail, tail_off = [], off
    for idx, rb in mapped_refs:
        table[idx][5] += tail_off
        table[idx] = tuple(table[idx])
        pad = (-rb.size) % 16
        ref_tail.append(np.concatenate([rb, np.zeros(pad, np.uint8)]))
        tail_off += rb.size + pad
    ref_np = np.concatenate(ref_parts + ref_tail)
    cand_nps = [np.concatenate(p) for p in cand_parts]
    tols = [(float(rng.choice([0.0, 1e-3, 0.25])), float(rng.choice([0.0, 1e-2, 0.125]))) for _ in table]
    equal_nan = bool(rng.integers(0, 2))
    ref = torch.from_numpy(ref_np.copy()).cuda()
    cands = [torch.from_numpy(c.copy()).cuda() for c in cand_nps]
    ck = B.Checker(table=table, num_candidates=K, equal_nan=equal_nan, device=0, tolerances=tols)
    try:
        ck.run(ref, cands)
        gpu = ck.read().copy()
        rep, cnt = ck.report(ref, cands, 4)
        with pytest.raises(B.GeakError):
            ck.ulp_histogram(ref, cands)                    # block-scaled entries: no ladder to count steps on
    finally:
        ck.close()
    cpu = np.zeros_like(gpu)
    for s, chk in enumerate(checks):
        atol, rtol = tols[s]
        for k in range(K):
            if chk[0] == "empty":
                b = a = np.zeros(0, np.float32); n, dt = 0, "f32"
            elif chk[0] == "plain":
                _, dt, n, start = chk
                w = synth.ELEM_SIZE[dt]
                b, a = ref_np[start:start + n * w], cand_nps[k][start:start + n * w]
            elif chk[0] == "gathered":
                _, dt, rows, cols, coff, cpitch, roff, rpitch, stride, _ = chk
                n = rows * cols
                b = oracle_mod.gather_rows(ref_np, rows, cols, dt, roff, rpitch, stride)
                a = oracle_mod.gather_rows(cand_nps[k], rows, cols, dt, coff, cpitch, 1)
            elif chk[0] == "mapped":
                _, coff, rows, cols, cpitch, roff, rpitch, stride, dt = table[chk[1]]
                n = rows * cols
                b = oracle_mod.gather_rows(ref_np, rows, cols, dt, roff, rpitch, stride)
                a = oracle_mod.gather_rows(cand_nps[k], rows, cols, dt, coff, cpitch, 1)
            else:
                _, fmt, n, tensors = chk
                b = mx.dequantize(tensors[0][0], tensors[0][1], n, fmt)
                a = mx.dequantize(tensors[k + 1][0], tensors[k + 1][1], n, fmt)
                dt = "f32"
            r = oracle_mod.check_segment(b, a, n, dt, atol, rtol, equal_nan)
            for f in cpu.dtype.names:
                cpu[s, k][f] = r[f]
            want = oracle_mod.report_segment(b, a, n, dt, atol, rtol, equal_nan, 4)
            assert int(cnt[s, k]) == len(want), (seed, s, k, chk[0])
            got = rep[s, k][:len(want)]
            assert (got["index"] == want["index"]).all(), (seed, s, k, chk[0])
            assert all(np.array_equal(got[f], want[f], equal_nan=True) for f in ("a", "b", "d", "tol")), (seed, s, k, chk[0])
    _assert_same(gpu, cpu, f"mixed table {seed}: {[c[0] for c in checks]}")
