"""Pins of the oracle's mismatch report (oracle_report_segment), CPU only.

The report is what the evaluator hands to the Reflector when the functionality test fails (GEAK
sections 4.1 and 4.2); the paper does not say what it holds, so the reading is fixed in
oracle/geak_oracle.c.  The pins: records derived by hand for exactly representable values, and the
structural facts that tie the report to the verdict records (which have pins of their own)."""
import numpy as np
import pytest


def _f32(x):
    return np.array(x, dtype=np.float32)


def test_hand_derived_records_f32(oracle_mod):
    # atol = 0.25, rtol = 0.5, b = [1, 1, 1, -2]: tol = [0.75, 0.75, 0.75, 1.25] (all exact)
    # a = [1.75, 1.75 + 2^-23, 0.25, -3.5]: d = [0.75, 0.75 + 2^-23, 0.75, 1.5] -> elements 1 and 3 fail
    b = _f32([1, 1, 1, -2])
    a = _f32([1.75, 1.75 + 2.0 ** -23, 0.25, -3.5])
    rep = oracle_mod.report_segment(b, a, 4, "f32", 0.25, 0.5, False, 8)
    assert len(rep) == 2
    assert [int(r["index"]) for r in rep] == [1, 3]
    assert float(rep[0]["a"]) == 1.75 + 2.0 ** -23 and float(rep[0]["b"]) == 1.0
    assert float(rep[0]["d"]) == 0.75 + 2.0 ** -23 and float(rep[0]["tol"]) == 0.75
    assert float(rep[1]["a"]) == -3.5 and float(rep[1]["b"]) == -2.0
    assert float(rep[1]["d"]) == 1.5 and float(rep[1]["tol"]) == 1.25
    # only the first M are kept
    rep1 = oracle_mod.report_segment(b, a, 4, "f32", 0.25, 0.5, False, 1)
    assert len(rep1) == 1 and int(rep1[0]["index"]) == 1
    assert len(oracle_mod.report_segment(b, a, 4, "f32", 0.25, 0.5, False, 0)) == 0


def test_hand_derived_records_16bit_and_int(oracle_mod):
    # binary16: b = 1.0 (0x3C00), a = 1 + 2^-9 (0x3C02), atol = rtol = 2^-11 -> tol = 2^-10, d = 2^-9
    b = np.array([0x3C00, 0x3C00], dtype=np.uint16)
    a = np.array([0x3C01, 0x3C02], dtype=np.uint16)
    rep = oracle_mod.report_segment(b, a, 2, "f16", 2.0 ** -11, 2.0 ** -11, False, 4)
    assert len(rep) == 1 and int(rep[0]["index"]) == 1
    assert float(rep[0]["a"]) == 1 + 2.0 ** -9 and float(rep[0]["b"]) == 1.0
    assert float(rep[0]["d"]) == 2.0 ** -9 and float(rep[0]["tol"]) == 2.0 ** -10
    # bfloat16: b = 1.0 (0x3F80), a = 1 + 2^-7 (0x3F81), atol = 0, rtol = 2^-8 -> tol = 2^-8 < d = 2^-7
    rep = oracle_mod.report_segment(np.array([0x3F80], dtype=np.uint16), np.array([0x3F81], dtype=np.uint16),
                                    1, "bf16", 0.0, 2.0 ** -8, False, 4)
    assert len(rep) == 1 and float(rep[0]["d"]) == 2.0 ** -7 and float(rep[0]["tol"]) == 2.0 ** -8
    # int32: exact difference, tolerance 0 whatever atol / rtol say
    b = np.array([5, -(2 ** 31), 7], dtype=np.int32)
    a = np.array([5, 2 ** 31 - 1, 9], dtype=np.int32)
    rep = oracle_mod.report_segment(b, a, 3, "i32", 100.0, 100.0, False, 4)
    assert [int(r["index"]) for r in rep] == [1, 2]
    assert float(rep[0]["d"]) == 2.0 ** 32 - 1 and float(rep[0]["tol"]) == 0.0
    assert float(rep[0]["a"]) == 2.0 ** 31 - 1 and float(rep[0]["b"]) == -(2.0 ** 31)
    assert float(rep[1]["d"]) == 2.0


def test_non_finite_elements(oracle_mod):
    inf, nan = np.inf, np.nan
    b = _f32([nan, nan, inf, inf, 1.0, inf])
    a = _f32([nan, 1.0, inf, -inf, inf, 2.0])
    # equal_nan: (nan, nan) passes; (1, nan) fails with d NaN; (inf, inf) passes; (-inf, inf) fails with d = inf;
    # (inf, 1) fails with d = inf and a finite tolerance; (2, inf) fails although d = inf <= tol = inf
    rep = oracle_mod.report_segment(b, a, 6, "f32", 1e-3, 1e-3, True, 16)
    assert [int(r["index"]) for r in rep] == [1, 3, 4, 5]
    assert np.isnan(rep[0]["d"]) and np.isnan(rep[0]["b"]) and np.isnan(rep[0]["tol"])
    assert rep[1]["d"] == inf and rep[1]["a"] == -inf and rep[1]["tol"] == inf
    assert rep[2]["d"] == inf and np.isfinite(rep[2]["tol"])
    assert rep[3]["d"] == inf and rep[3]["tol"] == inf and rep[3]["a"] == 2.0
    rep = oracle_mod.report_segment(b, a, 6, "f32", 1e-3, 1e-3, False, 16)
    assert [int(r["index"]) for r in rep] == [0, 1, 3, 4, 5]


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16", "i32"])
def test_report_agrees_with_verdict_record(oracle_mod, dtype):
    rng = np.random.default_rng(11)
    n = 5000
    if dtype == "i32":
        b = rng.integers(-50, 50, n, dtype=np.int32)
        a = b.copy()
        a[rng.random(n) < 0.01] += 1
    elif dtype == "f32":
        b = rng.standard_normal(n).astype(np.float32)
        a = (b + (rng.random(n) < 0.01) * 0.5).astype(np.float32)
    else:
        import torch
        td = torch.float16 if dtype == "f16" else torch.bfloat16
        bt = torch.from_numpy(rng.standard_normal(n).astype(np.float32)).to(td)
        at = (bt.float() + torch.from_numpy(((rng.random(n) < 0.01) * 0.5).astype(np.float32))).to(td)
        b, a = bt.view(torch.int16).numpy().view(np.uint16), at.view(torch.int16).numpy().view(np.uint16)
    rec = oracle_mod.check_segment(b, a, n, dtype, 1e-2, 1e-2, False)
    full = oracle_mod.report_segment(b, a, n, dtype, 1e-2, 1e-2, False, n)
    assert len(full) == int(rec["mismatch_count"]) > 10
    assert int(full[0]["index"]) == int(rec["first_mismatch"])
    assert (np.diff(full["index"]) > 0).all()
    assert float(np.nanmax(full["d"])) == float(rec["max_abs_err"])      # here the largest error is a mismatch
    some = oracle_mod.report_segment(b, a, n, dtype, 1e-2, 1e-2, False, 7)
    assert len(some) == 7 and (some == full[:7]).all()
    # every reported element, taken alone, is a mismatch with the same d; every other element is close
    esize = 2 if dtype in ("f16", "bf16") else 4
    reported = set(int(i) for i in full["index"])
    for r in full[:20]:
        i = int(r["index"])
        one = oracle_mod.check_segment(b, a, 1, dtype, 1e-2, 1e-2, False, ref_byte_offset=i * esize)
        assert int(one["mismatch_count"]) == 1 and float(one["max_abs_err"]) == float(r["d"])
    for i in range(0, n, 97):
        if i not in reported:
            one = oracle_mod.check_segment(b, a, 1, dtype, 1e-2, 1e-2, False, ref_byte_offset=i * esize)
            assert int(one["pass"]) == 1
