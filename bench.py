#!/usr/bin/env python3
"""Benchmark of the output-equivalence check on one MI355X.

A step is one geak_check_run over one batch of synthetic tensors that are already resident in HBM:
every kernel the call enqueues, i.e. the whole hot path.  With no --config the five seeded workloads
run one after the other in this process; the headline fields (value, ms_per_step, roofline,
cpu_baseline) are those of the largest one (fp32, 2^30 elements, 32 candidates: 132 GiB resident) and
"per_config" carries the same figures for each workload.  --config N runs and reports that one alone.

Prints ONE JSON line: throughput in verified GB/s (algorithmic bytes = (K + 1) tensors read once,
divided by the wall time of a step), the roofline entry of the compare kernel (its duration is taken
from HIP events recorded around it on the run's stream during the timed steps) and the CPU oracle
timed on a bounded sample of the same bytes.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth

# HBM bytes per compare-kernel launch from rocprofv3 counters (FETCH_SIZE + WRITE_SIZE, each scaled by
# what the same counter reads for a plain copy of known size; the summaries are under profiles/).
# They were taken in profiling runs of their own, not in the run that prints them, and describe the
# library whose build id is recorded with them: for any other build roofline.traffic is null.
MEASURED_TRAFFIC = {
    "build_id": "51dda1bf0b5a52f2",
    "bytes": {2: 8.7964e9, 3: 9.1980e9, 4: 1.2294e9, 5: 141.8672e9},
    "source": "profiles/compare_kernel_config*.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs, not this run)",
}

WORKLOADS = {
    1: "config1: fp32 1024x1024, K=8",
    2: "config2: fp16 8192x8192 Student-t(3)*0.5 with NaN/Inf, K=64, atol=rtol=1e-3, equal_nan",
    3: "config3: bf16 [16,32,4096,128], K=16, atol=1e-2, rtol=1.6e-2",
    4: "config4: ragged 1024 segments, log-uniform sizes to 2^20, mixed f32/f16/bf16/i32, K=4",
    5: "config5: fp32 2^30 elements, K=32, atol=1e-6, rtol=1e-5",
}
# bounded sample of each workload for the CPU baseline: (candidates, elements; 0 = all segments)
CPU_SAMPLE = {1: (8, 1 << 20), 2: (16, 1 << 26), 3: (8, 1 << 27), 4: (4, 0), 5: (8, 1 << 29)}


def measured_traffic(config: int, build_id: str):
    if build_id != MEASURED_TRAFFIC["build_id"]:
        return None
    return MEASURED_TRAFFIC["bytes"].get(config)


def cpu_baseline(w, max_candidates: int, max_elems: int):
    """The oracle as it stands, on the host cores, over a bounded sample of the workload."""
    import oracle
    from paper_2507_23194_amd import synth

    visible = oracle.host_cores()
    threads = max(1, min(16, visible))          # a one-GPU machine's share of its host is 16 cores
    ks = list(range(min(max_candidates, len(w.cands))))
    if w.segments is None:
        n = min(w.ref.numel(), max_elems)
        ref = synth.to_numpy_raw(w.ref[:n])
        cands = [synth.to_numpy_raw(w.cands[k][:n]) for k in ks]
        esize = synth.ELEM_SIZE[w.dtype]
        t0 = time.perf_counter()
        oracle.check_dense_chunked(ref, cands, w.dtype, w.atol, w.rtol, w.equal_nan, threads=threads)
        dt = time.perf_counter() - t0
        nbytes = (len(ks) + 1) * n * esize
        sample = f"first {n} elements of the reference and of candidates 0..{len(ks) - 1}"
    else:
        ref = synth.to_numpy_raw(w.ref)
        cands = [synth.to_numpy_raw(w.cands[k]) for k in ks]
        t0 = time.perf_counter()
        oracle.check_ragged(ref, cands, w.segments, w.atol, w.rtol, w.equal_nan, threads=threads)
        dt = time.perf_counter() - t0
        nbytes = (len(ks) + 1) * sum(n * synth.ELEM_SIZE[d] for (_, n, d) in w.segments)
        sample = f"all segments, candidates 0..{len(ks) - 1}"
    return {"value": nbytes / dt / 1e9, "unit": "GB/s", "cores": threads, "host_cores_visible": visible,
            "kind": "oracle", "sample": sample, "seconds": dt, "candidates_per_s": len(ks) / dt}


def run_config(cid: int, args, build_id: str):
    """Generate workload `cid`, time args.steps runs of the check on it, and return its figures."""
    import numpy as np
    import torch
    from paper_2507_23194_amd import binding as B
    from paper_2507_23194_amd import synth

    if cid == 0:                        # --dense: a profiling aid for other dtypes, never part of the default line
        dt, lg, kk = args.dense.split(":")
        w = synth.dense_noise(dt, int(lg), int(kk), device="cuda:0")
        WORKLOADS[0] = f"dense {dt} 2^{lg} elements, K={kk}, normal data with 2 % relative noise, atol=1e-2, rtol=0.1"
    else:
        w = synth.CONFIGS[cid](device="cuda:0")
    torch.cuda.synchronize()

    t_plan = time.perf_counter()
    if w.segments is None:
        ck = B.Checker(dense=(w.dtype, (w.ref.numel(),)), num_candidates=len(w.cands), atol=w.atol, rtol=w.rtol,
                       equal_nan=w.equal_nan, device=0)
    else:
        ck = B.Checker(w.segments, num_candidates=len(w.cands), atol=w.atol, rtol=w.rtol, equal_nan=w.equal_nan,
                       device=0)
    torch.cuda.synchronize()
    plan_ms = (time.perf_counter() - t_plan) * 1e3          # host planning, upload of the work table, workspace allocation: once per shape, untimed
    info = ck.info()
    alg_bytes = int(info.algorithmic_bytes)
    assert alg_bytes == w.algorithmic_bytes()

    for _ in range(args.warmup):
        ck.run(w.ref, w.cands)
    torch.cuda.synchronize()

    st = B.geak_check_profile_enable(ck.plan, args.steps)
    assert st == B.GEAK_OK
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        ck.run(w.ref, w.cands)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    kernel_ms = B.geak_check_profile_read(ck.plan, args.steps)
    B.geak_check_profile_enable(ck.plan, 0)

    # what a kernel that only reads the same bytes reaches on this machine (not part of the step)
    probe_gbps = None
    if len(w.cands) < 256:
        for _ in range(3):
            ck.read_probe(w.ref, w.cands)
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(10)]
        for a, b in ev:
            a.record()
            ck.read_probe(w.ref, w.cands)
            b.record()
        torch.cuda.synchronize()
        probe_ms = float(np.median([a.elapsed_time(b) for a, b in ev]))
        probe_gbps = alg_bytes / (probe_ms * 1e-3) / 1e9
        ck.run(w.ref, w.cands)                       # the probe used the workspace: produce the records again

    extras = {}
    if args.report > 0:
        ck.report(w.ref, w.cands, args.report)                      # warm-up (allocates its buffers)
        t0 = time.perf_counter()
        reps = 5
        for _ in range(reps):
            rrec, rcnt = ck.report(w.ref, w.cands, args.report)     # synchronises
        extras["report"] = {"max_records": args.report, "ms_per_call_incl_copy_back": (time.perf_counter() - t0) / reps * 1e3,
                            "pairs": int(rcnt.size), "records": int(rcnt.sum())}

    if args.graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            ck.run(w.ref, w.cands)                                   # warm-up on the capture stream
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            ck.run(w.ref, w.cands)
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        g_el = (time.perf_counter() - t0) / args.steps
        extras["graph_replay"] = {"ms_per_step": g_el * 1e3, "GBps": alg_bytes / g_el / 1e9}

    if args.ulp_histogram:
        for _ in range(3):
            ck.ulp_histogram_enqueue(w.ref, w.cands)                # warm-up (allocates its buffers on the first call)
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(10)]
        for a, b in ev:
            a.record()
            ck.ulp_histogram_enqueue(w.ref, w.cands)
            b.record()
        torch.cuda.synchronize()
        ulp_ms = float(np.median([a.elapsed_time(b) for a, b in ev]))
        hist = ck.ulp_histogram(w.ref, w.cands)
        numels = np.array([w.ref.numel()] if w.segments is None else [n for _, n, _ in w.segments], dtype=np.uint64)
        assert (hist.sum(axis=2) == numels[:, None]).all()           # every element counted once per pair
        extras["ulp_histogram"] = {"ms_per_call": ulp_ms, "GBps": alg_bytes / (ulp_ms * 1e-3) / 1e9,
                                   "frac_of_hbm_peak": alg_bytes / (ulp_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                                   "elements_within_1_ulp": float(hist[:, :, :2].sum() / max(1, hist.sum()))}

    rec = ck.read()
    n_fail = int((rec["pass"] == 0).sum())
    # the records must agree with what the generator planted (cheap sanity check, outside the timed region)
    for (s, k), e in w.expect.items():
        assert int(rec[s, k]["mismatch_count"]) == e["count"] and int(rec[s, k]["first_mismatch"]) == e["first"], (s, k)

    step_s = elapsed / args.steps
    gbps = alg_bytes / step_s / 1e9
    k_ms = float(np.mean(kernel_ms)) if len(kernel_ms) else float("nan")
    achieved = alg_bytes / (k_ms * 1e-3) / 1e9
    traffic = args.traffic_bytes if args.traffic_bytes is not None else measured_traffic(cid, build_id)
    storage = w.dtype if w.segments is None else "mixed(" + ",".join(sorted({d for _, _, d in w.segments})) + ")"
    out = {
        "config": cid,
        "workload": WORKLOADS[cid],
        "value": gbps,
        "unit": "GB/s",
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": step_s * 1e3,
        "pct_of_hbm_peak": 100.0 * gbps / HBM_PEAK_GBPS,
        "cache_resident": alg_bytes <= (256 << 20),          # fits the 256 MB last-level cache: not an HBM figure
        # the rule runs in binary32 for every floating dtype here (exact integer compare for i32); storage_dtype is what is read
        "dtype": "i32" if storage == "i32" else ("f32+i32" if w.segments is not None else "f32"),
        "storage_dtype": storage,
        "num_candidates": len(w.cands),
        "algorithmic_bytes": alg_bytes,
        "segments": 1 if w.segments is None else len(w.segments),
        "grid_blocks": int(info.grid_blocks),
        "work_items": int(info.num_items),
        "plan_ms": plan_ms,
        "candidates_per_sec": len(w.cands) / step_s,
        "verdicts_per_sec": rec.size / step_s,
        "failing_candidates": n_fail,
        "roofline": {"kernel": "compare_kernel", "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": traffic,
                     "traffic_source": (MEASURED_TRAFFIC["source"] if traffic is not None and args.traffic_bytes is None else None),
                     "kernel_ms_avg": k_ms, "kernel_ms_min": float(np.min(kernel_ms)) if len(kernel_ms) else None,
                     "read_only_kernel_GBps": probe_gbps,
                     "frac_of_read_only_kernel": (achieved / probe_gbps) if probe_gbps else None},
    }
    out.update(extras)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, *CPU_SAMPLE[cid])
    ck.close()
    del ck, w, rec
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=None, choices=sorted(WORKLOADS),
                    help="run this workload alone (default: all five, headline on config 5)")
    ap.add_argument("--dense", default=None, metavar="DTYPE:LOG2N:K",
                    help="instead of a configuration: one dense tensor of a floating dtype (f8e4m3:26:16, say) with "
                         "normal data, for profiles of dtypes the five configurations do not use; implies --no-cpu-baseline")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--traffic-bytes", type=float, default=None,
                    help="HBM bytes per compare launch from rocprofv3 counters, overriding the recorded figure "
                         "(reported as roofline.traffic; with --config only)")
    ap.add_argument("--report", type=int, default=0, metavar="M",
                    help="also time the mismatch report (first M mismatches per pair) that follows a failed check; "
                         "reported under \"report\", not part of the step")
    ap.add_argument("--graph", action="store_true",
                    help="also time the step replayed from a HIP graph (the launches of geak_check_run captured "
                         "once); reported under \"graph_replay\", the headline value stays the eager one")
    ap.add_argument("--ulp-histogram", action="store_true",
                    help="also time the ulp-distance histogram pass (a second read of all tensors, part of the error "
                         "trace of a failed check); reported under \"ulp_histogram\", not part of the step")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain element-wise copy of a known size (2 GiB read, 2 GiB written per launch), "
                         "for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: the check runs on one GPU only (no collectives, no sharding); use --gpus 1")

    import torch

    if args.calibrate_copy:
        torch.cuda.set_device(0)
        src = torch.ones(1 << 29, dtype=torch.float32, device="cuda:0")       # 2 GiB
        dst = torch.empty_like(src)
        for _ in range(5):
            torch.mul(src, 1.0, out=dst)                                       # one element-wise kernel: reads src, writes dst
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "torch.mul(src, 1.0, out=dst)", "bytes_read": src.numel() * 4,
                          "bytes_written": dst.numel() * 4, "launches": 5}))
        return
    from paper_2507_23194_amd import binding as B

    B.ensure_library()                  # loads what is built (compiles only when nothing is); raises if it was built from other sources
    build_id = B.geak_check_build_id()
    torch.cuda.set_device(0)
    if args.config is None and args.traffic_bytes is not None:
        sys.exit("bench.py: --traffic-bytes describes one workload; give --config with it")

    configs = [args.config] if args.config is not None else [1, 2, 3, 4, 5]
    if args.dense is not None:
        configs, args.no_cpu_baseline, args.config = [0], True, 0
    per_config = []
    for cid in configs:
        t0 = time.perf_counter()
        entry = run_config(cid, args, build_id)
        entry["wall_s_incl_generation_and_baseline"] = time.perf_counter() - t0
        per_config.append(entry)
        print(f"bench: {entry['workload'][:7]} {entry['value']:.0f} GB/s, step {entry['ms_per_step']:.3f} ms, "
              f"compare kernel {entry['roofline']['kernel_ms_avg']:.3f} ms", file=sys.stderr, flush=True)

    head = per_config[-1]               # the one asked for, or config 5: the largest single-GPU workload
    out = {
        "metric": "verified_bytes_per_sec",
        "value": head["value"],
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": head["dtype"],
        "data": "synthetic",
        "config": {"workload": head["workload"], "storage_dtype": head["storage_dtype"], "num_candidates": head["num_candidates"],
                   "algorithmic_bytes": head["algorithmic_bytes"], "segments": head["segments"],
                   "grid_blocks": head["grid_blocks"], "work_items": head["work_items"], "plan_ms": head["plan_ms"]},
        "pct_of_hbm_peak": head["pct_of_hbm_peak"],
        "candidates_per_sec": head["candidates_per_sec"],
        "verdicts_per_sec": head["verdicts_per_sec"],
        "failing_candidates": head["failing_candidates"],
        "build_id": build_id,
        "roofline": head["roofline"],
    }
    for extra in ("report", "graph_replay", "ulp_histogram", "cpu_baseline"):
        if extra in head:
            out[extra] = head[extra]
    if args.config is None:
        out["per_config"] = per_config
    print(json.dumps(out))


if __name__ == "__main__":
    main()
