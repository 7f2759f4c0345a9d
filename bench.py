#!/usr/bin/env python3
"""Benchmark of the hot path: one step = one whole reduction (redux_sum / redux_sum_segmented)
over a seeded synthetic array already resident in HBM.

Default workload: C3, the n = 2^30 + 12345 binary16 sum the headline metric is quoted on.
Prints ONE JSON line (see the keys below).  Usage:

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--settle SECONDS] [--workload C1..C5]
                    [--variant auto|mfma|classic|multipass] [--seglen L] [--set NAME=VALUE] [--no-cpu-baseline]
                    [--no-by-variant] [--ab-rounds R] [--lean]

Order of events
    settle   `--settle` seconds (default 0.25) of untimed calls: after an idle period -- and generating the input on the
             host is one -- the device needs some tens of calls until its clocks and power state have settled (measured:
             the classic family runs 4 % slower for calls 6-40 after two idle seconds).  Reported in config.settle_s.
    warmup   W untimed calls.
    timed    EXACTLY K calls, bracketed by device synchronisation (wall clock -> `value`, `ms_per_step`) and by two HIP
             events on the stream the kernels are launched on (-> `roofline`).
    per call K more calls with one HIP event between every two (-> `config.median_us`, `config.min_us`; an event record
             costs about 1 us per call, which is why this is a pass of its own).
    families both kernel families in turn, two rounds of K calls each (-> `config.by_variant`).

`value`            whole-job throughput in GB/s: algorithmic bytes (2 B per binary16 element, 1 B per
                   int8 element) x K / wall time of the K timed calls.
`roofline`         the reduction kernel against the 8 TB/s HBM3E peak: `achieved` is the same algorithmic bytes over
                   the average duration of a call in the timed region, by HIP events.  For every workload a call is
                   one kernel launch (the block that finishes last adds up the block partials), so this is that
                   kernel's average launch duration plus the gap to the next launch.
`cpu_baseline`     the CPU oracle (untuned) timed on the same array on this host: all host cores (`value`, `cores`) and
                   one thread (`single_thread`).
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0

# Per launch of the dominant kernel, from the rocprofv3 summaries under profiles/ (kernel trace for the duration;
# FETCH_SIZE + WRITE_SIZE, scaled by what the same counters read for a plain copy of known size, for the HBM bytes).
# (workload, family actually run): (HBM bytes per launch, kernel, average kernel duration in us, summary).  Absent = not profiled.
PROFILED = {
    ('C1', 'classic'): (2246885, 'sum_flat_kernel<FloatClassic<0>, 8, true>', 4.74, 'profiles/redux_sum_f16_C1_C2.md'),
    ('C1', 'mfma'): (2252389, 'sum_flat_kernel<FloatMfmaT<0, 4>, 8, true>', 4.59, 'profiles/redux_sum_f16_C1_C2.md'),
    ('C2', 'classic'): (134380556, 'sum_flat_kernel<FloatClassic<0>, 8, true>', 22.28, 'profiles/redux_sum_f16_C1_C2.md'),
    ('C2', 'mfma'): (134386050, 'sum_flat_kernel<FloatMfmaT<0, 4>, 8, true>', 21.44, 'profiles/redux_sum_f16_C1_C2.md'),
    ('C3', 'classic'): (2147627295, 'sum_flat_kernel<FloatClassic<0>, 8, true>', 289.42, 'profiles/redux_sum_f16_C3.md'),
    ('C3', 'mfma'): (2147632757, 'sum_flat_kernel<FloatMfmaT<0, 4>, 8, true>', 288.99, 'profiles/redux_sum_f16_C3.md'),
    ('C4', 'classic'): (1073852100, 'sum_flat_kernel<I8Classic, 8, true>', 145.72, 'profiles/redux_sum_i8_C4.md'),
    ('C4', 'mfma'): (1073872601, 'sum_flat_kernel<I8MfmaT<4>, 8, true>', 144.00, 'profiles/redux_sum_i8_C4.md'),
    ('C5', 'classic'): (537420392, 'sum_segments_tiles_kernel<FloatClassic<0>, 8, true, 0>', 74.63, 'profiles/redux_sum_segmented_f16_C5.md'),
    ('C5', 'mfma'): (537417381, 'sum_segments_tiles_kernel<FloatMfmaT<0, 1>, 8, true, 1>', 74.48, 'profiles/redux_sum_segmented_f16_C5.md'),
}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--settle", type=float, default=0.25, metavar="SECONDS",
                    help="untimed calls for this long before the warm-up, so that clocks and power state have settled")
    ap.add_argument("--workload", default="C3", choices=["C1", "C2", "C3", "C4", "C5"])
    ap.add_argument("--variant", default="auto", choices=["auto", "mfma", "classic", "multipass"],
                    help="kernel family of redux_sum; 'multipass' times redux_sum_multipass (the level-by-level form) instead")
    ap.add_argument("--seglen", type=int, default=0, metavar="L",
                    help="with --workload C5: cut the same array into segments of L elements instead of 4096 "
                         "(to time and profile the short- and ragged-segment kernels)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-by-variant", action="store_true", help="skip the pass that times both kernel families")
    ap.add_argument("--ab-rounds", type=int, default=2, metavar="R",
                    help="rounds of the pass that times both kernel families, alternating, K calls per family and round "
                         "(mean and standard deviation over the rounds are reported)")
    ap.add_argument("--lean", action="store_true",
                    help="for runs under a profiler: warm-up and the K timed calls only (no settle phase, no per-call pass, "
                         "no families pass, no CPU baseline)")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MIB",
                    help="instead of the reduction, run --steps plain copies of MIB MiB (known traffic) "
                         "so that hardware byte counters can be calibrated under rocprofv3 --pmc")
    ap.add_argument("--set", action="append", default=[], metavar="NAME=VALUE",
                    help="library launch parameter (see redux_set_param), may be repeated")
    args = ap.parse_args()

    if args.lean:
        args.settle, args.no_by_variant, args.no_cpu_baseline = 0.0, True, True
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU by design (one reduction = one device's share); "
              "run it with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_1903_03640_amd import redux, workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU path to benchmark", file=sys.stderr)
        return 3
    redux.load()
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")

    if args.calibrate_copy:
        nbytes = args.calibrate_copy << 20
        src = torch.zeros(nbytes, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(args.steps):
            rc = redux.calibration_copy_raw(dst.data_ptr(), src.data_ptr(), nbytes, torch.cuda.current_stream().cuda_stream)
            assert rc == 0, rc
        torch.cuda.synchronize()
        print(json.dumps({"calibration_copy_bytes": nbytes, "launches": args.steps}))
        return 0

    cfg = workloads.CONFIGS[args.workload]
    if args.seglen:
        if not cfg.segmented or args.seglen < 1 or args.seglen > cfg.n:
            print("bench.py: --seglen needs --workload C5 and 1 <= L <= %d" % cfg.n, file=sys.stderr)
            return 2
        import dataclasses
        nseg = cfg.n // args.seglen
        cfg = dataclasses.replace(cfg, n=nseg * args.seglen, nseg=nseg, seglen=args.seglen)
    t0 = time.perf_counter()
    host = workloads.make(cfg)
    gen_s = time.perf_counter() - t0
    input_checksum = workloads.checksum(host)
    x = torch.from_numpy(host).to(dev)
    torch.cuda.synchronize()

    multipass = args.variant == "multipass"
    redux.set_variant("auto" if multipass else args.variant)
    for kv in args.set:
        name, val = kv.split("=")
        redux.set_param(name, int(val))

    # raw C-ABI calls: pointers and sizes, the current stream's handle
    stream = torch.cuda.current_stream()
    sh = stream.cuda_stream
    dt = redux._dtype_of(x)
    if cfg.segmented:
        out = torch.empty(cfg.nseg, dtype=torch.float32, device=dev)
        xp, op, nseg, seglen = x.data_ptr(), out.data_ptr(), cfg.nseg, cfg.seglen
        step = lambda: redux.sum_segmented_raw(xp, nseg, seglen, dt, op, sh)
    else:
        out = torch.empty(1, dtype=torch.float32 if cfg.dtype == "f16" else torch.int64, device=dev)
        xp, op, n = x.data_ptr(), out.data_ptr(), x.numel()
        if multipass:
            step = lambda: redux.sum_multipass_raw(xp, n, dt, op, sh)[0]
        else:
            step = lambda: redux.sum_raw(xp, n, dt, op, sh)

    def timed(k):
        """k calls between two events on the stream and two synchronisations: (wall seconds, device milliseconds)"""
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t = time.perf_counter()
        ev0.record(stream)
        for _ in range(k):
            rc = step()
        ev1.record(stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t
        assert rc == 0, rc
        return wall, ev0.elapsed_time(ev1)

    # ---- settle, warm-up -------------------------------------------------------------------------------------
    settle_calls = 0
    t_end = time.perf_counter() + max(0.0, args.settle)
    while time.perf_counter() < t_end:
        for _ in range(16):
            step()
        settle_calls += 16
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # ---- the timed region: exactly K calls ----------------------------------------------------------------------
    wall_s, dev_ms = timed(args.steps)
    result = out.cpu().numpy().copy()
    nbytes = cfg.nbytes
    ms_per_step = wall_s * 1e3 / args.steps
    value = nbytes * args.steps / wall_s / 1e9
    call_us = dev_ms * 1e3 / args.steps
    achieved = nbytes / (call_us * 1e-6) / 1e9

    # ---- per-call durations: one event between every two calls ------------------------------------------------
    per_call = None
    if not args.lean:
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
        torch.cuda.synchronize()
        evs[0].record(stream)
        for i in range(args.steps):
            step()
            evs[i + 1].record(stream)
        torch.cuda.synchronize()
        per_call = [evs[i].elapsed_time(evs[i + 1]) * 1e3 for i in range(args.steps)]

    variant_run = "multipass" if multipass else redux.resolved_variant(dt, cfg.segmented)
    prof = None if args.seglen or args.set else PROFILED.get((args.workload, variant_run))
    plan = (redux.plan_sum_segmented(cfg.nseg, cfg.seglen, dt, x.data_ptr(), torch.cuda.get_device_properties(0).multi_processor_count)
            if cfg.segmented else redux.plan_sum(x.numel(), dt, x.data_ptr(), torch.cuda.get_device_properties(0).multi_processor_count))

    # ---- both kernel families, same process, alternating ------------------------------------------------------
    by_variant = None
    if not multipass and not args.no_by_variant:
        samples = {"mfma": [], "classic": []}
        for rnd in range(max(1, args.ab_rounds)):
            for v in (("mfma", "classic") if rnd % 2 == 0 else ("classic", "mfma")):
                redux.set_variant(v)
                for _ in range(max(5, args.warmup)):
                    step()
                samples[v].append(timed(args.steps)[1] * 1e3 / args.steps)
        redux.set_variant(args.variant)
        by_variant = {v: {"us_per_call": round(statistics.mean(s), 3), "gbps": round(nbytes / (statistics.mean(s) * 1e-6) / 1e9, 1),
                          "pct_of_hbm_peak": round(100.0 * nbytes / (statistics.mean(s) * 1e-6) / 1e9 / HBM_PEAK_GBPS, 2),
                          "sd_us": round(statistics.stdev(s), 3) if len(s) > 1 else None,
                          "rounds_us": [round(q, 3) for q in s]} for v, s in samples.items()}

    line = {
        "metric": "achieved HBM GB/s for the fp16 sum (algorithmic bytes / time), 1x MI355X"
                  if args.workload == "C3" else "achieved HBM GB/s (algorithmic bytes / time), 1x MI355X",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 6),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if cfg.dtype == "f16" else "int32",
        "data": "synthetic",
        "config": {
            "workload": "%s: n=%d %s %s seed %d%s" % (
                cfg.name, cfg.n, cfg.dtype, cfg.dist, cfg.seed,
                " segmented %dx%d" % (cfg.nseg, cfg.seglen) if cfg.segmented else ""),
            "variant": variant_run,
            "input_bytes": nbytes,
            "input_checksum": "%016x" % input_checksum,
            "gelem_per_s": round(cfg.n / wall_s * args.steps / 1e9, 2),
            "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
            "settle_s": args.settle,
            "settle_calls": settle_calls,
            "median_us": round(statistics.median(per_call), 3) if per_call else None,
            "min_us": round(min(per_call), 3) if per_call else None,
            "launches_per_call": 1 + (1 if plan.finish == 2 else 0) if not multipass else None,
            "by_variant": by_variant,
        },
        "roofline": {
            "bound": "hbm",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBPS, 4),
            "traffic": prof[0] if prof else None,
            "call_avg_us": round(call_us, 3),
            "kernel": prof[1] if prof else None,
            "kernel_avg_us_profiled": prof[2] if prof else None,
            "profile": prof[3] if prof else None,
        },
    }

    # ---- check the timed result and time the oracle beside it (host cores, not the target) ----------
    if not args.no_cpu_baseline:
        import oracle

        def one_thread():
            if cfg.segmented:
                return oracle.sum_segmented_f16(host, cfg.nseg, cfg.seglen)
            return oracle.sum_f16(host) if cfg.dtype == "f16" else oracle.sum_i8(host)

        def all_cores():
            if cfg.segmented:
                return oracle.sum_segmented_f16_chunks(host, cfg.nseg, cfg.seglen)
            return oracle.sum_f16_chunks(host) if cfg.dtype == "f16" else oracle.sum_i8_chunks(host)

        def run_for(fn, budget_s, max_reps):
            reps, spent, res = 0, 0.0, None
            while spent < budget_s and reps < max_reps:
                t = time.perf_counter()
                res = fn()
                spent += time.perf_counter() - t
                reps += 1
            return res, reps, spent

        want, reps1, cpu1_s = run_for(one_thread, 6.0, 40)
        want_mc, repsn, cpun_s = run_for(all_cores, 6.0, 200)
        cores = oracle.max_threads()
        if cfg.dtype == "i8":
            ok = int(result[0]) == want[0] == want_mc[0]
        else:
            tol = 1e-4 * np.asarray(want[1])
            ok = bool(np.all(np.abs(result.astype(np.float64) - np.asarray(want[0])) <= tol) and
                      np.all(np.abs(np.asarray(want_mc[0]) - np.asarray(want[0])) <= 1e-12 * np.asarray(want[1])))
        line["cpu_baseline"] = {
            "value": round(nbytes * repsn / cpun_s / 1e9, 3),
            "unit": "GB/s",
            "cores": cores,
            "kind": "oracle",
            "sample": "the whole %s array: %d passes of the chunked oracle on %d threads (%.1f s) and %d passes of the "
                      "single-threaded binary64 pairwise (int64 for int8) oracle (%.1f s)" % (
                          cfg.name, repsn, cores, cpun_s, reps1, cpu1_s),
            "single_thread": {"value": round(nbytes * reps1 / cpu1_s / 1e9, 3), "unit": "GB/s", "cores": 1},
        }
        line["config"]["matches_oracle"] = ok
        if not ok:
            print(json.dumps(line))
            print("bench.py: GPU result does not match the oracle", file=sys.stderr)
            return 1
    line["config"]["host_generate_s"] = round(gen_s, 2)
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
