#!/usr/bin/env python3
"""Benchmark of the hot path: one step = one whole reduction (redux_sum / redux_sum_segmented)
over a seeded synthetic array already resident in HBM.

Default workload: C3, the n = 2^30 + 12345 binary16 sum the headline metric is quoted on.
Prints ONE JSON line (see the keys below).  Usage:

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C1..C5] [--variant auto|mfma|classic|multipass]
                    [--seglen L] [--set NAME=VALUE] [--no-cpu-baseline]

`value`            whole-job throughput in GB/s: algorithmic bytes (2 B per binary16 element, 1 B per
                   int8 element) x K / wall time of K back-to-back calls, bracketed by device
                   synchronisation.
`roofline`         the reduction kernel against the 8 TB/s HBM3E peak: `achieved` uses the same
                   algorithmic bytes over the average launch duration measured with HIP events
                   recorded on the stream the kernels are launched on.
`cpu_baseline`     the CPU oracle (single thread, untuned) timed on the same array on this host.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0

# HBM traffic per launch measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE, scaled by the
# factor a plain copy kernel of known size reads on the same counters); see profiles/.
# Keyed by (workload, variant actually run).  None = not measured.
MEASURED_TRAFFIC_BYTES = {
    ("C3", "mfma"): 2147593438, ("C3", "classic"): 2147600392,     # profiles/redux_sum_f16_C3.md
    ("C4", "mfma"): 1073853054, ("C4", "classic"): 1073842846,     # profiles/redux_sum_i8_C4.md
    ("C5", "mfma"): 537411811, ("C5", "classic"): 537421025,       # profiles/redux_sum_segmented_f16_C5.md
}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="C3", choices=["C1", "C2", "C3", "C4", "C5"])
    ap.add_argument("--variant", default="auto", choices=["auto", "mfma", "classic", "multipass"],
                    help="kernel family of redux_sum; 'multipass' times redux_sum_multipass (the level-by-level form) instead")
    ap.add_argument("--seglen", type=int, default=0, metavar="L",
                    help="with --workload C5: cut the same array into segments of L elements instead of 4096 "
                         "(to time and profile the short- and ragged-segment kernels)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MIB",
                    help="instead of the reduction, run --steps plain copies of MIB MiB (known traffic) "
                         "so that hardware byte counters can be calibrated under rocprofv3 --pmc")
    ap.add_argument("--set", action="append", default=[], metavar="NAME=VALUE",
                    help="library launch parameter (see redux_set_param), may be repeated")
    args = ap.parse_args()

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
    x = torch.from_numpy(host).to(dev)
    torch.cuda.synchronize()

    multipass = args.variant == "multipass"
    redux.set_variant("auto" if multipass else args.variant)
    for kv in args.set:
        name, val = kv.split("=")
        redux.set_param(name, int(val))

    if cfg.segmented:
        out = torch.empty(cfg.nseg, dtype=torch.float32, device=dev)
        step = lambda: redux.sum_segmented(x, cfg.nseg, cfg.seglen, out=out)
    else:
        out = torch.empty(1, dtype=torch.float32 if cfg.dtype == "f16" else torch.int64, device=dev)
        step = (lambda: redux.sum_multipass(x, out=out)) if multipass else (lambda: redux.sum(x, out=out))

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    stream = torch.cuda.current_stream()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record(stream)
    for _ in range(args.steps):
        step()
    ev1.record(stream)
    torch.cuda.synchronize()
    wall_s = time.perf_counter() - t0
    dev_ms = ev0.elapsed_time(ev1)

    result = out.cpu().numpy().copy()
    nbytes = cfg.nbytes
    ms_per_step = wall_s * 1e3 / args.steps
    value = nbytes * args.steps / wall_s / 1e9
    launch_us = dev_ms * 1e3 / args.steps
    achieved = nbytes / (launch_us * 1e-6) / 1e9

    variant_run = "multipass" if multipass else redux.resolved_variant(redux._dtype_of(x), cfg.segmented)
    traffic = None if args.seglen else MEASURED_TRAFFIC_BYTES.get((args.workload, variant_run))

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
            "gelem_per_s": round(cfg.n / wall_s * args.steps / 1e9, 2),
            "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
        },
        "roofline": {
            "bound": "hbm",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBPS, 4),
            "traffic": traffic,
            "kernel_avg_us": round(launch_us, 3),
        },
    }

    # ---- check the timed result and time the oracle beside it (host cores, not the target) ----------
    if not args.no_cpu_baseline:
        import oracle
        reps, cpu_s = 0, 0.0
        while cpu_s < 8.0 and reps < 40:
            t0 = time.perf_counter()
            if cfg.segmented:
                want = oracle.sum_segmented_f16(host, cfg.nseg, cfg.seglen)
            elif cfg.dtype == "f16":
                want = oracle.sum_f16(host)
            else:
                want = oracle.sum_i8(host)
            cpu_s += time.perf_counter() - t0
            reps += 1
        if cfg.dtype == "i8":
            ok = int(result[0]) == want[0]
        else:
            ok = bool(np.all(np.abs(result.astype(np.float64) - np.asarray(want[0])) <= 1e-4 * np.asarray(want[1])))
        line["cpu_baseline"] = {
            "value": round(nbytes * reps / cpu_s / 1e9, 3),
            "unit": "GB/s",
            "cores": 1,
            "kind": "oracle",
            "sample": "the whole %s array, %d passes of the binary64 pairwise (int64 for int8) oracle, %.1f s" % (
                cfg.name, reps, cpu_s),
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
