#!/usr/bin/env python3
"""Benchmark of the sample-path engine on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input: one ``fcs_run`` of the
parameter grid (64 arrival rates x 32 activation budgets x 128 replicas = 262,144 sample paths of 50,000
slots under the flow-control rule, the largest sweep that one GPU takes), tables already resident in HBM.
Prints ONE JSON line:

* ``value``: simulated request-steps per second (sum over paths and slots of |P_t|);
* ``roofline``: the HBM reading that the metric names (algorithmic bytes = 8 B per request-step: one read
  and one write of a per-request token counter) next to what the kernel really moves and to the bound that
  does hold for it, the issue rate of the scalar instruction stream of a path (``roofline.issue``);
* ``all_configs``: the same figures for the other four benchmark configurations, one pass each;
* ``event_skipping``: the tiny configuration and the timed one again with runs of uneventful slots advanced
  in one go (same outputs; reported apart because it changes what a "step" costs);
* ``cpu_baseline``: the CPU oracle timed on a bounded sample of the same workload on the host cores.
"""
from __future__ import annotations

import argparse
import glob
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

BYTES_PER_REQUEST_STEP = 8.0
HBM_PEAK_GBS = 8000.0
N_SIMD = 1024          # 256 compute units x 4
CLOCK_HZ = 2.4e9
DEFAULT_CONFIG = 3


def cpu_baseline(wl, target_seconds: float = 15.0):
    """Times the oracle as it stands on a bounded sample of the workload: the same few replicas of every
    cell over the full horizon, cells spread over the host threads."""
    from concurrent.futures import ThreadPoolExecutor

    import numpy as np

    import oracle
    cores = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "16")))
    oracle.lib()
    n_cells = len(wl.cells)

    def run_cells(cells, ids):
        """request-steps of the listed replicas of the listed cells"""
        if len(cells) >= cores:  # many cells: one host thread per cell at a time
            with ThreadPoolExecutor(cores) as ex:
                parts = ex.map(lambda ci: int(oracle.run_cell(wl, ci, replica_ids=ids, n_threads=1)
                                              ["counters"]["sum_p"].sum()), cells)
                return sum(parts)
        return sum(int(oracle.run_cell(wl, ci, replica_ids=ids, n_threads=cores)["counters"]["sum_p"].sum())
                   for ci in cells)

    # calibrate on replica 0 of a strided subset of the cells, then size the sample for about target_seconds
    cal = list(range(0, n_cells, max(1, n_cells // cores)))[:cores]
    t0 = time.perf_counter()
    rs_cal = run_cells(cal, [0])
    dt_cal = max(time.perf_counter() - t0, 1e-3)
    threads_cal = cores if len(cal) >= cores else 1                 # one replica per call: one thread at a time
    per_replica = rs_cal / len(cal) * n_cells                       # request-steps of one replica of every cell
    rate = rs_cal / dt_cal * cores / max(threads_cal, 1)            # what all host threads together may reach
    k = int(max(1, min(wl.n_replicas, round(target_seconds * rate / max(per_replica, 1.0)))))
    if n_cells < cores:
        k = max(cores, (k // cores) * cores)
        k = min(k, wl.n_replicas)
    stride = max(1, wl.n_replicas // k)
    ids = np.arange(k) * stride
    t0 = time.perf_counter()
    total = run_cells(list(range(n_cells)), ids)
    dt = time.perf_counter() - t0
    return {"value": total / dt, "unit": "request-steps/s", "cores": cores, "kind": "oracle",
            "sample": f"replicas 0, {stride}, .. ({k} of {wl.n_replicas}) of each of the {n_cells} cells x "
                      f"{wl.n_steps} slots ({total} request-steps in {dt:.2f} s)"}


def source_hash():
    h = hashlib.sha256()
    for f in sorted(glob.glob(os.path.join(ROOT, "paper_2604_11001_amd", "csrc", "*"))):
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()


def committed_counters(config_index):
    """Per-launch figures of the committed rocprofv3 counter runs of a configuration (HBM bytes fetched and
    written, scalar instructions per path and slot), or {} once the kernel sources differ from the ones the
    counters were taken on."""
    path = os.path.join(ROOT, "profiles", f"fcs_sim_kernel_cfg{config_index}_counters.txt")
    if not os.path.exists(path):
        return {}
    vals = {}
    for ln in open(path):
        if ln.startswith("#") or ":" not in ln:
            continue
        k, v = ln.split(":", 1)
        vals[k.strip()] = v.strip()
    if vals.get("source_sha256") != source_hash():
        return {}
    return vals


def time_passes(torch, eng, steps, warmup):
    """`steps` timed launches after `warmup` untimed ones: wall time of the timed region and the duration of
    every launch by HIP events on the launch stream."""
    for _ in range(warmup):
        eng.run()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    t0 = time.perf_counter()
    for a, b in ev:
        a.record()
        eng.run()
        b.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return wall, [a.elapsed_time(b) for a, b in ev]


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=DEFAULT_CONFIG,
                    help="index of the benchmark configuration of the timed line (default 3, the parameter grid)")
    ap.add_argument("--workload", choices=("known-classes", "alpha-sweep", "budget-forms", "unknown-types",
                                           "known-types", "timed-study"),
                    default=None,
                    help="instead of --config: known-classes = the known-lengths study of Section 4.1 under "
                         "Algorithm 1 (three classes, Poisson rate 5 and budget 4 each, M = 16492); alpha-sweep = "
                         "the same three classes with unknown types under the alpha-protection greedy baseline "
                         "for four values of alpha, and the greedy baseline; budget-forms = configuration 1's "
                         "workload under Algorithm 2 with three forms of the activation budget B_t; "
                         "unknown-types = Section 4.1's three classes with unknown types under Algorithm 2, "
                         "alpha-protection, the MC benchmark and greedy; known-types = the same classes with "
                         "known types under Algorithm 1, alpha-protection, the MC benchmark with every request "
                         "predicted at its own length, and greedy; timed-study = configuration 1's "
                         "mix under Algorithm 2 and greedy with slots of variable duration")
    ap.add_argument("--replicas", type=int, default=None)
    ap.add_argument("--slots", type=int, default=None)
    ap.add_argument("--lds-slots", type=int, default=0)
    ap.add_argument("--max-active", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-all-configs", action="store_true",
                    help="only the timed line: skip the one-pass measurements of the other configurations")
    ap.add_argument("--skip-idle", action="store_true",
                    help="event skipping: runs of slots without arrival, admission, prefill or completion are "
                         "advanced in one go (same results; reported apart from the step-synchronous line)")
    ap.add_argument("--path-times", action="store_true",
                    help="profiling aid: per cell, when the workgroups of its paths started and how long they took "
                         "in the last timed launch (from the device-clock counters), as path_times in the line")
    ap.add_argument("--cells", type=str, default="", help="profiling aid: comma-separated subset of the cells")
    ap.add_argument("--copy-mib", type=int, default=0,
                    help="profiling aid: first run a plain device copy of this many MiB (scale for HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this engine runs on one GPU; sample paths are independent, so several GPUs would "
              "each take a share of the replicas with no exchange. Run with --gpus 1.", file=sys.stderr)
        return 2

    import torch

    import paper_2604_11001_amd as fcs
    from workloads import configs

    if not torch.cuda.is_available():
        print("bench.py: no HIP device", file=sys.stderr)
        return 3

    def build(bound, config=None):
        """The workload; `bound` computes the stability bound that the budgets of the configurations use."""
        if config is not None:
            return configs.make(config, bound)
        if args.workload == "known-classes":
            w = configs.known_classes()
        elif args.workload == "alpha-sweep":
            w = configs.alpha_sweep()
        elif args.workload == "budget-forms":
            w = configs.budget_forms(bound)
        elif args.workload == "unknown-types":
            w = configs.unknown_types()
        elif args.workload == "known-types":
            w = configs.known_types()
        elif args.workload == "timed-study":
            w = configs.timed_study(bound)
        else:
            w = configs.make(args.config, bound)
        if args.replicas or args.slots:
            w = w.scaled(n_replicas=args.replicas, n_steps=args.slots)
        if args.cells:
            import dataclasses
            w = dataclasses.replace(w, cells=tuple(w.cells[int(i)] for i in args.cells.split(",")))
        return w

    def measure(w, steps, warmup, **engine_kw):
        """One engine on workload w: statistics only (per-request records and histograms are parity-test
        outputs), timed launches, counters."""
        w = w.scaled(max_requests=0)
        eng = fcs.Engine(w, **engine_kw)
        geo = eng.geometry()
        wall, kernel_ms = time_passes(torch, eng, steps, warmup)
        _, summary = eng.stats()
        n_paths = eng.n_paths
        times = None
        if args.path_times:
            import numpy as np
            ctr, _ = eng.stats(profiling=True)
            start, end = ctr["clock_start"].astype(np.int64), ctr["clock_end"].astype(np.int64)
            t0, tick_ms = start.min(), 1e-5            # the device wall clock runs at 100 MHz
            times = {"launch_ms": float((end.max() - t0) * tick_ms), "cells": []}
            for ci in range(len(w.cells)):
                rows = slice(ci * eng.n_replicas, (ci + 1) * eng.n_replicas)
                d, b = (end[rows] - start[rows]) * tick_ms, (start[rows] - t0) * tick_ms
                times["cells"].append({"cell": ci, "label": w.cells[ci].label, "start_ms": [float(b.min()), float(b.max())],
                                       "duration_ms": {"mean": float(d.mean()), "p50": float(np.median(d)),
                                                       "p99": float(np.quantile(d, 0.99)), "max": float(d.max())}})
        eng.close()
        del eng
        torch.cuda.empty_cache()
        avg_ms = sum(kernel_ms) / len(kernel_ms)
        rs = int(summary["request_steps"])
        return {"wall": wall, "kernel_ms": avg_ms, "request_steps": rs, "geo": geo, "summary": summary,
                "paths": n_paths, "path_times": times,
                "achieved_gbs": rs * BYTES_PER_REQUEST_STEP / (avg_ms * 1e-3) / 1e9,
                "clocks_per_slot_and_simd": avg_ms * 1e-3 * CLOCK_HZ * N_SIMD / (n_paths * w.n_steps)}

    wl = build(fcs.stability_bound)
    plain = not (args.cells or args.replicas or args.slots or args.workload or args.lds_slots or args.max_active
                 or args.skip_idle or args.path_times)
    if args.workload:
        wl_label, kernel = args.workload, "fcs_sim_all_kernel"
    else:
        wl_label, kernel = f"configs[{args.config}] {wl.name}", "fcs_sim_kernel"
    copy_gbs = None
    if args.copy_mib > 0:
        src = torch.ones(args.copy_mib << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        # the same copy timed: what a plain kernel reaches of the HBM peak on this device (read + written bytes)
        cev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(5)]
        for a, b in cev:
            a.record()
            dst.copy_(src)
            b.record()
        torch.cuda.synchronize()
        copy_gbs = 2.0 * (args.copy_mib << 20) / (min(a.elapsed_time(b) for a, b in cev) * 1e-3) / 1e9
        del src, dst
        torch.cuda.empty_cache()

    engine_kw = dict(max_active=args.max_active, lds_slots=args.lds_slots)
    if args.skip_idle:
        engine_kw["skip_idle"] = True
    m = measure(wl, args.steps, args.warmup, **engine_kw)
    value = m["request_steps"] * args.steps / m["wall"]
    ctr = committed_counters(args.config) if plain else {}
    traffic = (int(ctr["fetch_bytes_per_launch"]) + int(ctr["write_bytes_per_launch"])
               if "fetch_bytes_per_launch" in ctr and "write_bytes_per_launch" in ctr else None)
    geo, summary = m["geo"], m["summary"]
    roof = {"bound": "hbm", "achieved": m["achieved_gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": m["achieved_gbs"] / HBM_PEAK_GBS, "traffic": traffic,
            "kernel": kernel, "kernel_ms": m["kernel_ms"], "bytes_per_request_step": BYTES_PER_REQUEST_STEP,
            "measured_hbm_gbs": None if traffic is None else traffic / (m["kernel_ms"] * 1e-3) / 1e9,
            "note": "achieved = algorithmic bytes (8 B per request-step, the accounting the metric names) over "
                    "kernel time. The kernel does not move them: the active set stays in LDS and registers and "
                    "decode growth is implicit in completion slots, so the HBM bytes really moved (traffic, "
                    "measured_hbm_gbs) are a few thousand times fewer and HBM does not bound the run. What "
                    "does is the issue rate of a path's instruction stream, see issue."}
    # the bound that holds: a SIMD issues at most one scalar instruction every 4 clocks, whatever the number
    # of wavefronts it holds, so a slot cannot take fewer clocks per SIMD than 4 x its scalar instructions
    issue = {"bound": "alu", "unit": "clocks per slot and SIMD (1,024 SIMDs at 2.4 GHz)",
             "achieved": m["clocks_per_slot_and_simd"]}
    if "salu_per_slot" in ctr:
        issue["scalar_instructions_per_slot"] = float(ctr["salu_per_slot"])
        issue["floor"] = 4.0 * float(ctr["salu_per_slot"])
        issue["frac"] = issue["floor"] / issue["achieved"]
    roof["issue"] = issue
    if copy_gbs is not None:
        roof["device_copy_gbs"] = copy_gbs

    line = {
        "metric": "simulated request-steps/sec (replicas x steps x active reqs); % of HBM roofline",
        "value": value, "unit": "request-steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": m["wall"] / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int32", "data": "synthetic",
        "config": {"workload": wl_label, "replicas": wl.n_replicas,
                   "slots": wl.n_steps, "cells": len(wl.cells), "paths": m["paths"],
                   "capacity": wl.capacity, "token_budget": wl.token_budget, "prefill_chunk": wl.prefill_chunk,
                   "request_steps_per_step": m["request_steps"], "lds_slots": geo["lds_slots"],
                   "lds_bytes_per_path": geo["lds_bytes"], "spill_slots": geo["spill_slots"],
                   "evictions": int(summary["evictions"]), "completed": int(summary["completed"]),
                   "skip_idle": bool(args.skip_idle)},
        "roofline": roof,
    }
    if m["path_times"] is not None:
        line["path_times"] = m["path_times"]
    if plain and not args.no_all_configs:
        # the other benchmark configurations, one warm-up and two timed passes each, same accounting
        rows = []
        for ci in range(len(configs.CONFIGS)):
            if ci == args.config:
                r = m
                w = wl
            else:
                w = build(fcs.stability_bound, ci)
                r = measure(w, 2, 1)
            rows.append({"config": ci, "workload": w.name, "paths": r["paths"], "slots": w.n_steps,
                         "kernel_ms": r["kernel_ms"], "request_steps": r["request_steps"],
                         "request_steps_per_s": r["request_steps"] / (r["kernel_ms"] * 1e-3),
                         "frac": r["achieved_gbs"] / HBM_PEAK_GBS,
                         "clocks_per_slot_and_simd": r["clocks_per_slot_and_simd"],
                         "lds_slots": r["geo"]["lds_slots"]})
        line["all_configs"] = rows
        # event skipping (runs of uneventful slots advanced in one go): same outputs, another accounting of
        # the time, so it is reported apart from the step-synchronous figures above
        skips = []
        for ci in (0, args.config):
            w = build(fcs.stability_bound, ci)
            r = measure(w, 2, 1, skip_idle=True)
            base = rows[ci]
            assert r["request_steps"] == base["request_steps"]
            skips.append({"config": ci, "workload": w.name, "kernel_ms": r["kernel_ms"],
                          "kernel_ms_step_synchronous": base["kernel_ms"],
                          "request_steps_per_s": r["request_steps"] / (r["kernel_ms"] * 1e-3)})
        line["event_skipping"] = skips
    if not args.no_cpu_baseline:
        import oracle
        line["cpu_baseline"] = cpu_baseline(build(oracle.stability_bound))
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
