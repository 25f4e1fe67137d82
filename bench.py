#!/usr/bin/env python3
"""Throughput of batched critical-path evaluation on one MI355X.

A step is one full cp_eval over one batch of candidate partitions: cost tables,
b-level sweep, critical-path length, t-level sweep and critical-vertex mask, with
the graph and the assignments already resident in HBM.  Both sweeps relax every
edge once per partition, so a step performs 2 * |E| * P edge relaxations.

Prints ONE JSON line.  `roofline` covers the dominant kernel (the b-level sweep),
timed with HIP events on the stream it runs on; `cpu_baseline` is the plain CPU
oracle timed on a bounded sample of the same partitions.
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

HBM_PEAK_GBS = 8000.0  # MI355X, published

# HBM bytes of one b-level sweep launch from hardware counters (rocprofv3 --pmc FETCH_SIZE and
# WRITE_SIZE in separate runs, each scaled by what the same counter reads for a 1 GiB device
# copy: x2.00 and x1.00; profiles/ holds the runs).  These are recorded values, not live ones:
# a figure belongs to one build of the kernels and one configuration, and is reported only
# while the sources it was taken on are unchanged and the configuration matches.
MEASURED_TRAFFIC = {
    "sources_sha256": "58b934d1b80cf7c4a2e9b0721b7a3c30d8d890266545b8b676540571ec8915e1",
    "runs": [
        # (workload, P, plan, out_layout) -> HBM bytes per launch of the dominant kernel: FETCH_SIZE x 2.00 +
        # WRITE_SIZE x 1.00 (KiB per dispatch, scaled by what the same counters read for a 1 GiB copy and fill)
        (("large_sparse", 256, 2, 1), (2 * 458523.3 + 2000005.9) * 1024),        # both sweeps in one launch
        (("large_sparse", 1024, 4, 1), (2 * 602781.3 + 4000023.4) * 1024),       # b-level sweep
        (("large_sparse", 16384, 4, 1), (2 * 9642261.2 + 64000490.5) * 1024),    # b-level sweep
    ],
}
TRAFFIC_SOURCES = ("kernels.hip", "window_shared.hip", "graph.cpp", "api.hip", "launch.hpp", "cpeval_internal.hpp",
                   "device_math.hpp")     # the sweep kernels, the packet layout, the choice of plan and shape


def sources_digest():
    import hashlib
    h = hashlib.sha256()
    for name in TRAFFIC_SOURCES:
        with open(os.path.join(ROOT, "paper_1711_01912_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def measured_traffic(workload, P, plan, out_layout):
    m = MEASURED_TRAFFIC
    if sources_digest() != m["sources_sha256"]:
        return None
    for key, nbytes in m["runs"]:
        if key == (workload, P, plan, out_layout):
            return float(nbytes)
    return None


def algorithmic_bytes_per_sweep(n, m, P, tick_bytes):
    """Gather model: per (vertex, partition) one device id read and one tick
    written; per (edge, partition) one device id and one tick read; plus the graph
    structure (12 bytes per vertex and per edge) once per 64 partitions."""
    data = (n + m) * P * (1 + tick_bytes)
    graph = (n * 12 + m * 12) * ((P + 63) // 64)
    return data + graph


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="large_sparse")
    ap.add_argument("--plan", type=int, default=0, help="0 auto, 1 wave-column, 2 resident-window, "
                    "3 / 4 shared window with 2 / 4 partitions per workgroup, 5 column slices, 6 streamed window")
    ap.add_argument("--batch", type=int, default=0, help="override the workload's batch size")
    ap.add_argument("--print-sources-digest", action="store_true",
                    help="print the digest MEASURED_TRAFFIC is keyed by (after taking the HBM counters anew) and exit")
    ap.add_argument("--out-layout", default="native", choices=("native", "vertex", "partition"),
                    help="layout of b, tl and the mask; native = the one the plan that runs produces directly "
                         "(partition-major for the resident-window plan, vertex-major for wave-column)")
    ap.add_argument("--cpu-sample", type=int, default=128, help="partitions the oracle is timed on (0 = skip)")
    ap.add_argument("--extras", action="store_true",
                    help="after the timed steps also time the consumers of the result (priority lists, one "
                         "critical path per partition, the list-scheduling simulation) and report them "
                         "under 'extras'")
    ap.add_argument("--calibrate-copy-mib", type=int, default=0,
                    help="also run a plain device copy of this many MiB (a known-size kernel to scale "
                         "hardware byte counters against)")
    args = ap.parse_args()
    if args.print_sources_digest:
        print(sources_digest())
        return
    if args.gpus != 1:
        print("bench.py measures one GPU: the path has no multi-GPU part; run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_1711_01912_amd as cpe
    from paper_1711_01912_amd import binding
    from workloads import make_workload

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    cpe.load_library()   # fails loudly if the HIP library was not built

    kw = {"P": args.batch} if args.batch else {}
    w = make_workload(args.workload, **kw)
    dev = "cuda:0"
    g = cpe.CpGraph.from_workload(w, device=dev)
    info = g.info
    T = info["min_tick_bytes"]
    a = torch.from_numpy(w.assignments).to(dev)
    P, n, m = w.P, w.n, w.m
    tdt = torch.int32 if T == 4 else torch.int64
    plan_used = args.plan if args.plan else binding.choose_plan(g, P, w.speeds, w.bandwidth, T)
    if args.out_layout == "native":
        out_layout = (cpe.OUT_VERTEX_MAJOR if plan_used in (cpe.PLAN_WAVE_COLUMN, cpe.PLAN_COLUMN_SLICE)
                      else cpe.OUT_PARTITION_MAJOR)
    else:
        out_layout = cpe.OUT_PARTITION_MAJOR if args.out_layout == "partition" else cpe.OUT_VERTEX_MAJOR
    rows, cols = (n, P) if out_layout == cpe.OUT_VERTEX_MAJOR else (P, n)
    out = {
        "cp": torch.empty(P, dtype=torch.int64, device=dev),
        "b": torch.empty((rows, cols), dtype=tdt, device=dev),
        "tl": torch.empty((rows, cols), dtype=tdt, device=dev),
        "mask": torch.empty((rows, (cols + 63) // 64), dtype=torch.int64, device=dev),
        "status": torch.empty(1, dtype=torch.int32, device=dev),
    }
    ws = torch.empty(binding.workspace_bytes(g, P, w.k, plan=args.plan, out_layout=out_layout, tick_bytes=T),
                     dtype=torch.uint8, device=dev)
    prof = cpe.CpProfile(max(args.steps, 1))

    def step(profile=None):
        cpe.cp_eval(g, a, w.speeds, w.bandwidth, out=out, workspace=ws, plan=args.plan, out_layout=out_layout,
                    profile=profile, check_status=False)

    if args.calibrate_copy_mib > 0:
        src = torch.empty(args.calibrate_copy_mib << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(prof)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    assert int(out["status"].item()) == 0
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    stages = {name: [] for name in binding.STAGE_NAMES}
    launches = (1, 1)
    for i in range(prof.count()):
        ms, launches = prof.read(i)
        for name, v in ms.items():
            stages[name].append(v)
    stage_ms = {name: float(np.mean(v)) for name, v in stages.items()}
    b_ms = stage_ms["blevel"]
    # the resident-window plan may run both sweeps in one launch (no t-level launch is reported
    # then): that launch is the dominant kernel and does the work of two sweeps
    paired = launches[1] == 0
    sweeps = 2 if paired else 1
    sweep_bytes = sweeps * algorithmic_bytes_per_sweep(n, m, P, T)
    b_launches = max(1, launches[0])
    achieved = sweep_bytes / (b_ms * 1e-3) / 1e9
    traffic = measured_traffic(args.workload, P, plan_used, out_layout)
    roofline = {
        # achieved / frac: the algorithmic bytes of the gather model (every relaxation fetches its
        # neighbour's value and device id) over the kernel's time.  The window plans serve those
        # gathers from LDS, so this is an effective rate; the bytes that really cross HBM are
        # `traffic` (a recorded counter value, see MEASURED_TRAFFIC), and `hbm_frac_measured` is
        # that over the same time against the same peak.
        "bound": "hbm", "model": "gather", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": achieved / HBM_PEAK_GBS,
        "traffic": traffic,
        "traffic_kind": "recorded rocprofv3 FETCH_SIZE + WRITE_SIZE of this build and configuration" if traffic else None,
        "hbm_frac_measured": traffic / (b_ms * 1e-3 / b_launches) / 1e9 / HBM_PEAK_GBS if traffic else None,
        "kernel": "b-level and t-level sweeps in one launch" if paired else "b-level sweep",
        "launches_per_step": b_launches,
        "avg_launch_us": b_ms * 1e3 / b_launches,
        "algorithmic_bytes_per_launch": sweep_bytes / b_launches,
        "relaxations_per_launch": sweeps * m * P / b_launches,
        "compulsory_frac": (sweeps * n * P * (1 + T)) / (b_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
    }

    extras = None
    if args.extras:
        extras = {}
        b_layout = out_layout
        max_b = int(out["cp"].max().item())

        def timed(fn, reps=5):
            fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps

        ms = timed(lambda: cpe.cp_pct_order(g, a, w.k, out["b"], max_b=max_b, b_layout=b_layout, check_status=False))
        extras["pct_order"] = {"ms": ms, "keys_per_s": n * P / (ms * 1e-3), "key_bits": max_b.bit_length()
                               + (w.k - 1).bit_length()}
        ms = timed(lambda: cpe.cp_critical_path(g, a, w.speeds, w.bandwidth, out["b"], out["cp"],
                                                b_layout=b_layout, check_status=False))
        extras["critical_path"] = {"ms": ms}
        if w.k <= 64:
            # the paper's Critical Path partition as a start, then three moves of the search
            t0 = time.perf_counter()
            seed = cpe.cp_seed_partition(g, w.speeds)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            found = cpe.cp_search(g, seed, w.speeds, w.bandwidth, max_moves=3, chunk=1024)
            torch.cuda.synchronize()
            t2 = time.perf_counter()
            extras["seed_partition"] = {"ms": (t1 - t0) * 1e3}
            extras["search"] = {"ms": (t2 - t1) * 1e3, "moves": int(len(found["moves"])),
                                "evaluated": int(found["evaluated"]),
                                "relaxations_per_s": float(found["evaluated"]) * m / (t2 - t1),
                                "cp_trace": [int(x) for x in found["cp_trace"]]}
        if w.k <= 64 and int(w.c.min()) >= 1:
            # the list-scheduling simulation under both policies, and the oracle's on a few partitions
            from oracle import cp_oracle
            sim_ws = {}
            for policy, name in ((cpe.POLICY_PCT, "pct"), (cpe.POLICY_FIFO, "fifo")):
                kwargs = dict(b=out["b"], b_layout=b_layout) if policy == cpe.POLICY_PCT else {}
                res = {}

                def run():
                    res["makespan"], _ = cpe.cp_simulate(g, a, w.speeds, w.bandwidth, policy, want_start=False,
                                                         check_status=False, **kwargs)
                ms = timed(run, reps=1 if n * P > 50_000_000 else 3)
                sample = min(16, P)
                b_ref = None
                if policy == cpe.POLICY_PCT:
                    rows_b = out["b"][:sample] if b_layout == cpe.OUT_PARTITION_MAJOR else out["b"][:, :sample].T
                    b_ref = rows_b.cpu().numpy().astype(np.int64)
                c0 = time.perf_counter()
                ref = cp_oracle.simulate(w.n, w.succ_ptr, w.succ_idx, w.succ_t, w.c, w.speeds, w.bandwidth,
                                         w.assignments[:sample], policy, b=b_ref, want_start=False, threads=16)
                c1 = time.perf_counter()
                assert np.array_equal(ref["makespan"], res["makespan"][:sample].cpu().numpy()), \
                    "GPU and oracle disagree on the makespan"
                extras["simulate_" + name] = {
                    "ms": ms, "vertex_starts_per_s": n * P / (ms * 1e-3),
                    "mean_makespan": float(res["makespan"].double().mean().item()),
                    "mean_cp": float(out["cp"].double().mean().item()),
                    "oracle_vertex_starts_per_s": n * sample / (c1 - c0), "oracle_threads": ref["threads"],
                    "oracle_sample": sample}

    cpu = None
    if args.cpu_sample > 0:
        from oracle import cp_oracle
        sample = min(args.cpu_sample, P)
        threads = min(16, len(os.sched_getaffinity(0)), sample)
        c0 = time.perf_counter()
        ref = cp_oracle.evaluate_workload(w, want=("cp",), threads=threads, partitions=slice(0, sample))
        c1 = time.perf_counter()
        assert np.array_equal(ref["cp"], out["cp"][:sample].cpu().numpy()), "GPU and oracle disagree on CP"
        cpu = {"value": 2.0 * m * sample / (c1 - c0), "unit": "relaxations/s", "cores": ref["threads"],
               "kind": "oracle", "sample": f"first {sample} of {P} partitions of the same workload, "
                                           f"both sweeps, {c1 - c0:.2f} s"}

    rec = {
        "metric": "edge-relaxations/sec (|E| x partitions) for batched critical-path eval",
        "value": 2.0 * m * P / (ms_per_step * 1e-3),
        "unit": "relaxations/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32" if T == 4 else "int64", "data": "synthetic",
        "config": {"workload": args.workload, "n": n, "m": m, "L": w.L, "P": P, "k": w.k,
                   "tick_bytes": T, "max_out_degree": info["max_out_degree"],
                   "raw_path_bound": info["raw_path_bound"],
                   "plan": {1: "wave-column", 2: "resident-window", 3: "shared-window-2", 4: "shared-window-4",
                            5: "column-slice", 6: "streamed-window"}[plan_used],
                   "out_layout": "vertex-major" if out_layout == cpe.OUT_VERTEX_MAJOR else "partition-major"},
        "stage_ms": stage_ms,
        "sweep_relaxations_per_s": sweeps * m * P / (b_ms * 1e-3),      # of the dominant kernel's stage
        "sweeps_in_dominant_kernel": sweeps,
        "ns_per_level": b_ms * 1e6 / w.L,                              # of that stage (both sweeps when paired)
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    if extras is not None:
        rec["extras"] = extras
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
