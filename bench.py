#!/usr/bin/env python3
"""Benchmark of the AD-PSGD per-event worker update on one MI355X.

A step is one adpsgd_run_events call on a slice of the seeded event schedule of
the headline configuration (n = 128 workers on a ring, d = 25.6 M fp32
parameters per replica, synthetic N(0, 1e-3) gradients, tau ~ U{0..16}); the
default 10 steps x 10 000 events are exactly that configuration's 100 000
events.  Inputs (the 13.1 GB model matrix) are resident in HBM before the timed
region; the schedule slices are generated on the host beforehand.

Prints ONE JSON line: worker updates/s, plus the HBM roofline of the fused
gossip-average + apply kernel (algorithmic bytes = 16 B per parameter per event:
read and write the two averaged rows) and the CPU oracle timed on this host.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth


def traffic_from_profiles():
    """HBM bytes per event of the fused kernel measured with rocprofv3 --pmc (FETCH_SIZE and
    WRITE_SIZE runs, scaled by a copy kernel of known size); kept as text under profiles/."""
    path = os.path.join(ROOT, "profiles", "fused_gossip_apply_cfg3_pmc.txt")
    try:
        m = re.search(r"^traffic_bytes_per_event:\s*([0-9.eE+]+)", open(path).read(), re.M)
        return float(m.group(1)) if m else None
    except OSError:
        return None


def cpu_baseline(cfg, graph, schedule, events):
    """The serial oracle, as it stands, on the first `events` events at full d (one host thread)."""
    import oracle
    sub = {k: (v[:events] if v is not None else None) for k, v in schedule.items()}
    X = np.zeros((cfg["n"], cfg["d"]), dtype=np.float32)      # untouched rows are never committed
    std = float(np.float32(cfg["synth_std"]))
    t0 = time.perf_counter()
    oracle.run_events(X, sub, oracle.MODEL_SYNTH, cfg["gamma"], synth_std=std, synth_seed=cfg["seed"])
    dt = time.perf_counter() - t0
    return {"value": events / dt, "unit": "worker updates/s", "cores": 1, "kind": "oracle",
            "sample": "first %d events of the same schedule at full size (n=%d, d=%d), %.1f s"
                      % (events, cfg["n"], cfg["d"], dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--events-per-step", type=int, default=10000)
    ap.add_argument("--cpu-events", type=int, default=16, help="events the CPU oracle is timed on (0 = skip)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch one plain 1 GiB device copy (reference point for rocprofv3 byte counters)")
    ap.add_argument("--d", type=int, default=0, help="override d (debugging only; the result is then not the headline)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (all n workers are simulated in one GPU's HBM); "
                 "--gpus %d is not supported" % args.gpus)

    import torch
    import paper_1710_06952_amd as P
    from workloads import get_config, ring_graph

    cfg = get_config(3)
    if args.d:
        cfg["d"] = args.d
    n, d = cfg["n"], cfg["d"]
    graph = ring_graph(n)
    std = float(np.float32(cfg["synth_std"]))
    E = args.events_per_step

    eng = P.Engine(graph, d, "synth", gamma=cfg["gamma"], T_max=cfg["T_max"], synth_std=std, synth_seed=cfg["seed"])
    eng.set_models(np.zeros(d, np.float32))
    scheds = [P.adpsgd_make_schedule(graph, E, seed=cfg["seed"], k_begin=s * E, T_max=cfg["T_max"])
              for s in range(args.warmup + args.steps)]

    if args.calibrate_copy:        # 2^28 floats read + 2^28 floats written by an elementwise copy kernel
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for s in range(args.warmup):
        eng.run_events(scheds[s])
    torch.cuda.synchronize()
    st0 = eng.get_stats()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()                      # same stream the library launches on (torch's current stream)
    t0 = time.perf_counter()
    for s in range(args.warmup, args.warmup + args.steps):
        eng.run_events(scheds[s])
    ev1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    gpu_s = ev0.elapsed_time(ev1) * 1e-3
    elapsed = max(wall, gpu_s)
    st1 = eng.get_stats()
    events = st1["events"] - st0["events"]
    launches = st1["fused_launches"] - st0["fused_launches"]

    # dominant kernel: per-launch duration from HIP events around every launch (second handle on
    # the same buffers with per-launch timing enabled, two steps of the same schedule)
    prof = P.Handle(graph, d, model=P.MODEL_SYNTH, X_ptr=eng.X.data_ptr(), ldx=eng.ld, gamma=cfg["gamma"],
                    T_max=cfg["T_max"], synth_std=std, synth_seed=cfg["seed"],
                    stream=torch.cuda.current_stream().cuda_stream, flags=P.FLAG_PROFILE)
    n_prof = min(2, len(scheds))
    for s in range(n_prof):
        prof.run_events(scheds[s])
    ps = prof.get_stats()
    prof.destroy()
    bytes_per_event = 16.0 * d                          # read x_i, x_j; write x_i, x_j (fp32)
    events_per_launch = ps["events"] / ps["fused_launches"]
    avg_launch_s = ps["fused_ms"] * 1e-3 / ps["fused_launches"]
    achieved = bytes_per_event * events_per_launch / avg_launch_s / 1e9
    traffic = traffic_from_profiles()          # measured bytes per event (rocprofv3 counters) ...
    if traffic is not None and d == 25_600_000:
        traffic *= events_per_launch           # ... per launch, like `achieved`
    else:
        traffic = None

    out = {
        "metric": "worker updates/sec and gossip+update HBM GB/s (% of peak) at n=128, d=25.6M",
        "value": events / elapsed,
        "unit": "worker updates/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": cfg["name"], "n": n, "d": d, "graph": "ring", "events_per_step": E,
                   "events": events, "tau": "U{0..%d}" % cfg["T_max"], "gamma": cfg["gamma"],
                   "gradient": "N(0,1e-3) Philox4x32-10 + Box-Muller, generated in registers",
                   "rounds": st1["rounds"] - st0["rounds"], "fused_launches": launches,
                   "algorithmic_GBs_whole_run": bytes_per_event * events / elapsed / 1e9},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "kernel": "fused_gossip_apply_kernel<synth>", "avg_launch_ms": avg_launch_s * 1e3,
                     "events_per_launch": events_per_launch, "bytes_per_event": bytes_per_event},
    }
    eng.close()
    del eng
    torch.cuda.empty_cache()
    if args.cpu_events > 0:
        out["cpu_baseline"] = cpu_baseline(cfg, graph, scheds[0], min(args.cpu_events, E))
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
