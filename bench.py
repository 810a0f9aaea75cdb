#!/usr/bin/env python3
"""Benchmark of the AD-PSGD per-event worker update on one MI355X.

Default (the headline): configuration 3 -- n = 128 workers on a ring, d = 25.6 M fp32
parameters per replica, synthetic N(0, 1e-3) gradients, tau ~ U{0..16}.  A step is one
adpsgd_run_events call on a slice of the seeded event schedule; the default 10 steps x
10 000 events are exactly that configuration's 100 000 events.  Inputs (the 13.1 GB
model matrix) are resident in HBM before the timed region; the schedule slices are
generated on the host beforehand.

Prints ONE JSON line: worker updates/s, plus the HBM roofline of the dominant kernel
(config 3: fused gossip-average + apply, algorithmic bytes = 16 B per parameter per
event: read and write the two averaged rows) and the CPU oracle timed on this host.

``--config 1|2|4|5`` times the other configurations the same way (data generated in GPU
memory; a step is a tenth of the configuration's events); those lines are context for the
gradient kernels, not the headline.  Their roofline object covers the kernels of one event
together (gradient launches + update kernel) against the method's own traffic per event with
the minibatch rows counted once.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth


KERNEL_SOURCES = ("device_common.hpp", "kernels_fused.hip", "kernels_grad_linear.hip", "kernels_mlp.hip")


def kernel_sources_sha256():
    """Fingerprint of the kernel sources a recorded counter run belongs to."""
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_1710_06952_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def traffic_from_profiles(config=3):
    """HBM bytes per event RECORDED from rocprofv3 --pmc runs (FETCH_SIZE and WRITE_SIZE, scaled by a copy
    kernel of known size) and kept as text under profiles/: the fused kernel of configuration 3, or all
    kernels of an event of the data configurations 2, 4 and 5.  Counters cannot be read inside this run, so
    the figure is a recorded one: it is returned with the name of its file, and only when the file carries the
    fingerprint of the kernel sources as they are now (a kernel changed since the counter run gives None)."""
    name, key = (("fused_gossip_apply_cfg3_pmc.txt", "traffic_bytes_per_event") if config == 3 else
                 ("data_configurations_hbm_traffic_pmc.txt", "traffic_bytes_per_event_cfg%d" % config))
    try:
        text = open(os.path.join(ROOT, "profiles", name)).read()
    except OSError:
        return None, None
    m = re.search(r"^%s:\s*([0-9.eE+]+)" % key, text, re.M)
    sha = re.search(r"^kernel_sources_sha256:\s*([0-9a-f]+)", text, re.M)
    if not m or not sha or sha.group(1) != kernel_sources_sha256():
        return None, None
    return float(m.group(1)), "profiles/" + name


def host_description():
    """CPU model string and core counts of the host the oracle is timed on."""
    model = "unknown"
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count()
    return {"cpu_model": model, "nproc": os.cpu_count(), "usable_cores": usable}


def cpu_baseline_synth(cfg, schedule, events):
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
                      % (events, cfg["n"], cfg["d"], dt), **host_description()}


def cpu_baseline_data(cfg, schedule, events, feats, targs, x0):
    """Oracle on the first `events` events of a data configuration (data copied to the host)."""
    import oracle
    import torch
    model = {"lsq": oracle.MODEL_LSQ, "logreg": oracle.MODEL_LOGREG, "mlp": oracle.MODEL_MLP}[cfg["model"]]
    if cfg["model"] == "mlp":
        din = cfg["mlp"][0]
        hf = [np.ascontiguousarray(f[:, :din].contiguous().view(torch.int16).cpu().numpy().view(np.uint16)) for f in feats]
    else:
        hf = [f.cpu().numpy() for f in feats]
    ht = [t.cpu().numpy() for t in targs]
    sub = {k: (v[:events] if v is not None else None) for k, v in schedule.items()}
    X = np.tile(x0, (cfg["n"], 1))
    t0 = time.perf_counter()
    oracle.run_events(X, sub, model, cfg["gamma"], M=cfg["M"], gscale=1.0 / cfg["M"], lam=cfg["lam"],
                      mlp=cfg.get("mlp", (0, 0, 0)), features=hf, targets=ht, mode=1)
    dt = time.perf_counter() - t0
    return {"value": events / dt, "unit": "worker updates/s", "cores": 1, "kind": "oracle",
            "sample": "first %d events of the same schedule at full size, %.1f s" % (events, dt), **host_description()}


def schedule_kwargs(cfg):
    n = cfg["n"]
    kw = dict(seed=cfg["seed"], T_max=cfg["T_max"], M=cfg["M"], rows=[max(cfg["rows"], 1)] * n)
    if cfg["tau_mode"] == "geometric":
        slow = np.arange(n) < cfg["n_slow"]
        kw.update(tau_mode=1, weight=np.where(slow, cfg["weight_slow"], cfg["weight_fast"]),
                  tau_num=np.where(slow, cfg["tau_slow"][0], cfg["tau_fast"][0]),
                  tau_den=np.where(slow, cfg["tau_slow"][1], cfg["tau_fast"][1]))
    return kw


def algorithmic_bytes_per_event(cfg):
    """The method's own traffic per event: rows of both replicas read and written (16 B per
    parameter), plus for the data models the gradient written and read once (8 B), the stale
    model read (4 B, or 2 B of bf16 shadow plus two bf16 shadow writes) and the minibatch rows read once."""
    d = cfg["d"]
    if cfg["model"] == "synth":
        return 16.0 * d
    if cfg["model"] == "mlp":
        return 16.0 * d + 8.0 * d + 2.0 * d + 4.0 * d + cfg["M"] * cfg["mlp"][0] * 2.0
    return 16.0 * d + 8.0 * d + 4.0 * d + 4.0 * cfg["M"] * d


def sync_bench(args):
    """The synchronous comparison schedule (every worker steps in every iteration and mixes with its ring
    neighbours) at the headline shape: --sync synth draws the gradients in registers (bound by the generator's
    arithmetic), --sync slots reads them from the pending slots as the data models do (bound by HBM: 12 B per
    parameter and worker update, 20 B with momentum buffers); the slots keep fixed values so that the mixing
    kernel alone is timed.  An even number of --steps alternates between two matrices, an odd one starts with an
    iteration in place; --sync-in-place keeps every iteration in place.  Context for the update kernels, not the
    headline."""
    import torch
    import paper_1710_06952_amd as P
    from workloads import get_config, hop_ring_graph, random_regular4_graph, ring_graph
    cfg = get_config(3)
    n, d = cfg["n"], args.d or cfg["d"]
    graph = {"ring": ring_graph, "reg4": lambda m: random_regular4_graph(m, cfg["seed"]), "hop": hop_ring_graph}[args.sync_graph](n)
    mom = args.momentum != 0.0 or args.weight_decay != 0.0
    if args.sync == "synth":
        eng = P.Engine(graph, d, "synth", gamma=cfg["gamma"], synth_std=float(np.float32(cfg["synth_std"])), synth_seed=cfg["seed"],
                       momentum=args.momentum, weight_decay=args.weight_decay, sync_in_place=args.sync_in_place)
        step = lambda S: eng.run_sync_steps(S)
        bytes_per_update = (16.0 if mom else 8.0) * d
    else:
        eng = P.Engine(graph, d, "external", gamma=cfg["gamma"], n_slots=n, momentum=args.momentum, weight_decay=args.weight_decay,
                       sync_in_place=args.sync_in_place)
        eng.workspace.normal_(0.0, 0.01)
        step = lambda S: eng.run_sync_steps_with(S, lambda worker, event, xhat, g: None)
        bytes_per_update = (20.0 if mom else 12.0) * d
    eng.set_models(np.zeros(d, np.float32))
    warm = max(args.warmup, 2) + ((max(args.warmup, 2) ^ args.steps) & 1)      # the parity of the timed call, and >= 2:
    step(warm)                                                                  # the handle's second matrix exists
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    step(args.steps)
    ev1.record()
    torch.cuda.synchronize()
    t = ev0.elapsed_time(ev1) * 1e-3
    achieved = bytes_per_update * n * args.steps / t / 1e9
    print(json.dumps({
        "metric": "worker updates/s (synchronous comparison schedule, gradients: %s)" % args.sync, "value": n * args.steps / t,
        "unit": "worker updates/s", "n_gpus": 1, "steps": args.steps, "warmup": warm, "ms_per_step": t / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "cfg3 shape, synchronous iterations on the %s" % {"ring": "ring", "reg4": "random 4-regular graph",
                                                                               "hop": "ring with the 2^i + 1 hop links"}[args.sync_graph],
                   "n": n, "d": d, "momentum": args.momentum,
                   "weight_decay": args.weight_decay},
        "roofline": {"bound": "hbm" if args.sync == "slots" else "alu", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                     "kernel": ("sync_ring_apply_kernel" if args.sync_graph == "ring" else "sync_mix_apply_kernel") + " (in place)"
                     if args.sync_in_place else
                     ("sync_ring_rows_kernel" if args.sync_graph == "ring" else "sync_graph_rows_kernel") +
                     " (pairs of iterations, out of place; an odd first one in place)",
                     "bytes_per_worker_update": bytes_per_update}}), flush=True)
    eng.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=3, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--events-per-step", type=int, default=0, help="default: a tenth of the configuration's events")
    ap.add_argument("--cpu-events", type=int, default=-1,
                    help="events the CPU oracle is timed on (0 = skip; default 50 for config 3, about a minute on one core; 0 otherwise)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch one plain 1 GiB device copy (reference point for rocprofv3 byte counters)")
    ap.add_argument("--momentum", type=float, default=0.0,
                    help="config 3 only: run the events with per-worker momentum buffers (24 B per parameter per event)")
    ap.add_argument("--weight-decay", type=float, default=0.0)
    ap.add_argument("--d", type=int, default=0, help="override d (debugging only; the result is then not the headline)")
    ap.add_argument("--sync", choices=["synth", "slots"], default=None,
                    help="time the synchronous comparison schedule at the headline shape instead (a step is one iteration)")
    ap.add_argument("--sync-graph", choices=["ring", "reg4", "hop"], default="ring",
                    help="with --sync: the ring (default), a random 4-regular graph, or the ring with the paper's 2^i + 1 hop links")
    ap.add_argument("--sync-in-place", action="store_true", help="with --sync: every iteration mixes in place (no second model matrix)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (all n workers are simulated in one GPU's HBM); "
                 "--gpus %d is not supported" % args.gpus)
    if args.sync:
        return sync_bench(args)

    import torch
    import paper_1710_06952_amd as P
    from workloads import (get_config, ring_graph, random_regular4_graph, linear_data_on_device,
                           mixture_data_on_device, mlp_init)

    cfg = get_config(args.config)
    if args.d:
        cfg["d"] = args.d
    n, d, M = cfg["n"], cfg["d"], cfg["M"]
    graph = ring_graph(n) if cfg["graph"] == "ring" else random_regular4_graph(n, cfg["seed"])
    E = args.events_per_step or max(cfg["K"] // 10, 1)
    cpu_events = args.cpu_events if args.cpu_events >= 0 else (50 if args.config == 3 else 0)
    synth = cfg["model"] == "synth"
    std = float(np.float32(cfg.get("synth_std", 0.0)))

    feats = targs = None
    x0 = np.zeros(d, np.float32)
    if synth:
        eng = P.Engine(graph, d, "synth", gamma=cfg["gamma"], T_max=cfg["T_max"], synth_std=std, synth_seed=cfg["seed"],
                       momentum=args.momentum, weight_decay=args.weight_decay)
    elif cfg["model"] == "mlp":
        feats, targs = mixture_data_on_device(n, cfg["rows"], din=cfg["mlp"][0], classes=cfg["mlp"][2], seed=cfg["seed"])
        x0 = mlp_init(*cfg["mlp"], seed=cfg["seed"])
        eng = P.Engine(graph, d, "mlp", M=M, gamma=cfg["gamma"], T_max=cfg["T_max"], mlp=cfg["mlp"])
    else:
        feats, targs = linear_data_on_device(cfg["model"], n, cfg["rows"], d, seed=cfg["seed"],
                                             feature_var=cfg.get("feature_var"))
        eng = P.Engine(graph, d, cfg["model"], M=M, gamma=cfg["gamma"], lam=cfg["lam"], T_max=cfg["T_max"])
    if feats is not None:
        eng.load_data(feats, targs)
    eng.set_models(x0)
    kw = schedule_kwargs(cfg)
    scheds = [P.adpsgd_make_schedule(graph, E, k_begin=s * E, **kw) for s in range(args.warmup + args.steps)]

    if args.calibrate_copy:        # 2^28 floats read + 2^28 floats written by a plain device copy
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

    # per-launch durations from HIP events around every launch: a second handle on the same
    # buffers with per-launch timing enabled, two steps of the same schedule
    prof = P.Handle(graph, d, model=eng.model, X_ptr=eng.X.data_ptr(), ldx=eng.ld, M=M, gamma=cfg["gamma"],
                    lam=cfg["lam"], T_max=cfg["T_max"], synth_std=std, synth_seed=cfg["seed"],
                    mlp=cfg.get("mlp", (0, 0, 0)), Xbf16_ptr=None if eng.Xbf16 is None else eng.Xbf16.data_ptr(),
                    workspace_ptr=None if eng.workspace is None else eng.workspace.data_ptr(),
                    workspace_bytes=0 if eng.workspace is None else eng.workspace.numel() * 4,
                    stream=torch.cuda.current_stream().cuda_stream, flags=P.FLAG_PROFILE,
                    momentum=args.momentum if synth else 0.0, weight_decay=args.weight_decay if synth else 0.0,
                    V_ptr=None if eng.V is None else eng.V.data_ptr())
    if feats is not None:
        for i, (f, t) in enumerate(eng._data):
            prof.load_data(i, f.data_ptr(), f.shape[0], f.stride(0), t.data_ptr())
    n_prof = min(2, len(scheds))
    for s in range(n_prof):
        prof.run_events(scheds[s])
    ps = prof.get_stats()
    prof.destroy()

    events_per_launch = ps["events"] / ps["fused_launches"]
    if synth:
        bytes_per_event = (24.0 if eng.V is not None else 16.0) * d   # read x_i, x_j; write x_i, x_j (+ v_i read and written)
        avg_launch_s = ps["fused_ms"] * 1e-3 / ps["fused_launches"]
        achieved = bytes_per_event * events_per_launch / avg_launch_s / 1e9
        traffic, traffic_source = traffic_from_profiles()   # recorded bytes per event (rocprofv3 counters) ...
        if traffic is not None and d == 25_600_000 and eng.V is None:
            traffic = traffic * events_per_launch            # ... per launch of this run
        else:
            traffic = traffic_source = None
        roof = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                "kernel": "fused_gossip_apply_kernel<synth>", "avg_launch_ms": avg_launch_s * 1e3,
                "events_per_launch": events_per_launch, "bytes_per_event": bytes_per_event}
    else:
        # the kernels of one event together: gradient launches + update (with a factored gradient the
        # update kernel does part of the gradient's work, so the two are not separated here); bytes = the
        # method's own traffic per event, minibatch rows counted once
        grad_rows_bytes = (M * cfg["mlp"][0] * 2.0 + 2.0 * d) if cfg["model"] == "mlp" else 4.0 * M * d
        per_grad_s = ps["grad_ms"] * 1e-3 / ps["events"]
        per_update_s = ps["fused_ms"] * 1e-3 / ps["events"]
        bytes_per_event = algorithmic_bytes_per_event(cfg)
        achieved = bytes_per_event / (per_grad_s + per_update_s) / 1e9
        traffic, traffic_source = traffic_from_profiles(args.config) if (not args.d and eng.V is None) else (None, None)
        roof = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBS,
                "traffic": traffic, "traffic_source": traffic_source,   # recorded bytes per event, as `achieved` is
                "kernel": "gradient + update kernels (per event)", "avg_gradient_us": per_grad_s * 1e6,
                "fused_us_per_event": per_update_s * 1e6, "bytes_per_event": bytes_per_event,
                "bytes_per_gradient": grad_rows_bytes, "events_per_launch": events_per_launch}

    out = {
        "metric": "worker updates/sec and gossip+update HBM GB/s (% of peak) at n=128, d=25.6M" if args.config == 3
                  else "worker updates/sec (configuration %d)" % args.config,
        "value": events / elapsed,
        "unit": "worker updates/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if cfg["model"] == "mlp" else "f32",
        "data": "synthetic",
        "config": {"workload": cfg["name"], "n": n, "d": d, "graph": cfg["graph"], "events_per_step": E,
                   "events": events, "M": M, "gamma": cfg["gamma"], "T_max": cfg["T_max"],
                   "rounds": st1["rounds"] - st0["rounds"], "fused_launches": launches,
                   "grad_launches": st1["grad_launches"] - st0["grad_launches"],
                   "algorithmic_GBs_whole_run": algorithmic_bytes_per_event(cfg) * events / elapsed / 1e9},
        "roofline": roof,
    }
    if synth:
        out["config"]["gradient"] = "N(0,1e-3) Philox4x32-10 + Box-Muller, generated in registers"
        if eng.V is not None:
            out["config"]["optimizer"] = {"momentum": args.momentum, "weight_decay": args.weight_decay}
            out["roofline"]["kernel"] = "fused_gossip_apply_kernel<synth, momentum>"
    # diagnostics (outside the timed region): consensus distance and mean model each read X once.  The second of two
    # calls is timed (the first one allocates the library's small result buffers), the output vector allocated before;
    # HIP events on the library's stream bracket each call: for the consensus distance its kernels, its 8-byte copy and
    # the wait for it; the mean model goes to device memory, which the call enqueues without waiting
    torch.cuda.synchronize()
    mean_dev = torch.empty(d, dtype=torch.float32, device="cuda:0")
    eng.consensus_distance()
    eng.h.mean_model_to_device(mean_dev.data_ptr())
    torch.cuda.synchronize()
    dv = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    dv[0].record()
    cd = eng.consensus_distance()
    dv[1].record()
    eng.h.mean_model_to_device(mean_dev.data_ptr())
    dv[2].record()
    torch.cuda.synchronize()
    t_cons, t_mean = dv[0].elapsed_time(dv[1]) * 1e-3, dv[1].elapsed_time(dv[2]) * 1e-3
    xbytes = 4.0 * n * d
    out["diagnostics"] = {"consensus_distance": cd, "consensus_ms": t_cons * 1e3, "consensus_GBs": xbytes / t_cons / 1e9,
                          "mean_model_ms": t_mean * 1e3, "mean_model_GBs": xbytes / t_mean / 1e9}
    del mean_dev
    if cfg["model"] in ("lsq", "logreg"):       # the objective reads every local row once
        eng.objective()
        t3 = time.perf_counter()
        fval = eng.objective()
        t4 = time.perf_counter()
        dbytes = 4.0 * n * cfg["rows"] * d
        out["diagnostics"].update({"objective_at_mean_model": fval, "objective_ms": (t4 - t3) * 1e3,
                                   "objective_GBs": dbytes / (t4 - t3) / 1e9})
    if cpu_events > 0:
        if synth:
            eng.close()
            del eng
            torch.cuda.empty_cache()
            out["cpu_baseline"] = cpu_baseline_synth(cfg, scheds[0], min(cpu_events, E))
        else:
            out["cpu_baseline"] = cpu_baseline_data(cfg, scheds[0], min(cpu_events, E), feats, targs, x0)
            eng.close()
    else:
        eng.close()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
