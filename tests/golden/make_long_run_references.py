#!/usr/bin/env python3
"""Writes tests/golden/long_run_cfg{2,4,5}.npz: the serial oracle's models along a run of ALL events of the data
configurations 2, 4 and 5 (20 000, 20 000 and 50 000 events), which is too long for the oracle to replay
inside the GPU suite (3.5 min, 15 min and 40 min of one host core).  Calls only oracle/ and the seeded input
generators of workloads/; nothing of the HIP library is imported, so no stored value comes from the GPU path.

    python tests/golden/make_long_run_references.py 2 4 5        # any subset; one process per configuration is fine

Workload: the configuration's n, d, M, step size, staleness law and graph (workloads/configs.py).  The local
data sets come from the host generators (numpy, seeded) and are cut down to what the tests can regenerate and
upload in seconds: configuration 2 keeps 256 of 4096 rows per worker, configuration 5 keeps 16 of 64; the
perceptron keeps all 8192.  The run is cut into CALLS self-contained calls (staleness restarts at a cut, as in
bench.py's steps); after every call the file keeps, per worker,
  coords            the sampled coordinates (seeded choice, the same for all workers and checkpoints)
  x[c][i, :]        the model of worker i at the sampled coordinates after call c            (fp32)
  amax[c][i]        max |x| over ALL coordinates of worker i (the denominator of the parity measure)
  l2[c][i], s[c][i] the Euclidean norm and the plain sum of ALL coordinates of worker i, in fp64
  loss_tail[c]      the mean minibatch loss of the call's last 200 events
tests/test_gpu_long_runs.py runs the same calls on the GPU and compares.
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from workloads import (get_config, logreg_data, lsq_data, mixture_data, mlp_init,  # noqa: E402
                       random_regular4_graph, ring_graph)

CALLS = 4
SAMPLED = 1024
ROWS = {2: 256, 4: 8192, 5: 16}


def schedule_kwargs(c, rows):
    n = c["n"]
    kw = dict(seed=c["seed"], T_max=c["T_max"], M=c["M"], rows=[rows] * n)
    if c["tau_mode"] == "geometric":
        slow = np.arange(n) < c["n_slow"]
        kw.update(tau_mode=1, weight=np.where(slow, c["weight_slow"], c["weight_fast"]),
                  tau_num=np.where(slow, c["tau_slow"][0], c["tau_fast"][0]),
                  tau_den=np.where(slow, c["tau_slow"][1], c["tau_fast"][1]))
    return kw


def workload(idx):
    """Graph, host data, initial model and the calls' schedules of one configuration (shared with the GPU test)."""
    c = get_config(idx)
    n, d, rows = c["n"], c["d"], ROWS[idx]
    g = ring_graph(n) if c["graph"] == "ring" else random_regular4_graph(n, c["seed"])
    if c["model"] == "mlp":
        feats, targs, _ = mixture_data(n, rows, din=c["mlp"][0], classes=c["mlp"][2], seed=c["seed"])
        x0 = mlp_init(*c["mlp"], seed=c["seed"])
    elif c["model"] == "logreg":
        feats, targs, _ = logreg_data(n, rows, d, seed=c["seed"])
        x0 = np.zeros(d, np.float32)
    else:
        feats, targs, _ = lsq_data(n, rows, d, seed=c["seed"], feature_var=1.0 / d)
        x0 = np.zeros(d, np.float32)
    per_call = c["K"] // CALLS
    skw = schedule_kwargs(c, rows)
    calls = [oracle.make_schedule(g, per_call, k_begin=q * per_call, **skw) for q in range(CALLS)]
    coords = np.sort(np.random.default_rng([c["seed"], 77, idx]).choice(d, size=min(SAMPLED, d), replace=False)).astype(np.int64)
    return c, g, feats, targs, x0, calls, coords


def main(which):
    for idx in which:
        t0 = time.time()
        c, g, feats, targs, x0, calls, coords = workload(idx)
        print("configuration %d: data ready after %.0f s" % (idx, time.time() - t0), flush=True)
        model = {"lsq": oracle.MODEL_LSQ, "logreg": oracle.MODEL_LOGREG, "mlp": oracle.MODEL_MLP}[c["model"]]
        X = np.tile(x0, (c["n"], 1))
        out = {"coords": coords, "events_per_call": np.int64(c["K"] // CALLS), "rows": np.int64(ROWS[idx])}
        for q, sched in enumerate(calls):
            r = oracle.run_events(X, sched, model, c["gamma"], M=c["M"], gscale=1.0 / c["M"], lam=c["lam"],
                                  mlp=c.get("mlp", (0, 0, 0)), features=feats, targets=targs, mode=1, want_loss=True)
            X64 = X.astype(np.float64)
            out["x%d" % q] = X[:, coords].copy()
            out["amax%d" % q] = np.max(np.abs(X), axis=1)
            out["l2_%d" % q] = np.sqrt((X64 * X64).sum(axis=1))
            out["s%d" % q] = X64.sum(axis=1)
            out["loss_tail%d" % q] = np.float64(r["loss"][-200:].mean())
            print("configuration %d: call %d of %d done after %.0f s, loss %.4f" % (idx, q + 1, CALLS, time.time() - t0,
                                                                                 out["loss_tail%d" % q]), flush=True)
        path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "long_run_cfg%d.npz" % idx)
        np.savez_compressed(path, **out)
        print("wrote %s (%.0f KB)" % (path, os.path.getsize(path) / 1e3), flush=True)


if __name__ == "__main__":
    main([int(a) for a in sys.argv[1:]] or [2, 4, 5])
