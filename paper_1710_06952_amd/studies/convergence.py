"""Convergence with respect to epochs, shaped like the paper's comparison of Sec. 5.2 (training loss
against epochs for 16 workers: the centralized synchronous baseline, the synchronous decentralized
one and AD-PSGD reach about the same loss after the same number of epochs).

Nothing here needs the paper's data or networks.  The workload is a small dense classifier
(in -> hidden, ReLU -> classes, softmax cross-entropy) on a seeded Gaussian mixture, every worker
with its own local samples of the same distribution; the optimizer is the experiments' (momentum 0.9,
weight decay 1e-4, a step size that is halved at fixed epochs).  Three schedules run on the same data,
all executed by the HIP library:

  complete     every iteration all workers take a gradient while ALL models are averaged:
               adpsgd_run_sync_steps on the complete graph, whose Metropolis weights are 1/n
               everywhere.  The mean model then follows minibatch SGD with n M samples (gradients
               taken at the workers' own models, which differ by one step only): the closest this
               schedule gets to the centralized synchronous baseline;
  d-psgd       the same iteration on the ring: each worker mixes with its two neighbours only;
  ad-psgd      adpsgd_run_events on the ring: one worker at a time, stale reads (tau uniform in
               {0..T_max}), pairwise averaging with one random neighbour.

An epoch is one pass over all workers' samples: n * rows / M gradient evaluations, i.e. that many
events, or 1/n of that many synchronous iterations.  After every epoch the objective over all
local data at the mean model (Algorithm 1's output) is read back with adpsgd_objective, and the
classification error (1 - accuracy) with adpsgd_classification_error.

    python -m paper_1710_06952_amd.studies.convergence [--n 16] [--epochs 12] [--json]
"""
from __future__ import annotations

import argparse
import json

import numpy as np

from .. import step_sizes


def ring(n):
    rowptr = np.arange(0, 2 * n + 1, 2, dtype=np.int32)
    col = np.array([[(i - 1) % n, (i + 1) % n] for i in range(n)], dtype=np.int32).reshape(-1)
    return rowptr, col


def complete(n):
    rowptr = np.arange(0, n * (n - 1) + 1, n - 1, dtype=np.int32)
    col = np.array([j for i in range(n) for j in range(n) if j != i], dtype=np.int32)
    return rowptr, col


def make_problem(n, rows, dims, seed):
    """Per worker `rows` samples of a `classes`-component Gaussian mixture (unit noise around seeded
    means of norm ~ 3), and one initial model N(0, 1/fan_in) shared by all workers."""
    din, hid, classes = dims
    rng = np.random.default_rng([seed, 11])
    means = 3.0 * rng.standard_normal((classes, din)) / np.sqrt(din)
    feats, labels = [], []
    for _ in range(n):
        y = rng.integers(0, classes, size=rows)
        feats.append((means[y] + rng.standard_normal((rows, din))).astype(np.float32))
        labels.append(y.astype(np.int32))
    x0 = np.concatenate([
        (rng.standard_normal(din * hid) / np.sqrt(din)), np.zeros(hid),
        (rng.standard_normal(hid * classes) / np.sqrt(hid)), np.zeros(classes)]).astype(np.float32)
    return feats, labels, x0


def run_study(n=16, dims=(64, 256, 10), rows=2048, M=32, epochs=12, T_max=4, gamma=0.02, halve_every=4,
              momentum=0.9, weight_decay=1e-4, seed=0, device="cuda:0"):
    import torch
    from .. import Engine, adpsgd_make_schedule
    din, hid, classes = dims
    d = din * hid + hid + hid * classes + classes
    feats, labels, x0 = make_problem(n, rows, dims, seed)
    dev_feats = [torch.from_numpy(f).to(device).to(torch.bfloat16).contiguous() for f in feats]
    dev_labels = [torch.from_numpy(y).to(device) for y in labels]
    events_per_epoch = n * rows // M
    iters_per_epoch = events_per_epoch // n

    def engine(graph):
        eng = Engine(graph, d, "mlp", M=M, gamma=gamma, T_max=T_max, mlp=dims, n_slots=max(n, T_max + 1),
                     momentum=momentum, weight_decay=weight_decay, device=device)
        eng.load_data(dev_feats, dev_labels)
        eng.set_models(x0)
        return eng

    curves = {}
    for name, graph in (("complete", complete(n)), ("d-psgd", ring(n))):
        eng = engine(graph)
        curve, errs = [eng.objective()], [eng.classification_error()]
        spread = 0.0
        rng = np.random.default_rng([seed, 12])
        for e in range(epochs):
            batch = rng.integers(0, rows, size=(iters_per_epoch, n, M)).astype(np.int32)
            # the step size of an iteration is that of the first of its n gradient evaluations
            g = step_sizes.step_decay(events_per_epoch, events_per_epoch, gamma, 0.5, halve_every,
                                      k_begin=e * events_per_epoch)[::n][:iters_per_epoch]
            eng.run_sync_steps(iters_per_epoch, batch, gamma=g)
            curve.append(eng.objective())
            errs.append(eng.classification_error())
            spread = max(spread, eng.consensus_distance())
        curves[name] = {"objective": curve, "error": errs, "max_consensus_distance": spread}
        eng.close()
    eng = engine(ring(n))
    curve, errs, spread = [eng.objective()], [eng.classification_error()], [0.0]
    sched = adpsgd_make_schedule(ring(n), epochs * events_per_epoch, seed=seed, T_max=T_max, M=M, rows=[rows] * n)
    sched["gamma"] = step_sizes.step_decay(epochs * events_per_epoch, events_per_epoch, gamma, 0.5, halve_every)

    def after_epoch(_events):
        curve.append(eng.objective())
        errs.append(eng.classification_error())
        spread[0] = max(spread[0], eng.consensus_distance())

    # one schedule for the whole run, executed an epoch per call; the calls look ahead, so the result is that of one call
    eng.run_events_in_pieces(sched, events_per_epoch, between=after_epoch)
    curves["ad-psgd"] = {"objective": curve, "error": errs, "max_consensus_distance": spread[0]}
    eng.close()
    return {"n": n, "dims": list(dims), "rows": rows, "M": M, "epochs": epochs, "T_max": T_max, "gamma": gamma,
            "halve_every": halve_every, "momentum": momentum, "weight_decay": weight_decay,
            "events_per_epoch": events_per_epoch, "curves": curves}


def format_table(res):
    names = list(res["curves"])
    lines = ["epoch | " + " | ".join("%20s" % (m + " loss / error") for m in names), "-" * (8 + 23 * len(names))]
    for e in range(res["epochs"] + 1):
        lines.append("%5d | " % e + " | ".join("%11.5f / %6.4f" % (res["curves"][m]["objective"][e], res["curves"][m]["error"][e])
                                             for m in names))
    lines.append("max consensus distance: " + ", ".join("%s %.3g" % (m, res["curves"][m]["max_consensus_distance"]) for m in names))
    return "\n".join(lines)


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--n", type=int, default=16)
    ap.add_argument("--rows", type=int, default=2048)
    ap.add_argument("--M", type=int, default=32)
    ap.add_argument("--epochs", type=int, default=12)
    ap.add_argument("--T-max", type=int, default=4)
    ap.add_argument("--gamma", type=float, default=0.02)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--json", action="store_true", help="print the results as one JSON object")
    a = ap.parse_args(argv)
    res = run_study(a.n, rows=a.rows, M=a.M, epochs=a.epochs, T_max=a.T_max, gamma=a.gamma, seed=a.seed)
    print(json.dumps(res) if a.json else format_table(res))


if __name__ == "__main__":
    main()
