"""Simulated wall-clock study of a slow worker, shaped like the paper's robustness experiment
(Sec. 5.4, "Robustness against slow computation": one of 16 workers slowed down 2x-100x, table of
time per epoch and speed-up for AD-PSGD against the synchronous algorithms; with --slow link the
companion experiment, "Robustness against slow communication", where one network link is slowed).

Nothing here needs the paper's data: the objective is a synthetic consistent least-squares problem
whose samples every worker can draw (the shared-data strategy of the remark in Sec. 3.1, as in the
paper's experiment, so that a slow worker changes staleness and update frequency but not the
objective), every worker's gradient time is drawn from its own clock (mean 1, the slow worker's mean = the
slowdown), and the time axis is simulated:

  AD-PSGD      every worker loops on its own; an event happens when a worker's clock fires.  The
               staleness of event k is the number of events since that worker last read its model,
               tau_k = k - (index of its previous event) - 1, which is what Algorithm 1's
               x^_k = X_{k - tau_k} means for a worker that reads, computes, then updates.
  synchronous  (D-PSGD) an iteration ends when the slowest worker is done: its duration is the
               maximum of the n clocks.

Both schedules are executed by the HIP library (adpsgd_run_events / adpsgd_run_sync_steps); this file
only builds schedules and keeps the simulated clock; the objective at the mean model comes from the
library too (adpsgd_objective).

    python -m paper_1710_06952_amd.studies.heterogeneity [--n 16] [--d 4096] [--epochs 40]
"""
from __future__ import annotations

import argparse
import json

import numpy as np


def ring(n):
    rowptr = np.arange(0, 2 * n + 1, 2, dtype=np.int32) if n > 2 else np.arange(0, n + 1, dtype=np.int32) * (n - 1)
    col = []
    for i in range(n):
        if n == 2:
            col += [1 - i]
        elif n > 2:
            col += [(i - 1) % n, (i + 1) % n]
    return rowptr, np.array(col, dtype=np.int32)


def make_problem(n, d, rows, seed, noise=0.01):
    """One data set for all workers: A (rows x d) with entries N(0, 1/d) (unit-norm rows),
    b = A x* + noise; returned as per-worker lists that all name the same arrays."""
    rng = np.random.default_rng([seed, 1])
    xstar = rng.standard_normal(d).astype(np.float32)
    A = (rng.standard_normal((rows, d)) / np.sqrt(d)).astype(np.float32)
    b = (A.astype(np.float64) @ xstar + noise * rng.standard_normal(rows)).astype(np.float32)
    return [A] * n, [b] * n


def objective(x, feats, targs):
    x = np.asarray(x, dtype=np.float64)
    return float(0.5 * np.mean((feats[0].astype(np.float64) @ x - targs[0]) ** 2))


def draw_durations(rng, mean, exponential):
    return rng.exponential(mean) if exponential else np.asarray(mean, dtype=np.float64).copy()


def clock_schedule(graph, K, mean_time, M, rows, seed, exponential=True, comm_time=0.0, slow_link=None, link_slowdown=1.0):
    """Event order of free-running workers.  Returns the schedule arrays and the simulated time of
    every event.  mean_time[i] = mean duration of one gradient on worker i; an event also takes
    comm_time for the exchange with its neighbour, times link_slowdown on the link slow_link = (a, b)."""
    rowptr, col = graph
    n = len(rowptr) - 1
    rng = np.random.default_rng([seed, 2])
    mean_time = np.asarray(mean_time, dtype=np.float64)

    def pick_neighbour(i):
        deg = rowptr[i + 1] - rowptr[i]
        return int(col[rowptr[i] + rng.integers(deg)]) if deg > 0 else i

    def exchange(i, j):
        slow = slow_link is not None and {i, j} == set(slow_link)
        return comm_time * (link_slowdown if slow else 1.0)

    nxt = np.array([pick_neighbour(i) for i in range(n)])            # partner of each worker's next event
    t_next = draw_durations(rng, mean_time, exponential) + np.array([exchange(i, nxt[i]) for i in range(n)])
    last_read = np.zeros(n, dtype=np.int64)        # logical time at which the worker last read its model
    worker = np.zeros(K, np.int32)
    nbr = np.zeros(K, np.int32)
    tau = np.zeros(K, np.int32)
    when = np.zeros(K, np.float64)
    for k in range(K):
        i = int(np.argmin(t_next))
        worker[k] = i
        nbr[k] = nxt[i]
        when[k] = t_next[i]
        tau[k] = k - last_read[i]
        last_read[i] = k + 1                        # it reads again right after its update
        nxt[i] = pick_neighbour(i)
        t_next[i] += (rng.exponential(mean_time[i]) if exponential else mean_time[i]) + exchange(i, nxt[i])
    batch = rng.integers(0, rows, size=(K, M)).astype(np.int32)
    return {"worker": worker, "neighbour": nbr, "tau": tau, "batch_idx": batch}, when


def sync_clock(S, mean_time, seed, exponential=True, comm_time=0.0, link_slowdown=1.0):
    """Simulated end time of every synchronous iteration: each lasts as long as its slowest worker
    plus its slowest exchange (every link is used in every iteration)."""
    rng = np.random.default_rng([seed, 3])
    mean_time = np.asarray(mean_time, dtype=np.float64)
    dur = np.array([draw_durations(rng, mean_time, exponential).max() for _ in range(S)]) + comm_time * max(link_slowdown, 1.0)
    return np.cumsum(dur)


def smooth(v, window):
    c = np.cumsum(np.insert(np.asarray(v, dtype=np.float64), 0, 0.0))
    out = np.empty(len(v))
    for k in range(len(v)):
        lo = max(0, k + 1 - window)
        out[k] = (c[k + 1] - c[lo]) / (k + 1 - lo)
    return out


def first_time_below(curve, when, target):
    hit = np.nonzero(curve <= target)[0]
    return float(when[hit[0]]) if hit.size else float("inf")


def run_study(n=16, d=4096, rows=1024, M=8, epochs=40, slowdowns=(1, 2, 10, 100), seed=0, exponential=True,
              target=0.2, device="cuda:0", slow="worker", comm_time=0.25):
    """slow = "worker": one worker's gradients take `slowdown` times longer (no exchange cost);
    slow = "link": gradients take unit time everywhere, an exchange takes comm_time, and the link between
    workers n/2 and n/2 + 1 is `slowdown` times slower."""
    from .. import Engine
    graph = ring(n)
    feats, targs = make_problem(n, d, rows, seed)
    gamma = 0.5 * M                                  # removes half of the minibatch residual per step
    grads_per_epoch = rows // M                      # gradient evaluations in one pass over the data
    K = epochs * grads_per_epoch
    S = K // n
    f0 = objective(np.zeros(d), feats, targs)
    rows_out = []
    for slowdown in slowdowns:
        mean_time = np.ones(n)
        link_kw = {}
        if slow == "worker":
            mean_time[n // 2] = float(slowdown)      # the slowed worker
        else:
            link_kw = dict(comm_time=comm_time, link_slowdown=float(slowdown))
        # ---- AD-PSGD
        sched, when = clock_schedule(graph, K, mean_time, M, rows, seed, exponential,
                                     slow_link=(n // 2, (n // 2 + 1) % n) if link_kw else None, **link_kw)
        T_max = int(sched["tau"].max())
        eng = Engine(graph, d, "lsq", M=M, gamma=gamma, T_max=T_max, n_slots=T_max + 1 + 2 * n, device=device)
        eng.load_data(feats, targs)
        eng.set_models(np.zeros(d, np.float32))
        eng.run_events(sched, want_loss=True)
        loss_a = smooth(eng.get_loss(), 4 * n)
        f_a = eng.objective()                        # at the mean model, over all data, on the GPU
        eng.close()
        # ---- synchronous iterations (all workers step together, mixing with both ring neighbours)
        when_s = sync_clock(S, mean_time, seed, exponential, **link_kw)
        batch = np.random.default_rng([seed, 4]).integers(0, rows, size=(S, n, M)).astype(np.int32)
        eng = Engine(graph, d, "lsq", M=M, gamma=gamma, n_slots=n, device=device)
        eng.load_data(feats, targs)
        eng.set_models(np.zeros(d, np.float32))
        eng.run_sync_steps(S, batch, want_loss=True)
        loss_s = smooth(eng.get_loss().reshape(S, n).mean(1), 4)
        f_s = eng.objective()
        eng.close()
        rows_out.append({
            "slowdown": slowdown,
            "adpsgd_time_per_epoch": float(when[-1] / epochs),
            "adpsgd_speedup": float(grads_per_epoch * epochs / when[-1]),       # against one worker of unit speed
            "sync_time_per_epoch": float(when_s[-1] / epochs),
            "sync_speedup": float(grads_per_epoch * epochs / when_s[-1]),
            "adpsgd_time_to_target": first_time_below(loss_a, when, target * f0),
            "sync_time_to_target": first_time_below(loss_s, when_s, target * f0),
            "adpsgd_final_objective": f_a,
            "sync_final_objective": f_s,
            "max_staleness": T_max,
        })
    return {"n": n, "d": d, "rows": rows, "M": M, "epochs": epochs, "gamma": gamma, "initial_objective": f0,
            "target_objective": target * f0, "clock": "exponential" if exponential else "deterministic", "slow": slow,
            "results": rows_out}


def format_table(res):
    lines = ["slowdown |  AD-PSGD time/epoch  speed-up  time-to-target |  sync time/epoch  speed-up  time-to-target | max tau",
             "-" * 112]
    for r in res["results"]:
        lines.append("%7dx | %19.2f %9.2f %15.1f | %16.2f %9.2f %15.1f | %7d" % (
            r["slowdown"], r["adpsgd_time_per_epoch"], r["adpsgd_speedup"], r["adpsgd_time_to_target"],
            r["sync_time_per_epoch"], r["sync_speedup"], r["sync_time_to_target"], r["max_staleness"]))
    return "\n".join(lines)


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--n", type=int, default=16)
    ap.add_argument("--d", type=int, default=4096)
    ap.add_argument("--rows", type=int, default=1024)
    ap.add_argument("--M", type=int, default=8)
    ap.add_argument("--epochs", type=int, default=40)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--deterministic-clocks", action="store_true")
    ap.add_argument("--slow", choices=["worker", "link"], default="worker", help="what is slowed down")
    ap.add_argument("--json", action="store_true", help="print the results as one JSON object")
    a = ap.parse_args(argv)
    res = run_study(a.n, a.d, a.rows, a.M, a.epochs, seed=a.seed, exponential=not a.deterministic_clocks, slow=a.slow)
    print(json.dumps(res) if a.json else format_table(res))


if __name__ == "__main__":
    main()
