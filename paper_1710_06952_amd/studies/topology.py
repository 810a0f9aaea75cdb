"""Consensus rate against topology: the paper's remark (Sec. 3.3) that adding links to the ring makes
the spectral quantity rho of the theory section smaller and the scalability better, shown numerically.

For pairwise gossip averaging W_k is a symmetric projection, so rho = lambda_2(E[W_k^T W_k]) =
lambda_2(E W_k) with  E W = I - (1/n) sum_i (1/deg i) sum_{j in N(i)} (e_i - e_j)(e_i - e_j)^T / 2.
The consensus lemma bounds the EXPECTED squared distance to the mean by rho^K times its initial value; here
the library runs K pure gossip events (synthetic gradients of standard deviation 0) on a random
initial X with many independent columns and reports the measured contraction next to that bound.  One
sequence of events typically contracts faster than the expectation (the logarithm of a product of
random contractions concentrates below the logarithm of its mean), so the measured distance sits
below rho^K; the ordering of the topologies is the paper's point.  K is shortened for fast topologies
so that the distance stays well above the rounding floor.

    python -m paper_1710_06952_amd.studies.topology [--n 32] [--d 65536] [--events 2000]
"""
from __future__ import annotations

import argparse
import json

import numpy as np


def ring(n):
    return (np.arange(0, 2 * n + 1, 2, dtype=np.int32),
            np.array([v for i in range(n) for v in ((i - 1) % n, (i + 1) % n)], dtype=np.int32))


def hop_ring(n):
    """Ring plus links at distance 2^i + 1, i = 0 .. floor(log2(n - 1))."""
    hops = {1}
    i = 0
    while (1 << i) <= n - 1:
        hops.add(((1 << i) + 1) % n)
        i += 1
    hops.discard(0)
    nb = [sorted({(v + h) % n for h in hops} | {(v - h) % n for h in hops} - {v}) for v in range(n)]
    rowptr = np.cumsum([0] + [len(x) for x in nb]).astype(np.int32)
    return rowptr, np.array([j for x in nb for j in x], dtype=np.int32)


def complete(n):
    nb = [[j for j in range(n) if j != i] for i in range(n)]
    rowptr = np.cumsum([0] + [len(x) for x in nb]).astype(np.int32)
    return rowptr, np.array([j for x in nb for j in x], dtype=np.int32)


def expected_W(graph):
    rowptr, col = graph
    n = len(rowptr) - 1
    EW = np.eye(n)
    for i in range(n):
        deg = rowptr[i + 1] - rowptr[i]
        for e in range(rowptr[i], rowptr[i + 1]):
            j = col[e]
            v = np.zeros(n)
            v[i], v[j] = 1.0, -1.0
            EW -= np.outer(v, v) / (2.0 * n * deg)
    return EW


def rho(graph):
    return float(np.sort(np.linalg.eigvalsh(expected_W(graph)))[-2])


def measure(graph, d, events, seed=0, device="cuda:0"):
    """Consensus distance before and after `events` pure gossip events, run by the library."""
    from .. import Engine, adpsgd_make_schedule
    n = len(graph[0]) - 1
    eng = Engine(graph, d, "synth", gamma=0.0, synth_std=0.0, device=device)
    x0 = np.random.default_rng(seed).standard_normal((n, d)).astype(np.float32)
    eng.set_models(x0, broadcast=False)
    c0 = eng.consensus_distance()
    half = events // 2
    eng.run_events(adpsgd_make_schedule(graph, half, seed=seed, k_begin=0))
    c1 = eng.consensus_distance()
    eng.run_events(adpsgd_make_schedule(graph, events - half, seed=seed, k_begin=half))
    c2 = eng.consensus_distance()
    mean_moved = float(np.abs(eng.get_mean_model() - x0.astype(np.float64).mean(0)).max())
    eng.close()
    return {"initial": c0, "after_half": c1, "after_all": c2,
            "rate_per_event": float((c2 / c1) ** (1.0 / (events - half))), "mean_moved": mean_moved}


def run_study(n=32, d=65536, events=2000, seed=0, device="cuda:0"):
    out = []
    for name, g in (("ring", ring(n)), ("ring + 2^i+1 hops", hop_ring(n)), ("complete", complete(n))):
        r = rho(g)
        k = int(min(events, max(2, np.ceil(np.log(1e-4) / np.log(r)))))      # rho^K >= 1e-4
        m = measure(g, d, k, seed, device)
        out.append({"topology": name, "degree": int(g[0][1] - g[0][0]), "rho": r, "events": k, "bound": r ** k, **m})
    return {"n": n, "d": d, "events": events, "results": out}


def format_table(res):
    lines = ["topology             degree        rho   events K   measured rate/event   distance ratio after K   bound rho^K",
             "-" * 113]
    for r in res["results"]:
        lines.append("%-20s %6d   %.6f   %8d   %19.6f   %23.3e   %11.3e" % (
            r["topology"], r["degree"], r["rho"], r["events"], r["rate_per_event"], r["after_all"] / r["initial"], r["bound"]))
    return "\n".join(lines)


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--n", type=int, default=32)
    ap.add_argument("--d", type=int, default=65536)
    ap.add_argument("--events", type=int, default=2000)
    ap.add_argument("--json", action="store_true")
    a = ap.parse_args(argv)
    res = run_study(a.n, a.d, a.events)
    print(json.dumps(res) if a.json else format_table(res))


if __name__ == "__main__":
    main()
