"""The slow-worker study: its schedule builder (CPU) and one tiny end-to-end run (GPU)."""
import numpy as np
import pytest

import oracle
import paper_1710_06952_amd as P
from paper_1710_06952_amd.studies import heterogeneity as H


def test_clock_schedule_staleness_counts_the_events_since_the_workers_last_read():
    n, K = 6, 500
    g = H.ring(n)
    mean = np.ones(n)
    mean[2] = 10.0
    s, when = H.clock_schedule(g, K, mean, M=3, rows=20, seed=1)
    assert np.all(np.diff(when) >= 0)
    last = {}
    for k in range(K):
        i = s["worker"][k]
        assert s["tau"][k] == k - (last[i] + 1 if i in last else 0)
        assert s["neighbour"][k] in ((i - 1) % n, (i + 1) % n)
        last[i] = k
    share = np.bincount(s["worker"], minlength=n) / K
    assert share[2] < 0.05 and share[0] > 0.12          # the slow worker updates about ten times less often
    assert s["batch_idx"].shape == (K, 3) and s["batch_idx"].min() >= 0 and s["batch_idx"].max() < 20
    # the library's planner accepts it, and the oracle runs it
    r_round, u_round, slot, R = P.adpsgd_plan_rounds(n, s["worker"], s["neighbour"], s["tau"], int(s["tau"].max()) + 1)
    assert R <= K and (r_round <= u_round).all()


def test_deterministic_equal_clocks_give_round_robin_with_staleness_n_minus_1():
    n, K = 5, 60
    s, when = H.clock_schedule(H.ring(n), K, np.ones(n), M=1, rows=4, seed=0, exponential=False)
    assert np.array_equal(s["worker"], np.arange(K) % n)
    assert np.array_equal(s["tau"][n:], np.full(K - n, n - 1))
    assert np.allclose(when, 1 + np.arange(K) // n)
    assert np.allclose(H.sync_clock(7, [1, 1, 3, 1], 0, exponential=False), 3 * np.arange(1, 8))


def test_slow_link_delays_only_the_events_that_use_it():
    n, K = 6, 600
    g = H.ring(n)
    s, when = H.clock_schedule(g, K, np.ones(n), M=1, rows=4, seed=3, exponential=False, comm_time=0.5,
                               slow_link=(2, 3), link_slowdown=20.0)
    assert np.all(np.diff(when) >= 0)
    prev = {}
    for k in range(K):
        i, j = int(s["worker"][k]), int(s["neighbour"][k])
        took = when[k] - prev.get(i, 0.0)
        assert np.isclose(took, 1.0 + (10.0 if {i, j} == {2, 3} else 0.5))
        prev[i] = when[k]
    share = np.bincount(s["worker"], minlength=n) / K
    assert share[2] < share[0] and share[3] < share[5]          # the two ends of the slow link update less often
    # a synchronous iteration waits for the slow link every time
    assert np.allclose(H.sync_clock(5, np.ones(n), 0, exponential=False, comm_time=0.5, link_slowdown=20.0), 11.0 * np.arange(1, 6))


def test_objective_and_smoothing_helpers():
    feats, targs = H.make_problem(3, 16, 8, seed=2, noise=0.0)
    assert all(f is feats[0] for f in feats) and len(feats) == 3          # shared data
    xstar = np.linalg.lstsq(feats[0].astype(np.float64), targs[0].astype(np.float64), rcond=None)[0]
    assert H.objective(xstar, feats, targs) < 1e-12 < H.objective(np.zeros(16), feats, targs)
    assert np.allclose(H.smooth([1, 3, 5, 7], 2), [1, 2, 4, 6])
    assert H.first_time_below(np.array([3.0, 2.0, 1.0]), np.array([10.0, 20.0, 30.0]), 2.0) == 20.0
    assert H.first_time_below(np.array([3.0]), np.array([1.0]), 2.0) == float("inf")


@pytest.mark.gpu
def test_study_runs_end_to_end_on_a_tiny_problem():
    res = H.run_study(n=4, d=256, rows=64, M=4, epochs=12, slowdowns=(1, 10), seed=0, target=0.1)
    assert [r["slowdown"] for r in res["results"]] == [1, 10]
    fast, slow = res["results"]
    for r in res["results"]:
        assert r["adpsgd_final_objective"] < 0.2 * res["initial_objective"]
        assert r["sync_final_objective"] < 0.2 * res["initial_objective"]
    # without a straggler both use the four workers; with one the synchronous schedule waits for it
    assert fast["adpsgd_speedup"] > 2.5 and fast["sync_speedup"] > 1.5
    assert slow["adpsgd_speedup"] > 2.5 > 1.0 > slow["sync_speedup"]
    assert slow["adpsgd_time_to_target"] < slow["sync_time_to_target"]
    assert "slowdown" in H.format_table(res)
    # the library's objective agrees with the plain numpy evaluation of the same problem
    feats, targs = H.make_problem(4, 256, 64, 0)
    eng = P.Engine(H.ring(4), 256, "lsq", M=4, gamma=0.1)
    eng.load_data(feats, targs)
    eng.set_models(np.zeros(256, np.float32))
    assert np.isclose(eng.objective(), H.objective(np.zeros(256), feats, targs), rtol=1e-5)
    assert np.isclose(eng.objective(), res["initial_objective"], rtol=1e-5)
    eng.close()
    link = H.run_study(n=4, d=256, rows=64, M=4, epochs=6, slowdowns=(1, 50), seed=0, target=0.1, slow="link")
    a, b = link["results"]
    assert b["sync_speedup"] < 0.2 * a["sync_speedup"]          # every synchronous iteration waits for the link
    assert b["adpsgd_speedup"] > 0.25 * a["adpsgd_speedup"]     # AD-PSGD only loses the exchanges that use it


def _rel_err(x_gpu, x_ref):
    num = np.max(np.abs(x_gpu.astype(np.float64) - x_ref.astype(np.float64)), axis=1)
    den = np.maximum(np.max(np.abs(x_ref.astype(np.float64)), axis=1), 1e-30)
    return float(np.max(num / den))


@pytest.mark.gpu
@pytest.mark.parametrize("exponential", [True, False])
def test_clock_derived_schedules_match_the_oracle(exponential):
    """The study's two schedules for one worker slowed down ten times (Sec. 5.4, robustness against slow
    computation): the events of free-running workers with the staleness their clocks imply, and the synchronous
    iterations beside them, each executed by the HIP library and by the serial oracle on the same data, final
    models and per-event losses compared at the fp32 parity bound."""
    n, d, rows, M, epochs, seed = 16, 2051, 96, 4, 30, 3
    graph = H.ring(n)
    feats, targs = H.make_problem(n, d, rows, seed)
    gamma = 0.5 * M
    K = epochs * (rows // M)
    mean_time = np.ones(n)
    mean_time[n // 2] = 10.0
    sched, when = H.clock_schedule(graph, K, mean_time, M, rows, seed, exponential)
    T_max = int(sched["tau"].max())
    share = np.bincount(sched["worker"], minlength=n) / K
    assert share[n // 2] < 0.3 * share[0] and T_max >= n - 1        # the slow worker is rare and the reads are stale
    print("clock schedule (%s): K=%d, T_max=%d" % ("exp" if exponential else "det", K, T_max), flush=True)
    eng = P.Engine(graph, d, "lsq", M=M, gamma=gamma, T_max=T_max, n_slots=T_max + 1 + 2 * n)
    eng.load_data(feats, targs)
    eng.set_models(np.zeros(d, np.float32))
    eng.run_events(sched, want_loss=True)
    Xg, lg = eng.get_models(), eng.get_loss()
    eng.close()
    Xr = np.zeros((n, d), np.float32)
    r = oracle.run_events(Xr, sched, oracle.MODEL_LSQ, gamma, M=M, gscale=1.0 / M, features=feats, targets=targs,
                          want_loss=True)
    assert _rel_err(Xg, Xr) <= 1e-5
    assert np.allclose(lg, r["loss"], rtol=2e-4, atol=1e-7)
    Xf = np.zeros((n, d), np.float32)                               # the same events with fresh reads differ
    oracle.run_events(Xf, dict(sched, tau=np.zeros(K, np.int32)), oracle.MODEL_LSQ, gamma, M=M, gscale=1.0 / M,
                      features=feats, targets=targs)
    assert _rel_err(Xf, Xr) > 1e-3

    S = K // n
    batch = np.random.default_rng([seed, 4]).integers(0, rows, size=(S, n, M)).astype(np.int32)
    eng = P.Engine(graph, d, "lsq", M=M, gamma=gamma, n_slots=n)
    eng.load_data(feats, targs)
    eng.set_models(np.zeros(d, np.float32))
    eng.run_sync_steps(S, batch, want_loss=True)
    Xg, lg = eng.get_models(), eng.get_loss().reshape(S, n)
    eng.close()
    Xr = np.zeros((n, d), np.float32)
    r = oracle.run_sync_steps(Xr, batch, oracle.metropolis_weights(graph), oracle.MODEL_LSQ, gamma, M=M, gscale=1.0 / M,
                              features=feats, targets=targs, want_loss=True)
    assert _rel_err(Xg, Xr) <= 1e-5
    assert np.allclose(lg, r["loss"], rtol=2e-4, atol=1e-7)
