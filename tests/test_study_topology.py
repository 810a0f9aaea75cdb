"""The topology study: spectral quantity rho of the theory section (CPU) and measured consensus rates (GPU)."""
import numpy as np
import pytest

from paper_1710_06952_amd.studies import topology as T
from workloads import hop_ring_graph, ring_graph


@pytest.mark.parametrize("n", [4, 8, 16, 33])
def test_rho_closed_forms(n):
    assert np.isclose(T.rho(T.ring(n)), 1 - (1 - np.cos(2 * np.pi / n)) / n, atol=1e-12)      # ring Laplacian spectrum
    assert np.isclose(T.rho(T.complete(n)), 1 - 1 / (n - 1), atol=1e-12)                       # E W = (1 - a) I + a 11^T / n
    EW = T.expected_W(T.hop_ring(n))
    assert np.allclose(EW, EW.T) and np.allclose(EW.sum(0), 1) and (EW >= -1e-15).all()       # doubly stochastic
    if n >= 8:
        assert T.rho(T.complete(n)) < T.rho(T.hop_ring(n)) < T.rho(T.ring(n)) < 1


def test_graphs_agree_with_the_shared_generators():
    for n in (8, 16, 32):
        for mine, ref in ((T.ring(n), ring_graph(n)), (T.hop_ring(n), hop_ring_graph(n))):
            assert np.array_equal(mine[0], ref[0]) and np.array_equal(mine[1], ref[1])


@pytest.mark.gpu
def test_measured_consensus_rate_follows_rho():
    res = T.run_study(n=16, d=8192, events=600, seed=1)
    rates = {r["topology"]: r for r in res["results"]}
    for r in res["results"]:
        assert r["mean_moved"] < 1e-5                      # averaging keeps the mean model
        assert r["after_all"] < r["after_half"] < r["initial"]
        # the lemma bounds the expectation; one sequence of events typically contracts faster, and
        # never by less than rho per event on average over a long run (slack 3 on the ratio)
        assert r["after_all"] / r["initial"] <= 3 * r["bound"], r
        assert r["rate_per_event"] < 1
    # the denser graphs mix far faster than the ring (their mutual order is within the scatter of one run)
    assert max(rates["complete"]["rate_per_event"], rates["ring + 2^i+1 hops"]["rate_per_event"]) < rates["ring"]["rate_per_event"] - 0.02
    assert "rho" in T.format_table(res)
