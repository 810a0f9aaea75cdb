"""The convergence study: its inputs (CPU) and the shape of its result (GPU)."""
import numpy as np
import pytest

import paper_1710_06952_amd as P
from paper_1710_06952_amd.studies import convergence as C
from workloads import graph_is_valid, ring_graph


def test_graphs_and_problem():
    for n in (3, 8, 16):
        assert graph_is_valid(*C.complete(n))
        r = C.ring(n)
        assert np.array_equal(r[0], ring_graph(n)[0]) and np.array_equal(r[1], ring_graph(n)[1])
        ws, we = P.adpsgd_metropolis_weights(C.complete(n))          # complete graph: plain averaging over all workers
        assert np.allclose(ws, 1.0 / n) and np.allclose(we, 1.0 / n)
    feats, labels, x0 = C.make_problem(4, 100, (16, 64, 5), seed=1)
    assert len(feats) == 4 and feats[0].shape == (100, 16) and labels[0].dtype == np.int32
    assert x0.shape == (16 * 64 + 64 + 64 * 5 + 5,) and not np.array_equal(feats[0], feats[1])
    assert set(np.unique(np.concatenate(labels))) <= set(range(5))


@pytest.mark.gpu
def test_the_three_schedules_converge_alike_per_epoch():
    res = C.run_study(n=8, dims=(32, 128, 6), rows=1024, M=32, epochs=6, T_max=3, gamma=0.02, halve_every=3, seed=2)
    curves = {k: np.array(v["objective"]) for k, v in res["curves"].items()}
    assert set(curves) == {"complete", "d-psgd", "ad-psgd"}
    start = curves["complete"][0]
    for name, c in curves.items():
        assert c[0] == start and np.isfinite(c).all()
        assert c[-1] < 0.5 * start, (name, c)
    for v in res["curves"].values():
        assert v["error"][-1] < 0.5 * v["error"][0] and 0 <= v["error"][-1] < 0.5
    finals = np.array([c[-1] for c in curves.values()])
    assert finals.max() <= 1.3 * finals.min(), curves                  # about the same loss after the same epochs
    spread = {k: v["max_consensus_distance"] for k, v in res["curves"].items()}
    assert 0 < spread["complete"] < spread["d-psgd"] and spread["ad-psgd"] > 0    # full averaging keeps the workers closest
    assert "epoch" in C.format_table(res)
