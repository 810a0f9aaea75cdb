"""The entry point that allocates nothing (adpsgd_consensus_distance_static: block partials and weights in a fixed
device array of the library) against the entry point it is a variant of, through the C ABI."""
import numpy as np
import pytest

import oracle
from workloads import ring_graph

pytestmark = pytest.mark.gpu


def test_static_consensus_distance_equals_the_allocating_entry_point():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1710_06952_amd as P
    P.lib()
    out = torch.full((2,), -1.0, dtype=torch.float64, device="cuda:0")
    # two calls in a row on the shared array, the second on a smaller input (fewer partials, fewer weights);
    # then the first size again
    for n, d, seed in ((24, 700001, 1), (6, 1500, 2), (24, 700001, 3)):
        print("static consensus distance n=%d d=%d" % (n, d), flush=True)
        g = ring_graph(n)
        eng = P.Engine(g, d, "synth", gamma=0.1, T_max=2, synth_std=0.05, synth_seed=seed)
        eng.set_models(np.random.default_rng(seed).standard_normal((n, d)).astype(np.float32), broadcast=False)
        eng.run_events(oracle.make_schedule(g, 40, seed=seed, T_max=2))
        p = np.random.default_rng(seed + 10).random(n)
        p /= p.sum()
        ref_u, ref_w = eng.consensus_distance(), eng.consensus_distance(p)
        out.fill_(-1.0)
        eng.h.consensus_distance_static(out.data_ptr())
        eng.h.consensus_distance_static(out.data_ptr() + 8, p)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        assert got[0] == ref_u and got[1] == ref_w                  # the same kernels on the same grid: the same bits
        X = eng.get_models()
        assert np.isclose(got[0], oracle.consensus_distance(X), rtol=1e-9)
        assert np.isclose(got[1], oracle.consensus_distance_weighted(X, p), rtol=1e-9)
        # invalid weights are refused and nothing is written
        out.fill_(-1.0)
        with pytest.raises(P.AdpsgdError) as ei:
            eng.h.consensus_distance_static(out.data_ptr(), np.full(n, 2.0 / n))
        assert ei.value.code == -1
        torch.cuda.synchronize()
        assert float(out[0].item()) == -1.0
        eng.close()


def test_static_consensus_distance_rejects_more_workers_than_its_weights_hold():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1710_06952_amd as P
    n, d = 4100, 8
    g = ring_graph(n)
    eng = P.Engine(g, d, "synth", gamma=0.1, synth_std=0.05)
    eng.set_models(np.random.default_rng(0).standard_normal((n, d)).astype(np.float32), broadcast=False)
    out = torch.zeros(1, dtype=torch.float64, device="cuda:0")
    with pytest.raises(P.AdpsgdError) as ei:
        eng.h.consensus_distance_static(out.data_ptr(), np.full(n, 1.0 / n))
    assert ei.value.code == -1 and "4096" in str(ei.value)
    eng.h.consensus_distance_static(out.data_ptr())                  # without weights any n fits
    torch.cuda.synchronize()
    assert float(out[0].item()) == eng.consensus_distance()
    eng.close()
