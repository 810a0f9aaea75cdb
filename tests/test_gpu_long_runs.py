"""GPU parity along long runs of the data configurations (2, 4 and 5) at their full n, d, M, step size and
staleness law, in two ways.

1. ALL events of each configuration (20 000, 20 000 and 50 000) against models of the serial oracle that were
   written beforehand by tests/golden/make_long_run_references.py (a script that calls only the oracle and the
   seeded generators: replaying these runs takes the oracle 3.5, 15 and 40 minutes of one core, too long for this
   suite).  The run is cut into four self-contained calls (as bench.py's steps are); after every call the GPU's
   models are compared with the stored ones: at 1024 sampled coordinates of every worker under the parity measure
   (max error over the worker's max |x|), and over all coordinates through max |x|, the Euclidean norm and the
   sum.  The test regenerates the same host data from the same seeds.
2. A prefix of each run against the oracle replayed live (one thread per configuration, side by side), with the
   data generated in GPU memory: the error is checked at four points, so that "the error does not grow with the
   length of a run" is tested and not only observed.

Local data sets are cut down where the oracle's host copy would not fit a test (the rows a minibatch samples do
not change what an event computes): configuration 2 keeps 256 of 4096 rows per worker, configuration 5 keeps 16
of 64; the perceptron keeps all 8192.  Configuration 3 is covered over all its 100 000 events on sampled
coordinates in test_gpu_parity.py.
"""
import importlib.util
import os
import queue
import threading
import time

import numpy as np
import pytest

import oracle
from workloads import get_config, random_regular4_graph, ring_graph

pytestmark = pytest.mark.gpu

TOL = 1e-5                # fp32 models, the task's bound
MLP_TOL_BF16 = 2e-2       # bf16 weights of the perceptron, the task's bound
# The perceptron's fp32 master cannot be held to the fp32 bound: a hidden activation whose fp32 (GPU) and fp64
# (oracle) sums fall on different sides of a bf16 rounding boundary moves by 2^-8 relative.  Same bound as in the
# other perceptron tests; measured at this shape on MI355X: 0.9e-5 ... 1.2e-5 at all checkpoints.
MLP_TOL_MASTER = 2e-3
CHECKPOINTS = 4
LIVE_RUNS = {2: dict(K=4000, rows=256), 4: dict(K=1200, rows=8192), 5: dict(K=1200, rows=16)}

_GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _references_module():
    spec = importlib.util.spec_from_file_location("make_long_run_references", os.path.join(_GOLDEN, "make_long_run_references.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def rel_err(x_gpu, x_ref):
    num = np.max(np.abs(x_gpu.astype(np.float64) - x_ref.astype(np.float64)), axis=1)
    den = np.maximum(np.max(np.abs(x_ref.astype(np.float64)), axis=1), 1e-30)
    return float(np.max(num / den))


@pytest.fixture(scope="module")
def P():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1710_06952_amd as pkg
    pkg.lib()
    return pkg


# ------------------------------------------------------------------ 1. all events, against stored oracle models
@pytest.fixture(scope="module")
def host_workloads():
    """The three host workloads are generated side by side while the first tests run (numpy's generators release
    the interpreter lock): {idx: (thread, box)}, box["value"] = (c, g, feats, targs, x0, calls, coords)."""
    mod = _references_module()
    started = {}
    for idx in (4, 2, 5):
        box = {}

        def work(idx=idx, box=box):
            try:
                box["value"] = mod.workload(idx)
            except BaseException as e:      # reported by the waiting test
                box["error"] = repr(e)

        th = threading.Thread(target=work, daemon=True)
        th.start()
        started[idx] = (th, box)
    return started


@pytest.mark.parametrize("idx", [4, 2, 5])
def test_all_events_against_stored_oracle_models(P, host_workloads, idx, capsys):
    from workloads import bf16_bits_to_f32
    ref = np.load(os.path.join(_GOLDEN, "long_run_cfg%d.npz" % idx), allow_pickle=False)
    th, box = host_workloads[idx]
    th.join()
    assert "error" not in box, box.get("error")
    c, g, feats, targs, x0, calls, coords = box.pop("value")
    assert np.array_equal(coords, ref["coords"]) and len(calls) == CHECKPOINTS
    assert int(ref["events_per_call"]) * CHECKPOINTS == c["K"]             # the whole run
    n, d, M = c["n"], c["d"], c["M"]
    mlp = c["model"] == "mlp"
    skw = _references_module().schedule_kwargs(c, int(ref["rows"]))
    eng = P.Engine(g, d, c["model"], M=M, gamma=c["gamma"], lam=c["lam"], T_max=c["T_max"], **(dict(mlp=c["mlp"]) if mlp else {}))
    eng.load_data(feats, targs)
    del feats, targs
    eng.set_models(x0)
    for q, sched in enumerate(calls):
        per_call = len(sched["worker"])
        lib_sched = P.adpsgd_make_schedule(g, per_call, k_begin=q * per_call, **skw)
        assert all(np.array_equal(sched[k], lib_sched[k]) for k in sched)
        eng.run_events(lib_sched, want_loss=True)
        X, loss = eng.get_models(), eng.get_loss()
        amax = ref["amax%d" % q].astype(np.float64)
        sampled = np.max(np.abs(X[:, coords].astype(np.float64) - ref["x%d" % q]), axis=1) / amax
        X64 = X.astype(np.float64)
        e_amax = np.max(np.abs(np.max(np.abs(X64), axis=1) - amax) / amax)
        e_l2 = np.max(np.abs(np.sqrt((X64 * X64).sum(axis=1)) - ref["l2_%d" % q]) / ref["l2_%d" % q])
        e_sum = np.max(np.abs(X64.sum(axis=1) - ref["s%d" % q]) / (amax * d))
        del X64
        line = ("configuration %d after %6d events (stored oracle models): sampled coordinates %.3e, max|x| %.1e, norm %.1e, "
                "sum %.1e" % (idx, (q + 1) * per_call, sampled.max(), e_amax, e_l2, e_sum))
        tol = MLP_TOL_MASTER if mlp else TOL
        assert sampled.max() <= tol and e_amax <= tol and e_l2 <= tol and e_sum <= tol, line
        want = float(ref["loss_tail%d" % q])
        assert abs(float(loss[-200:].mean()) - want) <= (5e-2 if mlp else 2e-4) * abs(want) + 1e-6, line
        if mlp:
            Xb = bf16_bits_to_f32(eng.get_bf16_models())
            eb = np.max(np.max(np.abs(Xb[:, coords].astype(np.float64) - oracle.round_bf16(ref["x%d" % q])), axis=1) / amax)
            line += ", bf16 weights %.3e" % eb
            assert eb <= MLP_TOL_BF16, line
        with capsys.disabled():
            print("\n" + line, flush=True)
    eng.close()


# ------------------------------------------------------------------ 2. a prefix, against the oracle replayed live
def _gpu_run(P, idx):
    """The GPU side of one configuration: returns what the oracle thread needs (host data, the calls' schedules,
    the initial model) and the GPU's models / bf16 weights / losses after every call."""
    import torch
    from workloads import linear_data_on_device, mixture_data_on_device, mlp_init
    c, K, rows = get_config(idx), LIVE_RUNS[idx]["K"], LIVE_RUNS[idx]["rows"]
    n, d, M = c["n"], c["d"], c["M"]
    g = ring_graph(n) if c["graph"] == "ring" else random_regular4_graph(n, c["seed"])
    kw = {}
    if c["model"] == "mlp":
        feats, targs = mixture_data_on_device(n, rows, din=c["mlp"][0], classes=c["mlp"][2], seed=c["seed"])
        x0, kw = mlp_init(*c["mlp"], seed=c["seed"]), dict(mlp=c["mlp"])
    else:
        feats, targs = linear_data_on_device(c["model"], n, rows, d, seed=c["seed"])
        x0 = np.zeros(d, np.float32)
    eng = P.Engine(g, d, c["model"], M=M, gamma=c["gamma"], lam=c["lam"], T_max=c["T_max"], **kw)
    eng.load_data(feats, targs)
    eng.set_models(x0)
    per_call = K // CHECKPOINTS
    skw = _references_module().schedule_kwargs(c, rows)
    calls, gpu = [], []
    for q in range(CHECKPOINTS):
        sched = P.adpsgd_make_schedule(g, per_call, k_begin=q * per_call, **skw)
        ref = oracle.make_schedule(g, per_call, k_begin=q * per_call, **skw)
        assert all(np.array_equal(sched[k], ref[k]) for k in ref)
        eng.run_events(sched, want_loss=True)
        gpu.append(dict(X=eng.get_models(), loss=eng.get_loss(), Xb=eng.get_bf16_models() if c["model"] == "mlp" else None))
        calls.append(ref)
    eng.close()
    if c["model"] == "mlp":
        din = c["mlp"][0]
        hf = [np.ascontiguousarray(f[:, :din].contiguous().view(torch.int16).cpu().numpy().view(np.uint16)) for f in feats]
    else:
        hf = [f.cpu().numpy() for f in feats]
    ht = [t.cpu().numpy() for t in targs]
    del feats, targs, eng
    torch.cuda.empty_cache()
    return dict(cfg=c, x0=x0, feats=hf, targs=ht, calls=calls, gpu=gpu)


def _oracle_replay(run, out):
    """Thread body: the oracle's chain of calls from the initial model; one message per checkpoint."""
    try:
        c = run["cfg"]
        model = {"lsq": oracle.MODEL_LSQ, "logreg": oracle.MODEL_LOGREG, "mlp": oracle.MODEL_MLP}[c["model"]]
        Xr = np.tile(run["x0"], (c["n"], 1))
        for q, sched in enumerate(run["calls"]):
            t0 = time.time()
            r = oracle.run_events(Xr, sched, model, c["gamma"], M=c["M"], gscale=1.0 / c["M"], lam=c["lam"],
                                  mlp=c.get("mlp", (0, 0, 0)), features=run["feats"], targets=run["targs"], mode=1,
                                  want_loss=True)
            out.put(("checkpoint", q, Xr.copy(), r["loss"], time.time() - t0))
        out.put(("done",))
    except BaseException as e:          # reported by the waiting test
        out.put(("error", repr(e)))


@pytest.fixture(scope="module")
def replays(P):
    started = {}
    for idx in sorted(LIVE_RUNS):
        print("long run, configuration %d: %d events on the GPU" % (idx, LIVE_RUNS[idx]["K"]), flush=True)
        run = _gpu_run(P, idx)
        q = queue.Queue()
        th = threading.Thread(target=_oracle_replay, args=(run, q), daemon=True)
        th.start()
        started[idx] = (run, q, th)
    return started


@pytest.mark.parametrize("idx", sorted(LIVE_RUNS))
def test_error_along_a_run_against_the_live_oracle(replays, idx, capsys):
    from workloads import bf16_bits_to_f32
    run, q, th = replays[idx]
    c, per_call = run["cfg"], LIVE_RUNS[idx]["K"] // CHECKPOINTS
    errs = []
    while True:
        msg = q.get(timeout=900)
        if msg[0] == "error":
            pytest.fail("oracle replay of configuration %d failed: %s" % (idx, msg[1]))
        if msg[0] == "done":
            break
        _, at, Xr, loss_r, secs = msg
        g = run["gpu"][at]
        e = rel_err(g["X"], Xr)
        line = "configuration %d after %6d events: max rel err %.3e (oracle %.0f s)" % (idx, (at + 1) * per_call, e, secs)
        if c["model"] == "mlp":
            eb = rel_err(bf16_bits_to_f32(g["Xb"]), oracle.round_bf16(Xr))
            line += ", bf16 weights %.3e" % eb
            assert eb <= MLP_TOL_BF16 and e <= MLP_TOL_MASTER, line
            assert np.allclose(g["loss"], loss_r, rtol=5e-2, atol=5e-3), line
        else:
            assert e <= TOL, line
            assert np.allclose(g["loss"], loss_r, rtol=2e-4, atol=1e-6), line
        with capsys.disabled():
            print("\n" + line, flush=True)
        errs.append(e)
        run["gpu"][at] = None               # free the checkpoint
    th.join()
    assert len(errs) == CHECKPOINTS
    if c["model"] != "mlp":
        # no growth along the run: the last checkpoint is no worse than a few times the first
        assert errs[-1] <= max(4 * errs[0], TOL / 4), errs
