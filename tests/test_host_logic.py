"""CPU-side tests of the HIP library's host logic (no GPU needed): the shared
library loads and exports every declared symbol, its schedule generator agrees
bit for bit with the oracle's own, and the round planner keeps serial semantics.
"""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
import paper_1710_06952_amd as P
from paper_1710_06952_amd import binding as B
from workloads import get_config, hop_ring_graph, lsq_data, random_regular4_graph, ring_graph

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "adpsgd.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = sorted(set(re.findall(r"\b(adpsgd_[a-z0-9_]+)\s*\(", header)))
    assert len(declared) >= 14
    L = P.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert sorted(P.EXPORTS) == declared
    # the four calls the method is specified by
    for name in ("adpsgd_create", "adpsgd_load_data", "adpsgd_run_events", "adpsgd_get_models"):
        assert name in declared


def _graph_for(cfg):
    return {"ring": ring_graph, "hopring": hop_ring_graph}.get(cfg["graph"], lambda n: random_regular4_graph(n, cfg["seed"]))(cfg["n"])


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5])
def test_schedule_generators_agree_bit_for_bit(idx):
    cfg = get_config(idx)
    g = _graph_for(cfg)
    n, K = cfg["n"], min(cfg["K"], 5000)
    kw = dict(seed=cfg["seed"], T_max=cfg["T_max"], M=cfg["M"], rows=[max(cfg["rows"], 1)] * n)
    if cfg["tau_mode"] == "geometric":
        slow = np.arange(n) < cfg["n_slow"]
        kw.update(tau_mode=1, weight=np.where(slow, cfg["weight_slow"], cfg["weight_fast"]),
                  tau_num=np.where(slow, cfg["tau_slow"][0], cfg["tau_fast"][0]),
                  tau_den=np.where(slow, cfg["tau_slow"][1], cfg["tau_fast"][1]))
    for k_begin in (0, 123456789012):
        a = P.adpsgd_make_schedule(g, K, k_begin=k_begin, **kw)
        b = oracle.make_schedule(g, K, k_begin=k_begin, **kw)
        for key in ("worker", "neighbour", "tau"):
            assert np.array_equal(a[key], b[key]), key
        if cfg["M"] > 0:
            assert np.array_equal(a["batch_idx"], b["batch_idx"])


def test_schedule_generator_rejects_bad_arguments():
    g = ring_graph(4)
    with pytest.raises(P.AdpsgdError):
        P.adpsgd_make_schedule(g, 10, M=4, rows=[0, 1, 1, 1])
    with pytest.raises(P.AdpsgdError):
        P.adpsgd_make_schedule(g, 10, tau_mode=1, T_max=3)          # geometric without (num, den)
    with pytest.raises(P.AdpsgdError):
        P.adpsgd_make_schedule(g, 10, weight=[0, 0, 0, 0])
    # the graph is checked before its arrays are indexed: neighbour out of range, not symmetric, rowptr not monotone,
    # two components
    for rowptr, col in (([0, 2, 4, 6, 8], [3, 1, 0, 2, 1, 3, 2, 9]), ([0, 1, 1], [1]), ([0, 2, 1, 2], [1, 2, 0]),
                        ([0, 1, 2, 3, 4], [1, 0, 3, 2])):
        with pytest.raises(P.AdpsgdError) as ei:
            P.adpsgd_make_schedule((np.array(rowptr, np.int32), np.array(col, np.int32)), 10)
        assert ei.value.code == -2


def test_create_validates_graph_and_buffers_before_touching_the_gpu():
    L = P.lib()

    def create(rowptr, col, d=8, **kw):
        rowptr, col = np.asarray(rowptr, np.int32), np.asarray(col, np.int32)
        g = B.Graph(rowptr.size - 1, rowptr.ctypes.data_as(C.POINTER(C.c_int32)), col.ctypes.data_as(C.POINTER(C.c_int32)))
        o = B.Opts()
        o.model, o.X, o.ldx = B.MODEL_SYNTH, 4096, 8
        for k, v in kw.items():
            setattr(o, k, v)
        h = C.c_void_p()
        rc = L.adpsgd_create(C.byref(h), C.byref(g), d, C.byref(o))
        assert rc != 0 and not h.value
        return rc, L.adpsgd_last_error(None).decode()

    assert create([0, 1, 2, 2], [1, 0])[0] == B.ERR_GRAPH             # vertex 2 unreachable
    assert create([0, 1, 1], [1])[0] == B.ERR_GRAPH                   # not symmetric
    assert create([0, 1, 2], [0, 1])[0] == B.ERR_GRAPH                # self loops
    assert create([0, 2, 4], [1, 1, 0, 0])[0] == B.ERR_GRAPH          # duplicate edge
    rc, msg = create([0, 1, 2], [1, 0], X=4100)
    assert rc == B.ERR_ARG and "aligned" in msg
    assert create([0, 1, 2], [1, 0], ldx=6)[0] == B.ERR_ARG           # ldx < d
    assert create([0, 1, 2], [1, 0], model=B.MODEL_LSQ, M=4)[0] == B.ERR_ARG   # no workspace


# ----------------------------------------------------------------------------- planner
def _validate_plan(n, sched, n_slots, r_round, u_round, slot, R, with_grad=True):
    """Executes the plan symbolically (row versions) and asserts that it equals the serial order."""
    w, j, tau = sched["worker"], sched["neighbour"], sched["tau"]
    K = len(w)
    assert u_round.min() >= 0 and u_round.max() <= R - 1
    # serial reference: version of every row as seen by each read, order of updates per row
    version = np.zeros(n, np.int64)
    seen_serial = np.zeros(K, np.int64)
    by_s = [[] for _ in range(K + 1)]
    for k in range(K):
        by_s[k - tau[k]].append(k)
    for t in range(K):
        for k in by_s[t]:
            seen_serial[k] = version[w[k]]
        version[w[t]] += 1
        if j[t] != w[t]:
            version[j[t]] += 1
    # planned execution: reads of a round, then its updates
    version[:] = 0
    order_u = np.argsort(u_round, kind="stable")
    order_r = np.argsort(r_round, kind="stable") if with_grad else []
    pu = pr = 0
    last_u_event = -np.ones(n, np.int64)
    for r in range(R):
        while with_grad and pr < K and r_round[order_r[pr]] == r:
            k = order_r[pr]
            assert version[w[k]] == seen_serial[k], "stale read sees the wrong state"
            assert r_round[k] <= u_round[k]
            pr += 1
        touched = set()
        while pu < K and u_round[order_u[pu]] == r:
            k = order_u[pu]
            rows = {w[k], j[k]}
            assert not (rows & touched), "two updates of one round share a row"
            touched |= rows
            for row in rows:
                assert last_u_event[row] < k, "updates of a row out of event order"
                last_u_event[row] = k
                version[row] += 1
            pu += 1
    assert pu == K and (not with_grad or pr == K)
    if with_grad:
        assert slot.min() >= 0 and slot.max() < n_slots
        for s in range(n_slots):
            ks = np.where(slot == s)[0]
            ks = ks[np.argsort(r_round[ks], kind="stable")]
            for a, b in zip(ks[:-1], ks[1:]):
                assert r_round[b] > u_round[a], "slot rewritten before its gradient was consumed"


def _check_plan(n, sched, n_slots, with_grad=True):
    w, j, tau = sched["worker"], sched["neighbour"], sched["tau"]
    r_round, u_round, slot, R = P.adpsgd_plan_rounds(n, w, j, tau, n_slots, with_grad)
    assert u_round.max() == R - 1
    _validate_plan(n, sched, n_slots, r_round, u_round, slot, R, with_grad)
    assert P.adpsgd_verify_plan(n, w, j, tau, n_slots, r_round, u_round, slot, R, with_grad)
    return R


def test_pieces_of_one_schedule_are_its_slices():
    """piece_of_run: events k_begin .. generated on their own are exactly the slice of the schedule generated in
    one go (the generator is counter based; only the clipping of tau at the start differs), in both
    implementations; without the flag the first events of a piece have their staleness cut at the piece's start."""
    g = random_regular4_graph(12, 2)
    kw = dict(seed=5, T_max=7, M=3, rows=[20] * 12)
    full = oracle.make_schedule(g, 500, **kw)
    clipped = 0
    for a, b in ((0, 60), (60, 61), (61, 300), (300, 500)):
        mine = P.adpsgd_make_schedule(g, b - a, k_begin=a, piece_of_run=True, **kw)
        ref = oracle.make_schedule(g, b - a, k_begin=a, piece_of_run=True, **kw)
        alone = P.adpsgd_make_schedule(g, b - a, k_begin=a, **kw)
        for key in ("worker", "neighbour", "tau", "batch_idx"):
            assert np.array_equal(mine[key], full[key][a:b]) and np.array_equal(ref[key], full[key][a:b])
            if key != "tau":
                assert np.array_equal(alone[key], full[key][a:b])
        assert np.array_equal(alone["tau"], np.minimum(full["tau"][a:b], np.arange(b - a)))
        clipped += int((alone["tau"] != full["tau"][a:b]).sum())
    assert clipped > 0


@pytest.mark.parametrize("n,T,graph", [(8, 3, "ring"), (64, 8, "ring"), (16, 4, "reg4"), (6, 0, "ring"), (1, 0, "ring")])
def test_planner_keeps_serial_semantics(n, T, graph):
    g = ring_graph(n) if graph == "ring" else random_regular4_graph(n, 1)
    sched = oracle.make_schedule(g, 3000, seed=n, T_max=T)
    R_min = _check_plan(n, sched, T + 1)
    R_more = _check_plan(n, sched, 4 * (T + 1) + 8)
    assert R_more <= R_min
    _check_plan(n, sched, 0, with_grad=False)
    from workloads import with_identity_events
    ident = dict(sched, neighbour=with_identity_events(sched["worker"], sched["neighbour"], 0.3, seed=n))   # W_k = I events
    assert (ident["neighbour"] == ident["worker"]).sum() > 500
    assert _check_plan(n, ident, T + 1) <= R_min
    if T > 0:      # fewer slots than the largest staleness + 1 cannot hold the in-flight gradients
        with pytest.raises(P.AdpsgdError):
            P.adpsgd_plan_rounds(n, sched["worker"], sched["neighbour"], sched["tau"], T)


def test_planner_packs_many_pairs_per_round_on_the_large_ring():
    n = 128
    sched = oracle.make_schedule(ring_graph(n), 20000, seed=0, T_max=16)
    _, u_round, _, R = P.adpsgd_plan_rounds(n, sched["worker"], sched["neighbour"], sched["tau"], 0, False)
    assert 20000 / R > 15          # far from one event per launch
    assert np.bincount(u_round).max() <= n // 2


def test_planner_with_heterogeneous_geometric_staleness():
    cfg = get_config(5)
    n = cfg["n"]
    g = random_regular4_graph(n, 0)
    slow = np.arange(n) < cfg["n_slow"]
    sched = oracle.make_schedule(g, 4000, seed=0, T_max=cfg["T_max"], tau_mode=1,
                                 weight=np.where(slow, 1, 10), tau_num=np.where(slow, 20, 2),
                                 tau_den=np.where(slow, 21, 3))
    assert sched["tau"].max() > 40
    _check_plan(n, sched, cfg["T_max"] + 1)


def test_planned_rounds_reproduce_the_oracle_bit_for_bit():
    """Execute the plan on the CPU (gradients from the oracle's own routine, updates in
    numpy fp32) and compare with the oracle's serial run: reordering into rounds is exact."""
    n, d, rows, K, M, T = 8, 24, 16, 600, 4, 5
    g = ring_graph(n)
    feats, targs, _ = lsq_data(n, rows, d, seed=1)
    sched = oracle.make_schedule(g, K, seed=2, T_max=T, M=M, rows=[rows] * n)
    from workloads import with_identity_events
    sched["neighbour"] = with_identity_events(sched["worker"], sched["neighbour"], 0.2, seed=5)   # some events have W_k = I
    X_ref = np.zeros((n, d), np.float32)
    X_ref[:] = np.random.default_rng(0).standard_normal(d).astype(np.float32)
    X = X_ref.copy()
    oracle.run_events(X_ref, sched, oracle.MODEL_LSQ, 0.02, M=M, gscale=1.0 / M, features=feats, targets=targs, mode=0)
    w, j, tau = sched["worker"], sched["neighbour"], sched["tau"]
    r_round, u_round, slot, R = P.adpsgd_plan_rounds(n, w, j, tau, T + 3, True)
    slots = {}
    for r in range(R):
        for k in np.where(r_round == r)[0]:
            slots[slot[k]] = oracle.minibatch_gradient(oracle.MODEL_LSQ, X[w[k]], feats[w[k]], targs[w[k]],
                                                       sched["batch_idx"][k], 1.0 / M)[0]
        for k in np.random.default_rng(r).permutation(np.where(u_round == r)[0]):   # any order inside a round
            avg = (X[w[k]] + X[j[k]]) * np.float32(0.5)
            X[j[k]] = avg
            X[w[k]] = avg - np.float32(0.02) * slots[slot[k]]
    assert np.array_equal(X, X_ref)


def test_planner_with_multi_pair_events_reproduces_the_oracle():
    """Events whose W_k averages several disjoint pairs: execute the plan on the CPU (every pair of an
    event in the event's round) and compare with the oracle bit for bit."""
    from workloads import random_extra_pairs
    n, d, rows, K, M, T = 10, 16, 12, 500, 3, 4
    g = random_regular4_graph(n, 2)
    feats, targs, _ = lsq_data(n, rows, d, seed=1)
    sched = oracle.make_schedule(g, K, seed=3, T_max=T, M=M, rows=[rows] * n)
    extra = random_extra_pairs(g, sched["worker"], sched["neighbour"], max_extra=3, seed=4)
    X_ref = np.tile(np.random.default_rng(0).standard_normal(d).astype(np.float32), (n, 1))
    X = X_ref.copy()
    oracle.run_events(X_ref, sched, oracle.MODEL_LSQ, 0.02, M=M, gscale=1.0 / M, features=feats, targets=targs,
                      mode=0, extra_pairs=extra)
    w, j, tau = sched["worker"], sched["neighbour"], sched["tau"]
    r_round, u_round, slot, R = P.adpsgd_plan_rounds(n, w, j, tau, T + 2, True, extra_pairs=extra)
    R_plain = P.adpsgd_plan_rounds(n, w, j, tau, T + 2, True)[3]
    assert R >= R_plain                       # more rows per event can only lengthen the chains
    slots = {}
    for r in range(R):
        for k in np.where(r_round == r)[0]:
            slots[slot[k]] = oracle.minibatch_gradient(oracle.MODEL_LSQ, X[w[k]], feats[w[k]], targs[w[k]],
                                                       sched["batch_idx"][k], 1.0 / M)[0]
        touched = set()
        for k in np.where(u_round == r)[0]:
            pairs = [(w[k], j[k])] + [(extra[1][q], extra[2][q]) for q in range(extra[0][k], extra[0][k + 1])]
            for a, b in pairs:
                assert a not in touched and b not in touched
                touched.update((a, b))
            for a, b in pairs[1:]:
                X[a] = X[b] = (X[a] + X[b]) * np.float32(0.5)
            avg = (X[w[k]] + X[j[k]]) * np.float32(0.5)
            X[j[k]] = avg
            X[w[k]] = avg - np.float32(0.02) * slots[slot[k]]
    assert np.array_equal(X, X_ref)


def test_planner_for_the_waitfree_variant_reproduces_the_oracle():
    """Wait-free variant: a read may be compensated with the worker's own pending gradient.  Execute
    the plan on the CPU -- the gradients of a round all see the slots as they were when the round
    began, so a gradient planned into the same round as the one it depends on would be caught -- and
    compare with the oracle's serial run bit for bit."""
    n, d, rows, K, M, T = 4, 20, 16, 500, 3, 6
    g = ring_graph(n)
    feats, targs, _ = lsq_data(n, rows, d, seed=1)
    sched = oracle.make_schedule(g, K, seed=5, T_max=T, M=M, rows=[rows] * n)
    gam = (0.01 + 0.005 * (np.arange(K) % 5)).astype(np.float32)
    X_ref = np.tile(np.random.default_rng(0).standard_normal(d).astype(np.float32), (n, 1))
    X = X_ref.copy()
    oracle.run_events(X_ref, sched, oracle.MODEL_LSQ, 0.0, M=M, gscale=1.0 / M, features=feats, targets=targs,
                      gamma_k=gam, mode=0, local_compensation=True)
    w, j, tau = sched["worker"], sched["neighbour"], sched["tau"]
    r_round, u_round, slot, R, prev = P.adpsgd_plan_rounds(n, w, j, tau, T + 2, True, local_compensation=True)
    # the pending event, recomputed here from its definition
    last = {}
    for k in range(K):
        kp = last.get(w[k], -1)
        want = kp if kp >= 0 and kp - tau[kp] <= k - tau[k] <= kp else -1
        assert prev[k] == want
        last[w[k]] = k
    assert (prev >= 0).sum() > K // 10          # the case under test really occurs
    slots = {}
    for r in range(R):
        at_start = dict(slots)
        for k in np.where(r_round == r)[0]:
            xh = X[w[k]]
            if prev[k] >= 0:
                assert r_round[prev[k]] < r <= u_round[prev[k]]
                xh = xh - gam[prev[k]] * at_start[slot[prev[k]]]
            slots[slot[k]] = oracle.minibatch_gradient(oracle.MODEL_LSQ, xh, feats[w[k]], targs[w[k]],
                                                       sched["batch_idx"][k], 1.0 / M)[0]
        for k in np.where(u_round == r)[0]:
            avg = (X[w[k]] + X[j[k]]) * np.float32(0.5)
            X[j[k]] = avg
            X[w[k]] = avg - gam[k] * slots[slot[k]]
    assert np.array_equal(X, X_ref)
    # without the switch the plan ignores the extra dependency
    assert len(P.adpsgd_plan_rounds(n, w, j, tau, T + 2, True)) == 4


@pytest.mark.parametrize("comp", [False, True])
def test_calls_that_look_ahead_reproduce_one_long_run(comp):
    """A run split into calls keeps the staleness across the boundaries when every call looks ahead to
    the first events of the next one: their early stale reads are evaluated now and carried in their
    slots.  The plans of the calls, executed one after another on the CPU, must give the oracle's single
    run over the whole schedule bit for bit (also with calls shorter than the look-ahead, and for the
    wait-free variant), every plan must pass the library's own check, and a call that does not look
    ahead far enough is refused."""
    n, d, rows, K, M, T = 6, 20, 16, 900, 3, 6
    g = ring_graph(n)
    feats, targs, _ = lsq_data(n, rows, d, seed=2)
    sched = oracle.make_schedule(g, K, seed=9, T_max=T, M=M, rows=[rows] * n)
    gam = (0.01 + 0.005 * (np.arange(K) % 4)).astype(np.float32)
    X_ref = np.tile(np.random.default_rng(1).standard_normal(d).astype(np.float32), (n, 1))
    X = X_ref.copy()
    oracle.run_events(X_ref, sched, oracle.MODEL_LSQ, 0.0, M=M, gscale=1.0 / M, features=feats, targets=targs,
                      gamma_k=gam, mode=0, local_compensation=comp)
    W, J, TAU = sched["worker"], sched["neighbour"], sched["tau"]
    n_slots = T + 3
    cuts = [0, 130, 133, 137, 400, 403, 900]          # calls of 130, 3, 4, 263, 3 and 497 events
    slots, pending, carried_reads = {}, {}, 0
    for a, b in zip(cuts[:-1], cuts[1:]):
        end = min(b + T, K)                           # look T events ahead (nothing after the last call)
        w, j, tau = W[a:end], J[a:end], TAU[a:end]
        carried = np.array([pending.get(a + k, -1) for k in range(end - a)], np.int32)
        carried_reads += int((carried >= 0).sum())
        out = P.adpsgd_plan_rounds(n, w, j, tau, n_slots, True, local_compensation=comp, n_apply=b - a, carried_slot=carried)
        r_round, u_round, slot, R = out[:4]
        prev = out[4] if comp else np.full(end - a, -1)
        assert P.adpsgd_verify_plan(n, w, j, tau, n_slots, r_round, u_round, slot, R, prev=prev if comp else None,
                                    n_apply=b - a, carried_slot=carried)
        assert np.all(u_round[b - a:] == -1) and np.all(u_round[:b - a] >= 0)
        check = lambda rr, uu, ss: P.adpsgd_verify_plan(n, w, j, tau, n_slots, rr, uu, ss, R, prev=prev if comp else None,
                                                        n_apply=b - a, carried_slot=carried)
        if end > b:                                   # damaged plans of a call that looks ahead are caught
            uu = u_round.copy()
            uu[b - a] = 0                             # an update for an event that is only looked ahead to
            assert not check(r_round, uu, slot)
            kept = [k for k in range(b - a, end - a) if slot[k] >= 0]          # gradients this call leaves pending
            fresh = [k for k in range(end - a) if r_round[k] >= 0 and (not kept or k != kept[0])]
            if kept and fresh:
                ss = slot.copy()
                ss[fresh[-1]] = slot[kept[0]]         # their slot given to another gradient
                assert not check(r_round, u_round, ss)
            moved = [k for k in range(end - a) if carried[k] >= 0]
            if moved:
                rr = r_round.copy()
                rr[moved[0]] = 0                      # a carried gradient evaluated again
                assert not check(rr, u_round, slot)
        for k in range(end - a):
            s_k = k - tau[k]
            if carried[k] >= 0:
                assert slot[k] == carried[k] and r_round[k] == -1 and s_k < 0
            elif s_k < b - a:
                assert r_round[k] >= 0 and slot[k] >= 0
            else:
                assert r_round[k] == -1 and slot[k] == -1 and k >= b - a
        for r in range(R):
            at_start = dict(slots)
            for k in np.where(r_round == r)[0]:
                xh = X[w[k]]
                if prev[k] >= 0:
                    xh = xh - gam[a + prev[k]] * at_start[slot[prev[k]]]
                slots[slot[k]] = oracle.minibatch_gradient(oracle.MODEL_LSQ, xh, feats[w[k]], targs[w[k]],
                                                           sched["batch_idx"][a + k], 1.0 / M)[0]
            for k in np.where(u_round == r)[0]:
                avg = (X[w[k]] + X[j[k]]) * np.float32(0.5)
                X[j[k]] = avg
                X[w[k]] = avg - gam[a + k] * slots[slot[k]]
        pending = {a + k: int(slot[k]) for k in range(b - a, end - a)}
    assert carried_reads > 10
    assert np.array_equal(X, X_ref)
    # the staleness at the boundaries matters: self-contained calls (tau clipped at the start of a call) differ
    call_start = np.array(cuts)[np.searchsorted(cuts, np.arange(K), side="right") - 1]
    clipped = dict(sched, tau=np.minimum(TAU, np.arange(K) - call_start).astype(np.int32))
    Xc = np.tile(np.random.default_rng(1).standard_normal(d).astype(np.float32), (n, 1))
    oracle.run_events(Xc, clipped, oracle.MODEL_LSQ, 0.0, M=M, gscale=1.0 / M, features=feats, targets=targs,
                      gamma_k=gam, mode=0, local_compensation=comp)
    assert not np.array_equal(Xc, X_ref)
    # an event whose read time lies before the call and that nobody carried is refused
    k0 = next(k for k in range(131, K) if TAU[k] > 1)
    with pytest.raises(P.AdpsgdError):
        P.adpsgd_plan_rounds(n, W[k0 - 1:k0 + 50], J[k0 - 1:k0 + 50], TAU[k0 - 1:k0 + 50], n_slots, True)


def test_metropolis_weights_agree_with_the_oracle_bit_for_bit():
    for g in (ring_graph(8), random_regular4_graph(16, 3), ring_graph(2), ring_graph(1)):
        w_self, w_edge = P.adpsgd_metropolis_weights(g)
        W = oracle.metropolis_weights(g)
        n = len(g[0]) - 1
        assert np.array_equal(w_self, np.diag(W))
        for i in range(n):
            for e in range(g[0][i], g[0][i + 1]):
                assert w_edge[e] == W[i, g[1][e]]
        assert np.count_nonzero(W) == n + len(w_edge)
    # an irregular graph: star with 4 leaves
    rowptr = np.array([0, 4, 5, 6, 7, 8], np.int32)
    col = np.array([1, 2, 3, 4, 0, 0, 0, 0], np.int32)
    w_self, w_edge = P.adpsgd_metropolis_weights((rowptr, col))
    assert np.array_equal(w_edge, np.full(8, np.float32(0.2))) and w_self[1] == np.float32(0.8)
    assert np.array_equal(np.diag(oracle.metropolis_weights((rowptr, col))), w_self)


def test_plan_verifier_agrees_with_the_symbolic_execution_on_damaged_plans():
    """The library's own plan check (its race detector) against this file's symbolic execution: single
    entries of correct plans are perturbed; the two must reach the same verdict every time, and both
    verdicts must occur."""
    rng = np.random.default_rng(11)
    verdicts = {True: 0, False: 0}
    for trial in range(6):
        n, T, K = int(rng.integers(3, 12)), int(rng.integers(0, 6)), 120
        g = ring_graph(n) if trial % 2 else random_regular4_graph(max(n, 6), trial)
        n = len(g[0]) - 1
        sched = oracle.make_schedule(g, K, seed=trial, T_max=T)
        w, j, tau = sched["worker"], sched["neighbour"], sched["tau"]
        n_slots = T + 2
        r0, u0, s0, R = P.adpsgd_plan_rounds(n, w, j, tau, n_slots, True)
        for m in range(60):
            r_round, u_round, slot = r0.copy(), u0.copy(), s0.copy()
            k = int(rng.integers(K))
            what = m % 4
            if what == 0:
                u_round[k] = max(0, u_round[k] - int(rng.integers(1, 3)))
            elif what == 1:
                u_round[k] = min(R - 1, u_round[k] + int(rng.integers(1, 3)))
            elif what == 2:
                r_round[k] = int(np.clip(r_round[k] + int(rng.integers(-2, 3)), 0, R - 1))
            else:
                slot[k] = int(rng.integers(n_slots))
            try:
                _validate_plan(n, sched, n_slots, r_round, u_round, slot, R, True)
                mine = True
            except AssertionError:
                mine = False
            theirs = P.adpsgd_verify_plan(n, w, j, tau, n_slots, r_round, u_round, slot, R, True)
            assert mine == theirs, (trial, m, k, what)
            verdicts[mine] += 1
    assert verdicts[True] > 20 and verdicts[False] > 100


def test_plan_verifier_covers_extra_pairs_and_the_waitfree_dependency():
    from workloads import random_extra_pairs
    n, K, T = 10, 300, 4
    g = random_regular4_graph(n, 2)
    sched = oracle.make_schedule(g, K, seed=3, T_max=T)
    w, j, tau = sched["worker"], sched["neighbour"], sched["tau"]
    extra = random_extra_pairs(g, w, j, max_extra=3, seed=4)
    r, u, s, R = P.adpsgd_plan_rounds(n, w, j, tau, T + 2, True, extra_pairs=extra)
    assert P.adpsgd_verify_plan(n, w, j, tau, T + 2, r, u, s, R, extra_pairs=extra)
    # a plan made without the extra pairs lets them collide with other updates of the round
    r2, u2, s2, R2 = P.adpsgd_plan_rounds(n, w, j, tau, T + 2, True)
    assert not P.adpsgd_verify_plan(n, w, j, tau, T + 2, r2, u2, s2, R2, extra_pairs=extra)
    # wait-free variant: the compensated read needs its pending gradient
    n = 4
    g = ring_graph(n)
    sched = oracle.make_schedule(g, K, seed=5, T_max=6)
    w, j, tau = sched["worker"], sched["neighbour"], sched["tau"]
    r, u, s, R, prev = P.adpsgd_plan_rounds(n, w, j, tau, 8, True, local_compensation=True)
    assert P.adpsgd_verify_plan(n, w, j, tau, 8, r, u, s, R, prev=prev)
    r3, u3, s3, R3 = P.adpsgd_plan_rounds(n, w, j, tau, 8, True)           # planned without the dependency
    assert (prev >= 0).any() and not P.adpsgd_verify_plan(n, w, j, tau, 8, r3, u3, s3, R3, prev=prev)


def test_the_abi_is_usable_from_plain_c(tmp_path):
    """The header compiles as C11 with -Wall -Wextra -Werror, and a C program linked against the library runs
    the host-only entry points (schedule generator, planner, plan check, Metropolis weights)."""
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    lib_dir = os.path.dirname(str(P.LIB_PATH))
    exe = str(tmp_path / "host_only")
    rocm_lib = "/opt/rocm/lib"
    subprocess.check_call(["gcc", "-std=c11", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(root, "include"),
                           os.path.join(root, "tests", "c_abi", "host_only.c"), "-o", exe, "-L", lib_dir, "-ladpsgd",
                           "-Wl,-rpath," + lib_dir, "-Wl,-rpath," + rocm_lib])
    env = dict(os.environ, LD_LIBRARY_PATH=rocm_lib + ":" + os.environ.get("LD_LIBRARY_PATH", ""))
    out = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=60)
    assert out.returncode == 0, (out.returncode, out.stdout, out.stderr)
    assert "c abi ok" in out.stdout


# ------------------------------------------------------------------ step-size rules of the experiments (Sec. 5.2, 5.3)
def test_step_size_rules_of_the_experiments():
    from paper_1710_06952_amd import step_sizes as ss
    epe = 40                                    # events per epoch
    K = 130 * epe
    halving = ss.step_decay(K, epe, 1.0, factor=0.5, every=25)               # start at 1, halve every 25 epochs
    assert halving.dtype == np.float32 and len(halving) == K
    assert halving[0] == 1.0 and halving[25 * epe - 1] == 1.0 and halving[25 * epe] == 0.5
    assert halving[50 * epe] == 0.25 and halving[-1] == 2.0 ** -5
    tenth = ss.step_decay(K, epe, 0.1, factor=0.1, milestones=(81, 122))     # /10 at the 81st and the 122nd epoch
    assert np.all(tenth[:80 * epe] == np.float32(0.1)) and np.isclose(tenth[80 * epe], 0.01)
    assert np.isclose(tenth[121 * epe - 1], 0.01) and np.isclose(tenth[121 * epe], 0.001)
    # a run split into calls sees the same values
    parts = np.concatenate([ss.step_decay(1000, epe, 1.0, k_begin=0), ss.step_decay(K - 1000, epe, 1.0, k_begin=1000)])
    assert np.array_equal(parts, halving)
    # warm-up: linear from 0.1 to the scaled step over 5 epochs, untouched afterwards
    scaled = ss.step_decay(K, epe, 0.8, factor=0.1, milestones=(81, 122))
    warm = ss.with_linear_warmup(scaled, epe, 5, 0.1)
    assert warm[0] == np.float32(0.1) and np.all(np.diff(warm[:5 * epe]) > 0)
    assert np.isclose(warm[5 * epe // 2], 0.45) and np.array_equal(warm[5 * epe:], scaled[5 * epe:])
    late = ss.with_linear_warmup(ss.step_decay(300, epe, 0.8, k_begin=150), epe, 5, 0.1, k_begin=150)
    assert np.allclose(late[:50], warm[150:200]) and np.all(late[50:] == np.float32(0.8))
    with pytest.raises(ValueError):
        ss.step_decay(10, 0, 1.0)


def test_stored_long_run_references_match_their_recipe():
    """tests/golden/long_run_cfg*.npz (the oracle's models along the full runs of configurations 2, 4, 5, written by
    tests/golden/make_long_run_references.py) carry what the GPU test expects: the whole run in four calls, the
    sampled coordinates the script's seed gives, one row per worker, finite values, losses that fall."""
    import importlib.util
    from workloads import get_config
    gold = os.path.join(ROOT, "tests", "golden")
    spec = importlib.util.spec_from_file_location("make_long_run_references", os.path.join(gold, "make_long_run_references.py"))
    mk = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mk)
    for idx in (2, 4, 5):
        c = get_config(idx)
        ref = np.load(os.path.join(gold, "long_run_cfg%d.npz" % idx), allow_pickle=False)
        assert int(ref["events_per_call"]) * mk.CALLS == c["K"] and int(ref["rows"]) == mk.ROWS[idx]
        coords = np.sort(np.random.default_rng([c["seed"], 77, idx]).choice(c["d"], size=mk.SAMPLED, replace=False))
        assert np.array_equal(ref["coords"], coords)
        for q in range(mk.CALLS):
            x, amax = ref["x%d" % q], ref["amax%d" % q]
            assert x.shape == (c["n"], mk.SAMPLED) and x.dtype == np.float32 and np.isfinite(x).all()
            assert amax.shape == (c["n"],) and (amax > 0).all() and (np.abs(x).max(axis=1) <= amax).all()
            assert (ref["l2_%d" % q] >= amax).all() and np.isfinite(ref["s%d" % q]).all()
        assert float(ref["loss_tail%d" % (mk.CALLS - 1)]) < float(ref["loss_tail0"])
