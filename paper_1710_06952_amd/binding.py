"""ctypes binding of libadpsgd.so: the same entry points as include/adpsgd.h,
argument marshalling only.  Every step of the update path runs in the HIP
library; there is no fallback: a missing library raises at import of the symbol
table, a failing call raises AdpsgdError with the library's message.
"""
from __future__ import annotations

import ctypes as C
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
LIB_PATH = _HERE / "libadpsgd.so"

OK, ERR_ARG, ERR_GRAPH, ERR_SCHEDULE, ERR_STATE, ERR_HIP, ERR_CALLBACK = 0, -1, -2, -3, -4, -5, -6
MODEL_LSQ, MODEL_LOGREG, MODEL_SYNTH, MODEL_MLP, MODEL_EXTERNAL = 0, 1, 2, 3, 4
FLAG_PROFILE, FLAG_DENSE_GRADIENT, FLAG_VERIFY_PLAN, FLAG_SYNC_IN_PLACE = 1, 2, 4, 8

EXPORTS = [
    "adpsgd_create", "adpsgd_destroy", "adpsgd_last_error", "adpsgd_load_data", "adpsgd_set_models",
    "adpsgd_run_events", "adpsgd_run_events_with", "adpsgd_get_models", "adpsgd_get_mean_model", "adpsgd_consensus_distance", "adpsgd_consensus_distance_weighted",
    "adpsgd_consensus_distance_static",
    "adpsgd_get_bf16_models", "adpsgd_classification_error", "adpsgd_get_momentum", "adpsgd_get_stats", "adpsgd_make_schedule", "adpsgd_plan_rounds",
    "adpsgd_synth_gradient", "adpsgd_run_sync_steps", "adpsgd_run_sync_steps_with", "adpsgd_metropolis_weights",
    "adpsgd_get_event_count", "adpsgd_set_event_count", "adpsgd_verify_plan", "adpsgd_objective", "adpsgd_objective_weighted", "adpsgd_count_nonfinite",
]


class AdpsgdError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("adpsgd error %d: %s" % (code, msg))
        self.code = code


class Graph(C.Structure):
    _fields_ = [("n", C.c_int32), ("rowptr", C.POINTER(C.c_int32)), ("col", C.POINTER(C.c_int32))]


class Opts(C.Structure):
    _fields_ = [("model", C.c_int32), ("M", C.c_int32), ("gamma", C.c_float), ("lambda_", C.c_float),
                ("grad_sum", C.c_int32), ("T_max", C.c_int32), ("synth_std", C.c_float),
                ("synth_seed", C.c_uint64), ("mlp_in", C.c_int32), ("mlp_hidden", C.c_int32),
                ("mlp_out", C.c_int32), ("X", C.c_void_p), ("ldx", C.c_int64), ("Xbf16", C.c_void_p),
                ("workspace", C.c_void_p), ("workspace_bytes", C.c_int64), ("stream", C.c_void_p),
                ("flags", C.c_int32), ("momentum", C.c_float), ("weight_decay", C.c_float), ("V", C.c_void_p),
                ("local_compensation", C.c_int32)]


class Schedule(C.Structure):
    _fields_ = [("K", C.c_int64), ("worker", C.POINTER(C.c_int32)), ("neighbour", C.POINTER(C.c_int32)),
                ("tau", C.POINTER(C.c_int32)), ("batch_idx", C.POINTER(C.c_int32)),
                ("gamma", C.POINTER(C.c_float)), ("extra_ptr", C.POINTER(C.c_int64)),
                ("extra_a", C.POINTER(C.c_int32)), ("extra_b", C.POINTER(C.c_int32)), ("lookahead", C.c_int64)]


class GradRequest(C.Structure):
    _fields_ = [("worker", C.c_int32), ("reserved", C.c_int32), ("event", C.c_int64), ("xhat", C.c_void_p), ("g", C.c_void_p)]


GRADIENT_FN = C.CFUNCTYPE(C.c_int, C.c_void_p, C.c_int32, C.POINTER(GradRequest), C.c_void_p)


class SyncSchedule(C.Structure):
    _fields_ = [("S", C.c_int64), ("batch_idx", C.POINTER(C.c_int32)), ("gamma", C.POINTER(C.c_float)),
                ("w_self", C.POINTER(C.c_float)), ("w_edge", C.POINTER(C.c_float))]


class SchedParams(C.Structure):
    _fields_ = [("graph", Graph), ("weight", C.POINTER(C.c_int32)), ("tau_mode", C.c_int32),
                ("T_max", C.c_int32), ("tau_num", C.POINTER(C.c_int32)), ("tau_den", C.POINTER(C.c_int32)),
                ("M", C.c_int32), ("rows", C.POINTER(C.c_int32)), ("piece_of_run", C.c_int32)]


class Stats(C.Structure):
    _fields_ = [("events", C.c_int64), ("rounds", C.c_int64), ("fused_launches", C.c_int64),
                ("grad_launches", C.c_int64), ("max_round_pairs", C.c_int64), ("slots", C.c_int64),
                ("fused_ms", C.c_double), ("grad_ms", C.c_double)]


_lib = None


def _preload_hip_runtime():
    """One process must use ONE HIP runtime: device pointers and streams handed over by PyTorch
    belong to the libamdhip64 that PyTorch bundles.  Load that copy first (same SONAME as the one
    libadpsgd.so was linked against), so the dynamic loader resolves our dependency to it."""
    import importlib.util
    spec = importlib.util.find_spec("torch")
    if spec is None or not spec.submodule_search_locations:
        return
    cand = Path(list(spec.submodule_search_locations)[0]) / "lib" / "libamdhip64.so"
    if cand.exists():
        C.CDLL(str(cand), mode=C.RTLD_GLOBAL)


def lib():
    """Load libadpsgd.so (built in-tree by paper_1710_06952_amd.build).  Fails loudly."""
    global _lib
    if _lib is None:
        if not LIB_PATH.exists():
            raise ImportError("%s is missing: run `python -m paper_1710_06952_amd.build` "
                              "(there is no CPU fallback)" % LIB_PATH)
        _preload_hip_runtime()
        L = C.CDLL(str(LIB_PATH))
        vp, i32, i64, u64 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64
        P = C.POINTER
        L.adpsgd_create.argtypes = [P(vp), P(Graph), i64, P(Opts)]
        L.adpsgd_destroy.argtypes = [vp]
        L.adpsgd_destroy.restype = None
        L.adpsgd_last_error.argtypes = [vp]
        L.adpsgd_last_error.restype = C.c_char_p
        L.adpsgd_load_data.argtypes = [vp, i32, vp, i64, i64, vp]
        L.adpsgd_set_models.argtypes = [vp, vp, i64, i32]
        L.adpsgd_run_events.argtypes = [vp, P(Schedule), vp]
        L.adpsgd_get_models.argtypes = [vp, vp, i64, i32]
        L.adpsgd_get_mean_model.argtypes = [vp, vp, i32]
        L.adpsgd_consensus_distance.argtypes = [vp, P(C.c_double)]
        L.adpsgd_consensus_distance_weighted.argtypes = [vp, P(C.c_double), P(C.c_double)]
        L.adpsgd_consensus_distance_static.argtypes = [vp, P(C.c_double), vp]
        L.adpsgd_get_bf16_models.argtypes = [vp, vp, i64, i32]
        L.adpsgd_get_momentum.argtypes = [vp, vp, i64, i32]
        L.adpsgd_get_stats.argtypes = [vp, P(Stats)]
        L.adpsgd_make_schedule.argtypes = [P(SchedParams), u64, u64, i64, P(i32), P(i32), P(i32), P(i32)]
        L.adpsgd_plan_rounds.argtypes = [i32, i64, P(i32), P(i32), P(i32), i32, i32, P(i32), P(i32), P(i32), P(i32),
                                         P(i64), P(i32), P(i32), i32, P(i64), i64, P(i32)]
        L.adpsgd_synth_gradient.argtypes = [u64, u64, C.c_float, i64, vp, vp]
        L.adpsgd_run_sync_steps.argtypes = [vp, P(SyncSchedule), vp]
        L.adpsgd_verify_plan.argtypes = [i32, i64, P(i32), P(i32), P(i32), i32, i32, P(i32), P(i32), P(i32), i32,
                                         P(i64), P(i32), P(i32), P(i64), i64, P(i32)]
        L.adpsgd_objective.argtypes = [vp, vp, P(C.c_double)]
        L.adpsgd_objective_weighted.argtypes = [vp, vp, P(C.c_double), P(C.c_double)]
        L.adpsgd_run_events_with.argtypes = [vp, P(Schedule), GRADIENT_FN, vp]
        L.adpsgd_run_sync_steps_with.argtypes = [vp, P(SyncSchedule), GRADIENT_FN, vp]
        L.adpsgd_classification_error.argtypes = [vp, vp, P(C.c_double)]
        L.adpsgd_count_nonfinite.argtypes = [vp, P(i64)]
        L.adpsgd_get_event_count.argtypes = [vp, P(u64)]
        L.adpsgd_set_event_count.argtypes = [vp, u64]
        L.adpsgd_metropolis_weights.argtypes = [P(Graph), P(C.c_float), P(C.c_float)]
        _lib = L
    return _lib


def _i32p(a):
    return None if a is None else a.ctypes.data_as(C.POINTER(C.c_int32))


def _as_i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _graph_struct(graph):
    rowptr, col = _as_i32(graph[0]), _as_i32(graph[1])
    return Graph(rowptr.size - 1, _i32p(rowptr), _i32p(col)), (rowptr, col)


def _check(h, rc):
    if rc != OK:
        raise AdpsgdError(rc, (lib().adpsgd_last_error(h) or b"").decode())


def adpsgd_make_schedule(graph, K, seed=0, k_begin=0, T_max=0, tau_mode=0, weight=None, tau_num=None,
                         tau_den=None, M=0, rows=None, piece_of_run=False):
    """Host-only: the random choices of Algorithm 1 for K events (see adpsgd.h)."""
    g, keep = _graph_struct(graph)
    weight, tau_num, tau_den, rows = map(_as_i32, (weight, tau_num, tau_den, rows))
    p = SchedParams(g, _i32p(weight), tau_mode, T_max, _i32p(tau_num), _i32p(tau_den), M, _i32p(rows),
                    1 if piece_of_run else 0)
    worker, nbr, tau = (np.zeros(K, np.int32) for _ in range(3))
    batch = np.zeros((K, M), np.int32) if M > 0 else None
    rc = lib().adpsgd_make_schedule(C.byref(p), seed, k_begin, K, _i32p(worker), _i32p(nbr), _i32p(tau), _i32p(batch))
    if rc != OK:
        raise AdpsgdError(rc, "adpsgd_make_schedule: bad argument")
    del keep
    return {"worker": worker, "neighbour": nbr, "tau": tau, "batch_idx": batch}


def _extra_arrays(extra_pairs):
    if extra_pairs is None:
        return None, None, None
    return (np.ascontiguousarray(extra_pairs[0], dtype=np.int64), _as_i32(extra_pairs[1]), _as_i32(extra_pairs[2]))


def adpsgd_plan_rounds(n, worker, neighbour, tau, n_slots, with_gradients=True, extra_pairs=None,
                       local_compensation=False, n_apply=-1, carried_slot=None):
    """Host-only: the round planner on its own; returns (r_round, u_round, slot, n_rounds), and with
    local_compensation also prev (the event whose pending gradient each read is compensated with).
    n_apply / carried_slot: a call that looks ahead, or continues one that did (see the header)."""
    worker, neighbour, tau = map(_as_i32, (worker, neighbour, tau))
    K = worker.size
    r, u, s = (np.zeros(K, np.int32) for _ in range(3))
    nr = C.c_int32(0)
    prev = np.zeros(K, np.int64)
    ep, ea, eb = _extra_arrays(extra_pairs)
    rc = lib().adpsgd_plan_rounds(n, K, _i32p(worker), _i32p(neighbour), _i32p(tau), n_slots,
                                  1 if with_gradients else 0, _i32p(r), _i32p(u), _i32p(s), C.byref(nr),
                                  None if ep is None else ep.ctypes.data_as(C.POINTER(C.c_int64)), _i32p(ea), _i32p(eb),
                                  1 if local_compensation else 0, prev.ctypes.data_as(C.POINTER(C.c_int64)),
                                  n_apply, _i32p(_as_i32(carried_slot)))
    if rc != OK:
        raise AdpsgdError(rc, "adpsgd_plan_rounds failed")
    if local_compensation:
        return r, u, s, nr.value, prev
    return r, u, s, nr.value


def adpsgd_verify_plan(n, worker, neighbour, tau, n_slots, r_round, u_round, slot, n_rounds, with_gradients=True,
                       extra_pairs=None, prev=None, n_apply=-1, carried_slot=None):
    """Host-only: True when the plan keeps the serial semantics of the events."""
    worker, neighbour, tau, r_round, u_round, slot = map(_as_i32, (worker, neighbour, tau, r_round, u_round, slot))
    ep, ea, eb = _extra_arrays(extra_pairs)
    pv = None if prev is None else np.ascontiguousarray(prev, dtype=np.int64)
    i64p = lambda a: None if a is None else a.ctypes.data_as(C.POINTER(C.c_int64))
    rc = lib().adpsgd_verify_plan(n, worker.size, _i32p(worker), _i32p(neighbour), _i32p(tau), n_slots,
                                  1 if with_gradients else 0, _i32p(r_round), _i32p(u_round), _i32p(slot), n_rounds,
                                  i64p(ep), _i32p(ea), _i32p(eb), i64p(pv), n_apply, _i32p(_as_i32(carried_slot)))
    if rc not in (OK, ERR_STATE):
        raise AdpsgdError(rc, "adpsgd_verify_plan: bad argument")
    return rc == OK


def adpsgd_metropolis_weights(graph):
    """Host-only: (w_self[n], w_edge[nnz]) aligned with the graph's CSR arrays."""
    g, keep = _graph_struct(graph)
    w_self = np.zeros(g.n, np.float32)
    w_edge = np.zeros(max(int(np.asarray(graph[0])[-1]), 1), np.float32)
    rc = lib().adpsgd_metropolis_weights(C.byref(g), w_self.ctypes.data_as(C.POINTER(C.c_float)),
                                         w_edge.ctypes.data_as(C.POINTER(C.c_float)))
    del keep
    if rc != OK:
        raise AdpsgdError(rc, "adpsgd_metropolis_weights failed")
    return w_self, w_edge[:int(np.asarray(graph[0])[-1])]


def adpsgd_synth_gradient(seed, k, std, d, out_ptr, stream=0):
    rc = lib().adpsgd_synth_gradient(seed, k, std, d, out_ptr, stream)
    if rc != OK:
        raise AdpsgdError(rc, "adpsgd_synth_gradient failed")


def _gradient_trampoline(gradient_fn):
    """The C callback around a Python gradient function, and the list that catches what it raises
    (an exception must not propagate through the C frames)."""
    raised = []

    def trampoline(_user, count, requests, stream):
        try:
            gradient_fn([(requests[t].worker, requests[t].event, requests[t].xhat, requests[t].g) for t in range(count)],
                        stream or 0)
            return 0
        except BaseException as exc:
            raised.append(exc)
            return 1

    return GRADIENT_FN(trampoline), raised


class Handle:
    """Owns one adpsgd_t*.  Methods mirror the C entry points one to one; device
    pointers are plain integers (e.g. ``tensor.data_ptr()``)."""

    def __init__(self, graph, d, *, model, X_ptr, ldx, M=0, gamma=0.0, lam=0.0, grad_sum=False, T_max=0,
                 synth_std=0.0, synth_seed=0, mlp=(0, 0, 0), Xbf16_ptr=None, workspace_ptr=None,
                 workspace_bytes=0, stream=0, flags=0, momentum=0.0, weight_decay=0.0, V_ptr=None,
                 local_compensation=False):
        g, keep = _graph_struct(graph)
        o = Opts(model, M, gamma, lam, 1 if grad_sum else 0, T_max, synth_std, synth_seed, mlp[0], mlp[1], mlp[2],
                 X_ptr, ldx, Xbf16_ptr, workspace_ptr, workspace_bytes, stream or None, flags,
                 momentum, weight_decay, V_ptr, 1 if local_compensation else 0)
        self._h = C.c_void_p()
        self.n, self.d, self.M, self.model = g.n, d, M, model
        rc = lib().adpsgd_create(C.byref(self._h), C.byref(g), d, C.byref(o))
        del keep
        if rc != OK:
            self._h = None
            raise AdpsgdError(rc, (lib().adpsgd_last_error(None) or b"").decode())

    def destroy(self):
        h, self._h = getattr(self, "_h", None), None
        if h:
            try:
                lib().adpsgd_destroy(h)
            except TypeError:       # interpreter shutdown: the module globals are already gone
                pass

    __del__ = destroy

    def load_data(self, worker, features_ptr, rows, ld, targets_ptr):
        _check(self._h, lib().adpsgd_load_data(self._h, worker, features_ptr, rows, ld, targets_ptr))

    def set_models(self, x, ld_in=0, on_device=False):
        """x: numpy fp32 array (host) or an integer device pointer (on_device=True)."""
        if on_device:
            ptr = x
        else:
            x = np.ascontiguousarray(x, dtype=np.float32)
            ptr = x.ctypes.data
        _check(self._h, lib().adpsgd_set_models(self._h, ptr, ld_in, 1 if on_device else 0))

    def run_events(self, schedule, loss_ptr=None):
        worker, nbr, tau = (_as_i32(schedule[k]) for k in ("worker", "neighbour", "tau"))
        batch = _as_i32(schedule.get("batch_idx"))
        gam = schedule.get("gamma")
        gam = None if gam is None else np.ascontiguousarray(gam, dtype=np.float32)
        ep, ea, eb = _extra_arrays(schedule.get("extra_pairs"))
        s = Schedule(worker.size, _i32p(worker), _i32p(nbr), _i32p(tau), _i32p(batch),
                     None if gam is None else gam.ctypes.data_as(C.POINTER(C.c_float)),
                     None if ep is None else ep.ctypes.data_as(C.POINTER(C.c_int64)), _i32p(ea), _i32p(eb),
                     int(schedule.get("lookahead", 0)))
        _check(self._h, lib().adpsgd_run_events(self._h, C.byref(s), loss_ptr))

    def run_events_with(self, schedule, gradient_fn):
        """MODEL_EXTERNAL: gradient_fn(requests, stream) gets a list of (worker, event, xhat_ptr, g_ptr)
        tuples (device pointers as integers) and the stream as an integer; it enqueues the work that
        writes every requested gradient.  An exception inside it aborts the run and is raised again here."""
        worker, nbr, tau = (_as_i32(schedule[k]) for k in ("worker", "neighbour", "tau"))
        gam = schedule.get("gamma")
        gam = None if gam is None else np.ascontiguousarray(gam, dtype=np.float32)
        ep, ea, eb = _extra_arrays(schedule.get("extra_pairs"))
        s = Schedule(worker.size, _i32p(worker), _i32p(nbr), _i32p(tau), None,
                     None if gam is None else gam.ctypes.data_as(C.POINTER(C.c_float)),
                     None if ep is None else ep.ctypes.data_as(C.POINTER(C.c_int64)), _i32p(ea), _i32p(eb),
                     int(schedule.get("lookahead", 0)))
        callback, raised = _gradient_trampoline(gradient_fn)
        rc = lib().adpsgd_run_events_with(self._h, C.byref(s), callback, None)
        if raised:
            raise raised[0]
        _check(self._h, rc)

    def run_sync_steps(self, steps, batch_idx=None, gamma=None, weights=None, loss_ptr=None):
        """steps iterations of the synchronous comparison schedule; batch_idx (steps, n, M);
        weights = (w_self, w_edge) or None for Metropolis weights."""
        fp = lambda a: None if a is None else a.ctypes.data_as(C.POINTER(C.c_float))
        batch = _as_i32(batch_idx)
        gam = None if gamma is None else np.ascontiguousarray(gamma, dtype=np.float32)
        ws = we = None
        if weights is not None:
            ws = np.ascontiguousarray(weights[0], dtype=np.float32)
            we = np.ascontiguousarray(weights[1], dtype=np.float32)
        s = SyncSchedule(steps, _i32p(batch), fp(gam), fp(ws), fp(we))
        _check(self._h, lib().adpsgd_run_sync_steps(self._h, C.byref(s), loss_ptr))

    def run_sync_steps_with(self, steps, gradient_fn, gamma=None, weights=None):
        """MODEL_EXTERNAL: the synchronous comparison schedule with gradient_fn as in run_events_with."""
        fp = lambda a: None if a is None else a.ctypes.data_as(C.POINTER(C.c_float))
        gam = None if gamma is None else np.ascontiguousarray(gamma, dtype=np.float32)
        ws = we = None
        if weights is not None:
            ws = np.ascontiguousarray(weights[0], dtype=np.float32)
            we = np.ascontiguousarray(weights[1], dtype=np.float32)
        s = SyncSchedule(steps, None, fp(gam), fp(ws), fp(we))
        callback, raised = _gradient_trampoline(gradient_fn)
        rc = lib().adpsgd_run_sync_steps_with(self._h, C.byref(s), callback, None)
        if raised:
            raise raised[0]
        _check(self._h, rc)

    def get_event_count(self):
        out = C.c_uint64(0)
        _check(self._h, lib().adpsgd_get_event_count(self._h, C.byref(out)))
        return out.value

    def set_event_count(self, events):
        _check(self._h, lib().adpsgd_set_event_count(self._h, events))

    def get_models(self, out=None, ld_out=None, on_device=False):
        if on_device:
            _check(self._h, lib().adpsgd_get_models(self._h, out, ld_out, 1))
            return None
        res = np.empty((self.n, self.d), dtype=np.float32)
        _check(self._h, lib().adpsgd_get_models(self._h, res.ctypes.data, self.d, 0))
        return res

    def get_bf16_models(self):
        res = np.empty((self.n, self.d), dtype=np.uint16)
        _check(self._h, lib().adpsgd_get_bf16_models(self._h, res.ctypes.data, self.d, 0))
        return res

    def get_momentum(self):
        res = np.empty((self.n, self.d), dtype=np.float32)
        _check(self._h, lib().adpsgd_get_momentum(self._h, res.ctypes.data, self.d, 0))
        return res

    def get_mean_model(self):
        res = np.empty(self.d, dtype=np.float32)
        _check(self._h, lib().adpsgd_get_mean_model(self._h, res.ctypes.data, 0))
        return res

    def mean_model_to_device(self, out_device_ptr):
        """The mean model into d floats of device memory, enqueued on the handle's stream (no wait)."""
        _check(self._h, lib().adpsgd_get_mean_model(self._h, out_device_ptr, 1))

    def objective(self, x_ptr=None, p=None):
        """f at a device vector (integer pointer), or at the mean model when x_ptr is None; p: the workers'
        probabilities (default 1 / n)."""
        out = C.c_double(0.0)
        if p is None:
            _check(self._h, lib().adpsgd_objective(self._h, x_ptr, C.byref(out)))
        else:
            p = np.ascontiguousarray(p, dtype=np.float64)
            if p.shape != (self.n,):
                raise ValueError("p must have one entry per worker")
            _check(self._h, lib().adpsgd_objective_weighted(self._h, x_ptr, p.ctypes.data_as(C.POINTER(C.c_double)), C.byref(out)))
        return out.value

    def classification_error(self, x_ptr=None):
        """Fraction of the local samples misclassified at a device vector, or at the mean model."""
        out = C.c_double(0.0)
        _check(self._h, lib().adpsgd_classification_error(self._h, x_ptr, C.byref(out)))
        return out.value

    def count_nonfinite(self):
        out = C.c_int64(0)
        _check(self._h, lib().adpsgd_count_nonfinite(self._h, C.byref(out)))
        return out.value

    def consensus_distance(self, p=None):
        """(1/n) sum_i |mean - x^i|^2, or sum_i p_i |mean - x^i|^2 with update probabilities p."""
        out = C.c_double(0.0)
        if p is None:
            _check(self._h, lib().adpsgd_consensus_distance(self._h, C.byref(out)))
        else:
            p = np.ascontiguousarray(p, dtype=np.float64)
            if p.shape != (self.n,):
                raise ValueError("p must have one entry per worker")
            _check(self._h, lib().adpsgd_consensus_distance_weighted(self._h, p.ctypes.data_as(C.POINTER(C.c_double)), C.byref(out)))
        return out.value

    def consensus_distance_static(self, out_device_ptr, p=None):
        """The consensus distance without any allocation by the library: the result (one double) is written to
        the device address out_device_ptr, asynchronously on the handle's stream."""
        pp = None
        if p is not None:
            p = np.ascontiguousarray(p, dtype=np.float64)
            if p.shape != (self.n,):
                raise ValueError("p must have one entry per worker")
            pp = p.ctypes.data_as(C.POINTER(C.c_double))
        _check(self._h, lib().adpsgd_consensus_distance_static(self._h, pp, out_device_ptr))

    def get_stats(self):
        st = Stats()
        _check(self._h, lib().adpsgd_get_stats(self._h, C.byref(st)))
        return {name: getattr(st, name) for name, _ in Stats._fields_}
