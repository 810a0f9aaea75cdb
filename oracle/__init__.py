"""AD-PSGD serial CPU oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.

Thin ctypes wrapper around ``adpsgd_oracle.c`` (plain C, one thread).  Only the
tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import this
package; the HIP library never does, and this package never imports the HIP
library.  Argument marshalling only: all arithmetic is in the C file, each
function of which names the passage of the paper it follows (Algorithm 1 and
the matrix form of the update at the start of the theory section).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "adpsgd_oracle.c"
_LIB = _HERE / "liboracle.so"

MODEL_LSQ, MODEL_LOGREG, MODEL_SYNTH, MODEL_MLP = 0, 1, 2, 3


def build(force: bool = False) -> Path:
    """Compile the oracle with gcc.  No contraction of a*b+c into an FMA: the
    three elementwise operations of an event keep their separate roundings."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(".so.tmp%d" % os.getpid())
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fPIC",
             "-shared", "-o", str(tmp), str(_SRC), "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(str(build()))
        _lib.oracle_minibatch_gradient.restype = C.c_double
        _lib.oracle_consensus_distance.restype = C.c_double
        _lib.oracle_consensus_distance_weighted.restype = C.c_double
        _lib.oracle_count_misclassified.restype = C.c_int64
    return _lib


def _p(a, ty):
    return None if a is None else a.ctypes.data_as(C.POINTER(ty))


def philox4x32_10(ctr, key):
    c = np.ascontiguousarray(ctr, dtype=np.uint32)
    k = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().oracle_philox4x32_10(_p(c, C.c_uint32), _p(k, C.c_uint32), _p(out, C.c_uint32))
    return out


def make_schedule(graph, K, seed=0, k_begin=0, T_max=0, tau_mode=0, weight=None,
                  tau_num=None, tau_den=None, M=0, rows=None, piece_of_run=False):
    """Random choices of Algorithm 1 for K events: worker i_k, neighbour j_k,
    staleness tau_k and the M minibatch indices.  ``graph`` = (rowptr, col)."""
    rowptr = np.ascontiguousarray(graph[0], dtype=np.int32)
    col = np.ascontiguousarray(graph[1], dtype=np.int32)
    n = rowptr.size - 1
    i32 = lambda a: None if a is None else np.ascontiguousarray(a, dtype=np.int32)
    weight, tau_num, tau_den, rows = i32(weight), i32(tau_num), i32(tau_den), i32(rows)
    if M > 0 and rows is None:
        raise ValueError("rows (local sample counts) needed when M > 0")
    worker = np.zeros(K, dtype=np.int32)
    nbr = np.zeros(K, dtype=np.int32)
    tau = np.zeros(K, dtype=np.int32)
    batch = np.zeros((K, M), dtype=np.int32) if M > 0 else None
    rc = lib().oracle_make_schedule(
        C.c_int32(n), _p(rowptr, C.c_int32), _p(col, C.c_int32), _p(weight, C.c_int32),
        C.c_int32(tau_mode), C.c_int32(T_max), _p(tau_num, C.c_int32), _p(tau_den, C.c_int32),
        C.c_int32(M), _p(rows, C.c_int32), C.c_uint64(seed), C.c_uint64(k_begin), C.c_int64(K),
        _p(worker, C.c_int32), _p(nbr, C.c_int32), _p(tau, C.c_int32), _p(batch, C.c_int32),
        C.c_int32(1 if piece_of_run else 0))
    if rc != 0:
        raise ValueError("oracle_make_schedule: bad argument")
    return {"worker": worker, "neighbour": nbr, "tau": tau, "batch_idx": batch}


def synth_grad(seed, k, std, coords):
    coords = np.ascontiguousarray(coords, dtype=np.int64)
    g = np.zeros(coords.size, dtype=np.float32)
    lib().oracle_synth_grad(C.c_uint64(seed), C.c_uint64(k), C.c_double(std),
                            C.c_int64(coords.size), _p(coords, C.c_int64), _p(g, C.c_float))
    return g


def round_bf16(x):
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty_like(x)
    lib().oracle_round_bf16(C.c_int64(x.size), _p(x, C.c_float), _p(out, C.c_float))
    return out


def _ptr_array(arrs):
    arr = (C.c_void_p * len(arrs))()
    for t, a in enumerate(arrs):
        arr[t] = a.ctypes.data
    return arr


def minibatch_gradient(model, xhat, features, targets, idx, gscale, lam=0.0, mlp=(0, 0, 0)):
    """g = gscale * sum_m grad F(xhat; xi_m) for one worker's data; returns (g, loss)."""
    xhat = np.ascontiguousarray(xhat, dtype=np.float32)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    assert features.flags.c_contiguous and targets.flags.c_contiguous
    g = np.zeros(xhat.size, dtype=np.float32)
    loss = lib().oracle_minibatch_gradient(
        C.c_int(model), C.c_int64(xhat.size), C.c_int(idx.size), C.c_double(gscale), C.c_double(lam),
        C.c_int(mlp[0]), C.c_int(mlp[1]), C.c_int(mlp[2]), _p(xhat, C.c_float),
        C.c_void_p(features.ctypes.data), C.c_int64(features.shape[1]),
        C.c_void_p(targets.ctypes.data), _p(idx, C.c_int32), _p(g, C.c_float))
    return g, loss


def count_misclassified(model, x, features, targets, mlp=(0, 0, 0)):
    """Rows of one worker's data whose predicted label (sign of a.x, or the largest logit of the
    perceptron) differs from the target."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    assert features.flags.c_contiguous and targets.flags.c_contiguous
    wrong = lib().oracle_count_misclassified(
        C.c_int(model), C.c_int64(x.size), C.c_int(mlp[0]), C.c_int(mlp[1]), C.c_int(mlp[2]), _p(x, C.c_float),
        C.c_void_p(features.ctypes.data), C.c_int64(features.shape[1]), C.c_void_p(targets.ctypes.data),
        C.c_int64(features.shape[0]))
    if wrong < 0:
        raise ValueError("count_misclassified: the model has no labels")
    return int(wrong)


def run_events(X, schedule, model, gamma, *, M=0, gscale=1.0, lam=0.0, mlp=(0, 0, 0),
               features=None, targets=None, gamma_k=None, synth_std=0.0, synth_seed=0,
               event_base=0, coords=None, mode=1, want_loss=False, want_g=False,
               momentum=0.0, weight_decay=0.0, V=None, extra_pairs=None, local_compensation=False):
    """Run the events of ``schedule`` on X (n x d fp32, C-contiguous) IN PLACE.

    mode 0 = literal snapshot history, mode 1 = parked gradients (same values).
    V (n x d fp32, updated in place) switches to the momentum / weight-decay form of the update.
    extra_pairs = (ptr[K+1], a[], b[]): further disjoint pairs averaged by W_k in event k.
    local_compensation: the wait-free variant (a worker applies its own pending gradient to the
    copy it reads before computing the next one).
    Returns a dict with optional 'loss' (K,) and 'g' (K, d)."""
    assert X.dtype == np.float32 and X.flags.c_contiguous and X.ndim == 2
    n, d = X.shape
    worker = np.ascontiguousarray(schedule["worker"], dtype=np.int32)
    nbr = np.ascontiguousarray(schedule["neighbour"], dtype=np.int32)
    tau = np.ascontiguousarray(schedule["tau"], dtype=np.int32)
    K = worker.size
    batch = schedule.get("batch_idx")
    if batch is not None:
        batch = np.ascontiguousarray(batch, dtype=np.int32)
    fptr = ldf = tptr = None
    keep = []
    if model != MODEL_SYNTH:
        assert features is not None and targets is not None and batch is not None
        assert batch.shape == (K, M)
        for f in features:
            assert f.flags.c_contiguous and f.ndim == 2
        keep = [list(features), list(targets)]
        fptr = _ptr_array(features)
        tptr = _ptr_array(targets)
        ldf = np.array([f.shape[1] for f in features], dtype=np.int64)
    if coords is not None:
        coords = np.ascontiguousarray(coords, dtype=np.int64)
        assert coords.size == d
    gk = None if gamma_k is None else np.ascontiguousarray(gamma_k, dtype=np.float32)
    if V is not None:
        assert V.dtype == np.float32 and V.flags.c_contiguous and V.shape == X.shape
    eptr = ea = eb = None
    if extra_pairs is not None:
        eptr = np.ascontiguousarray(extra_pairs[0], dtype=np.int64)
        ea = np.ascontiguousarray(extra_pairs[1], dtype=np.int32)
        eb = np.ascontiguousarray(extra_pairs[2], dtype=np.int32)
        assert eptr.size == K + 1 and ea.size == eb.size == eptr[-1]
    loss = np.zeros(K, dtype=np.float64) if want_loss else None
    glog = np.zeros((K, d), dtype=np.float32) if want_g else None
    rc = lib().oracle_run_events(
        C.c_int32(n), C.c_int64(d), _p(X, C.c_float), C.c_int64(d), C.c_int(model), C.c_int(M),
        C.c_double(gscale), C.c_double(lam), C.c_int(mlp[0]), C.c_int(mlp[1]), C.c_int(mlp[2]),
        fptr, _p(ldf, C.c_int64), tptr, C.c_float(gamma), _p(gk, C.c_float),
        C.c_double(synth_std), C.c_uint64(synth_seed), C.c_uint64(event_base),
        _p(coords, C.c_int64), C.c_int64(K), _p(worker, C.c_int32), _p(nbr, C.c_int32),
        _p(tau, C.c_int32), _p(batch, C.c_int32), C.c_int(mode), _p(loss, C.c_double),
        _p(glog, C.c_float), C.c_float(momentum), C.c_float(weight_decay), _p(V, C.c_float),
        C.c_int64(d), _p(eptr, C.c_int64), _p(ea, C.c_int32), _p(eb, C.c_int32),
        C.c_int(1 if local_compensation else 0))
    del keep
    if rc != 0:
        raise ValueError("oracle_run_events failed with code %d" % rc)
    return {"loss": loss, "g": glog}


def run_sync_steps(X, batch_idx, W, model, gamma, *, M=0, gscale=1.0, lam=0.0, mlp=(0, 0, 0),
                   features=None, targets=None, gamma_s=None, synth_std=0.0, synth_seed=0,
                   event_base=0, coords=None, steps=None, want_loss=False, want_g=False,
                   momentum=0.0, weight_decay=0.0, V=None):
    """Synchronous comparison schedule (D-PSGD): X <- W X - gamma G(X), IN PLACE, for ``steps``
    iterations (default: batch_idx.shape[0]).  batch_idx is (S, n, M); W is n x n, symmetric and
    doubly stochastic.  With V (n x d momentum buffers, updated in place) the step uses the
    experiments' optimizer on the mixed model.  Returns a dict with optional 'loss' (S, n) and
    'g' (S, n, d)."""
    assert X.dtype == np.float32 and X.flags.c_contiguous and X.ndim == 2
    n, d = X.shape
    W = np.ascontiguousarray(W, dtype=np.float32)
    assert W.shape == (n, n)
    fptr = ldf = tptr = None
    keep = []
    if model != MODEL_SYNTH:
        batch_idx = np.ascontiguousarray(batch_idx, dtype=np.int32)
        S = batch_idx.shape[0] if steps is None else steps
        assert batch_idx.shape == (S, n, M)
        for f in features:
            assert f.flags.c_contiguous and f.ndim == 2
        keep = [list(features), list(targets)]
        fptr = _ptr_array(features)
        tptr = _ptr_array(targets)
        ldf = np.array([f.shape[1] for f in features], dtype=np.int64)
    else:
        S = steps
        batch_idx = None
    if coords is not None:
        coords = np.ascontiguousarray(coords, dtype=np.int64)
        assert coords.size == d
    gs = None if gamma_s is None else np.ascontiguousarray(gamma_s, dtype=np.float32)
    if V is not None:
        assert V.dtype == np.float32 and V.flags.c_contiguous and V.shape == X.shape
    loss = np.zeros((S, n), dtype=np.float64) if want_loss else None
    glog = np.zeros((S, n, d), dtype=np.float32) if want_g else None
    rc = lib().oracle_run_sync_steps(
        C.c_int32(n), C.c_int64(d), _p(X, C.c_float), C.c_int64(d), C.c_int(model), C.c_int(M),
        C.c_double(gscale), C.c_double(lam), C.c_int(mlp[0]), C.c_int(mlp[1]), C.c_int(mlp[2]),
        fptr, _p(ldf, C.c_int64), tptr, C.c_float(gamma), _p(gs, C.c_float),
        C.c_double(synth_std), C.c_uint64(synth_seed), C.c_uint64(event_base),
        _p(coords, C.c_int64), C.c_int64(S), _p(batch_idx, C.c_int32), _p(W, C.c_float),
        _p(loss, C.c_double), _p(glog, C.c_float), C.c_float(momentum), C.c_float(weight_decay), _p(V, C.c_float))
    del keep
    if rc != 0:
        raise ValueError("oracle_run_sync_steps failed with code %d" % rc)
    return {"loss": loss, "g": glog}


def metropolis_weights(graph):
    rowptr = np.ascontiguousarray(graph[0], dtype=np.int32)
    col = np.ascontiguousarray(graph[1], dtype=np.int32)
    n = rowptr.size - 1
    W = np.zeros((n, n), dtype=np.float32)
    if lib().oracle_metropolis_weights(C.c_int32(n), _p(rowptr, C.c_int32), _p(col, C.c_int32), _p(W, C.c_float)) != 0:
        raise ValueError("oracle_metropolis_weights: bad graph")
    return W


def mean_model(X):
    n, d = X.shape
    out = np.zeros(d, dtype=np.float64)
    lib().oracle_mean_model(C.c_int32(n), C.c_int64(d), _p(X, C.c_float), C.c_int64(X.strides[0] // 4),
                            _p(out, C.c_double))
    return out


def consensus_distance(X):
    n, d = X.shape
    return lib().oracle_consensus_distance(C.c_int32(n), C.c_int64(d), _p(X, C.c_float),
                                           C.c_int64(X.strides[0] // 4))


def consensus_distance_weighted(X, p):
    """sum_i p_i |mean - x^i|^2 with the workers' update probabilities p (the definition of the proofs appendix)."""
    n, d = X.shape
    p = np.ascontiguousarray(p, dtype=np.float64)
    assert p.shape == (n,)
    return lib().oracle_consensus_distance_weighted(C.c_int32(n), C.c_int64(d), _p(X, C.c_float), C.c_int64(d),
                                                    _p(p, C.c_double))
