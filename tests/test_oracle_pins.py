"""Pins for the CPU oracle: everything the paper and the mathematics fix about
AD-PSGD's per-event update, checked against the oracle alone (no GPU).

Each test is chosen so that a plausible mistake in the oracle (a dropped term, a
wrong sign or index, a transposed operand, reading the wrong snapshot) fails it.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from workloads import ring_graph, random_regular4_graph, lsq_data, logreg_data

LSQ, LOGREG, SYNTH, MLP = oracle.MODEL_LSQ, oracle.MODEL_LOGREG, oracle.MODEL_SYNTH, oracle.MODEL_MLP


# --------------------------------------------------------------------------- generator
def test_philox_known_answers(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "philox4x32_10_kat.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        w = [int(t, 16) for t in r]
        out = oracle.philox4x32_10(w[0:4], w[4:6])
        assert [int(v) for v in out] == w[6:10]


def test_schedule_ranges_and_laws():
    n, K, M, T = 8, 40000, 4, 3
    g = ring_graph(n)
    rows = np.arange(10, 10 + n)
    s = oracle.make_schedule(g, K, seed=5, T_max=T, M=M, rows=rows)
    w, j, tau, b = s["worker"], s["neighbour"], s["tau"], s["batch_idx"]
    assert w.min() == 0 and w.max() == n - 1
    # neighbour is a ring neighbour of the worker
    assert np.all((j == (w - 1) % n) | (j == (w + 1) % n))
    # staleness within bounds and never beyond the events available
    assert tau.min() == 0 and tau.max() == T and np.all(tau <= np.arange(K))
    # minibatch indices address the worker's own rows
    assert np.all(b >= 0) and np.all(b < rows[w][:, None])
    # uniform laws (5-sigma binomial bands)
    for counts, p in ((np.bincount(w, minlength=n), 1 / n),
                      (np.bincount(tau[100:], minlength=T + 1), 1 / (T + 1))):
        tot = counts.sum()
        assert np.all(np.abs(counts - tot * p) < 5 * np.sqrt(tot * p * (1 - p)))
    left = np.mean(j == (w - 1) % n)
    assert abs(left - 0.5) < 5 * 0.5 / np.sqrt(K)
    # events are a pure function of (seed, k): a later window repeats the same draws
    s2 = oracle.make_schedule(g, 100, seed=5, k_begin=1000, T_max=T, M=M, rows=rows)
    assert np.array_equal(s2["worker"], w[1000:1100])
    assert np.array_equal(s2["neighbour"], j[1000:1100])
    assert np.array_equal(s2["batch_idx"], b[1000:1100])
    assert np.array_equal(s2["tau"][T:], tau[1000 + T:1100])
    # a different seed gives a different stream
    s3 = oracle.make_schedule(g, K, seed=6, T_max=T, M=M, rows=rows)
    assert np.mean(s3["worker"] == w) < 0.2


def test_schedule_weighted_workers_and_geometric_staleness():
    n, K = 6, 60000
    g = random_regular4_graph(n, seed=1)
    weight = np.array([10, 10, 1, 10, 1, 10])
    num = np.where(weight == 1, 20, 2)
    den = np.where(weight == 1, 21, 3)
    s = oracle.make_schedule(g, K, seed=3, T_max=400, tau_mode=1, weight=weight,
                             tau_num=num, tau_den=den)
    w, tau = s["worker"], s["tau"]
    p = weight / weight.sum()
    counts = np.bincount(w, minlength=n)
    assert np.all(np.abs(counts - K * p) < 5 * np.sqrt(K * p * (1 - p)))
    # P(tau >= t) = q^t  =>  mean q / (1 - q): 2 for the fast class, 20 for the slow one
    late = np.arange(K) > 2000
    fast, slow = tau[late & (weight[w] == 10)], tau[late & (weight[w] == 1)]
    assert abs(fast.mean() - 2.0) < 5 * np.sqrt(6.0 / fast.size)       # var = q/(1-q)^2 = 6
    assert abs(slow.mean() - 20.0) < 5 * np.sqrt(420.0 / slow.size)    # var = 420
    assert abs(np.mean(fast >= 3) - (2 / 3) ** 3) < 0.01
    # cap
    s = oracle.make_schedule(g, 5000, seed=3, T_max=7, tau_mode=1, weight=weight,
                             tau_num=num, tau_den=den)
    assert s["tau"].max() == 7


def test_synthetic_gradient_is_standard_normal():
    from scipy import stats
    coords = np.arange(200000)
    z = oracle.synth_grad(7, 3, 1.0, coords).astype(np.float64)
    assert abs(z.mean()) < 5 / np.sqrt(z.size)
    assert abs(z.var() - 1.0) < 5 * np.sqrt(2.0 / z.size)
    assert stats.kstest(z, "norm").pvalue > 1e-3
    assert abs(stats.kurtosis(z)) < 0.1
    # the four values of one generator call, and neighbouring events, are uncorrelated
    q = z.reshape(-1, 4)
    c = np.corrcoef(q.T)
    assert np.max(np.abs(c - np.eye(4))) < 0.03
    z2 = oracle.synth_grad(7, 4, 1.0, coords).astype(np.float64)
    assert abs(np.corrcoef(z, z2)[0, 1]) < 0.02
    # scaling by std and addressing by coordinate: a subset reproduces the same entries
    sub = np.array([5, 17, 4096, 199999])
    assert np.array_equal(oracle.synth_grad(7, 3, 1.0, sub), z[sub].astype(np.float32))
    g = oracle.synth_grad(7, 3, 0.25, coords)
    assert np.allclose(g, 0.25 * z, rtol=1e-6, atol=0)


# --------------------------------------------------------------------------- gradients
def test_lsq_gradient_matches_normal_equations():
    rng = np.random.default_rng(0)
    rows, d, M = 50, 33, 16
    A = rng.standard_normal((rows, d)).astype(np.float32)
    b = rng.standard_normal(rows).astype(np.float32)
    x = rng.standard_normal(d).astype(np.float32)
    idx = rng.integers(0, rows, M)
    g, loss = oracle.minibatch_gradient(LSQ, x, A, b, idx, 1.0 / M)
    Ab, bb = A[idx].astype(np.float64), b[idx].astype(np.float64)
    r = Ab @ x.astype(np.float64) - bb
    assert np.allclose(g, Ab.T @ r / M, rtol=1e-6, atol=1e-6)
    assert np.isclose(loss, 0.5 * np.mean(r * r), rtol=1e-12)
    # the paper's literal sum over the minibatch is M times the mean
    gs, ls = oracle.minibatch_gradient(LSQ, x, A, b, idx, 1.0)
    assert np.allclose(gs, M * (Ab.T @ r / M), rtol=1e-6, atol=1e-5)


def test_logreg_loss_and_gradient():
    rng = np.random.default_rng(1)
    rows, d, M, lam = 40, 21, 12, 0.3
    A = rng.standard_normal((rows, d)).astype(np.float32)
    y = np.where(rng.standard_normal(rows) > 0, 1.0, -1.0).astype(np.float32)
    x = (0.5 * rng.standard_normal(d)).astype(np.float32)
    idx = rng.integers(0, rows, M)
    g, loss = oracle.minibatch_gradient(LOGREG, x, A, y, idx, 1.0 / M, lam=lam)
    x64 = x.astype(np.float64)
    margins = y[idx] * (A[idx].astype(np.float64) @ x64)
    assert np.isclose(loss, np.mean(np.logaddexp(0.0, -margins)) + 0.5 * lam * x64 @ x64, rtol=1e-12)

    # the gradient is the derivative of the returned loss: central differences
    def loss_at(v):
        return oracle.minibatch_gradient(LOGREG, v.astype(np.float32), A, y, idx, 1.0 / M, lam=lam)[1]
    h = 2.0 ** -8          # exactly representable steps so that x +- h e is exact in fp32
    xq = np.round(x * 256) / 256
    gq, _ = oracle.minibatch_gradient(LOGREG, xq.astype(np.float32), A, y, idx, 1.0 / M, lam=lam)
    for e in range(d):
        step = np.zeros(d)
        step[e] = h
        fd = (loss_at(xq + step) - loss_at(xq - step)) / (2 * h)
        assert abs(fd - gq[e]) < 1e-4


def test_mlp_gradient_matches_autograd_with_same_roundings():
    torch = pytest.importorskip("torch")
    from workloads import mixture_data, mlp_init, bf16_bits_to_f32
    I, H, O, M, rows = 20, 24, 5, 8, 30
    feats, labels, _ = mixture_data(1, rows, din=I, classes=O, seed=2)
    x0 = mlp_init(I, H, O, seed=2)
    rng = np.random.default_rng(3)
    x0 = (x0 + 0.05 * rng.standard_normal(x0.size)).astype(np.float32)   # non-zero biases
    idx = rng.integers(0, rows, M)
    g, loss = oracle.minibatch_gradient(MLP, x0, feats[0], labels[0], idx, 1.0 / M, mlp=(I, H, O))

    def bf(t):   # round-to-nearest-even to bf16, kept in fp64
        return t.to(torch.float32).to(torch.bfloat16).to(torch.float64)

    class RoundGrad(torch.autograd.Function):      # identity forward, bf16-rounded backward
        @staticmethod
        def forward(ctx, t):
            return t
        @staticmethod
        def backward(ctx, gr):
            return bf(gr)

    p = torch.tensor(bf16_round_np(x0), dtype=torch.float64, requires_grad=True)
    W1 = p[:I * H].view(I, H); b1 = p[I * H:I * H + H]
    W2 = p[I * H + H:I * H + H + H * O].view(H, O); b2 = p[I * H + H + H * O:]
    Xb = torch.tensor(bf16_bits_to_f32(feats[0][idx]), dtype=torch.float64)
    pre = (Xb @ W1 + b1).to(torch.float32).to(torch.float64)
    pre = RoundGrad.apply(pre)
    hid = torch.relu(pre)
    hid = hid + (bf(hid) - hid).detach()           # forward sees the bf16-rounded activation
    logits = hid @ W2 + b2
    lt = torch.nn.functional.cross_entropy(logits, torch.tensor(labels[0][idx], dtype=torch.long),
                                           reduction="mean")
    lt.backward()
    ref = p.grad.numpy()
    assert np.isclose(loss, lt.item(), rtol=1e-9)
    # layer-2 and bias terms agree to rounding; layer-1 terms agree up to the bf16 rounding of
    # the back-propagated error (the oracle rounds after the 1/M scale, autograd before it is
    # scaled identically, so they agree exactly too)
    assert np.allclose(g, ref, rtol=2e-6, atol=1e-7)


def bf16_round_np(x):
    return oracle.round_bf16(x)


def test_classification_error_counts():
    """Predicted labels.  Logistic regression against numpy (sign of a.x, zero counts as +1).  The perceptron:
    a hand-made 2-2-2 network whose logits are relu(x) (prediction = index of the larger positive input,
    class 0 on ties), and the link to the loss on random data: a sample whose cross-entropy is below
    ln 2 has more than half of the probability on its label, so it cannot be counted as misclassified,
    and one whose loss exceeds ln(number of classes) has less than the uniform share, so it must be."""
    from workloads import mixture_data, mlp_init, f32_to_bf16_bits
    feats, targs, _ = logreg_data(1, 200, 33, seed=9)
    x = np.random.default_rng(2).standard_normal(33).astype(np.float32)
    want = int((np.where(feats[0].astype(np.float64) @ x.astype(np.float64) >= 0, 1.0, -1.0) != targs[0]).sum())
    assert 0 < want < 200 and oracle.count_misclassified(LOGREG, x, feats[0], targs[0]) == want
    assert oracle.count_misclassified(LOGREG, np.zeros(33, np.float32), feats[0], targs[0]) == int((targs[0] < 0).sum())
    with pytest.raises(ValueError):
        oracle.count_misclassified(LSQ, x, feats[0], targs[0])
    # W1 = I, b1 = 0, W2 = I, b2 = 0
    net = np.array([1, 0, 0, 1, 0, 0, 1, 0, 0, 1, 0, 0], np.float32)
    pts = np.array([[2.0, 1.0], [1.0, 2.0], [-1.0, -3.0], [0.5, 0.5], [-1.0, 0.25], [3.0, -1.0]], np.float32)
    predicted = np.array([0, 1, 0, 0, 1, 0], np.int32)
    xin = f32_to_bf16_bits(pts)
    assert oracle.count_misclassified(MLP, net, xin, predicted, mlp=(2, 2, 2)) == 0
    for flip in range(len(pts)):
        labels = predicted.copy()
        labels[flip] ^= 1
        assert oracle.count_misclassified(MLP, net, xin, labels, mlp=(2, 2, 2)) == 1
    # link to the loss
    dims = (8, 16, 4)
    f, lab, _ = mixture_data(1, 120, din=dims[0], classes=dims[2], seed=3)
    w = mlp_init(*dims, seed=3) * np.float32(3.0)
    losses = np.array([oracle.minibatch_gradient(MLP, w, f[0], lab[0], np.array([r]), 1.0, mlp=dims)[1] for r in range(120)])
    per_row = np.array([oracle.count_misclassified(MLP, w, f[0][r:r + 1], lab[0][r:r + 1], mlp=dims) for r in range(120)])
    assert oracle.count_misclassified(MLP, w, f[0], lab[0], mlp=dims) == per_row.sum()
    assert (losses < np.log(2)).any() and (losses > np.log(dims[2])).any()
    assert not per_row[losses < np.log(2)].any() and per_row[losses > np.log(dims[2])].all()


def test_bf16_rounding_is_nearest_even():
    import torch
    rng = np.random.default_rng(4)
    x = np.concatenate([rng.standard_normal(5000), [0.0, 1.0, 1.00390625, 1.01171875, -3.0e38, 1e-40]]
                       ).astype(np.float32)
    ref = torch.tensor(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(oracle.round_bf16(x), ref)


# --------------------------------------------------------------------------- the event
def _unit_quadratic_data(n, diag):
    """f_i(x) = sum_e diag[e] x_e^2 / 2 written as least squares: row e = sqrt(diag[e]) e_e, b = 0;
    a 'minibatch' listing every row once with scale 1 is the full gradient diag * x."""
    d = len(diag)
    A = np.diag(np.sqrt(np.asarray(diag, dtype=np.float64))).astype(np.float32)
    b = np.zeros(d, dtype=np.float32)
    return [A] * n, [b] * n


def test_hand_expanded_two_workers(golden_dir):
    cases = [l.split() for l in open(os.path.join(golden_dir, "alg1_two_workers_d1.txt"))
             if l.strip() and not l.startswith("#")]
    feats, targs = _unit_quadratic_data(2, [1.0])
    for name, i0, j0, t0, i1, j1, t1, e0, e1 in cases:
        for mode in (0, 1):
            X = np.array([[1.0], [3.0]], dtype=np.float32)
            sched = {"worker": [int(i0), int(i1)], "neighbour": [int(j0), int(j1)],
                     "tau": [int(t0), int(t1)], "batch_idx": np.zeros((2, 1), np.int32)}
            oracle.run_events(X, sched, LSQ, 0.5, M=1, gscale=1.0, features=feats, targets=targs, mode=mode)
            assert X[0, 0] == float(e0) and X[1, 0] == float(e1), name


def test_waitfree_hand_expanded(golden_dir):
    """Local compensation of the wait-free variant: values worked out by hand in the fixture."""
    cases = [l.split() for l in open(os.path.join(golden_dir, "waitfree_two_workers_d1.txt"))
             if l.strip() and not l.startswith("#")]
    feats, targs = _unit_quadratic_data(2, [1.0])
    assert len(cases) == 3
    for c in cases:
        name, comp, K = c[0], int(c[1]), int(c[2])
        taus = [int(t) for t in c[3:3 + K]]
        e0, e1 = float(c[3 + K]), float(c[4 + K])
        for mode in (0, 1):
            X = np.array([[1.0], [3.0]], dtype=np.float32)
            sched = {"worker": [0] * K, "neighbour": [1] * K, "tau": taus,
                     "batch_idx": np.zeros((K, 1), np.int32)}
            oracle.run_events(X, sched, LSQ, 0.5, M=1, gscale=1.0, features=feats, targets=targs,
                              mode=mode, local_compensation=bool(comp))
            assert (X[0, 0], X[1, 0]) == (e0, e1), (name, mode, X.ravel())


def test_waitfree_compensation_with_momentum_uses_the_buffered_gradient():
    """The computation thread of the wait-free appendix holds the buffered gradient g and the step size,
    nothing of the optimizer: its compensation stays  x - gamma g  when the update itself uses momentum.
    One worker, f(x) = x^2 / 2 (gradient x), gamma = mu = 1/2, x_0 = 1, tau = (0, 1, 1), by hand:
      event 0: g = 1,    v = 1,    x = 1/2
      event 1: reads 1,   compensated with g_0: 1/2;  g = 1/2;  v = 1/2 + 1/2 = 1;  x = 1/2 - 1/2 = 0
      event 2: reads 1/2, compensated with g_1: 1/4;  g = 1/4;  v = 1/2 + 1/4 = 3/4;  x = 0 - 3/8 = -3/8
    (compensating with gamma v_1 instead would read 0 and end at -1/4; without compensation event 1 has
    g = 1, v = 3/2, x = -1/4 and event 2 has g = 1/2, v = 5/4, x = -7/8)."""
    feats, targs = _unit_quadratic_data(1, [1.0])
    sched = {"worker": [0, 0, 0], "neighbour": [0, 0, 0], "tau": [0, 1, 1], "batch_idx": np.zeros((3, 1), np.int32)}
    for comp, want_x, want_v in ((True, -0.375, 0.75), (False, -0.875, 1.25)):
        for mode in (0, 1):
            X, V = np.array([[1.0]], np.float32), np.zeros((1, 1), np.float32)
            oracle.run_events(X, sched, LSQ, 0.5, M=1, gscale=1.0, features=feats, targets=targs, mode=mode,
                              momentum=0.5, weight_decay=0.0, V=V, local_compensation=comp)
            assert (X[0, 0], V[0, 0]) == (want_x, want_v), (comp, mode, X, V)


@pytest.mark.parametrize("model", [LSQ, LOGREG])
def test_waitfree_single_worker_is_fresh_sgd(model):
    """One worker, no neighbour, every gradient one event stale: the compensated read
    X_{k-1} - gamma g_{k-1} IS X_k, so the wait-free variant must reproduce SGD without any
    staleness bit for bit, while plain Algorithm 1 with the same schedule must not."""
    d, rows, M, K = 24, 64, 4, 60
    if model == LSQ:
        feats, targs, _ = lsq_data(1, rows, d, seed=11)
    else:
        feats, targs, _ = logreg_data(1, rows, d, seed=11)
    rng = np.random.default_rng(5)
    batch = rng.integers(0, rows, size=(K, M)).astype(np.int32)
    X0 = rng.standard_normal((1, d)).astype(np.float32)
    base = {"worker": np.zeros(K, np.int32), "neighbour": np.zeros(K, np.int32), "batch_idx": batch}
    stale = dict(base, tau=np.array([0] + [1] * (K - 1), np.int32))
    fresh = dict(base, tau=np.zeros(K, np.int32))
    kw = dict(M=M, gscale=1.0 / M, lam=0.01, features=feats, targets=targs)
    ref = X0.copy()
    oracle.run_events(ref, fresh, model, 0.05, **kw)
    for mode in (0, 1):
        X = X0.copy()
        oracle.run_events(X, stale, model, 0.05, mode=mode, local_compensation=True, **kw)
        assert np.array_equal(X, ref)
        # with no staleness nothing is ever pending: the switch must change nothing
        X = X0.copy()
        oracle.run_events(X, fresh, model, 0.05, mode=mode, local_compensation=True, **kw)
        assert np.array_equal(X, ref)
    X = X0.copy()
    oracle.run_events(X, stale, model, 0.05, **kw)
    assert not np.array_equal(X, ref)


def test_waitfree_modes_agree_on_random_schedule():
    """Literal snapshot history and parked gradients give the same bits with compensation on,
    with per-event step sizes (the compensation uses the pending event's own gamma)."""
    n, d, rows, M, K = 6, 20, 32, 2, 300
    graph = ring_graph(n)
    feats, targs, _ = lsq_data(n, rows, d, seed=3)
    sched = oracle.make_schedule(graph, K, seed=17, T_max=5, tau_mode=0, M=M, rows=[rows] * n)
    gk = (0.02 + 0.01 * (np.arange(K) % 7)).astype(np.float32)
    rng = np.random.default_rng(2)
    X0 = rng.standard_normal((n, d)).astype(np.float32)
    out = []
    for mode in (0, 1):
        X = X0.copy()
        oracle.run_events(X, sched, LSQ, 0.0, M=M, gscale=1.0 / M, features=feats, targets=targs,
                          gamma_k=gk, mode=mode, local_compensation=True)
        out.append(X)
    assert np.array_equal(out[0], out[1])
    X = X0.copy()
    oracle.run_events(X, sched, LSQ, 0.0, M=M, gscale=1.0 / M, features=feats, targets=targs, gamma_k=gk)
    assert not np.array_equal(X, out[0])


def _matrix_form_bruteforce(X0, diag, gamma, sched):
    """X_{k+1} = X_k W_k - gamma dg(X^_k) in exact rational arithmetic, with W_k and dg as
    explicit matrices and the whole history kept (columns = workers, as in the paper)."""
    n = len(X0)
    d = len(X0[0])
    Xk = [[Fraction(X0[i][e]) for i in range(n)] for e in range(d)]      # d x n
    hist = []
    for k, (i, j, tau) in enumerate(zip(sched["worker"], sched["neighbour"], sched["tau"])):
        hist.append([row[:] for row in Xk])
        W = [[Fraction(int(a == b)) for b in range(n)] for a in range(n)]
        if i != j:
            for a in (i, j):
                for b in (i, j):
                    W[a][b] -= Fraction(1, 2) * (1 if a == b else -1)
        XW = [[sum(Xk[e][a] * W[a][b] for a in range(n)) for b in range(n)] for e in range(d)]
        old = hist[k - tau]
        dg = [[Fraction(0)] * n for _ in range(d)]
        for e in range(d):
            dg[e][i] = Fraction(diag[e]) * old[e][i]
        Xk = [[XW[e][b] - Fraction(gamma) * dg[e][b] for b in range(n)] for e in range(d)]
    return [[float(Xk[e][i]) for e in range(d)] for i in range(n)]


@pytest.mark.parametrize("n", [2, 3])
def test_bruteforce_matrix_form_d4(n):
    diag = [1.0, 4.0, 0.25, 16.0]
    gamma = 0.0625
    X0 = [[1.0, -2.0, 3.0, 0.5], [3.0, 1.0, -1.0, 2.0], [-4.0, 0.25, 8.0, -1.0]][:n]
    if n == 2:
        sched = {"worker": [0, 1, 1, 0, 1], "neighbour": [1, 0, 0, 1, 0], "tau": [0, 1, 2, 0, 3]}
    else:
        sched = {"worker": [0, 2, 1, 1, 0, 2], "neighbour": [1, 1, 0, 2, 2, 0], "tau": [0, 1, 0, 3, 2, 4]}
    expect = _matrix_form_bruteforce(X0, diag, gamma, sched)
    feats, targs = _unit_quadratic_data(n, diag)
    full = dict(sched, batch_idx=np.tile(np.arange(4, dtype=np.int32), (len(sched["tau"]), 1)))
    for mode in (0, 1):
        X = np.array(X0, dtype=np.float32)
        oracle.run_events(X, full, LSQ, gamma, M=4, gscale=1.0, features=feats, targets=targs, mode=mode)
        assert np.array_equal(X.astype(np.float64), np.array(expect)), mode   # dyadic values: exact


def _random_problem(n, d, rows, K, M, T, seed, model=LSQ):
    g = ring_graph(n) if seed % 2 == 0 else random_regular4_graph(max(n, 5), seed)
    n = len(g[0]) - 1
    if model == LSQ:
        feats, targs, _ = lsq_data(n, rows, d, seed=seed)
    else:
        feats, targs, _ = logreg_data(n, rows, d, seed=seed)
    sched = oracle.make_schedule(g, K, seed=seed, T_max=T, M=M, rows=np.full(n, rows))
    rng = np.random.default_rng(seed + 100)
    X0 = rng.standard_normal((n, d)).astype(np.float32)
    return n, feats, targs, sched, X0


@pytest.mark.parametrize("model,seed", [(LSQ, 0), (LSQ, 1), (LOGREG, 2), (LOGREG, 3)])
def test_literal_history_equals_parked_gradients(model, seed):
    n, feats, targs, sched, X0 = _random_problem(6, 19, 12, 300, 5, 7, seed, model)
    Xa, Xb = X0.copy(), X0.copy()
    ra = oracle.run_events(Xa, sched, model, 0.01, M=5, gscale=0.2, lam=0.01, features=feats,
                           targets=targs, mode=0, want_loss=True, want_g=True)
    rb = oracle.run_events(Xb, sched, model, 0.01, M=5, gscale=0.2, lam=0.01, features=feats,
                           targets=targs, mode=1, want_loss=True, want_g=True)
    assert np.array_equal(Xa, Xb)
    assert np.array_equal(ra["g"], rb["g"]) and np.array_equal(ra["loss"], rb["loss"])
    assert sched["tau"].max() == 7      # the stale path was exercised
    # and staleness matters: forcing tau = 0 changes the result
    Xc = X0.copy()
    oracle.run_events(Xc, dict(sched, tau=np.zeros_like(sched["tau"])), model, 0.01, M=5, gscale=0.2,
                      lam=0.01, features=feats, targets=targs, mode=0)
    assert not np.array_equal(Xa, Xc)


def test_zero_staleness_equals_naive_loop():
    """tau = 0 for every event: x^ is the worker's current row, read before the average."""
    n, feats, targs, sched, X0 = _random_problem(6, 17, 10, 200, 4, 0, 4)
    X = X0.copy()
    oracle.run_events(X, sched, LSQ, 0.02, M=4, gscale=0.25, features=feats, targets=targs, mode=0)
    Y = X0.copy()
    for k in range(200):
        i, j = sched["worker"][k], sched["neighbour"][k]
        g, _ = oracle.minibatch_gradient(LSQ, Y[i], feats[i], targs[i], sched["batch_idx"][k], 0.25)
        avg = (Y[i] + Y[j]) * np.float32(0.5)
        Y[j] = avg
        Y[i] = avg - np.float32(0.02) * g
    assert np.array_equal(X, Y)


def test_per_event_postconditions_and_telescoping_sum():
    n, feats, targs, sched, X0 = _random_problem(6, 23, 12, 400, 5, 5, 6)
    gamma = 0.01
    X = X0.copy()
    total_g = np.zeros(23)
    for k in range(400):
        one = {key: (val[:k + 1] if val is not None else None) for key, val in sched.items()}
        before = X.copy()
        # replay the prefix so that stale reads see the true history, keep only the last event
        Y = X0.copy()
        r = oracle.run_events(Y, one, LSQ, gamma, M=5, gscale=0.2, features=feats, targets=targs,
                              mode=0, want_g=True)
        g = r["g"][k]
        i, j = sched["worker"][k], sched["neighbour"][k]
        X = Y
        others = [r_ for r_ in range(n) if r_ not in (i, j)]
        assert np.array_equal(X[others], before[others])                 # untouched rows bit-identical
        avg = (before[i].astype(np.float64) + before[j]) / 2
        assert np.allclose(X[j], avg, rtol=1e-6, atol=1e-7)                # both rows took the average
        assert np.allclose(X[i].astype(np.float64) - X[j], -gamma * g.astype(np.float64),
                           rtol=1e-5, atol=2e-7)                           # x_i - x_j = -gamma g_k
        # averaging preserves the sum over workers: the sum moves only by -gamma g_k
        assert np.allclose(X.sum(0, dtype=np.float64), before.sum(0, dtype=np.float64) - gamma * g,
                           rtol=0, atol=5e-6)
        total_g += g
        if k > 40:
            break
    Xf = X0.copy()
    r = oracle.run_events(Xf, sched, LSQ, gamma, M=5, gscale=0.2, features=feats, targets=targs,
                          mode=1, want_g=True)
    lhs = Xf.sum(0, dtype=np.float64)
    rhs = X0.sum(0, dtype=np.float64) - gamma * r["g"].sum(0, dtype=np.float64)
    assert np.allclose(lhs, rhs, rtol=0, atol=2e-5)


def test_pairwise_W_is_symmetric_doubly_stochastic_projection_and_oracle_applies_it():
    n, d = 5, 7
    rng = np.random.default_rng(8)
    X0 = rng.integers(-64, 64, (n, d)).astype(np.float32)   # integers: averages are exact
    for i in range(n):
        for j in range(n):
            if i == j:
                continue
            e = np.zeros((n, 1)); e[i] = 1; e[j] = -1
            W = np.eye(n) - 0.5 * (e @ e.T)
            assert np.array_equal(W, W.T) and np.all(W >= 0)
            assert np.allclose(W.sum(0), 1) and np.allclose(W.sum(1), 1)
            assert np.allclose(W @ W, W)
            X = X0.copy()
            sched = {"worker": [i], "neighbour": [j], "tau": [0]}
            oracle.run_events(X, sched, SYNTH, 0.0, synth_std=0.0)       # g = 0: pure X <- X W
            assert np.array_equal(X.astype(np.float64), W @ X0.astype(np.float64))


def test_equal_initial_models_gossip_is_a_noop():
    n, d = 8, 16
    x0 = np.random.default_rng(9).standard_normal(d).astype(np.float32)
    X = np.tile(x0, (n, 1))
    sched = oracle.make_schedule(ring_graph(n), 500, seed=1)
    oracle.run_events(X, sched, SYNTH, 0.0, synth_std=1.0, synth_seed=3)   # gamma = 0
    assert np.array_equal(X, np.tile(x0, (n, 1)))


def test_gossip_only_expectation_and_contraction_on_a_ring():
    """gamma = 0, X_0 = I: X_K = W_K ... W_1.  Independence gives E X_K = (E W)^K with
    E W = I - L/(2n) on a ring with uniform worker and neighbour (L = ring Laplacian), and the
    consensus lemma bounds E |1/n - prod W e_i|^2 by (n-1)/n rho^K, rho = lambda_2(E W^T W)
    = 1 - (1 - cos(2 pi/n))/n because W^T W = W for a pairwise average."""
    n, K, S = 8, 30, 3000
    L = 2 * np.eye(n) - np.roll(np.eye(n), 1, 0) - np.roll(np.eye(n), -1, 0)
    EW = np.eye(n) - L / (2 * n)
    rho = 1 - (1 - np.cos(2 * np.pi / n)) / n
    assert abs(rho - 0.963388) < 1e-6
    assert np.isclose(np.sort(np.linalg.eigvalsh(EW))[-2], rho)
    acc = np.zeros((n, n))
    dist = 0.0
    g = ring_graph(n)
    for s in range(S):
        X = np.eye(n, dtype=np.float32)
        oracle.run_events(X, oracle.make_schedule(g, K, seed=1000 + s), SYNTH, 0.0, synth_std=0.0)
        acc += X
        dist += np.sum((X.astype(np.float64) - 1.0 / n) ** 2)
        assert np.allclose(X.sum(0), 1.0) and np.allclose(X.sum(1), 1.0)    # product stays doubly stochastic
    mean = acc / S
    expect = np.linalg.matrix_power(EW, K)
    assert np.max(np.abs(mean - expect)) < 5 * 0.35 / np.sqrt(S)
    # sum over the n columns of the lemma's bound
    assert dist / S <= (n - 1) * rho ** K * 1.0 + 1e-9
    assert dist / S > 0.1 * (n - 1) * rho ** K          # and the bound is not vacuous here


def test_single_worker_is_vanilla_minibatch_sgd():
    """n = 1, T = 0: no neighbour, the update is x <- x - gamma * (1/M) sum_m grad F(x; xi_m)."""
    rows, d, M, K, gamma = 30, 9, 6, 150, 0.05
    feats, targs, _ = lsq_data(1, rows, d, seed=3)
    g = ring_graph(1)
    sched = oracle.make_schedule(g, K, seed=2, T_max=0, M=M, rows=[rows])
    assert np.all(sched["neighbour"] == 0) and np.all(sched["tau"] == 0)
    X = np.zeros((1, d), dtype=np.float32)
    oracle.run_events(X, sched, LSQ, gamma, M=M, gscale=1.0 / M, features=feats, targets=targs)
    x = np.zeros(d)
    A, b = feats[0].astype(np.float64), targs[0].astype(np.float64)
    for k in range(K):
        idx = sched["batch_idx"][k]
        x = x - gamma * A[idx].T @ (A[idx] @ x - b[idx]) / M
    assert np.allclose(X[0], x, rtol=1e-4, atol=1e-5)


def test_zero_noise_quadratic_reaches_the_closed_form_optimum():
    """All workers hold the same consistent system b = A x*, full batch, bounded staleness:
    consensus at x* is a fixed point of both steps and every replica converges to it."""
    n, rows, d = 6, 24, 8
    feats, targs, xstar = lsq_data(n, rows, d, seed=5, noise=0.0, shared=True)
    sol = np.linalg.lstsq(feats[0].astype(np.float64), targs[0].astype(np.float64), rcond=None)[0]
    assert np.allclose(sol, xstar, atol=1e-5)
    K = 6000
    sched = oracle.make_schedule(ring_graph(n), K, seed=4, T_max=3)
    sched["batch_idx"] = np.tile(np.arange(rows, dtype=np.int32), (K, 1))
    X = np.zeros((n, d), dtype=np.float32)
    oracle.run_events(X, sched, LSQ, 0.02, M=rows, gscale=1.0 / rows, features=feats, targets=targs)
    assert np.max(np.abs(X - sol[None, :])) < 1e-4
    assert oracle.consensus_distance(X) < 1e-9


def test_diagnostics_against_numpy():
    rng = np.random.default_rng(10)
    X = rng.standard_normal((7, 13)).astype(np.float32)
    mu = X.astype(np.float64).mean(0)
    assert np.allclose(oracle.mean_model(X), mu, rtol=1e-14)
    assert np.isclose(oracle.consensus_distance(X), np.mean(np.sum((X - mu) ** 2, axis=1)), rtol=1e-12)
    p = rng.random(7)
    p /= p.sum()
    assert np.isclose(oracle.consensus_distance_weighted(X, p), np.sum(p * np.sum((X - mu) ** 2, axis=1)), rtol=1e-12)
    assert np.isclose(oracle.consensus_distance_weighted(X, np.full(7, 1 / 7)), oracle.consensus_distance(X), rtol=1e-12)
    only3 = np.zeros(7)
    only3[3] = 1.0
    assert np.isclose(oracle.consensus_distance_weighted(X, only3), np.sum((X[3] - mu) ** 2), rtol=1e-12)


def test_coordinate_subset_of_synthetic_workload_follows_the_full_run():
    n, d, K = 8, 64, 300
    sched = oracle.make_schedule(ring_graph(n), K, seed=11, T_max=5)
    X = np.zeros((n, d), dtype=np.float32)
    oracle.run_events(X, sched, SYNTH, 0.1, synth_std=0.03, synth_seed=9, event_base=17)
    coords = np.array([0, 3, 5, 22, 63])
    Y = np.zeros((n, coords.size), dtype=np.float32)
    oracle.run_events(Y, sched, SYNTH, 0.1, synth_std=0.03, synth_seed=9, event_base=17, coords=coords)
    assert np.array_equal(Y, X[:, coords])
    # tau cannot matter when g ignores x
    Z = np.zeros((n, d), dtype=np.float32)
    oracle.run_events(Z, dict(sched, tau=np.zeros(K, np.int32)), SYNTH, 0.1, synth_std=0.03,
                      synth_seed=9, event_base=17)
    assert np.array_equal(Z, X)


# --------------------------------------------------------------------------- momentum / weight decay
def test_momentum_with_zero_coefficients_is_the_plain_event():
    n, feats, targs, sched, X0 = _random_problem(6, 19, 12, 200, 5, 4, 0, LSQ)
    Xa, Xb = X0.copy(), X0.copy()
    V = np.zeros_like(X0)
    oracle.run_events(Xa, sched, LSQ, 0.01, M=5, gscale=0.2, features=feats, targets=targs)
    r = oracle.run_events(Xb, sched, LSQ, 0.01, M=5, gscale=0.2, features=feats, targets=targs, V=V, want_g=True)
    assert np.array_equal(Xa, Xb)
    # with mu = 0 the buffer of a worker holds the last gradient it applied
    last = {}
    for k, i in enumerate(sched["worker"]):
        last[i] = k
    for i, k in last.items():
        assert np.array_equal(V[i], r["g"][k])


def test_single_worker_momentum_matches_library_sgd():
    """n = 1, T = 0: the update is the textbook SGD step with momentum and weight decay; compare
    with torch.optim.SGD fed the same minibatch gradients."""
    torch = pytest.importorskip("torch")
    rows, d, M, K, gamma, mu, wd = 30, 9, 6, 120, 0.05, 0.9, 0.01
    feats, targs, _ = lsq_data(1, rows, d, seed=3)
    sched = oracle.make_schedule(ring_graph(1), K, seed=2, T_max=0, M=M, rows=[rows])
    X = np.zeros((1, d), dtype=np.float32)
    V = np.zeros((1, d), dtype=np.float32)
    oracle.run_events(X, sched, LSQ, gamma, M=M, gscale=1.0 / M, features=feats, targets=targs,
                      momentum=mu, weight_decay=wd, V=V)
    p = torch.zeros(d, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([p], lr=gamma, momentum=mu, weight_decay=wd)
    A, b = torch.tensor(feats[0], dtype=torch.float64), torch.tensor(targs[0], dtype=torch.float64)
    for k in range(K):
        idx = torch.tensor(sched["batch_idx"][k], dtype=torch.long)
        opt.zero_grad()
        (0.5 * ((A[idx] @ p - b[idx]) ** 2).mean()).backward()
        opt.step()
    assert np.allclose(X[0], p.detach().numpy(), rtol=2e-4, atol=2e-5)


def test_momentum_constant_gradient_closed_form_and_sum_identity():
    """Synthetic gradient with std 0 and a constant offset is not available, so use gossip on a ring
    with n = 4 and the telescoped identity: the sum over workers moves by -gamma v_k at event k, and
    averaging never touches it; with wd = 0 the buffers obey v <- mu v + g exactly."""
    n, feats, targs, sched, X0 = _random_problem(6, 11, 10, 150, 4, 3, 2, LSQ)
    gamma, mu = 0.02, 0.8
    X, V = X0.copy(), np.zeros_like(X0)
    r = oracle.run_events(X, sched, LSQ, gamma, M=4, gscale=0.25, features=feats, targets=targs,
                          momentum=mu, weight_decay=0.0, V=V, want_g=True)
    Vref = np.zeros_like(X0, dtype=np.float64)
    total = np.zeros(11)
    for k, i in enumerate(sched["worker"]):
        Vref[i] = mu * Vref[i] + r["g"][k]
        total += Vref[i]
    assert np.allclose(V, Vref, rtol=1e-5, atol=1e-6)
    assert np.allclose(X.sum(0, dtype=np.float64), X0.sum(0, dtype=np.float64) - gamma * total, rtol=0, atol=5e-5)


def test_weight_decay_acts_on_the_averaged_model():
    """One event by hand: x_i = 2, x_j = 4, g = 0 (synthetic std 0): avg = 3, u = wd*3, v = u,
    x_i = 3 - gamma*wd*3, x_j = 3."""
    X = np.array([[2.0], [4.0]], dtype=np.float32)
    V = np.zeros_like(X)
    sched = {"worker": [0], "neighbour": [1], "tau": [0]}
    oracle.run_events(X, sched, SYNTH, 0.5, synth_std=0.0, momentum=0.9, weight_decay=0.25, V=V)
    assert X[1, 0] == 3.0 and V[0, 0] == 0.75 and X[0, 0] == 3.0 - 0.5 * 0.75 and V[1, 0] == 0.0
    oracle.run_events(X, sched, SYNTH, 0.5, synth_std=0.0, momentum=0.5, weight_decay=0.0, V=V)
    avg = (2.625 + 3.0) / 2
    assert V[0, 0] == 0.375 and X[0, 0] == np.float32(avg - 0.5 * 0.375) and X[1, 0] == np.float32(avg)


# --------------------------------------------------------------------------- general averaging matrix W_k
def test_multi_pair_W_is_doubly_stochastic_and_oracle_applies_it():
    """W_k = product of disjoint pairwise averagings: symmetric, doubly stochastic, idempotent;
    with g = 0 the oracle computes exactly X <- W X."""
    from workloads import random_extra_pairs
    n, d, K = 9, 5, 12
    g = random_regular4_graph(n, 3)
    sched = oracle.make_schedule(g, K, seed=6)
    extra = random_extra_pairs(g, sched["worker"], sched["neighbour"], max_extra=3, seed=1)
    assert extra[0][-1] > K // 2                       # the extension is exercised
    X0 = np.random.default_rng(2).integers(-512, 512, (n, d)).astype(np.float32) * 2.0 ** 20   # 12 exact halvings
    X = X0.copy()
    oracle.run_events(X, sched, SYNTH, 0.0, synth_std=0.0, extra_pairs=extra)
    ref = X0.astype(np.float64)
    for k in range(K):
        W = np.eye(n)
        pairs = [(sched["worker"][k], sched["neighbour"][k])] + [(extra[1][q], extra[2][q]) for q in range(extra[0][k], extra[0][k + 1])]
        rows = [r for pr in pairs for r in pr]
        assert len(set(rows)) == len(rows)             # disjoint
        for a, b in pairs:
            e = np.zeros((n, 1)); e[a] = 1; e[b] = -1
            W = W @ (np.eye(n) - 0.5 * e @ e.T)
        assert np.allclose(W, W.T) and np.all(W >= 0) and np.allclose(W.sum(0), 1) and np.allclose(W @ W, W)
        ref = W @ ref
    assert np.array_equal(X.astype(np.float64), ref)


def test_multi_pair_events_keep_the_gradient_semantics():
    """Extra pairs change only the averaging: the sum over workers still moves by -gamma g_k per event,
    literal and parked forms agree, and dropping the extras changes the result."""
    from workloads import random_extra_pairs
    n, feats, targs, sched, X0 = _random_problem(6, 13, 10, 200, 4, 3, 1, LSQ)   # seed 1: 4-regular graph
    g = random_regular4_graph(6, 1)
    extra = random_extra_pairs(g, sched["worker"], sched["neighbour"], max_extra=2, seed=2)
    Xa, Xb, Xc = X0.copy(), X0.copy(), X0.copy()
    ra = oracle.run_events(Xa, sched, LSQ, 0.02, M=4, gscale=0.25, features=feats, targets=targs, mode=0,
                           extra_pairs=extra, want_g=True)
    oracle.run_events(Xb, sched, LSQ, 0.02, M=4, gscale=0.25, features=feats, targets=targs, mode=1, extra_pairs=extra)
    oracle.run_events(Xc, sched, LSQ, 0.02, M=4, gscale=0.25, features=feats, targets=targs, mode=0)
    assert np.array_equal(Xa, Xb) and not np.array_equal(Xa, Xc)
    assert np.allclose(Xa.sum(0, dtype=np.float64), X0.sum(0, dtype=np.float64) - 0.02 * ra["g"].sum(0, dtype=np.float64),
                       rtol=0, atol=2e-5)


def test_identity_events_are_plain_gradient_steps_and_express_a_gradient_queue():
    """neighbour = worker (W_k = I) on a connected graph.  (1) With every event of that kind and no
    staleness each worker is textbook minibatch SGD on its own data.  (2) Two gradients queued before one
    communication step (wait-free appendix, computation thread): the averaging event followed by an
    identity event that reads the same model gives  avg - gamma (g1 + g2)  with both gradients taken at
    the worker's model from before the step."""
    n, rows, d, M, K, gamma = 3, 20, 7, 4, 60, 0.05
    feats, targs, _ = lsq_data(n, rows, d, seed=8)
    g = ring_graph(n)
    sched = oracle.make_schedule(g, K, seed=3, T_max=0, M=M, rows=[rows] * n)
    sched["neighbour"] = sched["worker"].copy()
    X0 = np.random.default_rng(2).standard_normal((n, d)).astype(np.float32)
    X = X0.copy()
    oracle.run_events(X, sched, LSQ, gamma, M=M, gscale=1.0 / M, features=feats, targets=targs)
    for i in range(n):
        x, A, b = X0[i].astype(np.float64), feats[i].astype(np.float64), targs[i].astype(np.float64)
        for k in np.nonzero(sched["worker"] == i)[0]:
            idx = sched["batch_idx"][k]
            x = x - gamma * A[idx].T @ (A[idx] @ x - b[idx]) / M
        assert np.allclose(X[i], x, rtol=1e-4, atol=1e-5)
    # (2) worker 0 averages with worker 1 and applies g1 (event 0), then applies the queued g2 (event 1, tau = 1)
    batch = np.array([[0, 1, 2, 3], [4, 5, 6, 7]], np.int32)
    queue = {"worker": np.array([0, 0], np.int32), "neighbour": np.array([1, 0], np.int32),
             "tau": np.array([0, 1], np.int32), "batch_idx": batch}
    X = X0.copy()
    oracle.run_events(X, queue, LSQ, gamma, M=M, gscale=1.0 / M, features=feats, targets=targs)
    x0, A, b = X0[0].astype(np.float64), feats[0].astype(np.float64), targs[0].astype(np.float64)
    grads = [A[idx].T @ (A[idx] @ x0 - b[idx]) / M for idx in batch]
    avg = 0.5 * (X0[0].astype(np.float64) + X0[1])
    assert np.allclose(X[0], avg - gamma * (grads[0] + grads[1]), rtol=1e-5, atol=1e-6)
    assert np.allclose(X[1], avg, rtol=1e-6, atol=1e-7) and np.array_equal(X[2], X0[2])
    fresh = A[batch[1]].T @ (A[batch[1]] @ (avg - gamma * grads[0]) - b[batch[1]]) / M
    assert not np.allclose(X[0], avg - gamma * (grads[0] + fresh), rtol=1e-5, atol=1e-6)   # the pin can tell tau = 1 from 0


def test_hop_ring_mixes_faster_than_the_ring():
    """The ring with extra 2^i + 1 hop links (Sec. 3.3.2) has a smaller rho = lambda_2(E W): closed
    form from the circulant Laplacian, and the oracle's gossip-only runs follow (E W)^K."""
    from workloads import hop_ring_graph
    n, K, S = 16, 40, 1500
    def expected_W(graph):
        rowptr, col = graph
        EW = np.zeros((n, n))
        for i in range(n):
            nb = col[rowptr[i]:rowptr[i + 1]]
            for j in nb:
                e = np.zeros((n, 1)); e[i] = 1; e[j] = -1
                EW += (np.eye(n) - 0.5 * e @ e.T) / (n * len(nb))
        return EW
    rho = {}
    for name, graph in (("ring", ring_graph(n)), ("hop", hop_ring_graph(n))):
        EW = expected_W(graph)
        rho[name] = np.sort(np.linalg.eigvalsh(EW))[-2]
        acc = np.zeros((n, n))
        for s in range(S):
            X = np.eye(n, dtype=np.float32)
            oracle.run_events(X, oracle.make_schedule(graph, K, seed=500 + s), SYNTH, 0.0, synth_std=0.0)
            acc += X
        assert np.max(np.abs(acc / S - np.linalg.matrix_power(EW, K))) < 5 * 0.35 / np.sqrt(S)
    assert np.isclose(rho["ring"], 1 - (1 - np.cos(2 * np.pi / n)) / n)
    assert rho["hop"] < rho["ring"] - 0.02


# ------------------------------------------------------------------ synchronous comparison schedule (D-PSGD)
def test_dpsgd_hand_expanded(golden_dir):
    cases = [l.split() for l in open(os.path.join(golden_dir, "dpsgd_two_workers_d1.txt"))
             if l.strip() and not l.startswith("#")]
    feats, targs = _unit_quadratic_data(2, [1.0])
    assert len(cases) == 5
    for a, S, e0, e1 in cases:
        a, S = float(a), int(S)
        X = np.array([[1.0], [3.0]], dtype=np.float32)
        W = np.array([[a, 1 - a], [1 - a, a]], np.float32)
        oracle.run_sync_steps(X, np.zeros((S, 2, 1), np.int32), W, LSQ, 0.5, M=1, gscale=1.0,
                              features=feats, targets=targs)
        assert (X[0, 0], X[1, 0]) == (float(e0), float(e1)), (a, S, X.ravel())


def test_dpsgd_identity_mixing_is_n_independent_sgd_runs():
    """W = I: worker i is plain minibatch SGD on its own data -- the single-worker case of the event
    oracle (itself pinned against a textbook loop), bit for bit."""
    n, d, rows, M, S = 3, 12, 20, 4, 40
    feats, targs, _ = lsq_data(n, rows, d, seed=4)
    rng = np.random.default_rng(1)
    batch = rng.integers(0, rows, size=(S, n, M)).astype(np.int32)
    X0 = rng.standard_normal((n, d)).astype(np.float32)
    X = X0.copy()
    oracle.run_sync_steps(X, batch, np.eye(n, dtype=np.float32), LSQ, 0.05, M=M, gscale=1.0 / M,
                          features=feats, targets=targs)
    for i in range(n):
        xi = X0[i:i + 1].copy()
        sched = {"worker": np.zeros(S, np.int32), "neighbour": np.zeros(S, np.int32), "tau": np.zeros(S, np.int32),
                 "batch_idx": np.ascontiguousarray(batch[:, i, :])}
        oracle.run_events(xi, sched, LSQ, 0.05, M=M, gscale=1.0 / M, features=[feats[i]], targets=[targs[i]])
        assert np.array_equal(xi[0], X[i])


def test_dpsgd_with_momentum_reduces_to_the_event_rule_and_to_a_closed_form():
    """Synchronous schedule with the experiments' optimizer.  (1) W = I: worker i is the single-worker
    event run with momentum (itself pinned against a library optimizer), bit for bit.  (2) Weight decay
    acts on the mixed model: with zero gradients one step gives  W X_0 (1 - gamma wd)  and  v = wd W X_0.
    (3) n = 1 with synthetic gradients: the recursion  v_t = mu v_{t-1} + g_t,  x_t = x_{t-1} - gamma v_t
    rebuilt in fp64 from the generator's draws.  (4) Zero coefficients leave the plain step."""
    n, d, rows, M, S, mu, wd = 3, 12, 20, 4, 30, 0.9, 1e-2
    feats, targs, _ = lsq_data(n, rows, d, seed=4)
    rng = np.random.default_rng(1)
    batch = rng.integers(0, rows, size=(S, n, M)).astype(np.int32)
    X0 = rng.standard_normal((n, d)).astype(np.float32)
    X, V = X0.copy(), np.zeros_like(X0)
    oracle.run_sync_steps(X, batch, np.eye(n, dtype=np.float32), LSQ, 0.05, M=M, gscale=1.0 / M,
                          features=feats, targets=targs, momentum=mu, weight_decay=wd, V=V)
    for i in range(n):
        xi, vi = X0[i:i + 1].copy(), np.zeros((1, d), np.float32)
        sched = {"worker": np.zeros(S, np.int32), "neighbour": np.zeros(S, np.int32), "tau": np.zeros(S, np.int32),
                 "batch_idx": np.ascontiguousarray(batch[:, i, :])}
        oracle.run_events(xi, sched, LSQ, 0.05, M=M, gscale=1.0 / M, features=[feats[i]], targets=[targs[i]],
                          momentum=mu, weight_decay=wd, V=vi)
        assert np.array_equal(xi[0], X[i]) and np.array_equal(vi[0], V[i])
    # (2)
    Wfull = np.full((n, n), 1.0 / n, np.float32)
    X, V = X0.copy(), np.zeros_like(X0)
    oracle.run_sync_steps(X, None, Wfull, SYNTH, 0.1, synth_std=0.0, steps=1, momentum=mu, weight_decay=wd, V=V)
    mixed = Wfull.astype(np.float64) @ X0.astype(np.float64)
    assert np.allclose(X, mixed * (1 - 0.1 * wd), rtol=1e-6, atol=1e-7)
    assert np.allclose(V, wd * mixed, rtol=1e-6, atol=1e-9)
    # (3)
    S2, gam = 12, 0.05
    Xs, Vs = np.zeros((1, d), np.float32), np.zeros((1, d), np.float32)
    oracle.run_sync_steps(Xs, None, np.ones((1, 1), np.float32), SYNTH, gam, synth_std=0.3, synth_seed=5,
                          event_base=7, steps=S2, momentum=mu, weight_decay=0.0, V=Vs)
    xs, vs = np.zeros(d), np.zeros(d)
    for t in range(S2):           # worker 0 of n = 1 draws event 7 + t in step t
        vs = mu * vs + oracle.synth_grad(5, 7 + t, 0.3, np.arange(d)).astype(np.float64)
        xs = xs - gam * vs
    assert np.abs(xs).max() > 0.05
    assert np.allclose(Xs[0], xs, rtol=1e-5, atol=1e-6) and np.allclose(Vs[0], vs, rtol=1e-5, atol=1e-6)
    # (4)
    Xa, Xb, Vb = X0.copy(), X0.copy(), np.zeros_like(X0)
    Wm = oracle.metropolis_weights(ring_graph(n))
    oracle.run_sync_steps(Xa, batch, Wm, LSQ, 0.05, M=M, gscale=1.0 / M, features=feats, targets=targs)
    oracle.run_sync_steps(Xb, batch, Wm, LSQ, 0.05, M=M, gscale=1.0 / M, features=feats, targets=targs,
                          momentum=0.0, weight_decay=0.0, V=Vb)
    assert np.array_equal(Xa, Xb)


def _path_plus_chord_graph():
    """A small irregular connected graph: path 0-1-2-3-4 plus the edges 1-3 and 1-4 (degrees 1..4)."""
    edges = [(0, 1), (1, 2), (2, 3), (3, 4), (1, 3), (1, 4)]
    nb = [[] for _ in range(5)]
    for a, b in edges:
        nb[a].append(b)
        nb[b].append(a)
    rowptr = np.cumsum([0] + [len(v) for v in nb]).astype(np.int32)
    col = np.array([j for v in nb for j in sorted(v)], np.int32)
    return rowptr, col


def test_metropolis_weights_are_symmetric_doubly_stochastic():
    g = _path_plus_chord_graph()
    W = oracle.metropolis_weights(g).astype(np.float64)
    assert np.array_equal(W, W.T) and (W >= 0).all()
    assert np.allclose(W.sum(0), 1, atol=1e-7) and np.allclose(W.sum(1), 1, atol=1e-7)
    assert W[0, 1] == np.float32(1 / 5) and W[2, 3] == np.float32(1 / 4) and W[0, 2] == 0   # 1/(1+max deg)
    ring = oracle.metropolis_weights(ring_graph(8))
    assert np.allclose(ring[ring > 0], 1 / 3, atol=1e-7) and (ring > 0).sum() == 24
    # second-largest eigenvalue modulus below one: repeated mixing reaches consensus
    assert np.sort(np.abs(np.linalg.eigvalsh(W)))[-2] < 1 - 1e-3


def test_dpsgd_gossip_only_is_a_matrix_power():
    """gamma = 0: X_S = W^S X_0 (numpy, fp64), and the mean of the workers does not move."""
    g = _path_plus_chord_graph()
    W = oracle.metropolis_weights(g)
    n, d, S = 5, 7, 25
    X0 = np.random.default_rng(3).standard_normal((n, d)).astype(np.float32)
    X = X0.copy()
    oracle.run_sync_steps(X, None, W, oracle.MODEL_SYNTH, 0.0, synth_std=1.0, steps=S)
    ref = np.linalg.matrix_power(W.astype(np.float64), S) @ X0.astype(np.float64)
    assert np.allclose(X, ref, rtol=0, atol=2e-6)
    assert np.allclose(X.mean(0), X0.mean(0), atol=1e-6)
    assert oracle.consensus_distance(X) < 0.05 * oracle.consensus_distance(X0)


def test_dpsgd_mean_moves_by_the_mean_gradient():
    """Doubly stochastic W: mean_{t+1} = mean_t - gamma * mean_i g_i, so after S steps the mean has moved
    by -sum_t gamma_t mean_i g_{t,i} (gradients logged), whatever the topology."""
    n, d, rows, M, S = 6, 10, 16, 3, 30
    W = oracle.metropolis_weights(random_regular4_graph(n, 1))
    feats, targs, _ = logreg_data(n, rows, d, seed=2)
    rng = np.random.default_rng(0)
    batch = rng.integers(0, rows, size=(S, n, M)).astype(np.int32)
    gam = (0.5 / (1 + np.arange(S) / 10)).astype(np.float32)
    X0 = rng.standard_normal((n, d)).astype(np.float32)
    X = X0.copy()
    r = oracle.run_sync_steps(X, batch, W, LOGREG, 0.0, M=M, gscale=1.0 / M, lam=0.01, features=feats,
                              targets=targs, gamma_s=gam, want_g=True, want_loss=True)
    moved = -(gam.astype(np.float64)[:, None, None] * r["g"].astype(np.float64)).sum(0).mean(0)
    assert np.allclose(X.astype(np.float64).mean(0) - X0.astype(np.float64).mean(0), moved, atol=5e-6)
    assert np.abs(moved).max() > 1e-2
    # the logged gradient of step 0 is the gradient at X_0, not at the mixed model
    g00, l00 = oracle.minibatch_gradient(LOGREG, X0[2], feats[2], targs[2], batch[0, 2], 1.0 / M, lam=0.01)
    assert np.array_equal(g00, r["g"][0, 2]) and l00 == r["loss"][0, 2]


def test_dpsgd_full_averaging_same_data_keeps_workers_equal():
    """W = 11^T / n (n = 4, exact in binary), every worker with the same data, minibatch and initial
    model: all replicas stay identical and follow single-worker SGD exactly."""
    n, d, rows, M, S = 4, 9, 12, 3, 25
    f1, t1, _ = lsq_data(1, rows, d, seed=8)
    feats, targs = [f1[0]] * n, [t1[0]] * n
    rng = np.random.default_rng(5)
    b1 = rng.integers(0, rows, size=(S, 1, M)).astype(np.int32)
    x0 = rng.standard_normal(d).astype(np.float32)
    X = np.tile(x0, (n, 1))
    oracle.run_sync_steps(X, np.repeat(b1, n, axis=1), np.full((n, n), 0.25, np.float32), LSQ, 0.1, M=M,
                          gscale=1.0 / M, features=feats, targets=targs)
    ref = x0[None].copy()
    oracle.run_sync_steps(ref, b1, np.ones((1, 1), np.float32), LSQ, 0.1, M=M, gscale=1.0 / M,
                          features=f1, targets=t1)
    assert all(np.array_equal(X[i], ref[0]) for i in range(n))


def test_dpsgd_synthetic_gradients_use_the_event_counter():
    """Worker i at step t draws event number base + t n + i of the synthetic generator."""
    n, d, S = 3, 8, 2
    X = np.zeros((n, d), np.float32)
    oracle.run_sync_steps(X, None, np.eye(n, dtype=np.float32), oracle.MODEL_SYNTH, 1.0, synth_std=0.5,
                          synth_seed=9, event_base=100, steps=S)
    for i in range(n):
        want = np.zeros(d, np.float32)
        for t in range(S):
            want = want - oracle.synth_grad(9, 100 + t * n + i, 0.5, np.arange(d))
        assert np.array_equal(X[i], want)
