"""Pins for the CPU oracle: closed forms, invariants, brute force and a library optimiser.

None of these compare the oracle with itself: each checks it against something the
mathematics of the problem fixes (the paper prints no formula or value for this path; the
problem statement is the L2-regularised GLM and its Fenchel dual, CoCoA with sigma = K and
adding, Section 2.2 and 5.1).
"""
import ctypes
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.optimize

from workloads import get_config, make_problem, round_permutations
from workloads.configs import k_for_round


# ----------------------------------------------------------------------------- helpers
def tiny_dense(n, d, seed, loss, separable=False):
    g = np.random.default_rng(seed)
    X = g.standard_normal((n, d)).astype(np.float32)
    if loss in ("hinge", "logistic"):
        wst = g.standard_normal(d)
        y = np.where(X.astype(np.float64) @ wst >= 0, 1.0, -1.0)
        if not separable:
            fl = g.random(n) < 0.2
            y[fl] *= -1
    else:
        y = X.astype(np.float64) @ g.standard_normal(d) + 0.3 * g.standard_normal(n)
    return X, y.astype(np.float32)


def to_csr(X):
    n, d = X.shape
    mask = X != 0
    row_ptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(mask.sum(axis=1), out=row_ptr[1:])
    col = np.nonzero(mask)[1].astype(np.int32)
    val = X[mask].astype(np.float32)
    return row_ptr, col, val


def bounds(n, rows):
    b = list(range(0, n, rows)) + [n]
    return np.array(b, dtype=np.int64)


def s_vec(loss, y):
    return np.ones(len(y)) if loss == "squared" else y.astype(np.float64)


def xlogx(a):
    return np.where(a > 0, a * np.log(np.where(a > 0, a, 1.0)), 0.0)


def w_of_alpha(loss, X, y, alpha, lam):
    n = X.shape[0]
    return X.astype(np.float64).T @ (alpha * s_vec(loss, y)) / (lam * n)


def primal(loss, X, y, w, lam):
    z = X.astype(np.float64) @ w
    if loss == "hinge":
        l = np.maximum(0.0, 1.0 - y * z)
    elif loss == "logistic":
        l = np.logaddexp(0.0, -y * z)
    else:
        l = 0.5 * (z - y) ** 2
    return 0.5 * lam * w @ w + l.mean()


def dual(loss, X, y, alpha, lam):
    w = w_of_alpha(loss, X, y, alpha, lam)
    if loss == "hinge":
        if np.any(alpha < -1e-15) or np.any(alpha > 1 + 1e-15):
            return -np.inf
        return alpha.mean() - 0.5 * lam * w @ w
    if loss == "logistic":
        if np.any(alpha < -1e-15) or np.any(alpha > 1 + 1e-15):
            return -np.inf
        a = np.clip(alpha, 0.0, 1.0)
        return -(xlogx(a) + xlogx(1.0 - a)).mean() - 0.5 * lam * w @ w
    return -(0.5 * alpha ** 2 - alpha * y).mean() - 0.5 * lam * w @ w


def run_rounds(o, K, rounds, seed=0, c2s=None):
    nchunks = o.chunk_bounds.size - 1
    if c2s is None:
        c2s = np.arange(nchunks) % K
    o.assign(K, c2s)
    hist = []
    for r in range(rounds):
        perms = round_permutations(seed, r, o.rows_per_solver())
        o.local_epoch(perms)
        o.aggregate()
        hist.append(o.gap())
    return hist


# ----------------------------------------------------------------------------- P1
@pytest.mark.parametrize("sparse", [False, True])
def test_gap_at_zero(oracle_mod, sparse):
    X, y = tiny_dense(50, 7, 1, "hinge")
    kw = dict(zip(("row_ptr", "col", "val"), to_csr(X))) if sparse else dict(X=X)
    o = oracle_mod.OracleCoCoA("hinge", 50, 7, 0.01, y, bounds(50, 16), **kw)
    P, D, G, FY = o.gap()
    assert (P, D, G, FY) == (1.0, 0.0, 1.0, 1.0)
    X, y = tiny_dense(50, 7, 2, "squared")
    kw = dict(zip(("row_ptr", "col", "val"), to_csr(X))) if sparse else dict(X=X)
    o = oracle_mod.OracleCoCoA("squared", 50, 7, 0.01, y, bounds(50, 16), **kw)
    P, D, G, FY = o.gap()
    want = 0.5 * np.mean(y.astype(np.float64) ** 2)
    assert D == 0.0 and abs(P - want) < 1e-14 and abs(G - want) < 1e-14 and abs(FY - want) < 1e-14
    X, y = tiny_dense(50, 7, 3, "logistic")
    kw = dict(zip(("row_ptr", "col", "val"), to_csr(X))) if sparse else dict(X=X)
    o = oracle_mod.OracleCoCoA("logistic", 50, 7, 0.01, y, bounds(50, 16), **kw)
    P, D, G, FY = o.gap()
    assert D == 0.0 and abs(P - np.log(2.0)) < 1e-14 and abs(G - np.log(2.0)) < 1e-14 and abs(FY - np.log(2.0)) < 1e-14


# ----------------------------------------------------------------------------- P2, P3, P4, P6
@pytest.mark.parametrize("loss", ["hinge", "squared", "logistic"])
@pytest.mark.parametrize("sparse", [False, True])
@pytest.mark.parametrize("K", [1, 3, 5])
def test_invariants_every_round(oracle_mod, loss, sparse, K):
    n, d, lam = 120, 9, 0.02
    X, y = tiny_dense(n, d, 3, loss)
    X[np.random.default_rng(5).random(X.shape) < 0.5] = 0.0     # make it genuinely sparse
    X[7] = 0.0                                                     # an all-zero row must be skipped
    kw = dict(zip(("row_ptr", "col", "val"), to_csr(X))) if sparse else dict(X=X)
    o = oracle_mod.OracleCoCoA(loss, n, d, lam, y, bounds(n, 13), **kw)
    o.assign(K, np.arange(o.chunk_bounds.size - 1) % K)
    prevD = dual(loss, X, y, o.alpha, lam)
    for r in range(8):
        perms = round_permutations(11, r, o.rows_per_solver())
        o.local_epoch(perms)
        o.aggregate()
        P, D, G, FY = o.gap()
        # P3: the shared vector is the image of alpha under the primal-dual map
        wa = w_of_alpha(loss, X, y, o.alpha, lam)
        assert np.linalg.norm(o.w - wa) <= 1e-12 * max(1.0, np.linalg.norm(wa))
        # P and D agree with their definitions written with numpy
        assert abs(P - primal(loss, X, y, o.w, lam)) < 1e-12 * max(1, abs(P))
        assert abs(D - dual(loss, X, y, o.alpha, lam)) < 1e-12 * max(1, abs(D))
        # P2 weak duality, P4 the two forms of the gap agree
        assert G >= -1e-13 and FY >= 0.0
        assert abs(G - FY) < 1e-12 * max(1.0, abs(P))
        # P6: sigma = K with adding never decreases the dual
        assert D >= prevD - 1e-13
        prevD = D
        if loss in ("hinge", "logistic"):
            assert o.alpha.min() >= 0.0 and o.alpha.max() <= 1.0
        assert o.alpha[7] == 0.0


# ----------------------------------------------------------------------------- P5
@pytest.mark.parametrize("K", [1, 4])
def test_ridge_closed_form(oracle_mod, K):
    n, d, lam = 200, 6, 0.05
    X, y = tiny_dense(n, d, 4, "squared")
    o = oracle_mod.OracleCoCoA("squared", n, d, lam, y, bounds(n, 32), X=X)
    hist = run_rounds(o, K, 2500 if K > 1 else 200)
    Xd, yd = X.astype(np.float64), y.astype(np.float64)
    wstar = np.linalg.solve(Xd.T @ Xd + lam * n * np.eye(d), Xd.T @ yd)
    assert np.linalg.norm(o.w - wstar) < 1e-9 * np.linalg.norm(wstar)
    assert np.max(np.abs(o.alpha - (yd - Xd @ wstar))) < 1e-8
    assert -1e-13 <= hist[-1][2] < 1e-12


def test_ridge_closed_form_on_workload(oracle_mod):
    cfg = get_config("dense_ridge", "mini")
    p = make_problem(cfg)
    p.lam = 1e-1          # the workload's own 1e-4 converges too slowly for a unit test
    o = oracle_mod.OracleCoCoA.from_problem(p)
    K = cfg["K"]
    c2s = oracle_mod.assign_greedy(p.chunk_nnz(), K)
    o.assign(K, c2s)
    for r in range(200):
        o.local_epoch(round_permutations(0, r, o.rows_per_solver()), keep_deltas=False)
        o.aggregate()
    Xd, yd = p.X.astype(np.float64), p.y.astype(np.float64)
    wstar = np.linalg.solve(Xd.T @ Xd + p.lam * p.n * np.eye(p.d), Xd.T @ yd)
    assert np.linalg.norm(o.w - wstar) < 1e-6 * np.linalg.norm(wstar)
    assert abs(o.gap()[2]) < 1e-10


# ----------------------------------------------------------------------------- P7
def _subproblem_value(loss, X, y, alpha, w, rows_k, dalpha_k, lam, sigma):
    """CoCoA local objective of worker k at the change dalpha_k of its dual variables,
    dropping the term that does not depend on dalpha_k:
    -1/n sum_{i in P_k} loss_i^*(-(alpha_i + dalpha_i)) - 1/n w.(A dalpha) - lam sigma/2 |A dalpha/(lam n)|^2
    with A's columns s_i x_i."""
    n = X.shape[0]
    a = alpha[rows_k] + dalpha_k
    Xk = X[rows_k].astype(np.float64)
    u = Xk.T @ (dalpha_k * s_vec(loss, y)[rows_k])
    if loss == "hinge":
        if np.any(a < 0) or np.any(a > 1):
            return -np.inf
        conj = -a
    elif loss == "logistic":
        if np.any(a < 0) or np.any(a > 1):
            return -np.inf
        conj = xlogx(a) + xlogx(1.0 - a)
    else:
        conj = 0.5 * a * a - a * y[rows_k]
    return -conj.sum() / n - (w @ u) / n - 0.5 * lam * sigma * (u @ u) / (lam * n) ** 2


@pytest.mark.parametrize("loss", ["hinge", "squared", "logistic"])
def test_single_step_is_argmax_of_local_objective(oracle_mod, loss):
    from oracle.cocoa import _load, _p
    L = _load()
    n, d, lam, sigma = 12, 5, 0.03, 3.0
    g = np.random.default_rng(8)
    X, y = tiny_dense(n, d, 9, loss)
    rp, col, val = to_csr(X)
    rows_k = np.array([1, 4, 6, 9], dtype=np.int64)
    for trial in range(24):
        boxed = loss in ("hinge", "logistic")
        code = {"hinge": 0, "squared": 1, "logistic": 2}[loss]
        alpha = g.random(n) if boxed else g.standard_normal(n)
        if boxed and trial % 3 == 0:
            alpha[rows_k] = g.integers(0, 2, size=rows_k.size).astype(np.float64)  # at the bounds
        w = g.standard_normal(d) * (3.0 if trial % 2 else 0.2)
        dalpha = np.zeros(rows_k.size)
        # some progress already made inside this pass
        dalpha[1:] = 0.1 * g.standard_normal(rows_k.size - 1)
        if boxed:
            dalpha = np.clip(alpha[rows_k] + dalpha, 0, 1) - alpha[rows_k]
        dalpha[0] = 0.0
        a_now = alpha.copy()
        a_now[rows_k] += dalpha
        # v = w + sigma * Delta w_k for the progress so far
        v = w + sigma * X[rows_k].astype(np.float64).T @ (dalpha * s_vec(loss, y)[rows_k]) / (lam * n)
        a_call, v_call = a_now.copy(), v.copy()
        one = np.array([rows_k[0]], dtype=np.int64)
        zero = np.zeros(1, dtype=np.int32)
        for sparse in (True, False):
            a_call, v_call = a_now.copy(), v.copy()
            if sparse:
                L.oracle_local_epoch_csr(code, 1, _p(one), _p(zero), _p(rp), _p(col),
                                         _p(val), _p(y), _p(a_call), _p(v_call), lam, n, sigma)
            else:
                L.oracle_local_epoch_dense(code, 1, _p(one), _p(zero), _p(X), d,
                                           _p(y), _p(a_call), _p(v_call), lam, n, sigma)
            delta = a_call[rows_k[0]] - a_now[rows_k[0]]
            # only that row's dual variable moved, and v moved along s_i x_i by sigma*delta/(lam n)
            moved = np.nonzero(a_call != a_now)[0]
            assert set(moved) <= {rows_k[0]}
            want_v = v + sigma * delta * s_vec(loss, y)[rows_k[0]] * X[rows_k[0]].astype(np.float64) / (lam * n)
            assert np.allclose(v_call, want_v, rtol=0, atol=1e-13)

            def f(dl):
                da = dalpha.copy()
                da[0] = dl
                return _subproblem_value(loss, X, y, alpha, w, rows_k, da, lam, sigma)

            if boxed:
                lo, hi = -alpha[rows_k[0]], 1.0 - alpha[rows_k[0]]
            else:
                lo, hi = delta - 5.0, delta + 5.0
            grid = np.linspace(lo, hi, 2001)
            vals = np.array([f(t) for t in grid])
            best = grid[np.argmax(vals)]
            res = scipy.optimize.minimize_scalar(lambda t: -f(t), bounds=(lo, hi), method="bounded",
                                                 options={"xatol": 1e-12})
            cand = max([best, res.x], key=f)
            assert abs(delta - cand) < 1e-3 * max(1.0, hi - lo)
            assert f(delta) >= f(cand) - 1e-12
            assert f(delta) >= vals.max() - 1e-12


# ----------------------------------------------------------------------------- P8
def test_hinge_tiny_grid_search(oracle_mod):
    lam = 0.3
    X = np.array([[1.0, 0.5], [-0.4, 1.0], [0.9, -0.2]], dtype=np.float32)
    y = np.array([1.0, -1.0, -1.0], dtype=np.float32)
    o = oracle_mod.OracleCoCoA("hinge", 3, 2, lam, y, bounds(3, 1), X=X)
    run_rounds(o, 1, 300)
    grid = np.linspace(0, 1, 51)
    bestD, besta = -np.inf, None
    for a in itertools.product(grid, repeat=3):
        Dv = dual("hinge", X, y, np.array(a), lam)
        if Dv > bestD:
            bestD, besta = Dv, np.array(a)
    Dor = dual("hinge", X, y, o.alpha, lam)
    assert Dor >= bestD - 1e-12
    assert np.max(np.abs(o.alpha - besta)) <= 0.021
    assert o.gap()[2] < 1e-10


@pytest.mark.parametrize("K", [1, 2, 4])
def test_hinge_matches_box_qp_solver(oracle_mod, K):
    """The dual optimum found by a library bound-constrained optimiser is what CoCoA converges to."""
    n, d, lam = 40, 4, 0.05
    X, y = tiny_dense(n, d, 21, "hinge")
    o = oracle_mod.OracleCoCoA("hinge", n, d, lam, y, bounds(n, 5), X=X)
    hist = run_rounds(o, K, 3000)
    Xd = X.astype(np.float64)
    A = Xd * y[:, None].astype(np.float64)
    Q = A @ A.T / (lam * n * n)

    def negD(a):
        return 0.5 * a @ Q @ a - a.mean(), Q @ a - 1.0 / n

    res = scipy.optimize.minimize(negD, np.zeros(n), jac=True, bounds=[(0, 1)] * n, method="L-BFGS-B",
                                  options={"maxiter": 20000, "ftol": 1e-16, "gtol": 1e-12})
    Dstar = -res.fun
    assert abs(hist[-1][1] - Dstar) < 1e-7
    assert hist[-1][2] < 1e-6
    wq = w_of_alpha("hinge", X, y, res.x, lam)
    assert np.linalg.norm(o.w - wq) < 1e-3 * np.linalg.norm(wq)


def test_separable_gap_goes_to_zero(oracle_mod):
    X, y = tiny_dense(60, 5, 33, "hinge", separable=True)
    o = oracle_mod.OracleCoCoA("hinge", 60, 5, 1e-2, y, bounds(60, 8), X=X)
    hist = run_rounds(o, 2, 1500)
    gaps = [h[2] for h in hist]
    assert gaps[-1] < 1e-8 and gaps[-1] >= -1e-14
    assert gaps[-1] < gaps[10] < gaps[0]


# ----------------------------------------------------------------------------- safe aggregation
@pytest.mark.parametrize("loss", ["hinge", "squared", "logistic"])
def test_sum_of_local_objectives_bounds_the_dual(oracle_mod, loss):
    """With sigma = K and adding, D(alpha + sum_k dalpha_k) >= sum_k G_k(dalpha_k), where G_k carries
    the 1/K share of -lam/2 |w|^2 (the separable lower bound CoCoA maximises)."""
    n, d, lam, K = 90, 6, 0.02, 3
    X, y = tiny_dense(n, d, 17, loss)
    o = oracle_mod.OracleCoCoA(loss, n, d, lam, y, bounds(n, 10), X=X)
    o.assign(K, np.arange(9) % K)
    for r in range(4):
        a0, w0 = o.alpha.copy(), o.w.copy()
        o.local_epoch(round_permutations(3, r, o.rows_per_solver()))
        o.aggregate()
        total = 0.0
        for k in range(K):
            rk = o.rows_of[k]
            total += _subproblem_value(loss, X, y, a0, w0, rk, o.alpha[rk] - a0[rk], lam, float(K))
            total += -0.5 * lam * (w0 @ w0) / K
        assert dual(loss, X, y, o.alpha, lam) >= total - 1e-12
        # and each local pass did improve its own objective over doing nothing
        for k in range(K):
            rk = o.rows_of[k]
            z = np.zeros(rk.size)
            assert _subproblem_value(loss, X, y, a0, w0, rk, o.alpha[rk] - a0[rk], lam, float(K)) >= \
                _subproblem_value(loss, X, y, a0, w0, rk, z, lam, float(K)) - 1e-14


@pytest.mark.parametrize("K", [1, 3])
def test_logistic_reaches_the_primal_optimum(oracle_mod, K):
    """Regularised logistic regression has a smooth primal: a library quasi-Newton method on P(w) gives
    w* to high accuracy; the oracle's rounds must close the gap and arrive at the same w and P."""
    n, d, lam = 150, 6, 0.05
    X, y = tiny_dense(n, d, 21, "logistic")
    o = oracle_mod.OracleCoCoA("logistic", n, d, lam, y, bounds(n, 25), X=X)
    hist = run_rounds(o, K, 120 if K == 1 else 400)
    Xd, yd = X.astype(np.float64), y.astype(np.float64)

    def f(w):
        z = Xd @ w
        val = 0.5 * lam * w @ w + np.logaddexp(0.0, -yd * z).mean()
        grad = lam * w - Xd.T @ (yd / (1.0 + np.exp(yd * z))) / n
        return val, grad

    res = scipy.optimize.minimize(f, np.zeros(d), jac=True, method="L-BFGS-B",
                                  options={"ftol": 1e-15, "gtol": 1e-12, "maxiter": 2000})
    P, D, G, FY = hist[-1]
    assert G < 1e-8 and abs(P - res.fun) < 1e-8
    assert np.linalg.norm(o.w - res.x) < 1e-4 * max(1.0, np.linalg.norm(res.x))
    # at the optimum the dual variables are the loss derivatives: a_i = 1 / (1 + exp(y_i x_i.w))
    assert np.max(np.abs(o.alpha - 1.0 / (1.0 + np.exp(yd * (Xd @ res.x))))) < 1e-3


def test_delta_w_is_image_of_delta_alpha(oracle_mod):
    n, d, lam, K = 64, 5, 0.1, 4
    X, y = tiny_dense(n, d, 2, "hinge")
    o = oracle_mod.OracleCoCoA("hinge", n, d, lam, y, bounds(n, 8), X=X)
    o.assign(K, np.array([0, 1, 2, 3, 3, 2, 1, 0]))
    a0 = o.alpha.copy()
    dws = o.local_epoch(round_permutations(0, 0, o.rows_per_solver()))
    for k in range(K):
        rk = o.rows_of[k]
        want = X[rk].astype(np.float64).T @ ((o.alpha[rk] - a0[rk]) * y[rk]) / (lam * n)
        assert np.allclose(dws[k], want, rtol=0, atol=1e-14)
    s = o.aggregate()
    assert np.allclose(s, sum(dws), rtol=0, atol=1e-15)


# ----------------------------------------------------------------------------- P9 assignment
def _lpt_reference(load, K, speed):
    order = sorted(range(len(load)), key=lambda c: (-load[c], c))
    L = [0] * K
    out = [None] * len(load)
    for c in order:
        fin = [Fraction(L[k] + load[c], speed[k] if speed else 1) for k in range(K)]
        best = min(range(K), key=lambda k: (fin[k], k))
        out[c] = best
        L[best] += load[c]
    return out


def test_assignment_matches_exact_rational_greedy(oracle_mod):
    g = np.random.default_rng(0)
    for trial in range(40):
        nchunks = int(g.integers(1, 60))
        K = int(g.integers(1, 12))
        load = g.integers(1, 50, size=nchunks) if trial % 2 else np.full(nchunks, 7)
        speed = None if trial % 3 == 0 else [int(x) for x in g.integers(1, 4, size=K)]
        got = oracle_mod.assign_greedy(load, K, speed)
        assert list(got) == _lpt_reference([int(x) for x in load], K, speed)
        assert got.min() >= 0 and got.max() < K and got.size == nchunks
    # huge loads must not overflow the comparison
    big = np.array([2**61, 2**61 - 1, 2**60], dtype=np.int64)
    assert list(oracle_mod.assign_greedy(big, 2, [3, 2])) == _lpt_reference([int(x) for x in big], 2, [3, 2])


def test_assignment_reaches_paper_heterogeneous_makespan(oracle_mod):
    """8 fast + 8 slow (1.5x slower) solvers, many equal chunks: fast solvers get 1.5x the load and
    the iteration takes 1.2 units (Section 5.4 methodology)."""
    nchunks = 16 * 600
    speed = [3] * 8 + [2] * 8
    c2s = oracle_mod.assign_greedy(np.ones(nchunks, dtype=np.int64), 16, speed)
    cnt = np.bincount(c2s, minlength=16)
    assert cnt.sum() == nchunks
    unit = nchunks / 16.0                      # one task on 1/16 of the data
    times = np.array([cnt[k] / unit * (1.0 if speed[k] == 3 else 1.5) for k in range(16)])
    assert abs(times.max() - 1.2) < 0.005
    assert abs(cnt[:8].mean() / cnt[8:].mean() - 1.5) < 0.01


def test_projection_examples_from_paper(oracle_mod):
    path = os.path.join(os.path.dirname(__file__), "golden", "projection_examples.txt")
    seen = 0
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, K, nodes, n_slow, sf, want, digits = line.split()
        got = oracle_mod.projected_round_time(None if K == "uni" else int(K), int(nodes),
                                              slow_factor=None if sf == "-" else float(sf),
                                              n_slow=int(n_slow))
        assert round(got, int(digits)) == float(want), name
        seen += 1
    assert seen == 4


# ----------------------------------------------------------------------------- P10 + contract
def test_state_travels_with_chunks_and_contract(oracle_mod):
    cfg = get_config("elastic", "mini")
    p = make_problem(cfg)
    o = oracle_mod.OracleCoCoA.from_problem(p)
    prev_gap = None
    from workloads.configs import speeds_for
    K = None
    gaps = []
    for r in range(cfg["rounds"]):
        Kr = k_for_round(cfg, r)
        if Kr != K:
            before = o.alpha.copy()
            K = Kr
            c2s = oracle_mod.assign_greedy(p.chunk_nnz(), K, speeds_for(cfg, K))
            o.assign(K, c2s)
            assert np.array_equal(before, o.alpha)
            owned = np.concatenate(o.rows_of)
            assert np.array_equal(np.sort(owned), np.arange(p.n))       # every row owned exactly once
        o.local_epoch(round_permutations(cfg["seed"], r, o.rows_per_solver()), keep_deltas=False)
        with pytest.raises(RuntimeError):
            o.assign(K, c2s)                                            # scheduler must wait
        with pytest.raises(RuntimeError):
            o.local_epoch(round_permutations(cfg["seed"], r, o.rows_per_solver()))
        o.aggregate()
        gaps.append(o.gap()[2])
    assert all(g >= 0 for g in gaps) and gaps[-1] < gaps[0]


def test_zero_chunk_solver_and_bad_tables(oracle_mod):
    X, y = tiny_dense(30, 4, 1, "hinge")
    o = oracle_mod.OracleCoCoA("hinge", 30, 4, 0.1, y, bounds(30, 10), X=X)
    o.assign(4, [0, 1, 3])                  # solver 2 owns nothing
    dws = o.local_epoch(round_permutations(0, 0, o.rows_per_solver()))
    assert np.all(dws[2] == 0.0)
    o.aggregate()
    with pytest.raises(ValueError):
        o.assign(2, [0, 1, 2])
    with pytest.raises(ValueError):
        o.assign(2, [0, 1])
    o.assign(2, [0, 1, 1])
    with pytest.raises(ValueError):
        o.local_epoch([np.arange(10, dtype=np.int32), np.zeros(20, dtype=np.int32)])


# ----------------------------------------------------------------------------- elastic net
# Regulariser lambda (|w|^2 / 2 + l1 |w|_1) (Section 2.2 speaks of generalised linear models in general).
# The pins: the lasso-type optimum from scikit-learn's coordinate descent (a different algorithm on the
# primal), optimality of that point under the oracle's own primal value, weak duality with a gap that
# closes, the primal vector as the soft-thresholded image of alpha, and l1 = 0 leaving everything as it was.
def test_elastic_net_squared_loss_matches_coordinate_descent(oracle_mod):
    from sklearn.linear_model import ElasticNet
    n, d, lam, l1 = 120, 10, 0.05, 4.0
    X, y = tiny_dense(n, d, 21, "squared")
    o = oracle_mod.OracleCoCoA("squared", n, d, lam, y, bounds(n, 16), X=X, l1=l1)
    hist = run_rounds(o, 3, 3000)
    # scikit-learn minimises 1/(2n) |y - Xw|^2 + a r |w|_1 + a (1 - r) / 2 |w|^2
    a, r = lam * (1.0 + l1), l1 / (1.0 + l1)
    ref = ElasticNet(alpha=a, l1_ratio=r, fit_intercept=False, tol=1e-14, max_iter=1000000)
    ref.fit(X.astype(np.float64), y.astype(np.float64))
    assert np.count_nonzero(ref.coef_ == 0.0) >= 1 and np.count_nonzero(ref.coef_) >= 2   # the term bites
    assert np.linalg.norm(o.w - ref.coef_) < 1e-7 * np.linalg.norm(ref.coef_)
    assert np.array_equal(o.w == 0.0, ref.coef_ == 0.0)
    P, D, G, _ = hist[-1]
    assert -1e-12 <= G < 1e-10
    # that point is optimal under the oracle's own primal value: no coordinate move of the other solver's
    # solution lowers it (a wrong weight of the |w|_1 term would move the optimum)
    o.w = ref.coef_.copy()
    P0 = o.gap()[0]
    for j in range(d):
        for step in (1e-4, -1e-4):
            o.w = ref.coef_.copy()
            o.w[j] += step
            assert o.gap()[0] >= P0 - 1e-13


@pytest.mark.parametrize("loss", ["hinge", "logistic"])
def test_elastic_net_duality(oracle_mod, loss):
    n, d, lam, l1 = 150, 12, 0.02, 0.8
    X, y = tiny_dense(n, d, 22, loss)
    o = oracle_mod.OracleCoCoA(loss, n, d, lam, y, bounds(n, 16), X=X, l1=l1)
    o.assign(3, np.arange(o.chunk_bounds.size - 1, dtype=np.int32) % 3)
    Xd, yd = X.astype(np.float64), y.astype(np.float64)
    prevD, gaps = -np.inf, []
    for r in range(1500):
        o.local_epoch(round_permutations(3, r, o.rows_per_solver()), keep_deltas=False)
        o.aggregate()
        P, D, G, FY = o.gap()
        # w is the soft-thresholded image of alpha
        v = Xd.T @ (o.alpha * yd) / (lam * n)
        assert np.max(np.abs(o.w - np.sign(v) * np.maximum(np.abs(v) - l1, 0.0))) < 1e-12
        assert G >= -1e-12 and D >= prevD - 1e-12          # weak duality; adding with sigma = K never lowers D
        assert abs(G - FY) < 1e-10 * max(1.0, abs(P))      # regulariser and its conjugate meet at w = grad g*(v)
        prevD = D
        gaps.append(G)
    assert gaps[-1] < 1e-4 * gaps[0]                       # ... and the gap closes: P and D bracket the optimum
    assert np.count_nonzero(o.w == 0.0) >= 1
    # the primal value at that w is minimal against a derivative-free search from it (non-smooth objective)
    def Pw(w):
        z = Xd @ w
        l = np.maximum(0.0, 1.0 - yd * z) if loss == "hinge" else np.logaddexp(0.0, -yd * z)
        return l.mean() + lam * (0.5 * w @ w + l1 * np.abs(w).sum())
    res = scipy.optimize.minimize(Pw, o.w, method="Powell", options={"xtol": 1e-10, "ftol": 1e-14, "maxiter": 20000})
    assert res.fun >= o.gap()[1] - 1e-9                    # nothing found below the dual value
    assert res.fun >= Pw(o.w) - 2.0 * gaps[-1]             # ... nor more than the remaining gap below the oracle's point
    assert abs(Pw(o.w) - o.gap()[0]) < 1e-12


def test_elastic_net_with_zero_l1_is_the_plain_round(oracle_mod):
    n, d, lam = 90, 7, 0.03
    X, y = tiny_dense(n, d, 23, "hinge")
    a = oracle_mod.OracleCoCoA("hinge", n, d, lam, y, bounds(n, 16), X=X)
    b = oracle_mod.OracleCoCoA("hinge", n, d, lam, y, bounds(n, 16), X=X, l1=0.0)
    ha, hb = run_rounds(a, 2, 20), run_rounds(b, 2, 20)
    assert ha == hb and np.array_equal(a.w, b.w) and np.array_equal(a.alpha, b.alpha)
