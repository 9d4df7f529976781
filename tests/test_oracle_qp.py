"""Pins for the oracle's quadratic-form objective (the dual SVM objective of the paper's section
"Dual SVM": 0.5 (a.y)^T K (a.y) - sum(a), s.t. y^T a = 0, 0 <= a <= c).

  * value / gradient by central differences; the difference form against differences of values;
  * no active bound: the minimiser solves Q x = -b with Q = diag(s) K diag(s);
  * box-constrained: brute force over all assignments {at l, free, at u} for n <= 7;
  * the dual SVM with the equality constraint (Algorithm 4) against scikit-learn's SVC on a precomputed
    Gaussian kernel: dual coefficients, objective value, y^T a = 0.
"""
import itertools

import numpy as np
import pytest

import oracle


def _spd(rng, n, shift=0.5):
    M = rng.standard_normal((n, n))
    return M @ M.T / n + shift * np.eye(n)


def test_value_gradient_and_difference_form():
    rng = np.random.default_rng(1)
    n = 9
    K, b = _spd(rng, n), rng.standard_normal(n)
    s = np.where(rng.random(n) < 0.5, -1.0, 1.0)
    obj = oracle.Objective(oracle.QP, K, b, sign=s)
    x = rng.standard_normal(n)
    f, g, row = oracle.fg(obj, x, want_rowvec=True)
    for i in range(n):
        h = 1e-5
        xp, xm = x.copy(), x.copy()
        xp[i] += h
        xm[i] -= h
        assert (oracle.f_only(obj, xp) - oracle.f_only(obj, xm)) / (2 * h) == pytest.approx(g[i], rel=1e-8, abs=1e-8)
    for scale in (1.0, 1e-4, 1e-9):
        xt = x + scale * rng.standard_normal(n)
        assert oracle.delta_f(obj, x, xt, row) == pytest.approx(oracle.f_only(obj, xt) - f, rel=1e-6, abs=1e-14 * abs(f))
    # f is a quadratic form: f(2x) - 2 f(x) = x^T Q x = 2 (f(x) - b.x)
    assert oracle.f_only(obj, 2 * x) - 2 * f == pytest.approx(2 * (f - b @ x), rel=1e-12)


@pytest.mark.parametrize("seed", [0, 1])
def test_without_active_bounds_the_minimiser_solves_the_linear_system(seed):
    rng = np.random.default_rng(seed)
    n = 12
    K, b = _spd(rng, n), rng.standard_normal(n)
    s = np.where(rng.random(n) < 0.5, -1.0, 1.0)
    obj = oracle.Objective(oracle.QP, K, b, sign=s)
    sol = oracle.Solver(obj, np.full(n, -np.inf), np.full(n, np.inf), np.zeros(n), 6, oracle.default_options(tol=1e-11))
    res = sol.solve()
    sol.close()
    Q = (s[:, None] * K) * s[None, :]
    assert res.info.status == oracle.CONVERGED
    np.testing.assert_allclose(res.x, np.linalg.solve(Q, -b), atol=1e-9)


def _box_qp_brute_force(Q, b, l, u):
    n = len(b)
    best = None
    for assign in itertools.product((0, 1, 2), repeat=n):       # 0 at l, 1 free, 2 at u
        a = np.array(assign)
        x = np.where(a == 0, l, u).astype(float)
        F = np.flatnonzero(a == 1)
        if F.size:
            rhs = -b[F] - Q[np.ix_(F, np.flatnonzero(a != 1))] @ x[a != 1]
            try:
                x[F] = np.linalg.solve(Q[np.ix_(F, F)], rhs)
            except np.linalg.LinAlgError:
                continue
            if np.any(x[F] < l[F] - 1e-12) or np.any(x[F] > u[F] + 1e-12):
                continue
        g = Q @ x + b
        if np.all(g[a == 0] >= -1e-10) and np.all(g[a == 2] <= 1e-10):
            fval = 0.5 * x @ Q @ x + b @ x
            if best is None or fval < best[1]:
                best = (x, fval)
    return best


@pytest.mark.parametrize("seed,n", [(0, 5), (1, 6), (2, 7)])
def test_box_constrained_against_enumeration_of_active_sets(seed, n):
    rng = np.random.default_rng(seed)
    K, b = _spd(rng, n), 2.0 * rng.standard_normal(n)
    s = np.where(rng.random(n) < 0.5, -1.0, 1.0)
    l, u = np.zeros(n), np.ones(n)
    Q = (s[:, None] * K) * s[None, :]
    x_ref, f_ref = _box_qp_brute_force(Q, b, l, u)
    obj = oracle.Objective(oracle.QP, K, b, sign=s)
    sol = oracle.Solver(obj, l, u, np.full(n, 0.5), 5, oracle.default_options(tol=1e-11))
    res = sol.solve()
    sol.close()
    assert res.info.status == oracle.CONVERGED
    np.testing.assert_allclose(res.x, x_ref, atol=1e-9)
    assert res.info.f == pytest.approx(f_ref, rel=1e-10, abs=1e-12)


@pytest.mark.parametrize("seed,n", [(3, 40), (4, 80)])
def test_dual_svm_against_scikit_learn(seed, n):
    from sklearn.svm import SVC
    rng = np.random.default_rng(seed)
    y = np.where(np.arange(n) % 2 == 0, 1.0, -1.0)
    X = rng.standard_normal((n, 3)) * 0.7 + 0.6 * y[:, None]
    D2 = ((X[:, None, :] - X[None, :, :]) ** 2).sum(-1)
    K = np.exp(-1.0 * D2)                                        # Gaussian kernel, gamma = 1 as in the paper
    c = 1.0
    svc = SVC(C=c, kernel="precomputed", tol=1e-10).fit(K, y)
    alpha_ref = np.zeros(n)
    alpha_ref[svc.support_] = np.abs(svc.dual_coef_[0])          # dual_coef_ holds y_i alpha_i
    obj = oracle.Objective(oracle.QP, K, -np.ones(n), sign=y).set_constraints(y[None, :], [0.0])
    a, lam, mu, info = oracle.auglag_solve(obj, np.zeros(n), np.full(n, c), np.zeros(n), 8,
                                           oracle.default_options(tol=1e-10), ctol=1e-10, max_outer=200)
    assert info.status == oracle.CONVERGED
    assert abs(y @ a) <= 1e-10 and np.all(a >= 0) and np.all(a <= c)
    Q = (y[:, None] * K) * y[None, :]
    f_ref = 0.5 * alpha_ref @ Q @ alpha_ref - alpha_ref.sum()
    assert info.f == pytest.approx(f_ref, rel=1e-7)
    np.testing.assert_allclose(a, alpha_ref, atol=2e-5)
    # the multiplier of y^T a = 0 is the SVM's bias up to sign: decision values of free support vectors are +-1
    free = (a > 1e-6) & (a < c - 1e-6)
    if free.any():
        margins = y[free] * (K[free] @ (a * y) + lam[0])
        np.testing.assert_allclose(margins, 1.0, atol=1e-5)
        assert lam[0] == pytest.approx(svc.intercept_[0], abs=1e-4)
