"""Pins for the oracle's augmented Lagrangian (Eq. (augLag), Algorithm 4 of the appendix) with linear
constraints on the least-squares objective.

The paper prints no worked example of Algorithm 4, so the pins are what the mathematics fixes:
  * the minimiser of an equality-constrained least-squares problem with no active bound solves the
    linear KKT system [A^T A, C^T; C, 0][x; nu] = [A^T b; d], and the multipliers converge to nu;
  * least squares over the simplex (the example problem of the section "Complete Framework": sum(x) = 1,
    x >= 0) against brute-force enumeration of supports, n <= 8;
  * inequality-constrained problems against scipy's trust-constr solver, and the KKT conditions of the constrained
    problem at the returned point (stationarity over the box, feasibility, mu >= 0, complementarity);
  * the value / gradient pair of Eq. (augLag) by central differences, and its limiting cases.
"""
import itertools

import numpy as np
import pytest
from scipy.optimize import Bounds, LinearConstraint, minimize

import oracle


def _problem(rng, rows, n, n_eq, n_in):
    A = rng.standard_normal((rows, n))
    b = rng.standard_normal(rows)
    C = rng.standard_normal((n_eq, n))
    E = rng.standard_normal((n_in, n))
    x_feas = rng.random(n)
    d = C @ x_feas
    e = E @ x_feas + rng.random(n_in) * 0.5          # x_feas is strictly feasible for the inequalities
    return A, b, C, d, E, e


def test_value_and_gradient_of_the_augmented_lagrangian_agree_by_central_differences():
    rng = np.random.default_rng(5)
    A, b, C, d, E, e = _problem(rng, 30, 7, 2, 3)
    lam, mu = rng.standard_normal(2), rng.random(3)
    obj = oracle.Objective(oracle.LSQ, A, b).set_constraints(C, d, E, e, lam=lam, mu=mu, rho=3.0)
    for _ in range(5):
        x = rng.standard_normal(7)
        f, g = oracle.fg(obj, x)
        for i in range(7):
            h = 1e-6
            xp, xm = x.copy(), x.copy()
            xp[i] += h
            xm[i] -= h
            fd = (oracle.f_only(obj, xp) - oracle.f_only(obj, xm)) / (2 * h)
            assert fd == pytest.approx(g[i], rel=1e-6, abs=1e-6)


def test_limiting_cases_of_the_penalty_terms():
    rng = np.random.default_rng(6)
    A, b, C, d, E, e = _problem(rng, 20, 5, 1, 2)
    plain = oracle.Objective(oracle.LSQ, A, b)
    x = rng.standard_normal(5)
    f0, g0 = oracle.fg(plain, x)
    # (i) multipliers zero and the point satisfies h = 0, g < 0: the penalties vanish
    d_here, e_here = C @ x, E @ x + 1.0
    obj = oracle.Objective(oracle.LSQ, A, b).set_constraints(C, d_here, E, e_here, rho=10.0)
    f1, g1 = oracle.fg(obj, x)
    assert f1 == pytest.approx(f0, rel=1e-14)
    np.testing.assert_allclose(g1, g0, rtol=1e-13, atol=1e-13)
    # (ii) an inequality row is inactive in the penalty exactly while g + mu/rho <= 0
    mu = np.array([0.5, 0.0])
    obj = oracle.Objective(oracle.LSQ, A, b).set_constraints(None, None, E, E @ x + np.array([0.5 / 10.0, 1.0]),
                                                             mu=mu, rho=10.0)
    f2, _ = oracle.fg(obj, x)
    assert f2 == pytest.approx(f0, rel=1e-14)            # g_0 + mu_0/rho = 0 exactly at the kink
    # (iii) equality row with h = 1, lambda = 2, rho = 4: rho/2 (1 + 2/4)^2 = 4.5
    obj = oracle.Objective(oracle.LSQ, A, b).set_constraints(C, C @ x - 1.0, lam=[2.0], rho=4.0)
    f3, g3 = oracle.fg(obj, x)
    assert f3 - f0 == pytest.approx(4.5, rel=1e-12)
    np.testing.assert_allclose(g3 - g0, 4.0 * 1.5 * C[0], rtol=1e-12)


def test_difference_form_matches_the_difference_of_values():
    rng = np.random.default_rng(7)
    A, b, C, d, E, e = _problem(rng, 25, 6, 2, 3)
    obj = oracle.Objective(oracle.LSQ, A, b).set_constraints(C, d, E, e, lam=rng.standard_normal(2), mu=rng.random(3),
                                                             rho=2.0)
    x = rng.standard_normal(6)
    f, _, row = oracle.fg(obj, x, want_rowvec=True)
    for scale in (1.0, 1e-3, 1e-8):
        xt = x + scale * rng.standard_normal(6)
        df = oracle.delta_f(obj, x, xt, row)
        assert df == pytest.approx(oracle.f_only(obj, xt) - f, rel=1e-6, abs=1e-13 * abs(f))


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_equality_constrained_least_squares_solves_the_kkt_system(seed):
    rng = np.random.default_rng(seed)
    n, n_eq = 9, 3
    A, b, C, d, _, _ = _problem(rng, 40, n, n_eq, 0)
    K = np.block([[A.T @ A, C.T], [C, np.zeros((n_eq, n_eq))]])
    sol = np.linalg.solve(K, np.concatenate([A.T @ b, d]))
    x_ref, nu = sol[:n], sol[n:]
    obj = oracle.Objective(oracle.LSQ, A, b).set_constraints(C, d)
    x, lam, mu, info = oracle.auglag_solve(obj, np.full(n, -np.inf), np.full(n, np.inf), np.zeros(n), 6,
                                           oracle.default_options(tol=1e-10), ctol=1e-9)
    assert info.status == oracle.CONVERGED
    assert info.violation <= 1e-9
    np.testing.assert_allclose(x, x_ref, atol=1e-7)
    np.testing.assert_allclose(lam, nu, rtol=1e-5, atol=1e-6)   # L = f + lambda^T h: same sign as the KKT system's nu
    assert info.f == pytest.approx(0.5 * np.sum((A @ x_ref - b) ** 2), rel=1e-7)


def _simplex_lsq_brute_force(A, b):
    """argmin 0.5||Ax-b||^2 s.t. sum(x) = 1, x >= 0 by enumerating supports."""
    n = A.shape[1]
    best = None
    for k in range(1, n + 1):
        for F in itertools.combinations(range(n), k):
            F = list(F)
            AF = A[:, F]
            K = np.block([[AF.T @ AF, np.ones((k, 1))], [np.ones((1, k)), np.zeros((1, 1))]])
            try:
                sol = np.linalg.solve(K, np.concatenate([AF.T @ b, [1.0]]))
            except np.linalg.LinAlgError:
                continue
            xF, nu = sol[:k], sol[k]
            if np.any(xF < -1e-12):
                continue
            x = np.zeros(n)
            x[F] = xF
            grad = A.T @ (A @ x - b) + nu                # stationarity needs grad_j >= 0 off the support
            off = np.setdiff1d(np.arange(n), F)
            if np.all(grad[off] >= -1e-10):
                fval = 0.5 * np.sum((A @ x - b) ** 2)
                if best is None or fval < best[1]:
                    best = (x, fval, nu)
    return best


@pytest.mark.parametrize("seed,n", [(0, 4), (1, 6), (2, 8)])
def test_least_squares_over_the_simplex_against_support_enumeration(seed, n):
    rng = np.random.default_rng(seed)
    A = rng.standard_normal((3 * n, n))
    b = A @ rng.dirichlet(np.ones(n) * 0.3) + 0.3 * rng.standard_normal(3 * n)
    x_ref, f_ref, nu = _simplex_lsq_brute_force(A, b)
    obj = oracle.Objective(oracle.LSQ, A, b).set_constraints(np.ones((1, n)), [1.0])
    x, lam, mu, info = oracle.auglag_solve(obj, np.zeros(n), np.full(n, np.inf), np.zeros(n), 5,
                                           oracle.default_options(tol=1e-10), ctol=1e-9)
    assert info.status == oracle.CONVERGED
    assert abs(x.sum() - 1.0) <= 1e-9 and np.all(x >= 0)
    np.testing.assert_allclose(x, x_ref, atol=1e-6)
    assert info.f == pytest.approx(f_ref, rel=1e-6)
    assert lam[0] == pytest.approx(nu, rel=1e-4, abs=1e-6)
    assert np.array_equal(x <= 1e-9, x_ref <= 1e-9)


@pytest.mark.parametrize("seed", [3, 4, 5])
def test_inequalities_and_a_box_against_scipy_and_the_kkt_conditions(seed):
    rng = np.random.default_rng(seed)
    n, n_eq, n_in = 8, 1, 4
    A, b, C, d, E, e = _problem(rng, 30, n, n_eq, n_in)
    l, u = np.zeros(n), np.full(n, 1.0)
    ref = minimize(lambda x: 0.5 * np.sum((A @ x - b) ** 2), np.full(n, 0.5), jac=lambda x: A.T @ (A @ x - b),
                   hess=lambda x: A.T @ A, method="trust-constr", bounds=Bounds(l, u),
                   constraints=[LinearConstraint(C, d, d), LinearConstraint(E, -np.inf, e)],
                   options={"gtol": 1e-12, "xtol": 1e-14, "barrier_tol": 1e-12, "maxiter": 2000})
    obj = oracle.Objective(oracle.LSQ, A, b).set_constraints(C, d, E, e)
    x, lam, mu, info = oracle.auglag_solve(obj, l, u, np.zeros(n), 6, oracle.default_options(tol=1e-10), ctol=1e-9,
                                           max_outer=200)
    assert info.status == oracle.CONVERGED
    np.testing.assert_allclose(x, ref.x, atol=1e-5)
    assert info.f == pytest.approx(ref.fun, rel=1e-6, abs=1e-8)
    # KKT conditions of the constrained problem
    assert np.all(x >= l) and np.all(x <= u)
    assert np.max(np.abs(C @ x - d)) <= 1e-9 and np.max(E @ x - e) <= 1e-9
    assert np.all(mu >= 0)
    assert np.max(np.abs(mu * (E @ x - e))) <= 1e-6                      # complementarity
    grad_lagr = A.T @ (A @ x - b) + C.T @ lam + E.T @ mu
    assert np.max(np.abs(x - np.clip(x - grad_lagr, l, u))) <= 1e-6       # stationarity over the box


def test_without_constraints_one_outer_iteration_is_the_box_solve():
    rng = np.random.default_rng(9)
    A, b = rng.standard_normal((30, 6)), rng.standard_normal(30)
    l, u = np.zeros(6), np.full(6, np.inf)
    plain = oracle.Objective(oracle.LSQ, A, b)
    s = oracle.Solver(plain, l, u, np.zeros(6), 5, oracle.default_options(tol=1e-10))
    ref = s.solve()
    s.close()
    obj = oracle.Objective(oracle.LSQ, A, b).set_constraints()
    x, lam, mu, info = oracle.auglag_solve(obj, l, u, np.zeros(6), 5, oracle.default_options(tol=1e-10))
    assert info.status == oracle.CONVERGED and info.outer == 1 and info.violation == 0.0
    np.testing.assert_array_equal(x, ref.x)
    assert info.inner_iters == ref.info.iters


def test_rho_is_doubled_exactly_when_the_violation_is_not_halved():
    # one variable, f = 0.5 c x^2, constraint x = 1: the inner minimiser is x = (rho - lambda)/(c + rho), so the
    # violation shrinks by the factor c/(c + rho) per outer iteration.  c = 1/4, rho = 1: factor 0.2, always
    # more than halved, rho must stay 1 and 0.2^k <= 1e-6 first holds at k = 9
    A, b = 0.5 * np.ones((1, 1)), np.zeros(1)
    obj = oracle.Objective(oracle.LSQ, A, b).set_constraints(np.ones((1, 1)), [1.0])
    x, lam, mu, info = oracle.auglag_solve(obj, [-np.inf], [np.inf], [0.0], 3, oracle.default_options(tol=1e-13),
                                           ctol=1e-6, max_outer=60)
    assert info.status == oracle.CONVERGED
    assert info.rho == 1.0
    assert info.outer == 9
    assert info.violation == pytest.approx(0.2 ** 9, rel=1e-6)
    assert lam[0] == pytest.approx(-0.25, abs=1e-6)
    # c = 9: factor 0.9 at rho = 1, not halved: rho must grow
    obj = oracle.Objective(oracle.LSQ, 3.0 * np.ones((1, 1)), b).set_constraints(np.ones((1, 1)), [1.0])
    x, lam, mu, info = oracle.auglag_solve(obj, [-np.inf], [np.inf], [0.0], 3, oracle.default_options(tol=1e-13),
                                           ctol=1e-6, max_outer=60)
    assert info.status == oracle.CONVERGED
    assert info.rho > 1.0
    assert x[0] == pytest.approx(1.0, abs=1e-6) and lam[0] == pytest.approx(-9.0, rel=1e-5)
