"""Pins for the oracle's regularised optimal-transport objective (the paper's section "Joint Probability
Distribution": min <M,P> + lambda r(P) s.t. P 1 = u, P^T 1 = v, P >= 0, r Gaussian or entropy) and for the
structured marginal constraints inside Eq. (augLag) / Algorithm 4.

  * value / gradient by central differences, the difference form against differences of values;
  * the Gaussian kind written out as the generic quadratic form (A = lambda I, b = vec(M)) with the marginal
    constraints as a DENSE 0/1 constraint matrix: a second, independent route through the oracle (itself pinned
    against scipy in the augmented-Lagrangian tests) that must give the same values, gradients, shifted constraint
    values, differences and the same Algorithm 4 result;
  * box only (no marginal terms): the entrywise closed forms max(0, -M/lambda) and exp(-M/lambda - 1);
  * M = 0: the closed-form couplings u 1^T/c + 1 v^T/r - 1/(rc) (Gaussian, when positive) and u v^T (entropy);
  * general M: the optimality structure P = max(0, -(M + a_i + b_j)/lambda) with the returned multipliers
    (Gaussian), log P + M/lambda additively separable (entropy), and scipy's SLSQP on the same problem.
"""
import numpy as np
import pytest
import scipy.optimize as so

import oracle
import workloads


def _marginal_matrix(rows, cols):
    """Dense K with K vec(P) = [P 1; P^T 1] for row-major vec."""
    K = np.zeros((rows + cols, rows * cols))
    for i in range(rows):
        K[i, i * cols:(i + 1) * cols] = 1.0
    for j in range(cols):
        K[rows + j, j::cols] = 1.0
    return K


def _random_problem(rng, rows, cols, signed=False):
    M = rng.random((rows, cols)) - (0.5 if signed else 0.0)
    u = rng.random(rows) + 0.1
    v = rng.random(cols) + 0.1
    return M, u / u.sum(), v / v.sum()


@pytest.mark.parametrize("kind", [oracle.OT_GAUSS, oracle.OT_ENTROPY])
@pytest.mark.parametrize("with_marginals", [False, True])
def test_value_gradient_and_difference_form(kind, with_marginals):
    rng = np.random.default_rng(3)
    rows, cols = 4, 6
    M, u, v = _random_problem(rng, rows, cols, signed=True)
    obj = oracle.Objective(kind, M, lam=0.7)
    if with_marginals:
        obj.set_marginals(u, v, lam=rng.standard_normal(rows + cols), rho=3.0)
    x = rng.random(rows * cols) + 0.05
    f, g, row = oracle.fg(obj, x, want_rowvec=True)
    assert row.shape == ((rows + cols) if with_marginals else 0,)
    for i in range(rows * cols):
        h = 1e-6
        xp, xm = x.copy(), x.copy()
        xp[i] += h
        xm[i] -= h
        assert (oracle.f_only(obj, xp) - oracle.f_only(obj, xm)) / (2 * h) == pytest.approx(g[i], rel=1e-7, abs=1e-8)
    for scale in (0.04, 1e-4, 1e-9):
        xt = x + scale * rng.standard_normal(x.size)
        assert oracle.delta_f(obj, x, xt, row) == pytest.approx(oracle.f_only(obj, xt) - f, rel=1e-6, abs=1e-14 * abs(f))
    # a step onto a tiny positive bound (the relative change rounds to -1): still the difference of the values
    xt = x.copy()
    xt[:4] = 1e-30
    assert np.isfinite(oracle.delta_f(obj, x, xt, row))
    assert oracle.delta_f(obj, x, xt, row) == pytest.approx(oracle.f_only(obj, xt) - f, rel=1e-9)
    # entries at zero: 0 log 0 = 0, and the difference form handles a zero at either end
    xz, xt = x.copy(), x.copy()
    xz[:5] = 0.0
    xt[3:8] = 0.0
    fz, _, rowz = oracle.fg(obj, xz, want_rowvec=True)
    assert np.isfinite(fz)
    assert oracle.delta_f(obj, xz, xt, rowz) == pytest.approx(oracle.f_only(obj, xt) - fz, rel=1e-9)


def test_gaussian_kind_equals_the_generic_quadratic_form_with_a_dense_constraint_matrix():
    rng = np.random.default_rng(5)
    rows, cols, lam, rho = 5, 4, 0.5, 2.5
    M, u, v = _random_problem(rng, rows, cols)
    mult = rng.standard_normal(rows + cols)
    ot = oracle.Objective(oracle.OT_GAUSS, M, lam=lam).set_marginals(u, v, lam=mult, rho=rho)
    n = rows * cols
    qp = oracle.Objective(oracle.QP, lam * np.eye(n), M.reshape(-1))
    qp.set_constraints(C_eq=_marginal_matrix(rows, cols), d=np.concatenate([u, v]), lam=mult, rho=rho)
    x = rng.random(n)
    f1, g1, r1 = oracle.fg(ot, x, want_rowvec=True)
    f2, g2, r2 = oracle.fg(qp, x, want_rowvec=True)
    assert f1 == pytest.approx(f2, rel=1e-14)
    np.testing.assert_allclose(g1, g2, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(r1, r2[n:], rtol=1e-13, atol=1e-15)     # the shifted constraint values h + lambda/rho
    xt = np.maximum(x + 0.1 * rng.standard_normal(n), 0.0)
    assert oracle.delta_f(ot, x, xt, r1) == pytest.approx(oracle.delta_f(qp, x, xt, r2), rel=1e-12)
    # Algorithm 4 through both routes: same multipliers, same point, same number of outer iterations
    opts = oracle.default_options(tol=1e-10, max_iter=5000)
    l, ub = np.zeros(n), np.full(n, np.inf)
    xa, la, _, ia = oracle.auglag_solve(ot, l, ub, np.zeros(n), 8, opts, ctol=1e-9)
    xb, lb_, _, ib = oracle.auglag_solve(qp, l, ub, np.zeros(n), 8, opts, ctol=1e-9)
    assert ia.status == ib.status == oracle.CONVERGED
    assert ia.outer == ib.outer
    np.testing.assert_allclose(xa, xb, atol=1e-8)
    np.testing.assert_allclose(la, lb_, atol=1e-7)
    assert ia.f == pytest.approx(ib.f, rel=1e-9)


def test_box_only_closed_forms():
    rng = np.random.default_rng(7)
    rows, cols, lam = 6, 5, 0.5
    M = rng.standard_normal((rows, cols))
    n = rows * cols
    opts = oracle.default_options(tol=1e-11, max_iter=2000)
    g = oracle.Solver(oracle.Objective(oracle.OT_GAUSS, M, lam=lam), np.zeros(n), np.full(n, np.inf), np.zeros(n), 6, opts)
    res = g.solve()
    g.close()
    assert res.info.status == oracle.CONVERGED
    np.testing.assert_allclose(res.x.reshape(rows, cols), np.maximum(0.0, -M / lam), atol=1e-9)
    # entropy: stationarity M + lam (log P + 1) = 0 inside the box [0.2, 3]
    lo, hi = 0.2, 3.0
    e = oracle.Solver(oracle.Objective(oracle.OT_ENTROPY, M, lam=lam), np.full(n, lo), np.full(n, hi), np.full(n, 1.0), 6, opts)
    res = e.solve()
    e.close()
    assert res.info.status == oracle.CONVERGED
    np.testing.assert_allclose(res.x.reshape(rows, cols), np.clip(np.exp(-M / lam - 1.0), lo, hi), atol=1e-8)


def _solve(kind, M, u, v, lam, lower, tol=1e-10, ctol=1e-9, m=10, max_iter=20000):
    rows, cols = M.shape
    n = rows * cols
    obj = oracle.Objective(kind, M, lam=lam).set_marginals(u, v)
    opts = oracle.default_options(tol=tol, max_iter=max_iter)
    x, mult, _, info = oracle.auglag_solve(obj, np.full(n, lower), np.full(n, np.inf), np.full(n, lower), m, opts, ctol=ctol)
    return x.reshape(rows, cols), mult, info


def test_zero_cost_closed_form_couplings():
    rng = np.random.default_rng(11)
    rows, cols = 5, 7
    u, v = rng.random(rows) + 1.0, rng.random(cols) + 1.0      # flat enough for the least-norm matrix to be positive
    u, v = u / u.sum(), v / v.sum()
    Z = np.zeros((rows, cols))
    # Gaussian: the least-norm matrix with these marginals (all its entries are positive for these u, v)
    P, _, info = _solve(oracle.OT_GAUSS, Z, u, v, 0.5, 0.0)
    closed = u[:, None] / cols + v[None, :] / rows - 1.0 / (rows * cols)
    assert closed.min() > 0
    assert info.status == oracle.CONVERGED and info.violation <= 1e-9
    np.testing.assert_allclose(P, closed, atol=1e-8)
    # entropy: the independent coupling
    P, _, info = _solve(oracle.OT_ENTROPY, Z, u, v, 0.5, 1e-30)
    assert info.status == oracle.CONVERGED and info.violation <= 1e-9
    np.testing.assert_allclose(P, np.outer(u, v), atol=1e-8)


def test_gaussian_solution_has_the_dual_structure_and_matches_slsqp():
    rng = np.random.default_rng(13)
    rows, cols, lam = 5, 6, 0.5
    M, u, v = _random_problem(rng, rows, cols)
    P, mult, info = _solve(oracle.OT_GAUSS, M, u, v, lam, 0.0)
    assert info.status == oracle.CONVERGED
    np.testing.assert_allclose(P.sum(1), u, atol=1e-8)
    np.testing.assert_allclose(P.sum(0), v, atol=1e-8)
    assert (P == 0).sum() > 0          # some entries sit on the bound: the max() below matters
    a, b = mult[:rows], mult[rows:]
    np.testing.assert_allclose(P, np.maximum(0.0, -(M + a[:, None] + b[None, :]) / lam), atol=1e-7)
    K, d = _marginal_matrix(rows, cols)[:-1], np.concatenate([u, v])[:-1]     # the last marginal row is implied by the others
    ref = so.minimize(lambda x: M.reshape(-1) @ x + 0.5 * lam * x @ x, np.outer(u, v).reshape(-1),
                      jac=lambda x: M.reshape(-1) + lam * x, method="SLSQP", bounds=[(0, None)] * (rows * cols),
                      constraints=[{"type": "eq", "fun": lambda x: K @ x - d, "jac": lambda x: K}],
                      options={"ftol": 1e-14, "maxiter": 1000})
    assert ref.success
    np.testing.assert_allclose(P.reshape(-1), ref.x, atol=1e-6)
    assert info.f == pytest.approx(ref.fun, abs=1e-9)


def test_entropy_solution_is_a_scaled_gibbs_kernel_and_matches_slsqp():
    rng = np.random.default_rng(17)
    rows, cols, lam = 4, 5, 0.5
    M, u, v = _random_problem(rng, rows, cols)
    P, _, info = _solve(oracle.OT_ENTROPY, M, u, v, lam, 1e-30)
    assert info.status == oracle.CONVERGED
    np.testing.assert_allclose(P.sum(1), u, atol=1e-8)
    np.testing.assert_allclose(P.sum(0), v, atol=1e-8)
    # P = diag(a) exp(-M/lam) diag(b): log P + M/lam has no interaction term
    T = np.log(P) + M / lam
    T = T - T.mean(0, keepdims=True) - T.mean(1, keepdims=True) + T.mean()
    assert np.abs(T).max() <= 1e-6
    K, d = _marginal_matrix(rows, cols)[:-1], np.concatenate([u, v])[:-1]     # the last marginal row is implied by the others
    ref = so.minimize(lambda x: M.reshape(-1) @ x + lam * np.sum(x * np.log(x)), np.outer(u, v).reshape(-1),
                      jac=lambda x: M.reshape(-1) + lam * (np.log(x) + 1.0), method="SLSQP",
                      bounds=[(1e-12, None)] * (rows * cols),
                      constraints=[{"type": "eq", "fun": lambda x: K @ x - d, "jac": lambda x: K}],
                      options={"ftol": 1e-14, "maxiter": 1000})
    assert ref.success
    np.testing.assert_allclose(P.reshape(-1), ref.x, atol=1e-6)


@pytest.mark.parametrize("dataset,reg", [(1, "gauss"), (2, "gauss"), (1, "entropy"), (2, "entropy")])
def test_generated_families_solve_to_a_coupling(dataset, reg):
    p = workloads.joint_probability(12, dataset=dataset, reg=reg, seed=4)
    P, _, info = _solve(p.kind, p.M, p.u, p.v, p.lam, p.lower, tol=1e-9, ctol=1e-8)
    assert info.status == oracle.CONVERGED, (info.status, info.outer, info.violation)
    assert P.min() >= p.lower
    np.testing.assert_allclose(P.sum(1), p.u, atol=1e-7)
    np.testing.assert_allclose(P.sum(0), p.v, atol=1e-7)
    assert P.sum() == pytest.approx(1.0, abs=1e-6)
