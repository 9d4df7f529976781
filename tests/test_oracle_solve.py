"""Pins for the oracle's whole iteration (Algorithm 1): the returned point is checked
against definitions that do not involve the oracle -- KKT conditions recomputed with numpy,
the closed-form least-squares solution, brute-force enumeration of active sets, and scipy's
independent solvers -- and the per-iteration invariants of Theorem 1 are checked along the
way."""
import itertools
import math

import numpy as np
import pytest
from scipy import optimize

import oracle
import workloads


def _numpy_grad(prob, x):
    A = prob.A.astype(np.float64)
    if prob.kind == workloads.OBJ_LSQ:
        return A.T @ (A @ x - prob.b)
    if prob.kind == workloads.OBJ_LSQ_L1SPLIT:
        c = prob.cols
        w = A.T @ (A @ (x[:c] - x[c:]) - prob.b)
        return np.concatenate([w + prob.lam, -w + prob.lam])
    from scipy.special import expit
    z = A @ x
    return -(A.T @ (prob.b * expit(-prob.b * z))) / prob.rows + prob.mu * x


def _numpy_f(prob, x):
    A = prob.A.astype(np.float64)
    if prob.kind == workloads.OBJ_LSQ:
        r = A @ x - prob.b
        return 0.5 * r @ r
    if prob.kind == workloads.OBJ_LSQ_L1SPLIT:
        c = prob.cols
        r = A @ (x[:c] - x[c:]) - prob.b
        return 0.5 * r @ r + prob.lam * x.sum()
    from scipy.special import log_expit
    return -log_expit(prob.b * (A @ x)).sum() / prob.rows + 0.5 * prob.mu * x @ x


def assert_kkt(prob, x, tol):
    """l <= x <= u, ||x - P(x - g)||_inf <= tol, and complementarity signs, with the gradient
    recomputed by numpy."""
    g = _numpy_grad(prob, x)
    assert np.all(x >= prob.l) and np.all(x <= prob.u)
    assert np.abs(x - np.clip(x - g, prob.l, prob.u)).max() <= tol
    at_l, at_u = x == prob.l, x == prob.u
    inside = ~at_l & ~at_u
    assert np.all(g[at_l & ~at_u] >= -tol)
    assert np.all(g[at_u & ~at_l] <= tol)
    # an interior coordinate is either stationary or closer than tol to a bound
    gap = np.minimum(x - prob.l, prob.u - x)
    assert np.all((np.abs(g[inside]) <= tol) | (gap[inside] <= tol))


# ---- closed form: no active bound -> least squares ---------------------------------------------

@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_unbounded_problem_gives_lstsq_solution(dtype):
    rng = np.random.default_rng(31)
    A = rng.normal(size=(60, 12)).astype(dtype)
    b = rng.normal(size=60)
    prob = workloads.Problem("free", workloads.OBJ_LSQ, A, b, np.full(12, -np.inf), np.full(12, np.inf),
                             np.zeros(12), m=6, tol=1e-10)
    res = oracle.solve_problem(prob)
    assert res.info.status == oracle.CONVERGED
    x_ls = np.linalg.lstsq(A.astype(np.float64), b, rcond=None)[0]
    np.testing.assert_allclose(res.x, x_ls, rtol=0, atol=1e-10)
    assert res.info.n_fixed == 0


def test_unbounded_problem_is_plain_lbfgs_with_every_pair_used():
    """With no bounds the free set is everything, Algorithm 2 returns d itself, and on a
    strictly convex quadratic every pair passes the gate: the method is textbook L-BFGS."""
    rng = np.random.default_rng(32)
    A = rng.normal(size=(40, 8))
    b = rng.normal(size=40)
    obj = oracle.Objective(oracle.LSQ, A, b)
    s = oracle.Solver(obj, np.full(8, -np.inf), np.full(8, np.inf), np.zeros(8), m=4,
                      options=oracle.default_options(tol=1e-9))
    k = 0
    while s.step() == oracle.RUNNING:
        k += 1
        assert s.mask.all()
        # branch 1 returns (x + d) - x, branch 2 returns d: equal up to the rounding of x + d
        np.testing.assert_allclose(s.p, s.d, rtol=0, atol=4e-16 * max(1.0, np.abs(s.x).max()))
        assert s.info.pairs_used == min(k - 1, 4)
    assert s.info.status == oracle.CONVERGED and k < 60
    s.close()


# ---- brute force over active sets --------------------------------------------------------------

def _brute_force_box_ls(A, b, l, u):
    """Exact minimiser of 0.5||Ax-b||^2 over the box by enumerating, for every coordinate,
    {at l, free, at u}, solving the free least-squares problem, and keeping the candidate that
    is feasible and has the right multiplier signs (unique for full-column-rank A)."""
    n = A.shape[1]
    choices = []
    for i in range(n):
        c = ["free"]
        if np.isfinite(l[i]):
            c.append("l")
        if np.isfinite(u[i]):
            c.append("u")
        choices.append(c)
    best = None
    for assign in itertools.product(*choices):
        x = np.zeros(n)
        F = [i for i, a in enumerate(assign) if a == "free"]
        for i, a in enumerate(assign):
            if a == "l":
                x[i] = l[i]
            elif a == "u":
                x[i] = u[i]
        if F:
            rhs = b - A @ x
            x[F] = np.linalg.lstsq(A[:, F], rhs, rcond=None)[0]
        if np.any(x < l - 1e-12) or np.any(x > u + 1e-12):
            continue
        g = A.T @ (A @ x - b)
        ok = all((a == "free" and abs(g[i]) < 1e-8) or (a == "l" and g[i] >= -1e-10) or
                 (a == "u" and g[i] <= 1e-10) for i, a in enumerate(assign))
        if ok:
            f = 0.5 * np.sum((A @ x - b) ** 2)
            if best is None or f < best[0]:
                best = (f, x)
    assert best is not None
    return best[1]


def test_nnls_matches_brute_force_active_set():
    with_active_bound = 0
    for seed in range(8):
        rng = np.random.default_rng(100 + seed)
        n = int(rng.integers(4, 11))
        prob = workloads.nnls(3 * n + 2, n, seed=200 + seed, zero_frac=0.5, nonzero="absnormal", m=4,
                              tol=1e-10, noise=1.0)
        x_bf = _brute_force_box_ls(prob.A, prob.b, prob.l, prob.u)
        res = oracle.solve_problem(prob)
        assert res.info.status == oracle.CONVERGED
        np.testing.assert_allclose(res.x, x_bf, rtol=0, atol=1e-9)
        assert np.array_equal(res.x == 0, x_bf == 0)            # identical active set
        with_active_bound += (x_bf == 0).sum() > 0
    assert with_active_bound >= 5                               # the instances do exercise the bound


@pytest.mark.parametrize("seed", range(4))
def test_two_sided_box_matches_brute_force(seed):
    rng = np.random.default_rng(300 + seed)
    n = int(rng.integers(3, 8))
    A = rng.normal(size=(2 * n + 3, n))
    b = rng.normal(size=2 * n + 3) * 3
    l = -0.3 * rng.random(n)
    u = 0.3 * rng.random(n)
    l[0] = -np.inf
    prob = workloads.Problem("box", workloads.OBJ_LSQ, A, b, l, u, np.clip(np.zeros(n), l, u), m=5, tol=1e-10)
    x_bf = _brute_force_box_ls(A, b, l, u)
    res = oracle.solve_problem(prob)
    assert res.info.status == oracle.CONVERGED
    np.testing.assert_allclose(res.x, x_bf, rtol=0, atol=1e-9)
    assert ((x_bf == l) | (x_bf == u)).sum() > 0


# ---- library cross-checks (same minimiser, different path) -------------------------------------

def test_c1_matches_scipy_nnls_and_meets_kkt():
    prob = workloads.config("C1")
    res = oracle.solve_problem(prob)
    assert res.info.status == oracle.CONVERGED
    assert res.info.pg2 <= 1e-8
    assert_kkt(prob, res.x, 1e-8)
    x_ref, _ = optimize.nnls(prob.A, prob.b)
    np.testing.assert_allclose(res.x, x_ref, rtol=0, atol=1e-8)
    assert np.array_equal(res.x == 0, x_ref == 0)
    assert res.info.f == pytest.approx(_numpy_f(prob, x_ref), rel=1e-12)
    # "30-40 iterations" is what the paper reports for its NNLS runs: soft sanity bound only
    assert 10 <= res.info.iters <= 120


def test_scaled_c5_matches_scipy_lsq_linear():
    prob = workloads.config("C5", scale=0.01)            # 1000 x 200, fp32 storage, box [0, 1]
    prob.tol, prob.tol_relative = 1e-8, False
    res = oracle.solve_problem(prob)
    assert res.info.status == oracle.CONVERGED
    assert_kkt(prob, res.x, 1e-7)
    ref = optimize.lsq_linear(prob.A.astype(np.float64), prob.b, bounds=(prob.l, prob.u), method="bvls",
                              tol=1e-14)
    np.testing.assert_allclose(res.x, ref.x, rtol=0, atol=1e-7)


def test_scaled_c3_matches_scipy_lbfgsb_objective_and_lasso_structure():
    prob = workloads.config("C3", scale=0.02)            # 200 x 400 -> 800 variables
    prob.tol, prob.tol_relative = 1e-9, False
    res = oracle.solve_problem(prob)
    assert res.info.status == oracle.CONVERGED
    assert_kkt(prob, res.x, 1e-8)
    c = prob.cols
    assert np.all(res.x[:c] * res.x[c:] == 0)            # p_i q_i = 0 at any KKT point with lam > 0
    ref = optimize.minimize(lambda x: (_numpy_f(prob, x), _numpy_grad(prob, x)), prob.x0, jac=True,
                            method="L-BFGS-B", bounds=list(zip(prob.l, prob.u)),
                            options=dict(maxiter=5000, ftol=1e-15, gtol=1e-10))
    assert res.info.f <= ref.fun * (1 + 1e-9)
    assert res.info.f == pytest.approx(ref.fun, rel=1e-7)


def test_scaled_c4_matches_scipy_lbfgsb():
    prob = workloads.config("C4", scale=0.01)            # 2000 x 20 logistic, box [-0.5, 0.5]
    prob.tol, prob.tol_relative = 1e-10, False
    res = oracle.solve_problem(prob)
    assert res.info.status == oracle.CONVERGED
    assert_kkt(prob, res.x, 1e-9)
    ref = optimize.minimize(lambda x: (_numpy_f(prob, x), _numpy_grad(prob, x)), prob.x0, jac=True,
                            method="L-BFGS-B", bounds=list(zip(prob.l, prob.u)),
                            options=dict(maxiter=5000, ftol=1e-16, gtol=1e-12))
    np.testing.assert_allclose(res.x, ref.x, rtol=0, atol=1e-6)
    assert res.info.f == pytest.approx(ref.fun, rel=1e-10)
    assert (np.abs(res.x) == 0.5).sum() > 0              # the box is active


# ---- invariants from the proof of Theorem 1 ----------------------------------------------------

@pytest.mark.parametrize("name,scale", [("C1", 1.0), ("C2", 0.02), ("C3", 0.01), ("C4", 0.005), ("C5", 0.005)])
def test_iteration_invariants(name, scale):
    prob = workloads.config(name, scale=scale)
    obj = oracle.Objective(prob.kind, prob.A, prob.b, prob.lam, prob.mu)
    opts = oracle.default_options(tol=1e-7, tol_relative=0, max_iter=400)
    s = oracle.Solver(obj, prob.l, prob.u, prob.x0, prob.m, opts)
    f_prev = s.info.f
    x_prev, g_prev = s.x, s.g
    iters = 0
    while s.step() == oracle.RUNNING:
        iters += 1
        info = s.info
        x = s.x
        assert np.all(x >= prob.l) and np.all(x <= prob.u)                  # feasible by construction
        assert info.f < f_prev or info.alpha * abs(info.gp) < 1e-15         # strict decrease
        # the accepted step satisfies the Armijo inequality, checked with numpy
        assert _numpy_f(prob, x) - _numpy_f(prob, x_prev) <= opts.armijo_c1 * info.alpha * info.gp + 1e-12 * abs(f_prev)
        assert info.gp < 0 and 0 < info.alpha <= min(1.0, info.alpha_ub)
        # the stored pair is (x+ - x, g+ - g)
        np.testing.assert_array_equal(s.S[-1], x - x_prev)
        np.testing.assert_allclose(s.Y[-1], s.g - g_prev, rtol=0, atol=0)
        assert s.npairs == min(iters, prob.m)
        # the cached ||y||^2 is the full-vector norm (as printed in Algorithm 3), not the masked one
        assert s.ynorm2[-1] == pytest.approx(s.Y[-1] @ s.Y[-1], rel=1e-14)
        # d vanishes on the fixed set
        assert np.all(s.d[s.mask == 0] == 0)
        f_prev, x_prev, g_prev = info.f, x, s.g
    assert s.info.status == oracle.CONVERGED
    assert s.info.iters == iters
    assert_kkt(prob, s.x, 1e-6)
    s.close()


def test_armijo_backtracking_on_a_hand_worked_quadratic():
    """f(x) = 0.5*(2x - 1)^2 from x = 0 with no stored pair: g = -2, d = p = 2 (projection branch,
    no bound).  f(alpha*2) - f(0) = -4 alpha + 8 alpha^2 and the Armijo bound is c1*alpha*(-4); with
    c1 = 0.5 the inequality holds iff alpha <= 1/4, so halving from 1 accepts alpha = 1/4 after two
    backtracks (there with equality, all numbers exact in binary) and lands on the minimiser 1/2."""
    obj = oracle.Objective(oracle.LSQ, np.array([[2.0]]), np.array([1.0]))
    s = oracle.Solver(obj, [-np.inf], [np.inf], [0.0], m=3, options=oracle.default_options(armijo_c1=0.5))
    assert s.step() == oracle.RUNNING
    info = s.info
    assert info.branch == 1 and info.gp == -4.0
    assert info.backtracks == 2 and info.alpha == 0.25
    assert s.x[0] == 0.5 and info.f == 0.0
    # with backtracking factor 1/4 the first reduced trial is already accepted
    s2 = oracle.Solver(obj, [-np.inf], [np.inf], [0.0], m=3,
                       options=oracle.default_options(armijo_c1=0.5, backtrack=0.25))
    s2.step()
    assert s2.info.backtracks == 1 and s2.info.alpha == 0.25
    # a bound that limits the step: u = 0.25 -> projection branch clips p to 0.25, alpha = 1 is accepted:
    # f(0.25) - f(0) = 0.125 - 0.5 = -0.375 <= 0.5 * 1 * (-2 * 0.25) = -0.25
    s3 = oracle.Solver(obj, [0.0], [0.25], [0.0], m=3, options=oracle.default_options(armijo_c1=0.5))
    s3.step()
    assert s3.info.branch == 1 and s3.info.alpha == 1.0 and s3.x[0] == 0.25 and s3.info.gp == -0.5
    for t in (s, s2, s3):
        t.close()


def test_skipping_the_projection_branch_reaches_the_same_optimum():
    prob = workloads.config("C1")
    a = oracle.solve_problem(prob)
    b = oracle.solve_problem(prob, always_branch2=1)
    assert a.info.status == b.info.status == oracle.CONVERGED
    np.testing.assert_allclose(a.x, b.x, rtol=0, atol=1e-8)
    assert a.info.f == pytest.approx(b.info.f, rel=1e-12)


def test_relative_tolerance_scales_with_initial_projected_gradient():
    prob = workloads.config("C2", scale=0.02)
    obj = oracle.Objective(prob.kind, prob.A, prob.b)
    g0 = _numpy_grad(prob, prob.x0)
    mask0 = oracle.free_mask(prob.x0, g0, prob.l, prob.u, 1e-10).astype(bool)
    res = oracle.solve_problem(prob, tol=1e-6, tol_relative=1)
    assert res.info.status == oracle.CONVERGED
    assert res.info.pg2 <= 1e-6 * np.linalg.norm(g0[mask0])
    assert res.info.pg2 > 1e-10 * np.linalg.norm(g0[mask0])     # it did not over-solve by orders


# ---- failure handling ---------------------------------------------------------------------------

def test_rejects_infeasible_start_and_crossed_bounds():
    A = np.eye(3)
    obj = oracle.Objective(oracle.LSQ, A, np.ones(3))
    with pytest.raises(ValueError):
        oracle.Solver(obj, np.zeros(3), np.ones(3), np.array([0.5, 2.0, 0.5]), m=3)
    with pytest.raises(ValueError):
        oracle.Solver(obj, np.array([0.0, 1.0, 0.0]), np.array([1.0, 0.5, 1.0]), np.full(3, 0.5), m=3)
    with pytest.raises(ValueError):
        oracle.Solver(obj, np.zeros(3), np.ones(3), np.array([0.5, np.nan, 0.5]), m=3)


def test_max_iter_status_and_start_at_optimum():
    prob = workloads.config("C1")
    res = oracle.solve_problem(prob, max_iter=3)
    assert res.info.status == oracle.MAX_ITER and res.info.iters == 3
    # starting at the optimum: converged with zero iterations
    opt = oracle.solve_problem(prob, tol=1e-9)
    prob2 = workloads.config("C1")
    prob2.x0 = opt.x
    res = oracle.solve_problem(prob2, tol=1e-8)
    assert res.info.status == oracle.CONVERGED and res.info.iters == 0


def test_coinciding_bounds_are_never_moved():
    rng = np.random.default_rng(77)
    A = rng.normal(size=(30, 6)); b = rng.normal(size=30)
    l = np.array([-np.inf, 0.2, 0.0, -1.0, 0.7, -np.inf]); u = np.array([np.inf, 0.2, 1.0, 1.0, 0.7, 0.0])
    x0 = np.clip(np.zeros(6), l, u)
    prob = workloads.Problem("pin", workloads.OBJ_LSQ, A, b, l, u, x0, m=3, tol=1e-10)
    res = oracle.solve_problem(prob)
    assert res.info.status == oracle.CONVERGED
    assert res.x[1] == 0.2 and res.x[4] == 0.7
    np.testing.assert_allclose(res.x, _brute_force_box_ls(A, b, l, u), rtol=0, atol=1e-9)
