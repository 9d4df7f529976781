"""Whole solves of randomly drawn small problems against the CPU oracle: objective kind, shape (single rows and
columns, sizes around the tile and wave widths), memory m, storage type, A-pass organisation and the kind of box
(none, one-sided, two-sided, mixed with infinities, coinciding bounds) all vary together.  What the method fixes is
compared: feasibility, that the reported f is the objective at the returned point (recomputed with numpy), and the
final objective value (both sides must converge; 1e-8 relative for fp64-stored matrices at the relative
stopping tolerance 1e-7 used here, 1e-4 for fp32-stored ones).  A second test draws strictly convex quadratic forms,
with and without equality rows (Algorithm 4), where the minimiser is unique and is compared itself."""
import math

import numpy as np
import pytest

import oracle
import paper_2203_16340_amd as L
import workloads
from gpu_helpers import DEV, host_gradient, host_objective

pytestmark = pytest.mark.gpu

SMALL = dict(rows=[1, 2, 7, 33, 64, 65, 130, 257, 400, 900], cols=[1, 2, 3, 8, 31, 64, 66, 128, 250, 513],
             m=[1, 2, 3, 5, 10, 12, 17])
LARGER = dict(rows=[5, 100, 511, 1025, 2300], cols=[4, 17, 100, 255, 1000, 1026, 2052], m=[1, 4, 10, 11, 20, 31])


def draw(pool, case):
    rng = np.random.default_rng(770000 + case)
    kind = int(rng.choice([workloads.OBJ_LSQ, workloads.OBJ_LSQ_L1SPLIT, workloads.OBJ_LOGISTIC_L2]))
    rows, cols, m = (int(rng.choice(pool[k])) for k in ("rows", "cols", "m"))
    dtype = np.float64 if rng.random() < 0.6 else np.float32
    a_pass = int(rng.choice([L.APASS_AUTO, L.APASS_TWO_PASS, L.APASS_FUSED]))
    A = (rng.standard_normal((rows, cols)) / math.sqrt(rows)).astype(dtype)
    n = 2 * cols if kind == workloads.OBJ_LSQ_L1SPLIT else cols
    b = np.where(rng.random(rows) < 0.5, -1.0, 1.0) if kind == workloads.OBJ_LOGISTIC_L2 else rng.standard_normal(rows)
    box = int(rng.integers(0, 5))
    if kind == workloads.OBJ_LSQ_L1SPLIT or box == 0:
        l, u = np.zeros(n), np.full(n, np.inf)
    elif box == 1:
        l, u = np.full(n, -np.inf), np.full(n, np.inf)
    elif box == 2:
        l, u = -rng.random(n), rng.random(n)
    elif box == 3:
        l = np.where(rng.random(n) < 0.5, -np.inf, -rng.random(n))
        u = np.where(rng.random(n) < 0.5, np.inf, rng.random(n))
    else:
        l = 0.3 * rng.standard_normal(n)
        u = l + np.where(rng.random(n) < 0.2, 0.0, rng.random(n))      # a fifth of the variables have l = u
    x0 = np.clip(0.5 * rng.standard_normal(n), l, u)
    prob = workloads.Problem("random", kind, np.ascontiguousarray(A), b, l, u, x0, m,
                             lam=0.05 if kind == workloads.OBJ_LSQ_L1SPLIT else 0.0,
                             mu=0.05 if kind == workloads.OBJ_LOGISTIC_L2 else 0.0,
                             tol=1e-7, tol_relative=True, max_iter=1500)
    return prob, a_pass


# Two draws zigzag for thousands of iterations (many bounds become active one at a time; with m = 1 the method is close
# to projected steepest descent): the oracle needs over a minute (case 112: 4057 iterations) or does not converge within
# 20000 iterations (case 103).  They keep a limit of 1500 iterations and a weaker comparison, stated below.
SLOW = {("larger", 103), ("larger", 112)}


@pytest.mark.parametrize("pool,case", [("small", c) for c in range(60)] + [("larger", c) for c in range(100, 116)])
def test_random_problem_matches_the_oracle(pool, case):
    prob, a_pass = draw(SMALL if pool == "small" else LARGER, case)
    slow = (pool, case) in SLOW
    prob.max_iter = 1500 if slow else 5000
    try:
        s = L.solver_for_problem(prob, DEV, a_pass=a_pass)
    except L.LbfgsbError as e:
        if e.code != L.E_UNSUPPORTED:
            raise
        s = L.solver_for_problem(prob, DEV, a_pass=L.APASS_AUTO)   # the fused pass does not take this shape
    f0 = s.info().f
    info = s.solve()
    x = s.x().cpu().numpy()
    s.close()
    ref = oracle.solve_problem(prob)
    assert np.all(x >= prob.l) and np.all(x <= prob.u)
    f_host = host_objective(prob, x)
    assert abs(info.f - f_host) <= 1e-8 * abs(f_host) + 1e-14
    # the benchmark spec's bound on the final objective: 1e-8 relative for fp64-stored matrices, 1e-4 for fp32-stored ones
    # (an objective that can be driven to zero -- more columns than rows -- is compared on the scale of its start value)
    tol = 1e-8 if prob.A.dtype == np.float64 else 1e-4
    slack = tol * max(abs(ref.info.f), 1e-10 * abs(f0))
    if slow:
        # both sides feasible, neither far from the other, and a side that converged is not above the one that did not
        assert info.status in (L.CONVERGED, L.MAX_ITER) and ref.info.status in (oracle.CONVERGED, oracle.MAX_ITER)
        assert abs(info.f - ref.info.f) <= 1e-2 * abs(ref.info.f)
        if info.status == L.CONVERGED:
            assert info.f <= ref.info.f + 1e-6 * abs(ref.info.f)
        if ref.info.status == oracle.CONVERGED:
            assert ref.info.f <= info.f + 1e-6 * abs(ref.info.f)
        return
    assert info.status == L.CONVERGED and ref.info.status == oracle.CONVERGED, (info.as_dict(), ref.info.status)
    assert abs(info.f - ref.info.f) <= slack, (info.f, ref.info.f)
    g = host_gradient(prob, x)
    mask = oracle.free_mask(x, g, prob.l, prob.u, 1e-10).astype(bool)
    assert np.linalg.norm(g[mask]) <= 1.5 * max(info.pg2, 1e-300) + 1e-9 * np.linalg.norm(g) + 1e-12


@pytest.mark.parametrize("case", range(24))
def test_random_quadratic_form_with_and_without_constraint_rows(case):
    """Strictly convex quadratic forms (unique minimiser, so the points themselves are compared): box only, or with
    one to three equality rows through Algorithm 4; sign vector or none, fp64 or fp32 matrix."""
    from gpu_helpers import rel_err, to_dev
    rng = np.random.default_rng(880000 + case)
    n = int(rng.choice([1, 2, 5, 64, 65, 130, 257, 513, 1030]))
    n_eq = int(rng.choice([0, 0, 1, 2, 3])) if n >= 5 else 0
    dtype = np.float64 if rng.random() < 0.7 else np.float32
    m = int(rng.choice([1, 3, 8, 12]))
    B = rng.standard_normal((n, max(n, 2)))
    K = (B @ B.T / n + 0.5 * np.eye(n)).astype(dtype)
    K = np.ascontiguousarray(0.5 * (K + K.T))
    b = 2.0 * rng.standard_normal(n)
    sign = np.where(rng.random(n) < 0.5, -1.0, 1.0) if rng.random() < 0.6 else None
    if rng.random() < 0.5:
        l, u = np.zeros(n), np.ones(n)
    else:
        l = np.where(rng.random(n) < 0.3, -np.inf, -rng.random(n))
        u = np.where(rng.random(n) < 0.3, np.inf, 1.0 + rng.random(n))
    x0 = np.clip(np.zeros(n), l, u)
    sd = to_dev(sign) if sign is not None else None
    ftol = 1e-8 if dtype == np.float64 else 1e-4
    if n_eq == 0:
        obj = oracle.Objective(oracle.QP, K, b, sign=sign)
        osol = oracle.Solver(obj, l, u, x0, m, oracle.default_options(tol=1e-9))
        ref = osol.solve()
        osol.close()
        sol = L.Solver(L.OBJ_QP, to_dev(K), to_dev(b), to_dev(l), to_dev(u), m, sign=sd, options=L.default_options(tol=1e-9))
        sol.set_x(to_dev(x0))
        info = sol.solve()
        x = sol.x().cpu().numpy()
        sol.close()
        assert ref.info.status == oracle.CONVERGED and info.status == L.CONVERGED, info.as_dict()
        assert np.all(x >= l) and np.all(x <= u)
        assert abs(info.f - ref.info.f) <= ftol * abs(ref.info.f) + 1e-12
        assert rel_err(x, ref.x) <= (1e-6 if dtype == np.float64 else 1e-3) or np.linalg.norm(ref.x) < 1e-9
        return
    x_feas = np.clip(0.5 * rng.random(n), l, u)
    Cm = rng.standard_normal((n_eq, n)) / math.sqrt(n)
    d = Cm @ x_feas
    obj = oracle.Objective(oracle.QP, K, b, sign=sign).set_constraints(Cm, d)
    x_ref, lam_ref, _, iref = oracle.auglag_solve(obj, l, u, x0, m, oracle.default_options(tol=1e-9), ctol=1e-9, max_outer=200)
    al = L.AuglagRows(L.OBJ_QP, to_dev(K), to_dev(b), to_dev(Cm), to_dev(d), to_dev(l), to_dev(u), m, sign=sd,
                      options=L.default_options(tol=1e-9), ctol=1e-9, max_outer=200)
    info = al.solve(to_dev(x0))
    x, lam = al.x().cpu().numpy(), al.lam().cpu().numpy()
    al.close()
    assert iref.status == oracle.CONVERGED and info.status == L.CONVERGED, info.as_dict()
    assert np.all(x >= l) and np.all(x <= u) and np.abs(Cm @ x - d).max() <= 1e-8
    assert rel_err(x, x_ref) <= (1e-5 if dtype == np.float64 else 1e-3)
    assert rel_err(lam, lam_ref) <= (1e-4 if dtype == np.float64 else 1e-2)
    assert info.f == pytest.approx(iref.f, rel=10 * ftol, abs=1e-10)
