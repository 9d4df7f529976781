"""The transport objective kinds (the paper's section "Joint Probability Distribution") and the marginal-constraint
entry point of Algorithm 4 against the CPU oracle.

Parity levels: (i) value, gradient and marginal residuals on identical inputs (1e-12 normwise), at shapes that
span several row blocks / column tiles with ragged tails, fp64 and fp32 cost matrices; (ii) single iterations of
Algorithm 1 from the same point (direction branch, step length, new iterate, new objective value); (iii) the box
solve without marginal terms; (iv) Algorithm 4 on the two generated families: coupling, multipliers, objective,
violation, number of outer iterations; (v) properties at a size the oracle does not reach.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2203_16340_amd as L
import workloads
from gpu_helpers import DEV, rel_err, to_dev

pytestmark = pytest.mark.gpu

KINDS = [(L.OBJ_OT_GAUSS, oracle.OT_GAUSS), (L.OBJ_OT_ENTROPY, oracle.OT_ENTROPY)]
KIND_IDS = ["gauss", "entropy"]
# rows x cols: one row block / one tile; several row blocks with a ragged last one; more than 512 rows (several rows
# per workgroup of the sum kernel); wider than one 256-column tile; a single row; a single column
SHAPES = [(5, 7), (37, 300), (1100, 19), (2100, 9), (40, 1000), (1, 130), (130, 1)]


def _problem(rng, rows, cols, dtype=np.float64):
    M = (rng.random((rows, cols)) - 0.3).astype(dtype)
    u, v = rng.random(rows) + 0.1, rng.random(cols) + 0.1
    return M, u / u.sum(), v / v.sum()


def _solver(kind, M, l, ub, m, lam, beta=None, omega=None, **opts):
    return L.Solver(kind, to_dev(M), to_dev(beta) if beta is not None else None, to_dev(l), to_dev(ub), m, lam=lam,
                    options=L.default_options(**opts), row_weight=to_dev(omega) if omega is not None else None)


@pytest.mark.parametrize("kinds", KINDS, ids=KIND_IDS)
@pytest.mark.parametrize("rows,cols", SHAPES)
@pytest.mark.parametrize("dtype", [np.float64, np.float32], ids=["f64", "f32"])
@pytest.mark.parametrize("with_marginals", [True, False], ids=["penalty", "plain"])
def test_value_gradient_and_marginal_residuals(kinds, rows, cols, dtype, with_marginals):
    kind, okind = kinds
    rng = np.random.default_rng(rows * 31 + cols)
    M, u, v = _problem(rng, rows, cols, dtype)
    n, lam, rho = rows * cols, 0.5, 2.5
    mult = rng.standard_normal(rows + cols)
    ref = oracle.Objective(okind, M, lam=lam)
    beta = omega = None
    if with_marginals:
        ref.set_marginals(u, v, lam=mult, rho=rho)
        beta, omega = np.concatenate([u, v]) - mult / rho, np.full(rows + cols, rho)
    x = rng.random(n) / n + 1e-6
    f_ref, g_ref, row_ref = oracle.fg(ref, x, want_rowvec=True)
    s = _solver(kind, M, np.full(n, 1e-30), np.full(n, np.inf), 3, lam, beta, omega)
    f, g, row = s.dbg_fg(to_dev(x), want_rowvec=True)
    assert abs(f - f_ref) <= 1e-12 * max(abs(f_ref), 1e-3)
    assert rel_err(g.cpu().numpy(), g_ref) <= 1e-12
    if with_marginals:
        assert rel_err(row.cpu().numpy(), row_ref) <= 1e-12
    s.close()


@pytest.mark.parametrize("kinds", KINDS, ids=KIND_IDS)
@pytest.mark.parametrize("rows,cols", [(37, 300), (1100, 19)])
def test_iterations_follow_the_oracle(kinds, rows, cols):
    kind, okind = kinds
    rng = np.random.default_rng(rows + cols)
    M, u, v = _problem(rng, rows, cols)
    n, lam, rho, lower = rows * cols, 0.5, 4.0, (0.0 if kind == L.OBJ_OT_GAUSS else 1e-30)
    mult = 0.01 * rng.standard_normal(rows + cols)
    l, ub = np.full(n, lower), np.full(n, np.inf)
    x0 = np.where(rng.random(n) < 0.5, lower, rng.random(n) / n)
    ref_obj = oracle.Objective(okind, M, lam=lam).set_marginals(u, v, lam=mult, rho=rho)
    ref = oracle.Solver(ref_obj, l, ub, x0, 5, oracle.default_options(tol=0.0))
    s = _solver(kind, M, l, ub, 5, lam, np.concatenate([u, v]) - mult / rho, np.full(rows + cols, rho), tol=0.0)
    s.set_x(to_dev(x0))
    for it in range(12):
        ref.step()
        info = s.step()
        ri = ref.info
        assert info.branch == ri.branch and info.backtracks == ri.backtracks, (it, info.as_dict())
        assert info.alpha == pytest.approx(ri.alpha, rel=1e-9)
        assert info.f == pytest.approx(ri.f, rel=1e-10), it
        assert rel_err(s.x().cpu().numpy(), ref.x) <= 1e-8, it
        assert rel_err(s.g().cpu().numpy(), ref.g) <= 1e-8, it
    ref.close()
    s.close()


@pytest.mark.parametrize("kinds", KINDS, ids=KIND_IDS)
def test_box_solve_without_marginal_terms(kinds):
    kind, okind = kinds
    rng = np.random.default_rng(9)
    rows, cols, lam = 70, 300, 0.5
    M = rng.standard_normal((rows, cols))
    n = rows * cols
    lo, hi = (0.0, np.inf) if kind == L.OBJ_OT_GAUSS else (0.2, 3.0)
    s = _solver(kind, M, np.full(n, lo), np.full(n, hi), 6, lam, tol=1e-10)
    s.set_x(to_dev(np.full(n, max(lo, 1.0) if kind == L.OBJ_OT_ENTROPY else 0.0)))
    info = s.solve()
    x = s.x().cpu().numpy().reshape(rows, cols)
    s.close()
    assert info.status == L.CONVERGED, info.as_dict()
    closed = np.maximum(0.0, -M / lam) if kind == L.OBJ_OT_GAUSS else np.clip(np.exp(-M / lam - 1.0), lo, hi)
    np.testing.assert_allclose(x, closed, atol=1e-9)


@pytest.mark.parametrize("kinds", KINDS, ids=KIND_IDS)
def test_box_solve_with_a_different_box_per_entry(kinds):
    """Bounds that differ from entry to entry (the kernels then stream l and u instead of taking one pair of
    numbers from the argument block): the separable problem still has an entrywise closed form."""
    kind, okind = kinds
    rng = np.random.default_rng(10)
    rows, cols, lam = 64, 310, 0.5
    M = rng.standard_normal((rows, cols))
    n = rows * cols
    lo = 0.05 + 0.2 * rng.random(n)
    hi = lo + 0.1 + rng.random(n)
    s = _solver(kind, M, lo, hi, 6, lam, tol=1e-10)
    s.set_x(to_dev(lo))
    info = s.solve()
    x = s.x().cpu().numpy()
    s.close()
    assert info.status == L.CONVERGED, info.as_dict()
    free = -M.reshape(-1) / lam if kind == L.OBJ_OT_GAUSS else np.exp(-M.reshape(-1) / lam - 1.0)
    np.testing.assert_allclose(x, np.clip(free, lo, hi), atol=1e-9)


def _run_gpu(p, tol, ctol, max_outer=100, max_iter=20000, dtype=np.float64, eps=1e-10):
    al = L.AuglagMarginals(p.kind, to_dev(p.M.astype(dtype)), to_dev(np.concatenate([p.u, p.v])), to_dev(p.l), to_dev(p.ub),
                           p.m, lam=p.lam, options=L.default_options(tol=tol, max_iter=max_iter, eps=eps),
                           ctol=ctol, max_outer=max_outer)
    info = al.solve(to_dev(p.x0))
    x = al.x().cpu().numpy()
    mult = al.lam().cpu().numpy()
    al.close()
    return x.reshape(p.rows, p.cols), mult, info


def _run_oracle(p, tol, ctol, max_outer=100, max_iter=20000):
    obj = oracle.Objective(p.kind, p.M, lam=p.lam).set_marginals(p.u, p.v)
    x, mult, _, info = oracle.auglag_solve(obj, p.l, p.ub, p.x0, p.m, oracle.default_options(tol=tol, max_iter=max_iter),
                                           ctol=ctol, max_outer=max_outer)
    return x.reshape(p.rows, p.cols), mult, info


@pytest.mark.parametrize("dataset,reg,size", [(1, "gauss", 40), (2, "gauss", 24), (1, "entropy", 16), (2, "entropy", 20)])
def test_joint_probability_against_the_oracle(dataset, reg, size):
    p = workloads.joint_probability(size, dataset=dataset, reg=reg, seed=6)
    P_ref, mult_ref, iref = _run_oracle(p, 1e-9, 1e-8)
    P, mult, info = _run_gpu(p, 1e-9, 1e-8)
    assert iref.status == oracle.CONVERGED and info.status == L.CONVERGED, info.as_dict()
    assert info.violation <= 1e-8
    assert P.min() >= p.lower
    np.testing.assert_allclose(P.sum(1), p.u, atol=1e-8)
    np.testing.assert_allclose(P.sum(0), p.v, atol=1e-8)
    assert rel_err(P, P_ref) <= 1e-5
    assert info.f == pytest.approx(iref.f, rel=1e-7, abs=1e-10)
    # the multipliers are determined up to the constant (+c on the rows, -c on the columns) the redundant
    # constraint leaves free; compare after removing it
    a, b = mult[:p.rows], mult[p.rows:]
    ar, br = mult_ref[:p.rows], mult_ref[p.rows:]
    assert rel_err(a[:, None] + b[None, :], ar[:, None] + br[None, :]) <= 1e-4
    assert abs(info.outer - iref.outer) <= 1 and info.rho == iref.rho


def test_fp32_cost_matrix_solves_the_same_problem():
    p = workloads.joint_probability(24, dataset=2, reg="gauss", seed=8, dtype=np.float32)
    P_ref, _, iref = _run_oracle(p, 1e-9, 1e-8)         # the oracle reads the same fp32 entries
    P, _, info = _run_gpu(p, 1e-9, 1e-8, dtype=np.float32)
    assert info.status == L.CONVERGED
    assert rel_err(P, P_ref) <= 1e-5
    assert info.f == pytest.approx(iref.f, rel=1e-7)


@pytest.mark.parametrize("dataset,reg", [(1, "gauss"), (2, "gauss"), (2, "entropy")])
def test_properties_at_a_larger_size(dataset, reg):
    size = 300
    p = workloads.joint_probability(size, dataset=dataset, reg=reg, seed=10)
    # Entries of P are 1e-5 and smaller here.  Eq. (ws) treats a variable within epsilon of its bound as sitting on it,
    # so with the default epsilon = 1e-10 the entropy's smallest (strictly positive) entries would be frozen there:
    # epsilon has to sit below the scale of the solution.
    P, mult, info = _run_gpu(p, 1e-8, 1e-8, max_iter=20000, eps=1e-10 if reg == "gauss" else 1e-20)
    assert info.status == L.CONVERGED, info.as_dict()
    assert P.min() >= p.lower
    assert np.abs(P.sum(1) - p.u).max() <= 1e-8 and np.abs(P.sum(0) - p.v).max() <= 1e-8
    a, b = mult[:p.rows], mult[p.rows:]
    if reg == "gauss":
        # optimality structure with the returned multipliers: the gradient of the augmented Lagrangian on the free
        # entries is below the inner tolerance 1e-8, so P is within 1e-8/lambda of the closed form
        closed = np.maximum(0.0, -(p.M + a[:, None] + b[None, :]) / p.lam)
        assert np.abs(P - closed).max() <= 1.5e-8 / p.lam
        assert info.f == pytest.approx(float((p.M * P).sum() + 0.5 * p.lam * (P * P).sum()), rel=1e-9)
    else:
        T = np.log(P) + p.M / p.lam
        T = T - T.mean(0, keepdims=True) - T.mean(1, keepdims=True) + T.mean()
        assert np.abs(T).max() <= 1e-6
        assert info.f == pytest.approx(float((p.M * P).sum() + p.lam * (P * np.log(P)).sum()), rel=1e-9)
    print(f"[transport] ds{dataset} {reg} {p.rows}x{p.cols}: outer {info.outer}, inner {info.inner_iters}, "
          f"violation {info.violation:.2e}, rho {info.rho}", flush=True)


# ---- at the sizes bench.py runs (10^6 and 2*10^6 variables): the long-vector Gram / direction kernels ----------------

@pytest.mark.parametrize("dataset,reg", [(1, "gauss"), (2, "gauss"), (1, "entropy"), (2, "entropy")])
def test_full_size_value_gradient_and_first_iterations(dataset, reg):
    """The oracle's cost is linear in the number of variables here, so it evaluates the full-size problem itself:
    value, gradient and marginal residuals at a feasible point, then the first iterations of Algorithm 1 step by step
    (direction branch, step length, iterate, gradient) on the augmented Lagrangian with non-zero multipliers."""
    p = workloads.joint_probability(1000, dataset=dataset, reg=reg, seed=4001)
    rng = np.random.default_rng(5)
    n, rho = p.n, 2.0
    mult = 1e-4 * rng.standard_normal(p.rows + p.cols)
    eps = 1e-10 if reg == "gauss" else 1e-20
    ref_obj = oracle.Objective(p.kind, p.M, lam=p.lam).set_marginals(p.u, p.v, lam=mult, rho=rho)
    x0 = np.where(rng.random(n) < 0.4, p.lower, rng.random(n) * 2.0 / n)
    f_ref, g_ref, row_ref = oracle.fg(ref_obj, x0, want_rowvec=True)
    s = _solver(p.kind, p.M, p.l, p.ub, p.m, p.lam, np.concatenate([p.u, p.v]) - mult / rho, np.full(p.rows + p.cols, rho),
                tol=0.0, eps=eps)
    f, g, row = s.dbg_fg(to_dev(x0), want_rowvec=True)
    assert abs(f - f_ref) <= 1e-12 * max(abs(f_ref), 1e-3)
    assert rel_err(g.cpu().numpy(), g_ref) <= 1e-12
    assert rel_err(row.cpu().numpy(), row_ref) <= 1e-12
    ref = oracle.Solver(ref_obj, p.l, p.ub, x0, p.m, oracle.default_options(tol=0.0, eps=eps))
    s.set_x(to_dev(x0))
    for it in range(14):          # past the point where the pair memory is full (m = 10)
        ref.step()
        info = s.step()
        ri = ref.info
        assert info.branch == ri.branch and info.backtracks == ri.backtracks, (it, info.as_dict())
        assert info.alpha == pytest.approx(ri.alpha, rel=1e-9)
        assert info.f == pytest.approx(ri.f, rel=1e-10, abs=1e-15), it
        assert info.n_fixed == ri.n_fixed, it
        assert rel_err(s.x().cpu().numpy(), ref.x) <= 1e-8, it
        assert rel_err(s.g().cpu().numpy(), ref.g) <= 1e-8, it
    ref.close()
    s.close()


@pytest.mark.parametrize("dataset", [1, 2])
def test_full_size_solve_properties(dataset):
    """bench.py's JP1G / JP2G run (same tolerances): a coupling with the dual structure of the Gaussian regulariser."""
    p = workloads.joint_probability(1000, dataset=dataset, reg="gauss", seed=4001)
    al = L.AuglagMarginals(p.kind, to_dev(p.M), to_dev(np.concatenate([p.u, p.v])), to_dev(p.l), to_dev(p.ub), p.m, lam=p.lam,
                           options=L.default_options(tol=1e-6, tol_relative=1, max_iter=5000), ctol=1e-6, max_outer=100)
    info = al.solve(to_dev(p.x0))
    P = al.x().cpu().numpy().reshape(p.rows, p.cols)
    mult = al.lam().cpu().numpy()
    al.close()
    assert info.status == L.CONVERGED, info.as_dict()
    assert P.min() >= 0.0
    assert np.abs(P.sum(1) - p.u).max() <= 1e-6 and np.abs(P.sum(0) - p.v).max() <= 1e-6
    a, b = mult[:p.rows], mult[p.rows:]
    closed = np.maximum(0.0, -(p.M + a[:, None] + b[None, :]) / p.lam)
    # inner tolerance: ||grad L [S]|| <= 1e-6 max(1, start value); the start value of the last inner solve is below 1
    assert np.abs(P - closed).max() <= 1.5e-6 / p.lam
    assert info.f == pytest.approx(float((p.M * P).sum() + 0.5 * p.lam * (P * P).sum()), rel=1e-9)
    print(f"[transport] full size ds{dataset}: outer {info.outer}, inner {info.inner_iters}, violation {info.violation:.2e}", flush=True)


@pytest.mark.parametrize("kinds", KINDS, ids=KIND_IDS)
def test_long_vector_runs_are_bit_reproducible(kinds):
    """163840 variables: 512 workgroups of the Gram kernel, partials added in two levels by whichever workgroups
    finish last -- the order of the additions must not depend on that."""
    kind, _ = kinds
    rng = np.random.default_rng(12)
    rows, cols = 512, 320
    M, u, v = _problem(rng, rows, cols)
    n, lam, rho, lower = rows * cols, 0.5, 3.0, (0.0 if kind == L.OBJ_OT_GAUSS else 1e-30)
    x0 = np.where(rng.random(n) < 0.5, lower, rng.random(n) / n)
    outs = []
    for _ in range(2):
        s = _solver(kind, M, np.full(n, lower), np.full(n, np.inf), 10, lam, np.concatenate([u, v]), np.full(rows + cols, rho),
                    tol=0.0)
        s.set_x(to_dev(x0))
        for _ in range(25):
            s.step(want_info=False)
        outs.append((s.x().clone(), s.g().clone(), s.info().f))
        s.close()
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1]) and outs[0][2] == outs[1][2]


def test_entropy_rejects_a_zero_lower_bound():
    M = np.zeros((4, 5))
    with pytest.raises(L.LbfgsbError) as e:
        _solver(L.OBJ_OT_ENTROPY, M, np.zeros(20), np.full(20, np.inf), 3, 0.5)
    assert e.value.code == L.E_BOUNDS


def test_timing_records_of_the_gram_kernel():
    """Transport kinds have no pass over a matrix: the benchmark's roofline figure times the Gram kernel instead, from
    the m-th iteration after lbfgsb_set_x on (pair memory full), and prices a launch at x, g, the newest y and the
    mask in full (25 bytes per variable with uniform bounds) plus the 2m pair vectors at the free variables."""
    rng = np.random.default_rng(77)
    rows, cols, m, lam, rho = 300, 500, 4, 0.5, 5.0
    M, u, v = _problem(rng, rows, cols)
    n = rows * cols
    s = _solver(L.OBJ_OT_GAUSS, M, np.zeros(n), np.full(n, np.inf), m, lam, np.concatenate([u, v]),
                np.full(rows + cols, rho), tol=0.0)
    s.set_x(to_dev(np.zeros(n)))
    s.enable_apass_timing(2)
    for _ in range(m + 6):
        s.step(want_info=False)
    info = s.info()
    count, total_ms, nbytes = s.apass_timing()
    assert count == 6
    assert nbytes == 25.0 * n + 16.0 * m * (n - info.n_fixed)
    assert 0 < info.n_fixed < n
    assert total_ms / count > 1e-3 * nbytes / 8e9
    s.close()
