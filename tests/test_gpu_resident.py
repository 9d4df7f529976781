"""The single-workgroup resident solver (small plain least squares: matrix in registers, vectors in LDS, whole
iterations without leaving the compute unit) against the oracle: iteration by iteration, whole solves, every
instantiation (tiles per lane x column chunks), both storage types, odd shapes and a padded leading dimension, the
in-kernel recomputation of the gradient, and its agreement with the multi-kernel organisations."""
import numpy as np
import pytest
import torch

import oracle
import paper_2203_16340_amd as L
import workloads
from gpu_helpers import DEV, active_set, kkt_residual, rel_err, to_dev

pytestmark = pytest.mark.gpu

# rows x cols: every instantiation (columns per lane x rows per group: 8x4, 4x8, 7x7, 8x8, 16x4) at its limits and
# inside them, odd sizes, a single row, a single column
SHAPES = [(60, 30), (128, 128), (120, 77), (256, 64), (250, 5), (200, 100), (224, 112), (208, 128), (256, 128), (30, 200),
          (128, 256), (61, 201), (1, 40), (40, 1), (7, 3)]


def _problem(rows, cols, seed, dtype=np.float64, upper=np.inf, m=5):
    return workloads.nnls(rows, cols, seed=seed, dtype=dtype, zero_frac=0.5, nonzero="absnormal", noise=0.5,
                          upper=upper, m=m, tol=1e-9)


def _solver(prob, A_dev=None, **opts):
    A = to_dev(prob.A) if A_dev is None else A_dev
    s = L.Solver(prob.kind, A, to_dev(prob.b), to_dev(prob.l), to_dev(prob.u), prob.m,
                 options=L.default_options(**opts))
    s.set_x(to_dev(prob.x0))
    return s


@pytest.mark.parametrize("dtype", [np.float64, np.float32], ids=["f64", "f32"])
@pytest.mark.parametrize("rows,cols", SHAPES)
def test_iterations_and_solve_follow_the_oracle(rows, cols, dtype):
    prob = _problem(rows, cols, seed=rows * 7 + cols, dtype=dtype, upper=(2.0 if (rows + cols) % 2 else np.inf))
    s = _solver(prob, tol=1e-9, a_pass=L.APASS_RESIDENT)
    assert s.apass_name == "resident"
    orc = oracle.Solver(oracle.Objective(prob.kind, prob.A, prob.b), prob.l, prob.u, prob.x0, prob.m,
                        oracle.default_options(tol=1e-9))
    tol = 1e-10 if dtype == np.float64 else 1e-6
    g0_norm = float(np.linalg.norm(orc.g))
    for k in range(4):
        ost = orc.step()
        info = s.step()
        assert info.status == ost
        if ost != oracle.RUNNING:
            break
        oi = orc.info
        assert (info.iters, info.branch, info.backtracks, info.pairs_used) == (oi.iters, oi.branch, oi.backtracks, oi.pairs_used)
        assert info.alpha == pytest.approx(oi.alpha, rel=1e-12)
        assert info.gp == pytest.approx(oi.gp, rel=tol) and info.f == pytest.approx(oi.f, rel=tol)
        assert rel_err(s.x().cpu().numpy(), orc.x) <= tol
        # (one row or one column: the first step can land on the minimiser, where the gradient is pure rounding)
        assert rel_err(s.g().cpu().numpy(), orc.g) <= 10 * tol or \
            np.linalg.norm(s.g().cpu().numpy() - orc.g) <= 1e-13 * g0_norm
    f0 = 0.5 * float(prob.b @ prob.b)                                # objective at x0 = 0
    ref = orc.solve()
    info = s.solve()
    x = s.x().cpu().numpy()
    assert info.status == L.CONVERGED == ref.info.status
    # (more columns than rows: the residual can be driven to zero and the minimiser is not unique, so the objective is
    # compared on the scale of its start value and the point through the KKT conditions only)
    assert abs(info.f - ref.info.f) <= (1e-8 if dtype == np.float64 else 1e-4) * max(abs(ref.info.f), 1e-10 * f0)
    if rows >= cols:
        assert np.array_equal(active_set(prob, x), active_set(prob, ref.x))
        assert rel_err(x, ref.x) <= 1e-6
    res, g_host = kkt_residual(prob, x)
    assert res <= 1e-7
    # what the other entry points read afterwards: gradient and free mask in device memory
    assert rel_err(s.g().cpu().numpy(), g_host) <= 1e-7 or np.linalg.norm(g_host) < 1e-6
    s.close(); orc.close()


def test_padded_leading_dimension_and_agreement_with_the_other_organisations():
    prob = _problem(200, 100, seed=5)
    buf = torch.zeros(200, 116, dtype=torch.float64, device=DEV)
    buf[:, :100] = to_dev(prob.A)
    results = []
    for a_pass, A_dev in ((L.APASS_RESIDENT, buf[:, :100]), (L.APASS_FUSED, None), (L.APASS_TWO_PASS, None)):
        s = _solver(prob, A_dev=A_dev, tol=1e-10, a_pass=a_pass)
        info = s.solve()
        assert info.status == L.CONVERGED
        results.append((s.x().cpu().numpy(), info.f, info.iters))
        s.close()
    for x, f, it in results[1:]:
        assert rel_err(results[0][0], x) <= 1e-8 and f == pytest.approx(results[0][1], rel=1e-10)
        assert abs(it - results[0][2]) <= 3


@pytest.mark.parametrize("refresh_every", [0, 1, 4])
def test_in_kernel_recomputation_of_the_gradient(refresh_every):
    """With refresh_every = 1 every iteration starts from a gradient computed from x; with 0 it is never recomputed
    except before convergence is declared.  All three follow the oracle, and the reported gradient is the true one."""
    prob = workloads.config("C1")
    ref = oracle.solve_problem(prob)
    s = _solver(prob, tol=1e-8, a_pass=L.APASS_RESIDENT, refresh_every=refresh_every)
    for _ in range(20):
        s.step(want_info=False)
    x, g = s.x().cpu().numpy(), s.g().cpu().numpy()
    g_true = prob.A.T @ (prob.A @ x - prob.b)
    assert rel_err(g, g_true) <= 1e-11
    info = s.solve()
    x = s.x().cpu().numpy()
    assert info.status == L.CONVERGED and info.iters == pytest.approx(ref.info.iters, abs=3)
    assert abs(info.f - ref.info.f) <= 1e-8 * abs(ref.info.f)
    assert np.array_equal(active_set(prob, x), active_set(prob, ref.x))
    assert kkt_residual(prob, x)[0] <= 1e-8
    # fevals: one per accepted trial plus the rejected ones plus the evaluations from scratch
    assert info.fevals >= info.iters + 1
    s.close()


def test_one_launch_per_solve_equals_one_launch_per_step():
    prob = workloads.config("C1")
    a = _solver(prob, tol=0.0, max_iter=30, a_pass=L.APASS_RESIDENT)
    b = _solver(prob, tol=0.0, max_iter=30, a_pass=L.APASS_RESIDENT)
    ia = a.solve()
    for _ in range(30):
        b.step(want_info=False)
    ib = b.step()                                   # 31st call: the iteration limit stops it
    assert ia.status == ib.status == L.MAX_ITER and ia.iters == ib.iters == 30
    assert torch.equal(a.x(), b.x()) and torch.equal(a.g(), b.g()) and ia.f == ib.f
    a.close(); b.close()


def test_selection_and_refusal():
    small = _problem(200, 100, seed=1)
    s = _solver(small)                              # AUTO
    assert s.apass_name == "resident"
    s.close()
    for a_pass, name in ((L.APASS_FUSED, "fused"), (L.APASS_TWO_PASS, "two_pass")):
        s = _solver(small, a_pass=a_pass)
        assert s.apass_name == name
        s.close()
    big = _problem(400, 100, seed=2)                # 13 rows per group of lanes: does not fit the registers
    s = _solver(big)
    assert s.apass_name != "resident"
    s.close()
    with pytest.raises(L.LbfgsbError) as e:
        _solver(big, a_pass=L.APASS_RESIDENT)
    assert e.value.code == L.E_UNSUPPORTED
    # other objective kinds and weighted rows keep the multi-kernel organisations
    logi = workloads.config("C4", scale=0.001)
    s = L.solver_for_problem(logi, DEV)
    assert s.apass_name != "resident"
    s.close()
    w = to_dev(np.ones(small.rows))
    s = L.Solver(small.kind, to_dev(small.A), to_dev(small.b), to_dev(small.l), to_dev(small.u), small.m, row_weight=w)
    assert s.apass_name != "resident"
    s.close()


def test_primitive_hooks_still_work_around_resident_steps():
    """The hooks run the multi-kernel kernels on the same workspace; a set_x afterwards restores the solver."""
    prob = workloads.config("C1")
    s = _solver(prob, tol=1e-8)
    assert s.apass_name == "resident"
    for _ in range(5):
        s.step(want_info=False)
    x5 = s.x().clone()
    f, g = s.dbg_fg(x5)
    assert rel_err(g.cpu().numpy(), prob.A.T @ (prob.A @ x5.cpu().numpy() - prob.b)) <= 1e-12
    s.set_x(to_dev(prob.x0))
    info = s.solve()
    ref = oracle.solve_problem(prob)
    assert info.status == L.CONVERGED and abs(info.f - ref.info.f) <= 1e-8 * abs(ref.info.f)
    s.close()
