"""The quadratic-form objective (dual SVM of the paper's section "Dual SVM"), the extra dense rows that
carry penalty terms, and Algorithm 4 with separately passed constraint rows, against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2203_16340_amd as L
import workloads
from gpu_helpers import DEV, rel_err, to_dev

pytestmark = pytest.mark.gpu


def _spd(rng, n, dtype=np.float64):
    M = rng.standard_normal((n, max(n, 2)))
    K = M @ M.T / n + 0.5 * np.eye(n)
    K = K.astype(dtype)
    return np.ascontiguousarray(0.5 * (K + K.T))


@pytest.mark.parametrize("a_pass", [L.APASS_TWO_PASS, L.APASS_FUSED], ids=["two_pass", "fused"])
@pytest.mark.parametrize("dtype", [np.float64, np.float32], ids=["f64", "f32"])
@pytest.mark.parametrize("n,with_sign", [(1, False), (37, True), (300, True), (1030, False), (2051, True), (5200, True)])
def test_fg_parity(n, with_sign, dtype, a_pass):
    rng = np.random.default_rng(n)
    K, b = _spd(rng, n, dtype), rng.standard_normal(n)
    s = np.where(rng.random(n) < 0.5, -1.0, 1.0) if with_sign else None
    ref = oracle.Objective(oracle.QP, K, b, sign=s)
    x = rng.standard_normal(n)
    f_ref, g_ref, row_ref = oracle.fg(ref, x, want_rowvec=True)
    try:
        sol = L.Solver(L.OBJ_QP, to_dev(K), to_dev(b), to_dev(np.full(n, -np.inf)), to_dev(np.full(n, np.inf)), 3,
                       sign=to_dev(s) if s is not None else None, options=L.default_options(a_pass=a_pass))
    except L.LbfgsbError as e:
        if e.code == L.E_UNSUPPORTED:
            pytest.skip("shape not supported by the fused pass (rows not 16-byte aligned)")
        raise
    f, g, row = sol.dbg_fg(to_dev(x), want_rowvec=True)
    tol = 1e-12 if dtype == np.float64 else 1e-5
    assert abs(f - f_ref) <= tol * max(abs(f_ref), np.linalg.norm(g_ref))
    assert rel_err(g.cpu().numpy(), g_ref) <= tol
    assert rel_err(row.cpu().numpy(), row_ref) <= tol
    assert sol.apass_name == ("fused" if a_pass == L.APASS_FUSED else "two_pass")
    sol.close()


@pytest.mark.parametrize("kind", ["lsq", "qp"])
def test_extra_rows_add_the_penalty_term(kind):
    rng = np.random.default_rng(17)
    n, n_eq, rho = 150, 4, 2.5
    C, d, lam = rng.standard_normal((n_eq, n)), rng.standard_normal(n_eq), rng.standard_normal(n_eq)
    if kind == "lsq":
        A, b = rng.standard_normal((400, n)), rng.standard_normal(400)
        ref = oracle.Objective(oracle.LSQ, A, b).set_constraints(C, d, lam=lam, rho=rho)
        mk = lambda extra: L.Solver(L.OBJ_LSQ, to_dev(A), to_dev(b), to_dev(np.full(n, -np.inf)),
                                    to_dev(np.full(n, np.inf)), 3, extra=extra)
    else:
        K, b = _spd(rng, n), rng.standard_normal(n)
        s = np.where(rng.random(n) < 0.5, -1.0, 1.0)
        ref = oracle.Objective(oracle.QP, K, b, sign=s).set_constraints(C, d, lam=lam, rho=rho)
        mk = lambda extra: L.Solver(L.OBJ_QP, to_dev(K), to_dev(b), to_dev(np.full(n, -np.inf)),
                                    to_dev(np.full(n, np.inf)), 3, sign=to_dev(s), extra=extra)
    x = rng.standard_normal(n)
    f_ref, g_ref = oracle.fg(ref, x)
    sol = mk((to_dev(C), to_dev(d - lam / rho), to_dev(np.full(n_eq, rho))))
    f, g = sol.dbg_fg(to_dev(x))
    assert abs(f - f_ref) <= 1e-12 * abs(f_ref)
    assert rel_err(g.cpu().numpy(), g_ref) <= 1e-12
    sol.close()


def test_box_constrained_quadratic_form_matches_the_oracle():
    rng = np.random.default_rng(23)
    n = 400
    K, b = _spd(rng, n), 3.0 * rng.standard_normal(n)
    s = np.where(rng.random(n) < 0.5, -1.0, 1.0)
    l, u = np.zeros(n), np.ones(n)
    obj = oracle.Objective(oracle.QP, K, b, sign=s)
    osol = oracle.Solver(obj, l, u, np.zeros(n), 8, oracle.default_options(tol=1e-10))
    ref = osol.solve()
    sol = L.Solver(L.OBJ_QP, to_dev(K), to_dev(b), to_dev(l), to_dev(u), 8, sign=to_dev(s),
                   options=L.default_options(tol=1e-10))
    sol.set_x(to_dev(np.zeros(n)))
    info = sol.solve()
    x = sol.x().cpu().numpy()
    assert ref.info.status == oracle.CONVERGED and info.status == L.CONVERGED
    assert abs(info.f - ref.info.f) <= 1e-8 * abs(ref.info.f)
    assert rel_err(x, ref.x) <= 1e-7
    assert np.array_equal((x <= 1e-10) | (x >= 1 - 1e-10), (ref.x <= 1e-10) | (ref.x >= 1 - 1e-10))
    # first iterations step by step
    osol.close()
    osol = oracle.Solver(obj, l, u, np.zeros(n), 8, oracle.default_options(tol=0.0))
    sol.set_x(to_dev(np.zeros(n)))
    for k in range(3):
        assert osol.step() == oracle.RUNNING
        gi, oi = sol.step(), osol.info
        assert (gi.branch, gi.backtracks, gi.pairs_used) == (oi.branch, oi.backtracks, oi.pairs_used)
        assert gi.alpha == pytest.approx(oi.alpha, rel=1e-12)
        assert gi.f == pytest.approx(oi.f, rel=1e-10)
        assert rel_err(sol.x().cpu().numpy(), osol.x) <= 1e-10
        assert rel_err(sol.g().cpu().numpy(), osol.g) <= 1e-9
    osol.close()
    sol.close()


def _svm_gpu(sp, tol, ctol, max_outer=200):
    n = sp.n
    al = L.AuglagRows(L.OBJ_QP, to_dev(sp.K), to_dev(-np.ones(n)), to_dev(sp.y[None, :].copy()), to_dev(np.zeros(1)),
                      to_dev(np.zeros(n)), to_dev(np.full(n, sp.c)), sp.m, sign=to_dev(sp.y),
                      options=L.default_options(tol=tol), ctol=ctol, max_outer=max_outer)
    info = al.solve(to_dev(np.zeros(n)))
    a, lam = al.x().cpu().numpy(), al.lam().cpu().numpy()
    al.close()
    return a, lam, info


def test_dual_svm_with_the_equality_constraint_matches_the_oracle():
    sp = workloads.svm_dual(300, 4, seed=5, separation=1.2, m=8)
    n = sp.n
    obj = oracle.Objective(oracle.QP, sp.K, -np.ones(n), sign=sp.y).set_constraints(sp.y[None, :], [0.0])
    a_ref, lam_ref, _, iref = oracle.auglag_solve(obj, np.zeros(n), np.full(n, sp.c), np.zeros(n), sp.m,
                                                  oracle.default_options(tol=1e-9), ctol=1e-9, max_outer=200)
    a, lam, info = _svm_gpu(sp, 1e-9, 1e-9)
    assert iref.status == oracle.CONVERGED and info.status == L.CONVERGED, info.as_dict()
    assert info.violation <= 1e-9 and abs(sp.y @ a) <= 1e-9
    assert np.all(a >= 0) and np.all(a <= sp.c)
    assert rel_err(a, a_ref) <= 1e-5
    assert lam[0] == pytest.approx(lam_ref[0], rel=1e-5, abs=1e-7)
    assert info.f == pytest.approx(iref.f, rel=1e-7)
    assert abs(info.outer - iref.outer) <= 1
    bound = lambda v: (v <= 1e-9) | (v >= sp.c - 1e-9)
    assert np.mean(bound(a) == bound(a_ref)) >= 0.99


def test_dual_svm_properties_at_a_larger_size():
    sp = workloads.svm_dual(3000, 10, seed=6, separation=1.0)
    a, lam, info = _svm_gpu(sp, 1e-7, 1e-8)
    assert info.status == L.CONVERGED, info.as_dict()
    assert abs(sp.y @ a) <= 1e-8 and np.all(a >= 0) and np.all(a <= sp.c)
    dec = sp.K @ (a * sp.y) + lam[0]                      # decision values; lambda is the bias
    free = (a > 1e-6) & (a < sp.c - 1e-6)
    assert free.sum() > 10
    np.testing.assert_allclose(sp.y[free] * dec[free], 1.0, atol=1e-4)
    assert np.all(sp.y[a <= 1e-9] * dec[a <= 1e-9] >= 1.0 - 1e-4)          # non-support vectors are outside the margin
    assert np.all(sp.y[a >= sp.c - 1e-9] * dec[a >= sp.c - 1e-9] <= 1.0 + 1e-4)
    Q = (sp.y[:, None] * sp.K) * sp.y[None, :]
    assert info.f == pytest.approx(0.5 * a @ Q @ a - a.sum(), rel=1e-9)
    assert np.mean(np.sign(dec) == sp.y) > 0.7


def test_argument_errors():
    K = to_dev(np.eye(4))
    with pytest.raises(ValueError):
        L.Solver(L.OBJ_QP, to_dev(np.ones((3, 4))), to_dev(np.ones(3)), to_dev(np.zeros(4)), to_dev(np.ones(4)), 3)
    with pytest.raises(L.LbfgsbError) as e:
        L.AuglagRows(L.OBJ_LOGISTIC_L2, K, to_dev(np.ones(4)), to_dev(np.ones((1, 4))), to_dev(np.zeros(1)),
                     to_dev(np.zeros(4)), to_dev(np.ones(4)), 3)
    assert e.value.code == L.E_INVALID_ARG
