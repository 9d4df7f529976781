"""Pins for the oracle's per-iteration primitives against things other than itself:
hand-worked truth tables (tests/golden), numpy/scipy library routines, finite differences,
and a dense BFGS-matrix construction of what Algorithm 3 must return."""
import math
import os

import numpy as np
import pytest

import oracle
import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _num(tok: str) -> float:
    return float(tok)  # float() understands 'inf' and '-inf'


# ---- Eq. (ws) --------------------------------------------------------------------------------

def _free_set_cases():
    rows = []
    with open(os.path.join(GOLDEN, "free_set_truth_table.txt")) as fh:
        for line in fh:
            line = line.split("#")[0].strip()
            if line:
                x, l, u, g, free = line.split()
                rows.append((_num(x), _num(l), _num(u), _num(g), int(free)))
    return rows


def test_free_set_truth_table():
    cases = _free_set_cases()
    assert len(cases) >= 30
    x, l, u, g, free = map(np.array, zip(*cases))
    got = oracle.free_mask(x, g, l, u, eps=0.125)
    assert got.tolist() == free.tolist()
    # one variable at a time as well (no cross-talk between coordinates)
    for xi, li, ui, gi, fi in cases:
        assert oracle.free_mask([xi], [gi], [li], [ui], eps=0.125)[0] == fi


def test_free_set_matches_set_formula_on_random_points():
    rng = np.random.default_rng(5)
    n, eps = 4000, 1e-3
    l = np.where(rng.random(n) < 0.2, -np.inf, rng.normal(size=n))
    u = np.where(rng.random(n) < 0.2, np.inf, np.where(np.isfinite(l), l, 0.0) + rng.random(n) * 2)
    # x: a mix of exactly-at-bound, within eps, interior
    t = rng.random(n)
    lo = np.where(np.isfinite(l), l, -3.0)
    hi = np.where(np.isfinite(u), u, 3.0)
    x = lo + t * (hi - lo)
    pick = rng.integers(0, 5, n)
    x = np.where((pick == 0) & np.isfinite(l), l, x)
    x = np.where((pick == 1) & np.isfinite(u), u, x)
    x = np.where((pick == 2) & np.isfinite(l), np.minimum(l + 0.5 * eps, hi), x)
    g = rng.normal(size=n) * (rng.random(n) > 0.1)      # some exact zeros
    fixed = set(np.flatnonzero((x <= l + eps) & (g >= 0))) | set(np.flatnonzero((x >= u - eps) & (g <= 0)))
    expect = np.array([0 if i in fixed else 1 for i in range(n)], dtype=np.uint8)
    assert 0.05 * n < len(fixed) < 0.95 * n
    assert np.array_equal(oracle.free_mask(x, g, l, u, eps), expect)


# ---- Algorithm 2 -----------------------------------------------------------------------------

def _project_cases():
    out = []
    with open(os.path.join(GOLDEN, "project_direction_cases.txt")) as fh:
        for line in fh:
            line = line.split("#")[0].strip()
            if not line:
                continue
            f = [t.strip() for t in line.split("|")]
            vec = lambda s: np.array([_num(t) for t in s.split()])
            out.append(dict(name=f[0], l=vec(f[1]), u=vec(f[2]), x=vec(f[3]), g=vec(f[4]), d=vec(f[5]),
                            branch=int(f[6]), p=vec(f[7]), alpha_ub=_num(f[8])))
    return out


@pytest.mark.parametrize("case", _project_cases(), ids=lambda c: c["name"])
def test_project_direction_worked_cases(case):
    p, branch, ub = oracle.project_direction(case["x"], case["g"], case["d"], case["l"], case["u"], eps=0.01)
    assert branch == case["branch"]
    np.testing.assert_allclose(p, case["p"], rtol=0, atol=1e-15)
    if math.isinf(case["alpha_ub"]):
        assert ub == math.inf
    else:
        assert ub == pytest.approx(case["alpha_ub"], rel=1e-14)


def test_project_direction_properties_random():
    """Branch 1: p = P(x+d) - x.  Branch 2 (proof of Theorem 1): p_i in {0, d_i},
    <g,p> <= <g,d> when d vanishes on the fixed set, ||p|| <= ||d||, and x + alpha p stays
    feasible for every alpha in [0, alpha_ub]."""
    rng = np.random.default_rng(11)
    eps = 1e-3
    seen = {1: 0, 2: 0}
    for trial in range(300):
        n = int(rng.integers(1, 12))
        l = -rng.random(n)
        u = rng.random(n)
        x = l + rng.random(n) * (u - l)
        snap = rng.integers(0, 4, n)
        x = np.where(snap == 0, l, np.where(snap == 1, u, x))
        g = rng.normal(size=n)
        mask = oracle.free_mask(x, g, l, u, eps).astype(bool)
        d = -g * rng.random(n) * (10.0 ** rng.integers(-4, 1))
        d[~mask] = 0.0
        p, branch, ub = oracle.project_direction(x, g, d, l, u, eps)
        seen[branch] += 1
        if branch == 1:
            np.testing.assert_array_equal(p, np.clip(x + d, l, u) - x)
            assert ub == 1.0
            assert p @ g <= -eps * (p @ p) and p @ p >= eps
        else:
            p1 = np.clip(x + d, l, u) - x
            assert not (p1 @ g <= -eps * (p1 @ p1) and p1 @ p1 >= eps)
            assert np.all((p == 0) | (p == d))
            assert g @ p <= g @ d + 1e-18
            assert np.linalg.norm(p) <= np.linalg.norm(d)
            for a in (0.0, 0.3 * ub, ub) if np.isfinite(ub) else (0.0, 1.0, 1e6):
                xa = x + a * p
                assert np.all(xa >= l - 1e-12) and np.all(xa <= u + 1e-12)
            if np.isfinite(ub) and np.any(p != 0):
                xa = x + 1.001 * ub * p - 0  # a hair beyond the bound must leave the box
                assert np.any(xa < l - 1e-15) or np.any(xa > u + 1e-15) or ub == 0.0
    assert seen[1] > 20 and seen[2] > 20
    # the remark after the corollary: the projection branch may be skipped
    p, branch, ub = oracle.project_direction([0.5], [1.0], [-0.2], [0.0], [1.0], eps, always_branch2=True)
    assert branch == 2 and p[0] == -0.2 and ub == pytest.approx(2.5)


# ---- objectives ------------------------------------------------------------------------------

def _small_objectives():
    rng = np.random.default_rng(3)
    A64 = rng.normal(size=(23, 7))
    A32 = rng.normal(size=(19, 5)).astype(np.float32)
    b = rng.normal(size=23)
    y = np.where(rng.random(19) < 0.5, -1.0, 1.0)
    return [
        ("lsq_f64", oracle.Objective(oracle.LSQ, A64, b)),
        ("lsq_f32", oracle.Objective(oracle.LSQ, A32, rng.normal(size=19))),
        ("l1split", oracle.Objective(oracle.LSQ_L1SPLIT, A64, b, lam=0.37)),
        ("logistic_f32", oracle.Objective(oracle.LOGISTIC_L2, A32, y, mu=0.05)),
        ("logistic_f64", oracle.Objective(oracle.LOGISTIC_L2, A64, np.where(b > 0, 1.0, -1.0), mu=1e-3)),
    ]


def _numpy_fg(obj, x):
    """The three objectives retyped from their definitions with numpy/scipy library calls."""
    from scipy.special import expit, log_expit
    A = obj.A.astype(np.float64)
    if obj.kind == oracle.LSQ:
        r = A @ x - obj.b
        return 0.5 * r @ r, A.T @ r
    if obj.kind == oracle.LSQ_L1SPLIT:
        c = A.shape[1]
        r = A @ (x[:c] - x[c:]) - obj.b
        w = A.T @ r
        return 0.5 * r @ r + obj.c.lam * x.sum(), np.concatenate([w + obj.c.lam, -w + obj.c.lam])
    z = A @ x
    N = A.shape[0]
    f = -log_expit(obj.b * z).sum() / N + 0.5 * obj.c.mu * x @ x
    g = -(A.T @ (obj.b * expit(-obj.b * z))) / N + obj.c.mu * x
    return f, g


@pytest.mark.parametrize("name,obj", _small_objectives(), ids=lambda v: v if isinstance(v, str) else "")
def test_fg_against_library_formulas_and_finite_differences(name, obj):
    rng = np.random.default_rng(17)
    n = obj.n
    for _ in range(3):
        x = rng.normal(size=n)
        f, g, row = oracle.fg(obj, x, want_rowvec=True)
        f_ref, g_ref = _numpy_fg(obj, x)
        assert f == pytest.approx(f_ref, rel=1e-13)
        np.testing.assert_allclose(g, g_ref, rtol=0, atol=1e-13 * max(1.0, np.abs(g_ref).max()))
        assert oracle.f_only(obj, x) == f
        # central differences: an independent check of the sign and scaling of every term
        h = 1e-6
        for i in range(n):
            e = np.zeros(n); e[i] = h
            fd = (oracle.f_only(obj, x + e) - oracle.f_only(obj, x - e)) / (2 * h)
            assert fd == pytest.approx(g[i], rel=2e-6, abs=2e-8)
        # the row vector is the residual / the margins
        A = obj.A.astype(np.float64)
        v = x if obj.kind != oracle.LSQ_L1SPLIT else x[:A.shape[1]] - x[A.shape[1]:]
        expect_row = A @ v - (obj.b if obj.kind != oracle.LOGISTIC_L2 else 0.0)
        np.testing.assert_allclose(row, expect_row, rtol=0, atol=1e-13)


def test_fg_respects_leading_dimension():
    rng = np.random.default_rng(2)
    big = rng.normal(size=(9, 11))
    view = big[:, :6]                      # ld = 11 > cols = 6
    b = rng.normal(size=9)
    x = rng.normal(size=6)
    f1, g1 = oracle.fg(oracle.Objective(oracle.LSQ, view, b), x)
    f2, g2 = oracle.fg(oracle.Objective(oracle.LSQ, np.ascontiguousarray(view), b), x)
    assert f1 == f2 and np.array_equal(g1, g2)


@pytest.mark.parametrize("name,obj", _small_objectives(), ids=lambda v: v if isinstance(v, str) else "")
def test_delta_f_equals_objective_difference(name, obj):
    """f(xt) - f(x) in its cancellation-free form: equals the plain difference for large
    steps, and the exact (rational-arithmetic) difference for tiny ones."""
    from fractions import Fraction
    rng = np.random.default_rng(23)
    n = obj.n
    x = rng.normal(size=n)
    _, _, row = oracle.fg(obj, x, want_rowvec=True)
    for scale in (1.0, 1e-3):
        xt = x + scale * rng.normal(size=n)
        plain = oracle.f_only(obj, xt) - oracle.f_only(obj, x)
        assert oracle.delta_f(obj, x, xt, row) == pytest.approx(plain, rel=1e-9 / scale, abs=1e-15)
    if obj.kind != oracle.LOGISTIC_L2:
        # exact reference with Fractions for a step of relative size 1e-9
        xt = x + 1e-9 * rng.normal(size=n)
        A = obj.A.astype(np.float64)
        c = A.shape[1]

        def exact_f(xx):
            v = [Fraction(t) for t in xx]
            if obj.kind == oracle.LSQ_L1SPLIT:
                vv = [v[j] - v[c + j] for j in range(c)]
            else:
                vv = v
            tot = Fraction(0)
            for r in range(A.shape[0]):
                res = sum(Fraction(A[r, j]) * vv[j] for j in range(c)) - Fraction(obj.b[r])
                tot += res * res / 2
            if obj.kind == oracle.LSQ_L1SPLIT:
                tot += Fraction(obj.c.lam) * sum(v)
            return tot

        exact = float(exact_f(xt) - exact_f(x))
        assert oracle.delta_f(obj, x, xt, row) == pytest.approx(exact, rel=1e-6)


def test_logistic_delta_f_where_the_margin_saturates():
    """softplus(a + da) - softplus(a) for a single row with a large margin a and a step da that undoes most of it:
    sigmoid(a) is 1 up to rounding and expm1(da) is nearly -1, so log1p(sigmoid(a) * expm1(da)) would take the
    logarithm of a difference of two numbers that agree to nine digits.  Reference: 60-digit decimal arithmetic on
    the definition log(1 + e^t)."""
    from decimal import Decimal, getcontext
    getcontext().prec = 60

    def softplus_exact(t):
        return (Decimal(1) + Decimal(t).exp()).ln()

    mu = 0.0
    for a, da in [(20.0, -25.0), (25.0, -29.5), (12.0, -11.0), (30.0, -29.0), (18.0, -3.0), (-20.0, 25.0), (3.0, -2.0),
                  (0.5, 1e-9), (40.0, -29.9), (35.0, -40.0)]:
        # one row, one variable, label y = -1: the loss is softplus(-y * X w) = softplus(w) with X = [[1]]
        obj = oracle.Objective(oracle.LOGISTIC_L2, np.array([[1.0]]), np.array([-1.0]), mu=mu)
        x, xt = np.array([a]), np.array([a + da])
        _, _, row = oracle.fg(obj, x, want_rowvec=True)
        exact = float(softplus_exact(a + da) - softplus_exact(a))
        got = oracle.delta_f(obj, x, xt, row)
        assert got == pytest.approx(exact, rel=1e-13, abs=1e-300), (a, da)


# ---- Algorithm 3 -----------------------------------------------------------------------------

def _dense_reference(S, Y, ynorm2, g, mask, eps):
    """What Algorithm 3 must return, built densely: start from H0 = gamma*I on the free
    coordinates (gamma = rho/||y||^2 of the newest pair if it passes its gate, else 1) and
    apply the BFGS inverse update H <- (I - s y^T/rho) H (I - y s^T/rho) + s s^T/rho for every
    masked pair that passes, oldest first; d[S] = -H g[S]."""
    F = np.flatnonzero(mask)
    k = len(F)
    Sm, Ym = S[:, F], Y[:, F]
    rho = np.einsum("ij,ij->i", Sm, Ym)
    ok = rho > eps * ynorm2
    H = np.eye(k)
    if len(rho) and ok[-1]:
        H *= rho[-1] / ynorm2[-1]
    for i in range(len(rho)):
        if ok[i]:
            V = np.eye(k) - np.outer(Ym[i], Sm[i]) / rho[i]
            H = V.T @ H @ V + np.outer(Sm[i], Sm[i]) / rho[i]
    d = np.zeros_like(g)
    d[F] = -H @ g[F]
    return d, int(ok.sum())


def _spd_pairs(rng, n, k, cond=50.0):
    Q, _ = np.linalg.qr(rng.normal(size=(n, n)))
    Hm = Q @ np.diag(np.linspace(1.0, cond, n)) @ Q.T
    S = rng.normal(size=(k, n))
    return S, S @ Hm


def test_two_loop_all_free_equals_textbook_bfgs():
    rng = np.random.default_rng(7)
    for n, k in ((6, 1), (20, 5), (50, 10)):
        S, Y = _spd_pairs(rng, n, k)
        g = rng.normal(size=n)
        mask = np.ones(n, dtype=np.uint8)
        yn = np.einsum("ij,ij->i", Y, Y)
        d, used = oracle.two_loop(S, Y, g, mask, eps=1e-10)
        ref, ref_used = _dense_reference(S, Y, yn, g, mask, 1e-10)
        assert used == ref_used == k
        np.testing.assert_allclose(d, ref, rtol=0, atol=1e-11 * np.linalg.norm(ref))
        assert g @ d < 0


def test_two_loop_masked_and_gated():
    rng = np.random.default_rng(8)
    hit_skip = hit_newest_fail = 0
    for trial in range(60):
        n = int(rng.integers(5, 40))
        k = int(rng.integers(1, 8))
        S, Y = _spd_pairs(rng, n, k)
        # make some pairs violate the curvature condition on the free set, as the appendix warns
        for i in range(k):
            if rng.random() < 0.35:
                Y[i] = -Y[i] if rng.random() < 0.5 else rng.normal(size=n)
        mask = (rng.random(n) < 0.7).astype(np.uint8)
        if mask.sum() == 0:
            mask[0] = 1
        g = rng.normal(size=n)
        eps = 10.0 ** rng.integers(-10, -1)
        yn = np.einsum("ij,ij->i", Y, Y)          # full-vector norms, as printed in the listing
        d, used = oracle.two_loop(S, Y, g, mask, eps, ynorm2=yn)
        ref, ref_used = _dense_reference(S, Y, yn, g, mask, eps)
        assert used == ref_used
        hit_skip += used < k
        rho_new = (S[-1] * Y[-1])[mask.astype(bool)].sum()
        hit_newest_fail += (not rho_new > eps * yn[-1]) and used > 0
        np.testing.assert_allclose(d, ref, rtol=0, atol=1e-10 * max(np.linalg.norm(ref), 1e-300))
        assert np.all(d[mask == 0] == 0.0)
        if np.any(g[mask.astype(bool)] != 0):
            assert g @ d < 0                       # descent (Eq. (1) in the proof of Theorem 1)
    assert hit_skip > 5 and hit_newest_fail > 0


def test_two_loop_no_pairs_is_masked_steepest_descent():
    g = np.array([1.0, -2.0, 3.0, -4.0])
    mask = np.array([1, 0, 1, 1], dtype=np.uint8)
    d, used = oracle.two_loop(np.empty((0, 4)), np.empty((0, 4)), g, mask, 1e-10)
    assert used == 0
    assert d.tolist() == [-1.0, 0.0, -3.0, 4.0]


def test_two_loop_gate_uses_full_norm_and_strict_inequality():
    # one pair, n = 2, mask keeps only coordinate 0:  rho = s0*y0 = 1, ||y||^2 (full) = 1 + 99 = 100.
    S = np.array([[1.0, 0.0]])
    Y = np.array([[1.0, math.sqrt(99.0)]])
    g = np.array([2.0, 5.0])
    mask = np.array([1, 0], dtype=np.uint8)
    yn = np.array([100.0])
    # eps*||y||^2 = 1 = rho  -> '>' fails -> pair unused -> d = -g on S
    d, used = oracle.two_loop(S, Y, g, mask, eps=0.01, ynorm2=yn)
    assert used == 0 and d.tolist() == [-2.0, 0.0]
    # slightly smaller eps -> used.  q = g0 - (s0 g0/rho) y0 = 0; scaled; + (alpha - beta) s0 = alpha = 2
    d, used = oracle.two_loop(S, Y, g, mask, eps=0.0099, ynorm2=yn)
    assert used == 1 and d.tolist() == [-2.0, 0.0]
    # with the masked norm (1.0) instead of the full norm the gate would pass at eps = 0.5;
    # with the full norm it must not
    d, used = oracle.two_loop(S, Y, g, mask, eps=0.5, ynorm2=yn)
    assert used == 0


def test_two_loop_scaling_by_newest_pair():
    # single pair s = (2, 0), y = (1, 0) on n = 2, all free: H = (I - s y^T/rho) gamma (I - y s^T/rho) + s s^T/rho
    # rho = 2, gamma = rho/||y||^2 = 2.  For g = (0, 1): H g = gamma * g = (0, 2).  For g = (1, 0): H g = s s^T g/rho = (2, 0).
    S = np.array([[2.0, 0.0]]); Y = np.array([[1.0, 0.0]])
    mask = np.ones(2, dtype=np.uint8)
    d, _ = oracle.two_loop(S, Y, np.array([0.0, 1.0]), mask, 1e-10)
    assert d.tolist() == [0.0, -2.0]
    d, _ = oracle.two_loop(S, Y, np.array([1.0, 0.0]), mask, 1e-10)
    assert d.tolist() == [-2.0, 0.0]


# ---- input generators (shared with the GPU tests): shape and distribution sanity --------------

def test_config_generators_match_their_recipes():
    p = workloads.config("C1")
    assert p.A.shape == (200, 100) and p.A.dtype == np.float64 and p.m == 5
    assert (p.x_true == 0).sum() == 50 and np.all(p.x_true >= 0)
    assert np.all(p.l == 0) and np.all(np.isinf(p.u)) and np.all(p.x0 == 0)
    assert abs(np.std(p.b - p.A @ p.x_true) - 0.01) < 0.002
    q = workloads.config("C1")
    assert np.array_equal(p.A, q.A) and np.array_equal(p.b, q.b)       # seeded
    p = workloads.config("C3", scale=0.02)
    assert p.n == 2 * p.cols and p.kind == workloads.OBJ_LSQ_L1SPLIT
    assert p.lam == pytest.approx(0.1 * np.abs(p.A.T @ p.b).max())
    assert abs(np.std(p.A) * math.sqrt(p.rows) - 1.0) < 0.05
    p = workloads.config("C4", scale=0.01)
    assert p.A.dtype == np.float32 and set(np.unique(p.b)) <= {-1.0, 1.0}
    assert np.all(p.l == -0.5) and np.all(p.u == 0.5) and p.mu == 1e-3
    p = workloads.config("C5", scale=0.01)
    assert p.A.dtype == np.float32 and np.all(p.u == 1.0) and p.m == 20
    assert (p.x_true == 0).sum() == round(0.9 * p.cols) and p.x_true.max() < 1.0
