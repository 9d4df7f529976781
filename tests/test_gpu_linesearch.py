"""The line search's hard paths on the GPU, iteration by iteration against the oracle:

  * logistic problems on which the Armijo search (section "Algorithm") really backtracks -- badly scaled
    features, so unit steps overshoot: the second stage of the search on the margins (eight step lengths per
    sweep), its one-at-a-time continuation beyond nine trials, the transposed pass over X after a rejected
    speculative first step, and the update reading that pass's partial columns all do work here;
  * exhausted searches for the quadratic, logistic and entropy kinds: pair memory cleared, one retry from
    steepest descent on the free set, then LINESEARCH_FAILED.  The oracle's branch for this is pinned by the
    hand-worked cases of tests/test_oracle_linesearch_exhausted.py; the same hand-worked cases run here too.

Every case asserts first that the ORACLE shows the behaviour the case is there for (so a change of recipe that
makes a case trivial fails loudly), then compares the GPU with it.  On the GPU an exhausted search ends the
lbfgsb_step call it happened in (memory cleared, iteration count unchanged); the retry is the next call.
"""
from fractions import Fraction as F

import numpy as np
import pytest
import torch

import oracle
import paper_2203_16340_amd as L
import workloads
from gpu_helpers import DEV, rel_err, to_dev

pytestmark = pytest.mark.gpu

A_PASSES = [L.APASS_FUSED, L.APASS_TWO_PASS]
A_PASS_IDS = ["fused", "two_pass"]


def _oracle_solver(prob, **opts):
    obj = oracle.Objective(prob.kind, prob.A, prob.b, prob.lam, prob.mu)
    return oracle.Solver(obj, prob.l, prob.u, prob.x0, prob.m, oracle.default_options(**opts))


def _gpu_iteration(s):
    """One iteration of Algorithm 1 in the oracle's sense: an lbfgsb_step call whose search is exhausted only clears
    the memory, the call after it is the retry."""
    before = s.info()
    for _ in range(2):
        info = s.step()
        if info.status != L.RUNNING or info.iters > before.iters:
            return info
        assert info.memory_resets == before.memory_resets + 1, info.as_dict()
    raise AssertionError("two lbfgsb_step calls neither advanced nor stopped: " + str(info.as_dict()))


def _follow(orc, s, iters, tol, what):
    """Advances both by `iters` iterations (or until both stop) and compares after each one.  Returns the oracle's
    per-iteration backtrack counts."""
    bts = []
    for k in range(iters):
        ost = orc.step()
        oi = orc.info
        info = _gpu_iteration(s)
        tag = (what, k, info.as_dict())
        assert info.status == ost, tag
        assert (info.iters, info.memory_resets) == (oi.iters, oi.memory_resets), tag
        x, g = s.x().cpu().numpy(), s.g().cpu().numpy()
        assert rel_err(x, orc.x) <= tol, tag
        assert rel_err(g, orc.g) <= 10 * tol, tag
        assert info.f == pytest.approx(oi.f, rel=tol, abs=1e-300), tag
        if ost != oracle.RUNNING:
            break
        assert (info.branch, info.backtracks, info.pairs_used) == (oi.branch, oi.backtracks, oi.pairs_used), tag
        assert info.alpha == pytest.approx(oi.alpha, rel=1e-12), tag
        assert info.gp == pytest.approx(oi.gp, rel=tol), tag
        bts.append(oi.backtracks)
    return bts


# ---- logistic objective: searches that backtrack ------------------------------------------------------------------

LOGISTIC_CASES = [
    # the first step needs 14 halvings (more than the 1 + 8 of the two batched stages), later ones 1
    dict(rows=700, cols=80, seed=0, feature_scale=20, column_spread=2, bound=5.0, random_start=False, label_noise=0.5, mu=1e-3, m=5),
    dict(rows=700, cols=80, seed=1, feature_scale=5, column_spread=1, bound=50.0, random_start=True, label_noise=0.1, mu=1e-5, m=10),
    # 300 columns: several column tiles; 18 halvings in the first iteration
    dict(rows=600, cols=300, seed=1, feature_scale=20, column_spread=2, bound=50.0, random_start=False, label_noise=0.1, mu=1e-5, m=10),
    dict(rows=700, cols=80, seed=0, feature_scale=1, column_spread=1.5, bound=50.0, random_start=True, label_noise=0.0, mu=1e-6, m=3),
    dict(rows=700, cols=80, seed=2, feature_scale=1, column_spread=1.5, bound=0.5, random_start=True, label_noise=0.5, mu=1e-3, m=5),
]


def _logistic(case, dtype):
    prob = workloads.logistic(dtype=np.float64, **case)
    prob.A = np.ascontiguousarray(prob.A.astype(dtype))
    return prob


@pytest.mark.parametrize("a_pass", A_PASSES, ids=A_PASS_IDS)
@pytest.mark.parametrize("dtype", [np.float64, np.float32], ids=["f64", "f32"])
@pytest.mark.parametrize("case", range(len(LOGISTIC_CASES)))
def test_logistic_backtracking_follows_the_oracle(case, dtype, a_pass):
    prob = _logistic(LOGISTIC_CASES[case], dtype)
    orc = _oracle_solver(prob, tol=0.0)
    s = L.solver_for_problem(prob, DEV, tol=0.0, a_pass=a_pass)
    assert s.apass_name == ("fused" if a_pass == L.APASS_FUSED else "two_pass")
    bts = _follow(orc, s, 16, 1e-8 if dtype == np.float64 else 1e-6, f"logistic case {case}")
    assert sum(1 for b in bts if b >= 1) >= 3, bts          # the oracle did backtrack in at least 3 iterations
    if case in (0, 2):
        assert max(bts) > 1 + 8, bts                        # ... and beyond the two batched stages
    orc.close(); s.close()


def test_the_logistic_cases_cover_every_stage_of_the_search():
    """Between them the cases above accept at the first trial, inside the second stage (1..8 halvings) and in the
    one-at-a-time continuation (9 or more), as counted by the oracle."""
    seen = set()
    for case in LOGISTIC_CASES:
        orc = _oracle_solver(_logistic(case, np.float64), tol=0.0)
        for _ in range(16):
            orc.step()
            b = orc.info.backtracks
            seen.add("first" if b == 0 else ("batch" if b <= 8 else "continuation"))
        orc.close()
    assert seen == {"first", "batch", "continuation"}


@pytest.mark.parametrize("case", [0, 1, 4])
def test_steps_enqueued_without_waiting_survive_rejected_first_steps(case):
    """lbfgsb_step(info = NULL) uses the short launch sequence of the logistic objective, which has no launches for a
    rejected first trial step: the solver parks itself, later steps return at once, and the library finishes the
    iteration and redoes the skipped steps when it next looks at the device state (here: in x()).  Sixteen such calls
    must leave exactly the state sixteen synchronous calls leave, on problems that backtrack in the first iteration
    (case 0: fourteen halvings) and several times later."""
    prob = _logistic(LOGISTIC_CASES[case], np.float64)
    a = L.solver_for_problem(prob, DEV, tol=0.0, a_pass=L.APASS_FUSED)
    b = L.solver_for_problem(prob, DEV, tol=0.0, a_pass=L.APASS_FUSED)
    for _ in range(16):
        a.step(want_info=False)
        b.step()
    xa, xb = a.x(), b.x()                       # (x() brings a parked solver up to date first)
    ia, ib = a.info(), b.info()
    assert ia.iters == ib.iters == 16 and ia.status == ib.status == L.RUNNING
    assert torch.equal(xa, xb) and torch.equal(a.g(), b.g())
    # f is a reported scalar that no decision reads (the Armijo test uses the difference): the short sequence carries it
    # as f + [f(x + a p) - f(x)], the full one evaluates it from the new margins, and which iterations run which
    # sequence differs between the two ways of stepping -- equal to rounding, not bit for bit
    assert ia.f == pytest.approx(ib.f, rel=1e-14) and ia.fevals == ib.fevals
    # and lbfgsb_solve from here on agrees too
    a2, b2 = a.solve(), b.solve()
    assert (a2.status, a2.iters) == (b2.status, b2.iters) and torch.equal(a.x(), b.x())
    a.close(); b.close()


def test_a_very_tall_matrix_takes_the_full_logistic_sequence():
    """The short launch sequence keeps two numbers per row of a workgroup in LDS; with more than about ten thousand
    rows per workgroup (here 5.3 million rows of 8 columns: 512 workgroups) they do not fit, and the library has to
    fall back to the full sequence instead of asking for more LDS than a workgroup can have.  Steps enqueued without
    waiting, steps with an info struct and the oracle must agree."""
    prob = workloads.logistic(rows=5_300_000, cols=8, seed=11, dtype=np.float32, label_noise=0.5, mu=1e-3, bound=0.5, m=5)
    a = L.solver_for_problem(prob, DEV, tol=0.0, a_pass=L.APASS_FUSED)
    b = L.solver_for_problem(prob, DEV, tol=0.0, a_pass=L.APASS_FUSED)
    assert a.apass_name == "fused"
    for _ in range(4):
        a.step(want_info=False)
        b.step()
    ia, ib = a.info(), b.info()
    assert ia.iters == ib.iters == 4 and ia.status == ib.status == L.RUNNING
    assert torch.equal(a.x(), b.x()) and torch.equal(a.g(), b.g())
    orc = _oracle_solver(prob, tol=0.0)
    for _ in range(4):
        orc.step()
    assert rel_err(a.x().cpu().numpy(), orc.x) <= 1e-6
    assert ia.f == pytest.approx(orc.info.f, rel=1e-6)
    orc.close(); a.close(); b.close()


# ---- exhausted searches ---------------------------------------------------------------------------------------------

def _hand_solver(a_diag, b, max_backtracks, a_pass):
    A = np.diag([float(v) for v in a_diag])
    inf = np.full(2, np.inf)
    s = L.Solver(L.OBJ_LSQ, to_dev(A), to_dev(np.array([float(v) for v in b])), to_dev(-inf), to_dev(inf), 3,
                 options=L.default_options(max_backtracks=max_backtracks, tol=1e-12, a_pass=a_pass))
    s.set_x(to_dev(np.zeros(2)))
    return s


def _floats(v):
    return np.array([float(t) for t in v])


@pytest.mark.parametrize("a_pass", [L.APASS_AUTO, L.APASS_TWO_PASS], ids=["auto", "two_pass"])
@pytest.mark.parametrize("max_backtracks", [0, 1, 2])
def test_hand_worked_reset_with_accepted_retry(max_backtracks, a_pass):
    """A = diag(5/4, 1/8), b = (-1, -512), x0 = 0 (worked out in tests/test_oracle_linesearch_exhausted.py):
    iteration 1 accepts p = -g at alpha = 1; in iteration 2 the quasi-Newton direction fails at alpha = 1, 1/2, 1/4,
    the memory is cleared and the retry p = -g is accepted at alpha = 1.  All numbers are binary fractions, so the
    iterates are compared exactly."""
    s = _hand_solver([F(5, 4), F(1, 8)], [F(-1), F(-512)], max_backtracks, a_pass)
    i1 = s.step()
    assert (i1.iters, i1.backtracks, i1.alpha, i1.memory_resets) == (1, 0, 1.0, 0)
    np.testing.assert_array_equal(s.x().cpu().numpy(), [-1.25, -64.0])
    np.testing.assert_array_equal(s.g().cpu().numpy(), _floats([F(-45, 64), F(63)]))
    i2 = s.step()                                               # exhausted: memory cleared, nothing moved
    assert (i2.status, i2.iters, i2.memory_resets) == (L.RUNNING, 1, 1), i2.as_dict()
    assert i2.backtracks == max_backtracks + 1
    np.testing.assert_array_equal(s.x().cpu().numpy(), [-1.25, -64.0])
    np.testing.assert_array_equal(s.g().cpu().numpy(), _floats([F(-45, 64), F(63)]))
    i3 = s.step()                                               # the retry
    assert (i3.status, i3.iters, i3.memory_resets, i3.backtracks, i3.alpha, i3.pairs_used) == (L.RUNNING, 2, 1, 0, 1.0, 0)
    assert i3.gp == float(-(F(45, 64) ** 2 + F(63) ** 2))
    np.testing.assert_array_equal(s.x().cpu().numpy(), _floats([F(-35, 64), F(-127)]))
    # one pair is stored again: the next direction uses it
    i4 = s.step()
    assert i4.pairs_used == 1 or i4.memory_resets == 2, i4.as_dict()
    s.close()


@pytest.mark.parametrize("a_pass", [L.APASS_AUTO, L.APASS_TWO_PASS], ids=["auto", "two_pass"])
def test_hand_worked_quasi_newton_step_when_backtracks_suffice(a_pass):
    """Same data with 3 backtracks allowed: the quasi-Newton direction (2025062713485/1341737956,
    -2340977197248/335434489) is accepted at alpha = 1/8, no reset."""
    d = [F(2025062713485, 1341737956), F(-2340977197248, 335434489)]
    s = _hand_solver([F(5, 4), F(1, 8)], [F(-1), F(-512)], 3, a_pass)
    s.step()
    info = s.step()
    assert (info.memory_resets, info.backtracks, info.alpha, info.pairs_used, info.iters) == (0, 3, 0.125, 1, 2)
    np.testing.assert_allclose(s.x().cpu().numpy(), _floats([F(-5, 4) + d[0] / 8, F(-64) + d[1] / 8]), rtol=1e-13)
    assert info.gp == pytest.approx(float(F(-45, 64) * d[0] + F(63) * d[1]), rel=1e-13)
    s.close()


@pytest.mark.parametrize("a_pass", [L.APASS_AUTO, L.APASS_TWO_PASS], ids=["auto", "two_pass"])
@pytest.mark.parametrize("through", ["step", "solve"])
def test_hand_worked_double_exhaustion_fails(through, a_pass):
    """A = diag(2, 1), b = (-1/8, -4), max_backtracks = 0: iteration 1 accepted, in iteration 2 the quasi-Newton
    direction and then the steepest-descent retry both raise f at alpha = 1 -> LINESEARCH_FAILED at x^1 = (-1/4, -4)."""
    s = _hand_solver([F(2), F(1)], [F(-1, 8), F(-4)], 0, a_pass)
    if through == "step":
        assert s.step().iters == 1
        i2 = s.step()
        assert (i2.status, i2.memory_resets, i2.iters) == (L.RUNNING, 1, 1)
        info = s.step()
        assert s.step().status == L.LINESEARCH_FAILED          # a stopped solver stays stopped
    else:
        info = s.solve()
    assert (info.status, info.memory_resets, info.iters) == (L.LINESEARCH_FAILED, 1, 1), info.as_dict()
    np.testing.assert_array_equal(s.x().cpu().numpy(), [-0.25, -4.0])
    np.testing.assert_array_equal(s.g().cpu().numpy(), [-0.75, 0.0])
    assert info.f == 9.0 / 128.0
    s.close()


@pytest.mark.parametrize("nb,expect", [(0, "fail"), (1, "fail"), (2, "accept")])
def test_hand_worked_empty_memory(nb, expect):
    """A = diag(2, 1), b = (-1/2, 0): f(x + alpha p) - f(x) = -alpha + 2 alpha^2 along p = -g = (-1, 0): rejected at
    alpha = 1 and 1/2, accepted at 1/4.  With no pair stored an exhausted search fails at once, no reset counted."""
    s = _hand_solver([F(2), F(1)], [F(-1, 2), F(0)], nb, L.APASS_AUTO)
    info = s.solve() if expect == "fail" else s.step()
    if expect == "fail":
        assert (info.status, info.memory_resets, info.iters) == (L.LINESEARCH_FAILED, 0, 0), info.as_dict()
        np.testing.assert_array_equal(s.x().cpu().numpy(), [0.0, 0.0])
    else:
        assert (info.status, info.backtracks, info.alpha, info.iters) == (L.RUNNING, 2, 0.25, 1)
        np.testing.assert_array_equal(s.x().cpu().numpy(), [-0.25, 0.0])
    s.close()


@pytest.mark.parametrize("a_pass", A_PASSES, ids=A_PASS_IDS)
@pytest.mark.parametrize("sigma_max,expect", [(1.3, "resets"), (1.6, "fails"), (2.5, "fails_at_once")])
def test_quadratic_exhaustion_follows_the_oracle(sigma_max, expect, a_pass):
    """400 x 300 least squares with singular values in [0.03, sigma_max] and max_backtracks = 0 (only the unit step
    is tried): several resets with accepted retries; resets and then a failed retry; failure in the first iteration."""
    prob = workloads.spectrum_lsq(400, 300, seed=0, sigma_min=0.03, sigma_max=sigma_max)
    orc = _oracle_solver(prob, tol=1e-9, max_backtracks=0)
    s = L.solver_for_problem(prob, DEV, tol=1e-9, max_backtracks=0, a_pass=a_pass)
    _follow(orc, s, 30, 1e-9, f"spectrum {sigma_max}")
    oi = orc.info
    if expect == "resets":
        assert oi.status == oracle.RUNNING and oi.memory_resets >= 2 and oi.iters == 30
    elif expect == "fails":
        assert oi.status == oracle.LINESEARCH_FAILED and oi.memory_resets >= 1 and oi.iters >= 2
    else:
        assert (oi.status, oi.memory_resets, oi.iters) == (oracle.LINESEARCH_FAILED, 0, 0)
    assert s.info().status == oi.status
    orc.close(); s.close()


@pytest.mark.parametrize("a_pass", A_PASSES, ids=A_PASS_IDS)
def test_quadratic_solve_reports_the_failure(a_pass):
    """lbfgsb_solve (not stepping by hand) through the resets to the failure: same final state as the oracle's solve."""
    prob = workloads.spectrum_lsq(400, 300, seed=0, sigma_min=0.03, sigma_max=1.6)
    ref = oracle.solve_problem(prob, tol=1e-9, max_backtracks=0)
    assert ref.info.status == oracle.LINESEARCH_FAILED and ref.info.memory_resets >= 1
    s = L.solver_for_problem(prob, DEV, tol=1e-9, max_backtracks=0, a_pass=a_pass)
    info = s.solve()
    assert (info.status, info.iters, info.memory_resets) == (L.LINESEARCH_FAILED, ref.info.iters, ref.info.memory_resets)
    assert rel_err(s.x().cpu().numpy(), ref.x) <= 1e-9
    assert info.f == pytest.approx(ref.info.f, rel=1e-9)
    s.close()


@pytest.mark.parametrize("a_pass", A_PASSES, ids=A_PASS_IDS)
@pytest.mark.parametrize("dtype", [np.float64, np.float32], ids=["f64", "f32"])
@pytest.mark.parametrize("case,expect", [(1, "resets"), (3, "resets"), (4, "fails"), (0, "fails_at_once"), (2, "fails_at_once")])
def test_logistic_exhaustion_follows_the_oracle(case, expect, dtype, a_pass):
    """The badly scaled logistic problems with max_backtracks = 0."""
    prob = _logistic(LOGISTIC_CASES[case], dtype)
    orc = _oracle_solver(prob, tol=1e-9, max_backtracks=0)
    s = L.solver_for_problem(prob, DEV, tol=1e-9, max_backtracks=0, a_pass=a_pass)
    # 16 iterations: all but one of the resets of these cases fall into the first ten, and on these badly conditioned
    # problems the two trajectories drift apart by a factor of ~3 per iteration from rounding-level differences
    _follow(orc, s, 16, 1e-8 if dtype == np.float64 else 1e-6, f"logistic case {case}, no backtracking allowed")
    oi = orc.info
    if expect == "resets":
        assert oi.status == oracle.RUNNING and oi.memory_resets >= 3 and oi.iters == 16
    elif expect == "fails":
        assert oi.status == oracle.LINESEARCH_FAILED and oi.memory_resets >= 1 and oi.iters >= 1
    else:
        assert (oi.status, oi.memory_resets, oi.iters) == (oracle.LINESEARCH_FAILED, 0, 0)
    assert s.info().status == oi.status
    # lbfgsb_solve from the start reaches the same end
    if expect != "resets":
        t = L.solver_for_problem(prob, DEV, tol=1e-9, max_backtracks=0, a_pass=a_pass)
        info = t.solve()
        assert (info.status, info.iters, info.memory_resets) == (oi.status, oi.iters, oi.memory_resets)
        assert torch.equal(t.x(), s.x())
        t.close()
    orc.close(); s.close()


def _entropy_problem(rows, cols, seed, lam, width, with_marginals):
    rng = np.random.default_rng(seed)
    M = rng.standard_normal((rows, cols))
    n = rows * cols
    lo = 0.05 + 0.2 * rng.random(n)
    hi = lo + width * (0.1 + rng.random(n))
    u, v = rng.random(rows) + 0.1, rng.random(cols) + 0.1
    mult = 0.01 * rng.standard_normal(rows + cols)
    return M, lo, hi, (u * cols * 0.3, v * rows * 0.3, mult, 0.01) if with_marginals else None


@pytest.mark.parametrize("rows,cols,seed,lam,width,marg,expect", [
    (64, 310, 10, 0.05, 1.0, False, "resets"),
    (300, 37, 4, 0.05, 0.1, False, "resets_then_converges"),
    (64, 310, 10, 0.5, 0.1, False, "fails"),
    (64, 310, 10, 0.5, 0.1, True, "fails"),
])
def test_entropy_exhaustion_follows_the_oracle(rows, cols, seed, lam, width, marg, expect):
    """The transport objective with the entropy regulariser over a box that differs from entry to entry (narrow
    boxes keep the projected steepest-descent step short enough for a unit step), max_backtracks = 0."""
    M, lo, hi, con = _entropy_problem(rows, cols, seed, lam, width, marg)
    n = rows * cols
    ref_obj = oracle.Objective(oracle.OT_ENTROPY, M, lam=lam)
    beta = omega = None
    if con is not None:
        u, v, mult, rho = con
        ref_obj.set_marginals(u, v, lam=mult, rho=rho)
        beta, omega = np.concatenate([u, v]) - mult / rho, np.full(rows + cols, rho)
    orc = oracle.Solver(ref_obj, lo, hi, lo.copy(), 5, oracle.default_options(tol=1e-9, max_backtracks=0))
    s = L.Solver(L.OBJ_OT_ENTROPY, to_dev(M), to_dev(beta) if beta is not None else None, to_dev(lo), to_dev(hi), 5,
                 lam=lam, options=L.default_options(tol=1e-9, max_backtracks=0),
                 row_weight=to_dev(omega) if omega is not None else None)
    s.set_x(to_dev(lo))
    _follow(orc, s, 40, 1e-8, f"entropy {rows}x{cols}")
    oi = orc.info
    if expect == "resets":
        assert oi.status == oracle.RUNNING and oi.memory_resets >= 2
    elif expect == "resets_then_converges":
        assert oi.status == oracle.CONVERGED and oi.memory_resets >= 1
    else:
        assert oi.status == oracle.LINESEARCH_FAILED and oi.memory_resets >= 1 and oi.iters >= 2
    assert s.info().status == oi.status
    orc.close(); s.close()
