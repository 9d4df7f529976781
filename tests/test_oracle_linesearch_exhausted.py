"""Pins for the oracle's handling of an EXHAUSTED line search.

The paper's section "Algorithm" asks for a backtracking search that satisfies the Armijo condition and
says nothing about a search that runs out of trial steps.  The reading taken (both implementations):
clear the pair memory and redo the iteration once from the steepest-descent direction on the free set;
if that search is exhausted too, stop with the status LINESEARCH_FAILED.

Each case is a 2-variable least-squares problem with a diagonal matrix, no bounds and x^0 = 0, small enough
to work by hand.  The expected numbers are written out as exact fractions below; the quasi-Newton
direction is re-derived in the test from the DENSE inverse BFGS matrix in rational arithmetic (a textbook
construction that shares nothing with the oracle's two-loop recursion), and every Armijo decision is
re-taken in rational arithmetic, so a mistake in the oracle's retry logic (memory not cleared, retry not
taken or taken twice, wrong status, iterate moved by a failed search) fails a comparison with numbers that
do not come from the oracle.
"""
from fractions import Fraction as F

import numpy as np
import pytest

import oracle

C1 = F(1, 10000)          # Armijo constant (the default 1e-4 is not a binary fraction; the decisions below have wide margins)


def _armijo(h, g, p, alpha):
    """f(x + alpha p) - f(x) <= c1 alpha <g,p> for f with Hessian diag(h), in exact arithmetic"""
    gp = g[0] * p[0] + g[1] * p[1]
    df = alpha * gp + alpha * alpha * (h[0] * p[0] * p[0] + h[1] * p[1] * p[1]) / 2
    return df <= C1 * alpha * gp


def _dense_bfgs_direction(s, y, g):
    """-H g with H the inverse BFGS update of (s.y / y.y) I by the pair (s, y), formed as a dense 2 x 2 matrix"""
    sy = s[0] * y[0] + s[1] * y[1]
    gamma = sy / (y[0] * y[0] + y[1] * y[1])
    rho = 1 / sy
    eye = [[F(1), F(0)], [F(0), F(1)]]
    V = [[eye[i][j] - rho * y[i] * s[j] for j in range(2)] for i in range(2)]          # I - rho y s^T
    H = [[sum(V[k][i] * gamma * V[k][j] for k in range(2)) + rho * s[i] * s[j] for j in range(2)] for i in range(2)]
    return [-(H[i][0] * g[0] + H[i][1] * g[1]) for i in range(2)]


def _solver(a_diag, b, max_backtracks, m=3):
    A = np.diag([float(v) for v in a_diag])
    obj = oracle.Objective(oracle.LSQ, A, np.array([float(v) for v in b]))
    opts = oracle.default_options(max_backtracks=max_backtracks, tol=1e-12)
    return oracle.Solver(obj, [-np.inf, -np.inf], [np.inf, np.inf], [0.0, 0.0], m=m, options=opts)


def _floats(v):
    return np.array([float(t) for t in v])


@pytest.mark.parametrize("max_backtracks", [0, 1, 2])
def test_exhausted_search_clears_the_memory_and_the_retry_succeeds(max_backtracks):
    """A = diag(5/4, 1/8), b = (-1, -512): Hessian diag(25/16, 1/64), g^0 = -A^T b = (5/4, 64).
    Iteration 1 (no pair): p = -g^0, alpha = 1 is accepted (every eigenvalue of the Hessian is below 2(1 - c1)):
      x^1 = (-5/4, -64), g^1 = (I - H) g^0 = (-45/64, 63), pair s = -g^0, y = H s = (-125/64, -1).
    Iteration 2: y is dominated by its second entry, so the scaling s.y / y.y is about 60 and the quasi-Newton
      direction overshoots along the first (stiff) coordinate: d ~ (1509, -6979), <g,d> ~ -4.4e5, d.Hd ~ 4.3e6, so
      alpha = 1, 1/2 and 1/4 all INCREASE f (the first acceptable one is 1/8).  With at most 0, 1 or 2 backtracks
      the search is exhausted -> memory cleared -> retry with
      p = -g^1, alpha = 1 accepted -> x^2 = x^1 - g^1 = (-35/64, -127), and the new pair is the only one stored."""
    h = [F(25, 16), F(1, 64)]
    g0 = [F(5, 4), F(64)]
    x1 = [-g0[0], -g0[1]]
    g1 = [(1 - h[0]) * g0[0], (1 - h[1]) * g0[1]]
    assert g1 == [F(-45, 64), F(63)]
    s, y = x1, [h[0] * x1[0], h[1] * x1[1]]
    d = _dense_bfgs_direction(s, y, g1)
    assert d == [F(2025062713485, 1341737956), F(-2340977197248, 335434489)]
    # the decisions, in exact arithmetic
    assert _armijo(h, g0, [-g0[0], -g0[1]], F(1))
    assert not _armijo(h, g1, d, F(1)) and not _armijo(h, g1, d, F(1, 2)) and not _armijo(h, g1, d, F(1, 4))
    assert _armijo(h, g1, d, F(1, 8))
    assert _armijo(h, g1, [-g1[0], -g1[1]], F(1))

    sol = _solver([F(5, 4), F(1, 8)], [F(-1), F(-512)], max_backtracks)
    assert sol.step() == oracle.RUNNING
    i1 = sol.info
    assert (i1.iters, i1.backtracks, i1.alpha, i1.memory_resets, i1.pairs_used) == (1, 0, 1.0, 0, 0)
    np.testing.assert_array_equal(sol.x, _floats(x1))
    np.testing.assert_array_equal(sol.g, _floats(g1))
    assert sol.step() == oracle.RUNNING
    i2 = sol.info
    assert i2.memory_resets == 1 and i2.iters == 2
    assert (i2.backtracks, i2.alpha, i2.pairs_used) == (0, 1.0, 0)            # the accepted search is the retry's
    assert i2.gp == float(-(g1[0] ** 2 + g1[1] ** 2))                           # <g, p> of the steepest-descent retry
    np.testing.assert_array_equal(sol.x, _floats([F(-35, 64), F(-127)]))
    np.testing.assert_array_equal(sol.d, _floats([-g1[0], -g1[1]]))            # the direction of the retry: -g on S
    assert sol.npairs == 1                                                     # old pair gone, new pair stored
    np.testing.assert_array_equal(sol.S[0], _floats([-g1[0], -g1[1]]))
    np.testing.assert_array_equal(sol.Y[0], _floats([-h[0] * g1[0], -h[1] * g1[1]]))
    # trial evaluations: x^0, 1 trial + 1 gradient, then (max_backtracks + 1) rejected trials, 1 trial + 1 gradient
    assert i2.fevals == 1 + 2 + (max_backtracks + 1) + 2
    sol.close()


def test_with_enough_backtracks_the_same_problem_needs_no_reset():
    """Same data, 3 backtracks allowed: the quasi-Newton direction is accepted at alpha = 1/8 (the exact
    decisions are asserted in the test above) and the memory is kept."""
    h = [F(25, 16), F(1, 64)]
    g1 = [F(-45, 64), F(63)]
    x1 = [F(-5, 4), F(-64)]
    d = [F(2025062713485, 1341737956), F(-2340977197248, 335434489)]
    sol = _solver([F(5, 4), F(1, 8)], [F(-1), F(-512)], 3)
    sol.step()
    assert sol.step() == oracle.RUNNING
    info = sol.info
    assert (info.memory_resets, info.backtracks, info.alpha, info.pairs_used, info.iters) == (0, 3, 0.125, 1, 2)
    np.testing.assert_allclose(sol.d, _floats(d), rtol=1e-14)
    np.testing.assert_allclose(sol.x, _floats([x1[0] + d[0] / 8, x1[1] + d[1] / 8]), rtol=1e-14)
    assert info.gp == pytest.approx(float(g1[0] * d[0] + g1[1] * d[1]), rel=1e-14)
    assert sol.npairs == 2
    sol.close()


def test_exhausted_twice_stops_with_linesearch_failed():
    """A = diag(2, 1), b = (-1/8, -4): Hessian diag(4, 1), g^0 = (1/4, 4).
    Iteration 1 (no pair): p = -g^0, <g,p> = -257/16, ||A p||^2 = 65/4: f(x + p) - f(x) = -257/16 + 65/8 = -127/16,
      accepted at alpha = 1.  x^1 = (-1/4, -4), g^1 = (I - H) g^0 = (-3/4, 0), pair s = (-1/4, -4), y = (-1, -4).
    Iteration 2, max_backtracks = 0:
      two-loop by hand: s.y = 65/4, y.y = 17; alpha_1 = s.g/s.y = 3/260; q = g - alpha_1 y = (-48/65, 3/65);
      scaled by 65/68: (-12/17, 3/68); beta = y.q/s.y = 36/1105; q += (3/260 - 36/1105) s
      -> d = -q = (12387/17680, -567/4420);  <g,d> = -37161/70720, d.Hd > 1.9: f rises at alpha = 1 -> exhausted
      -> memory cleared, retry p = -g^1 = (3/4, 0): <g,p> = -9/16, ||A p||^2 = 9/4, change of f = -9/16 + 9/8 = 9/16 > 0
      -> exhausted again with nothing left to clear -> LINESEARCH_FAILED; the iterate has not moved."""
    h = [F(4), F(1)]
    g0 = [F(1, 4), F(4)]
    x1 = [F(-1, 4), F(-4)]
    g1 = [F(-3, 4), F(0)]
    s, y = x1, [F(-1), F(-4)]
    d = _dense_bfgs_direction(s, y, g1)
    assert d == [F(12387, 17680), F(-567, 4420)]
    assert _armijo(h, g0, [-g0[0], -g0[1]], F(1))
    assert not _armijo(h, g1, d, F(1))
    assert not _armijo(h, g1, [-g1[0], -g1[1]], F(1))

    sol = _solver([F(2), F(1)], [F(-1, 8), F(-4)], 0)
    assert sol.step() == oracle.RUNNING
    np.testing.assert_array_equal(sol.x, _floats(x1))
    np.testing.assert_array_equal(sol.g, _floats(g1))
    f1 = sol.info.f
    assert f1 == 9.0 / 128.0
    assert sol.step() == oracle.LINESEARCH_FAILED
    info = sol.info
    assert info.status == oracle.LINESEARCH_FAILED
    assert info.memory_resets == 1 and info.iters == 1 and sol.npairs == 0
    np.testing.assert_array_equal(sol.x, _floats(x1))                          # a failed search moves nothing
    np.testing.assert_array_equal(sol.g, _floats(g1))
    assert info.f == f1
    np.testing.assert_array_equal(sol.d, _floats([-g1[0], -g1[1]]))            # the last direction tried: the retry's
    # a stopped solver stays stopped
    assert sol.step() == oracle.LINESEARCH_FAILED and sol.info.iters == 1
    sol.close()
    # the quasi-Newton direction itself, from a solver that is allowed to backtrack
    sol = _solver([F(2), F(1)], [F(-1, 8), F(-4)], 60)
    sol.step()
    sol.step()
    np.testing.assert_allclose(sol.d, _floats(d), rtol=1e-15)
    assert sol.info.memory_resets == 0
    sol.close()


def test_exhausted_with_an_empty_memory_fails_at_once():
    """A = diag(2, 1), b = (-1/2, 0): g^0 = (1, 0), p = (-1, 0), <g,p> = -1, ||A p||^2 = 4.
    f(x + alpha p) - f(x) = -alpha + 2 alpha^2: +1 at alpha = 1, 0 at 1/2 (not <= -c1/2), -1/8 at 1/4 (accepted).
    With fewer than 2 backtracks and no pair stored there is nothing to clear: LINESEARCH_FAILED, no reset counted."""
    for nb in (0, 1):
        sol = _solver([F(2), F(1)], [F(-1, 2), F(0)], nb)
        assert sol.step() == oracle.LINESEARCH_FAILED
        info = sol.info
        assert (info.memory_resets, info.iters, sol.npairs) == (0, 0, 0)
        np.testing.assert_array_equal(sol.x, [0.0, 0.0])
        assert info.fevals == 1 + (nb + 1)
        sol.close()
    sol = _solver([F(2), F(1)], [F(-1, 2), F(0)], 2)
    assert sol.step() == oracle.RUNNING
    info = sol.info
    assert (info.backtracks, info.alpha, info.iters) == (2, 0.25, 1)
    np.testing.assert_array_equal(sol.x, [-0.25, 0.0])
    assert info.f == 0.0                                                       # A x = b there
    sol.close()
