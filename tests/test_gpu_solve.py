"""End-to-end parity of the HIP solver with the CPU oracle on the benchmark configurations.

The two do not follow the same trajectory (reduction order and the Armijo test at the margin
differ), so what is compared is what the method fixes: the final objective value (1e-8 relative
for fp64-stored matrices, 1e-4 for fp32-stored ones), the final active set on the
well-conditioned configurations, and the KKT conditions recomputed on the host with numpy.  The
first iterations, where nothing is marginal yet, are compared step by step.
"""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2203_16340_amd as L
import workloads
from gpu_helpers import DEV, active_set, host_gradient, host_objective, kkt_residual, make_solver, rel_err, to_dev

pytestmark = pytest.mark.gpu

A_PASSES = [pytest.param(L.APASS_TWO_PASS, id="two_pass"), pytest.param(L.APASS_FUSED, id="fused")]


def _gpu_solver(prob, a_pass, **opts):
    try:
        return L.solver_for_problem(prob, DEV, a_pass=a_pass, **opts)
    except L.LbfgsbError as e:
        if e.code == L.E_UNSUPPORTED:
            pytest.skip("shape/objective not supported by the fused A pass")
        raise


def _compare_with_oracle(prob, a_pass, f_tol, same_active_set, kkt_tol, **opts):
    ref = oracle.solve_problem(prob)
    assert ref.info.status == oracle.CONVERGED
    s = _gpu_solver(prob, a_pass, **opts)
    info = s.solve()
    x = s.x().cpu().numpy()
    assert info.status == L.CONVERGED, info.as_dict()
    assert abs(info.f - ref.info.f) <= f_tol * abs(ref.info.f), (info.f, ref.info.f)
    # the reported f is the objective at the returned x
    assert info.f == pytest.approx(host_objective(prob, x), rel=1e-9)
    res, g = kkt_residual(prob, x)
    assert res <= kkt_tol, res
    # the solver's own stopping quantity agrees with the host's recomputation
    mask = oracle.free_mask(x, g, prob.l, prob.u, 1e-10).astype(bool)
    assert np.linalg.norm(g[mask]) <= 1.5 * max(info.pg2, 1e-300) + 1e-9 * np.linalg.norm(g)
    if same_active_set:
        assert np.array_equal(active_set(prob, x), active_set(prob, ref.x))
    # iteration counts are of the same order (soft: trajectories differ)
    assert info.iters <= 2 * ref.info.iters + 20
    s.close()
    return info, ref


@pytest.mark.parametrize("a_pass", A_PASSES)
def test_c1_full_size(a_pass):
    prob = workloads.config("C1")                         # NNLS 200 x 100 fp64, m = 5, tol 1e-8 absolute
    info, ref = _compare_with_oracle(prob, a_pass, 1e-8, True, 1e-8)
    assert info.pg2 <= 1e-8


@pytest.mark.parametrize("a_pass", A_PASSES)
@pytest.mark.parametrize("name,scale,f_tol,same_set", [
    ("C2", 0.1, 1e-8, True),      # 2000 x 500 fp64
    ("C3", 0.05, 1e-8, False),    # 500 x 1000 -> 2000 variables (not strictly convex: active sets may differ)
    ("C4", 0.02, 1e-4, False),    # 4000 x 40 fp32 logistic
    ("C5", 0.02, 1e-4, True),     # 2000 x 400 fp32, box [0, 1]
])
def test_scaled_configs(name, scale, f_tol, same_set, a_pass):
    prob = workloads.config(name, scale=scale)
    prob.tol, prob.tol_relative = 1e-9, True              # tight enough that f agrees to the stated bound
    g0 = host_gradient(prob, prob.x0)
    mask0 = oracle.free_mask(prob.x0, g0, prob.l, prob.u, 1e-10).astype(bool)
    _compare_with_oracle(prob, a_pass, f_tol, same_set, 1e-8 * max(1.0, np.linalg.norm(g0[mask0])))


@pytest.mark.parametrize("name,scale,same_set", [
    ("P1", 0.05, False),   # the paper's NNLS experiment (i): 145 x 435, U(0,1) entries, singular Gram matrix (minimiser not unique)
    ("P2", 0.02, True),    # the paper's NNLS experiment (ii): 592 x 296 Gaussian
])
def test_the_papers_nnls_recipes_scaled_down(name, scale, same_set):
    prob = workloads.config(name, scale=scale)
    prob.tol, prob.tol_relative = 1e-9, True
    g0 = host_gradient(prob, prob.x0)
    mask0 = oracle.free_mask(prob.x0, g0, prob.l, prob.u, 1e-10).astype(bool)
    _compare_with_oracle(prob, L.APASS_AUTO, 1e-8, same_set, 1e-8 * max(1.0, np.linalg.norm(g0[mask0])))


@pytest.mark.parametrize("a_pass", A_PASSES)
@pytest.mark.parametrize("name,scale", [("C1", 1.0), ("C2", 0.05), ("C3", 0.03), ("C4", 0.01), ("C5", 0.02)])
def test_first_iterations_match_step_by_step(name, scale, a_pass):
    """Iterations 1-3 from x0 = 0: same branch, same number of backtracks, same step length, and the
    iterate within rounding."""
    prob = workloads.config(name, scale=scale)
    obj = oracle.Objective(prob.kind, prob.A, prob.b, prob.lam, prob.mu)
    orc = oracle.Solver(obj, prob.l, prob.u, prob.x0, prob.m, oracle.default_options(tol=0.0))
    s = _gpu_solver(prob, a_pass, tol=0.0)
    tol = 1e-10 if prob.A.dtype == np.float64 else 1e-6
    for k in range(3):
        assert orc.step() == oracle.RUNNING
        info = s.step()
        oi = orc.info
        assert info.status == L.RUNNING and info.iters == k + 1
        assert (info.branch, info.backtracks, info.pairs_used) == (oi.branch, oi.backtracks, oi.pairs_used)
        assert info.alpha == pytest.approx(oi.alpha, rel=1e-12)
        assert info.gp == pytest.approx(oi.gp, rel=tol)
        assert info.f == pytest.approx(oi.f, rel=tol)
        assert rel_err(s.x().cpu().numpy(), orc.x) <= tol
        assert rel_err(s.g().cpu().numpy(), orc.g) <= tol * 10
    orc.close(); s.close()


def _width_case(case):
    kind, dtype, rows, cols = case
    if kind == "nnls":
        return workloads.nnls(rows, cols, seed=900 + cols, dtype=dtype, zero_frac=0.6, nonzero="uniform", m=6)
    if kind == "l1":
        return workloads.l1_split(rows, cols, seed=900 + cols, m=6)
    return workloads.logistic(rows, cols, seed=900 + cols, dtype=dtype, mu=1e-3, bound=0.5, m=6)


@pytest.mark.parametrize("case", [
    # widths between the tuned configurations: each takes a variant of the single-read pass of its own
    ("nnls", np.float64, 2300, 1500),      # fp64, 1025..2048 columns: 512-thread workgroups, two chunks per thread
    ("l1", np.float64, 900, 1800),         # the same variant with v = p - q
    ("nnls", np.float32, 1500, 300),       # fp32 up to 512 columns: 128-thread workgroups
    ("nnls", np.float32, 2500, 1800),      # fp32, 1025..2048 columns
    ("logistic", np.float64, 2500, 1200),  # logistic, fp64, 1025..2048 columns
    ("logistic", np.float32, 3000, 400),   # logistic, fp32 up to 512 columns
    ("logistic", np.float32, 3000, 900),   # logistic, fp32 up to 1024 columns
], ids=lambda c: f"{c[0]}-{np.dtype(c[1]).name}-{c[2]}x{c[3]}")
def test_first_iterations_on_the_widths_between_the_tuned_ones(case):
    """Iterations 1-4 against the oracle on the single-read pass (direction passes, deferred choice of Algorithm 2's
    branch, the short logistic sequence), each width on the pass's variant for it."""
    prob = _width_case(case)
    obj = oracle.Objective(prob.kind, prob.A, prob.b, prob.lam, prob.mu)
    orc = oracle.Solver(obj, prob.l, prob.u, prob.x0, prob.m, oracle.default_options(tol=0.0))
    s = _gpu_solver(prob, L.APASS_FUSED, tol=0.0)
    assert s.apass_name == "fused"
    tol = 1e-10 if prob.A.dtype == np.float64 else 1e-6
    for k in range(4):
        assert orc.step() == oracle.RUNNING
        info = s.step()
        oi = orc.info
        assert info.status == L.RUNNING and info.iters == k + 1
        assert (info.branch, info.backtracks, info.pairs_used) == (oi.branch, oi.backtracks, oi.pairs_used)
        assert info.alpha == pytest.approx(oi.alpha, rel=1e-12)
        assert info.gp == pytest.approx(oi.gp, rel=tol)
        assert info.f == pytest.approx(oi.f, rel=tol)
        assert rel_err(s.x().cpu().numpy(), orc.x) <= tol
        assert rel_err(s.g().cpu().numpy(), orc.g) <= tol * 10
    orc.close(); s.close()


@pytest.mark.parametrize("name,scale,a_pass", [("C1", 1.0, L.APASS_AUTO), ("C2", 0.05, L.APASS_FUSED), ("C2", 0.05, L.APASS_TWO_PASS),
                                               ("C3", 0.03, L.APASS_AUTO), ("C4", 0.01, L.APASS_FUSED), ("C4", 0.01, L.APASS_TWO_PASS)])
def test_history_ring_holds_what_each_step_reported(name, scale, a_pass):
    """The per-iteration records kept on the device while steps are enqueued without waiting equal what synchronous
    steps report one by one (and, for the first iterations, what the oracle did)."""
    prob = workloads.config(name, scale=scale)
    a = _gpu_solver(prob, a_pass, tol=0.0)
    b = _gpu_solver(prob, a_pass, tol=0.0)
    infos = [a.step() for _ in range(12)]
    for _ in range(12):
        b.step(want_info=False)
    hist = b.history()
    assert [r.iter for r in hist] == list(range(1, 13))
    for r, i in zip(hist, infos):
        assert (r.f, r.alpha, r.alpha_ub, r.gp, r.pg2, r.pginf) == (i.f, i.alpha, i.alpha_ub, i.gp, i.pg2, i.pginf)
        assert (r.branch, r.backtracks, r.pairs_used, r.n_fixed, r.memory_resets) == \
            (i.branch, i.backtracks, i.pairs_used, i.n_fixed, i.memory_resets)
    assert len(b.history(capacity=5)) == 5 and b.history(capacity=5)[-1].iter == 12 and b.history(capacity=5)[0].iter == 8
    orc = oracle.Solver(oracle.Objective(prob.kind, prob.A, prob.b, prob.lam, prob.mu), prob.l, prob.u, prob.x0, prob.m,
                        oracle.default_options(tol=0.0))
    for r in hist[:3]:
        orc.step()
        oi = orc.info
        assert (r.branch, r.backtracks, r.pairs_used, r.n_fixed) == (oi.branch, oi.backtracks, oi.pairs_used, oi.n_fixed)
        assert r.alpha == pytest.approx(oi.alpha, rel=1e-12) and r.f == pytest.approx(oi.f, rel=1e-6)
    b.set_x(torch.from_numpy(prob.x0).to(DEV))
    assert b.history() == []                        # lbfgsb_set_x clears the ring
    orc.close(); a.close(); b.close()


def test_history_ring_keeps_the_most_recent_records():
    prob = workloads.config("C2", scale=0.05)
    s = L.solver_for_problem(prob, DEV, tol=0.0, max_iter=300, a_pass=L.APASS_FUSED)
    info = s.solve()
    assert info.status == L.MAX_ITER and info.iters == 300
    hist = s.history()
    assert len(hist) == L.HISTORY_CAPACITY
    assert [r.iter for r in hist] == list(range(300 - L.HISTORY_CAPACITY + 1, 301))
    # (with tol = 0 the iteration runs on at the rounding floor, where the periodic recomputation of f moves its last digits)
    assert hist[-1].f == info.f and all(y.f <= x.f * (1 + 1e-12) for x, y in zip(hist, hist[1:]))
    s.close()


def test_iterates_stay_feasible_and_objective_decreases():
    prob = workloads.config("C5", scale=0.02)
    s = L.solver_for_problem(prob, DEV, tol=1e-10, tol_relative=1)
    f_prev = s.info().f
    for _ in range(40):
        info = s.step()
        if info.status != L.RUNNING:
            break
        x = s.x().cpu().numpy()
        assert np.all(x >= prob.l) and np.all(x <= prob.u)
        assert info.f <= f_prev
        assert info.gp < 0 and 0 < info.alpha <= min(1.0, info.alpha_ub)
        f_prev = info.f
    s.close()


def test_async_steps_equal_synchronous_steps():
    """lbfgsb_step(info = NULL) only enqueues; 12 of them give bit-identical state to 12 synchronised ones."""
    prob = workloads.config("C2", scale=0.05)
    a = L.solver_for_problem(prob, DEV, tol=0.0)
    b = L.solver_for_problem(prob, DEV, tol=0.0)
    for _ in range(12):
        a.step(want_info=False)
        b.step()
    assert torch.equal(a.x(), b.x()) and torch.equal(a.g(), b.g())
    assert a.info().f == b.info().f and a.info().iters == 12
    a.close(); b.close()


def test_solvers_on_their_own_streams_run_side_by_side():
    """Two solvers created on two non-default streams (default priority), their steps enqueued alternately without
    synchronising in between: each owns its workspace, scalar block and arrival counters, so both end bit-identical
    to the same problems solved one after the other on the default stream."""
    probs = [workloads.config("C2", scale=0.05), workloads.config("C4", scale=0.01)]
    ref = []
    for prob in probs:
        s = L.solver_for_problem(prob, DEV, tol=0.0)
        for _ in range(10):
            s.step(want_info=False)
        ref.append((s.x().clone(), s.info().f))
        s.close()
    streams = [torch.cuda.Stream(device=DEV), torch.cuda.Stream(device=DEV)]
    solvers = []
    for prob, st in zip(probs, streams):
        with torch.cuda.stream(st):
            solvers.append(L.solver_for_problem(prob, DEV, tol=0.0))
    for _ in range(10):
        for s, st in zip(solvers, streams):
            with torch.cuda.stream(st):
                s.step(want_info=False)
    for s, st, (x_ref, f_ref) in zip(solvers, streams, ref):
        with torch.cuda.stream(st):
            x, info = s.x().clone(), s.info()
        st.synchronize()
        assert info.iters == 10 and info.f == f_ref
        assert torch.equal(x, x_ref)
        s.close()


def test_steps_recorded_into_a_graph_replay_like_eager_steps():
    """lbfgsb_step(info = NULL) launches kernels only, so a run of steps can be recorded into a HIP graph.  Every
    replay (with eager work and a synchronisation in between) must leave exactly the state the same number of
    eager steps leaves.  refresh_every = 0: the periodic recomputation is scheduled by the host when a step is
    enqueued, and a recorded sequence would replay whatever pattern it was recorded with."""
    K, REPLAYS = 6, 3
    prob = workloads.config("C2", scale=0.05)
    st = torch.cuda.Stream(device=DEV)
    with torch.cuda.stream(st):
        x0 = torch.from_numpy(prob.x0).to(DEV)
        eager = L.solver_for_problem(prob, DEV, tol=0.0, refresh_every=0)
        rec = L.solver_for_problem(prob, DEV, tol=0.0, refresh_every=0)
        st.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=st):
            for _ in range(K):
                rec.step(want_info=False)
        rec.set_x(x0)                       # recording executes nothing: both start from x0
        for r in range(REPLAYS):
            graph.replay()
            for _ in range(K):
                eager.step(want_info=False)
            gi, ei = rec.info(), eager.info()                # synchronises
            assert gi.iters == ei.iters == K * (r + 1)
            assert gi.f == ei.f
            assert torch.equal(rec.x(), eager.x()) and torch.equal(rec.g(), eager.g())
            st.synchronize()
        eager.close(); rec.close()


def test_runs_are_bit_reproducible():
    prob = workloads.config("C3", scale=0.03)
    xs = []
    for _ in range(2):
        s = L.solver_for_problem(prob, DEV)
        s.solve()
        xs.append(s.x().clone())
        s.close()
    assert torch.equal(xs[0], xs[1])


def test_recurrence_refresh_keeps_residual_and_gradient_exact():
    """Least-squares kinds carry r and g by recurrence; with refresh_every = 4 and with no refresh at
    all the solver reaches the same optimum, and after a solve the carried gradient equals the
    gradient recomputed from x."""
    prob = workloads.config("C2", scale=0.05)
    prob.tol, prob.tol_relative = 1e-10, True
    outs = []
    for refresh in (4, 0, 32):
        s = L.solver_for_problem(prob, DEV, refresh_every=refresh)
        info = s.solve()
        assert info.status == L.CONVERGED
        x = s.x().cpu().numpy()
        g = s.g().cpu().numpy()
        assert rel_err(g, host_gradient(prob, x)) <= 1e-9 or np.linalg.norm(g - host_gradient(prob, x)) <= 1e-9 * np.linalg.norm(host_gradient(prob, prob.x0))
        outs.append((info.f, x))
        s.close()
    for f, x in outs[1:]:
        assert f == pytest.approx(outs[0][0], rel=1e-10)
        np.testing.assert_allclose(x, outs[0][1], rtol=0, atol=1e-7)


# ---- degenerate and failure cases ----------------------------------------------------------------

def test_error_codes_for_bad_problems():
    A = np.eye(3); b = np.ones(3)
    with pytest.raises(L.LbfgsbError) as e:
        make_solver(L.OBJ_LSQ, A, b, np.array([0.0, 1.0, 0.0]), np.array([1.0, 0.5, 1.0]), 3)
    assert e.value.code == L.E_BOUNDS
    with pytest.raises(L.LbfgsbError) as e:
        make_solver(L.OBJ_LSQ, A, b, np.array([0.0, np.nan, 0.0]), np.ones(3), 3)
    assert e.value.code == L.E_BOUNDS
    s = make_solver(L.OBJ_LSQ, A, b, np.zeros(3), np.ones(3), 3)
    with pytest.raises(L.LbfgsbError) as e:
        s.set_x(to_dev(np.array([0.5, 2.0, 0.5])))
    assert e.value.code == L.E_INFEASIBLE_X0
    with pytest.raises(L.LbfgsbError) as e:
        s.set_x(to_dev(np.array([0.5, np.nan, 0.5])))
    assert e.value.code == L.E_INFEASIBLE_X0
    with pytest.raises(L.LbfgsbError) as e:
        s.step()                                          # no iterate yet
    assert e.value.code == L.E_INVALID_ARG
    s.set_x(to_dev(np.full(3, 0.5)))                      # and it recovers
    assert s.solve().status == L.CONVERGED
    s.close()
    Abad = np.eye(3); Abad[1, 1] = np.inf
    s = make_solver(L.OBJ_LSQ, Abad, b, np.zeros(3), np.ones(3), 3)
    with pytest.raises(L.LbfgsbError) as e:
        s.set_x(to_dev(np.full(3, 0.5)))
    assert e.value.code == L.E_NONFINITE
    s.close()


def test_max_iter_and_start_at_optimum():
    prob = workloads.config("C1")
    s = L.solver_for_problem(prob, DEV, max_iter=3)
    info = s.solve()
    assert info.status == L.MAX_ITER and info.iters == 3
    s.close()
    ref = oracle.solve_problem(prob, tol=1e-10)
    prob.x0 = ref.x
    s = L.solver_for_problem(prob, DEV)
    info = s.solve()
    assert info.status == L.CONVERGED and info.iters == 0
    s.close()


@pytest.mark.parametrize("name,scale", [("C2", 0.05), ("C3", 0.05), ("C4", 0.02)])
@pytest.mark.parametrize("a_pass", A_PASSES)
def test_steps_behind_the_last_one_change_nothing(name, scale, a_pass):
    """Steps enqueued without waiting go on after the solver has stopped (the iteration limit here, then the tolerance):
    every kernel of such a step returns at once, whichever kernel of the sequence took the decision and through
    whichever copy of the scalar block the others learn of it.  Iterate, gradient, counts and status stay as they were,
    bit for bit, and the state equals that of a solver stopped by the same limit in lbfgsb_solve."""
    prob = workloads.config(name, scale=scale)
    a = _gpu_solver(prob, a_pass, tol=0.0, max_iter=5)
    for _ in range(5):
        a.step(want_info=False)
    a.step(want_info=False)                     # the step whose stopping test finds the limit reached
    at_limit = a.info()
    x5, g5 = a.x().clone(), a.g().clone()
    assert at_limit.status == L.MAX_ITER and at_limit.iters == 5
    for _ in range(4):
        a.step(want_info=False)
    after = a.info()
    assert torch.equal(a.x(), x5) and torch.equal(a.g(), g5)
    assert after.as_dict() == at_limit.as_dict()
    b = _gpu_solver(prob, a_pass, tol=0.0, max_iter=5)
    ib = b.solve()
    assert ib.status == L.MAX_ITER and ib.iters == 5
    assert torch.equal(b.x(), x5) and ib.f == at_limit.f
    a.close(); b.close()
    # stopped by the tolerance: later steps are no-ops too
    c = _gpu_solver(prob, a_pass, tol=1e-3, tol_relative=1)
    ic = c.solve()
    assert ic.status == L.CONVERGED
    xc = c.x().clone()
    for _ in range(3):
        c.step(want_info=False)
    assert torch.equal(c.x(), xc) and c.info().as_dict() == ic.as_dict()
    c.close()


def test_coinciding_and_infinite_bounds():
    rng = np.random.default_rng(77)
    A = rng.normal(size=(30, 6)); b = rng.normal(size=30)
    l = np.array([-np.inf, 0.2, 0.0, -1.0, 0.7, -np.inf]); u = np.array([np.inf, 0.2, 1.0, 1.0, 0.7, 0.0])
    prob = workloads.Problem("pin", workloads.OBJ_LSQ, A, b, l, u, np.clip(np.zeros(6), l, u), m=3, tol=1e-10)
    ref = oracle.solve_problem(prob)
    s = L.solver_for_problem(prob, DEV)
    info = s.solve()
    x = s.x().cpu().numpy()
    assert info.status == L.CONVERGED and x[1] == 0.2 and x[4] == 0.7
    np.testing.assert_allclose(x, ref.x, rtol=0, atol=1e-8)
    s.close()


def test_unbounded_least_squares_gives_lstsq_solution():
    rng = np.random.default_rng(31)
    A = rng.normal(size=(300, 40)); b = rng.normal(size=300)
    prob = workloads.Problem("free", workloads.OBJ_LSQ, A, b, np.full(40, -np.inf), np.full(40, np.inf), np.zeros(40),
                             m=8, tol=1e-10)
    s = L.solver_for_problem(prob, DEV)
    info = s.solve()
    assert info.status == L.CONVERGED and info.n_fixed == 0
    np.testing.assert_allclose(s.x().cpu().numpy(), np.linalg.lstsq(A, b, rcond=None)[0], rtol=0, atol=1e-9)
    s.close()


def test_single_variable_and_single_row():
    prob = workloads.Problem("one", workloads.OBJ_LSQ, np.array([[2.0]]), np.array([1.0]), np.array([0.0]),
                             np.array([0.25]), np.array([0.0]), m=1, tol=1e-12)
    s = L.solver_for_problem(prob, DEV)
    info = s.solve()
    assert info.status == L.CONVERGED and s.x().item() == 0.25
    s.close()


@pytest.mark.parametrize("a_pass,per_step", [(L.APASS_FUSED, 1), (L.APASS_TWO_PASS, 2)], ids=["fused", "two_pass"])
def test_timing_of_the_passes_over_the_matrix(a_pass, per_step):
    """The records behind the benchmark's roofline figure: one per launch that reads A (two per iteration when A is
    read twice), the matrix's size as bytes per launch, durations that add up to less than the wall time of the same
    steps, and the pause / resume / discard switch."""
    import time
    prob = workloads.config("C2", scale=0.1)
    s = _gpu_solver(prob, a_pass, tol=0.0, refresh_every=0)
    for _ in range(3):
        s.step(want_info=False)                       # untimed
    s.enable_apass_timing(2)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(10):
        s.step(want_info=False)
    torch.cuda.synchronize()
    wall_ms = 1e3 * (time.perf_counter() - t0)
    s.enable_apass_timing(0)                          # pause: the next steps are not recorded
    for _ in range(4):
        s.step(want_info=False)
    count, total_ms, nbytes = s.apass_timing()
    assert count == 10 * per_step
    assert nbytes == prob.rows * prob.cols * prob.A.dtype.itemsize
    assert 0.0 < total_ms < wall_ms
    assert total_ms / count > 1e-3 * nbytes / 8e9     # no launch moves its bytes faster than the memory's peak
    s.enable_apass_timing(1)                          # resume: records are kept and added to
    for _ in range(2):
        s.step(want_info=False)
    assert s.apass_timing()[0] == 12 * per_step
    s.enable_apass_timing(2)                          # discard
    assert s.apass_timing()[0] == 0
    s.close()


def test_benchmark_line_has_the_agreed_fields():
    """One run of bench.py on the smallest configuration in a process of its own: exactly one JSON line on stdout with
    the fields the harness reads, the roofline object and the oracle timed beside it."""
    import json
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--config", "C1", "--steps", "10", "--warmup", "2",
                        "--cpu-budget", "1"], capture_output=True, text=True, timeout=280)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 10 and d["warmup"] == 2 and d["higher_is_better"] is True
    assert d["unit"] == "iterations/s" and d["data"] == "synthetic" and d["dtype"] == "f64" and d["vs_baseline"] is None
    assert d["value"] > 0 and d["ms_per_step"] > 0 and d["value"] == pytest.approx(1e3 / d["ms_per_step"], rel=1e-6)
    assert "workload" in d["config"] and "model" not in d["config"]
    rf = d["roofline"]
    assert rf["bound"] == "hbm" and rf["unit"] == "GB/s" and rf["peak"] == 8000.0
    assert rf["frac"] == pytest.approx(rf["achieved"] / rf["peak"]) and "traffic" in rf
    assert "traffic_source" in rf and "step_frac" in d
    assert d["kkt"]["proj_grad_2norm_host"] >= 0 and d["kkt"]["tol_relative"] is False      # C1: absolute 1e-8
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["cores"] == 1 and cb["value"] > 0 and cb["unit"] == "iterations/s" and cb["sample"]
    assert cb["nproc"] >= 1 and isinstance(cb["cpu_model"], str)
    assert "configs" not in d                               # a named --config runs that workload only


def test_default_benchmark_line_reports_every_configuration():
    """Without --config the line is the headline workload (C2) with C1, C3, C4, C5 beside it.  Run here at 2 % of the
    sizes so that the test takes seconds; the records must still be complete."""
    import json
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--steps", "8", "--warmup", "2", "--cpu-budget", "1",
                        "--scale", "0.02"], capture_output=True, text=True, timeout=280)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    assert d["config"]["workload"].startswith("C2:")
    assert sorted(d["configs"]) == ["C1", "C3", "C4", "C5"]
    for name, rec in d["configs"].items():
        assert "error" not in rec, (name, rec)
        assert rec["workload"].startswith(name + ":") and rec["value"] > 0 and rec["steps_valid"] is True
        assert rec["kkt"]["status"] == L.CONVERGED and rec["kkt"]["feasible"] is True
        assert rec["roofline"]["bound"] == "hbm" and "traffic_source" in rec["roofline"]
        assert rec["step_frac"] is None or 0 < rec["step_frac"] < 1
