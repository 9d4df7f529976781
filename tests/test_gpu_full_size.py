"""Parity at the full sizes of the benchmark configurations C2-C5, in the launch configuration
bench.py times (default options: the fused single-read A pass, which for the logistic objective is the
speculative pass that also carries the first trial step).

A full oracle evaluation streams up to 8 GB through one core, so the oracle is asked for SAMPLED
outputs it can compute one by one, each of them an exact output of the full-size problem:
  * dense x, sampled rows I: the oracle evaluates the sub-problem (A[I], b[I]) -> the residuals /
    margins of rows I of the full problem;
  * sparse x (64 non-zeros), sampled columns J: with K = supp(x) u J the oracle evaluates the
    sub-problem (A[:, K], b) at x[K] -> the objective value, ALL residuals / margins and the gradient
    entries K of the full problem (the GPU still multiplies with every column).
End to end, the solve is checked through properties that hold at any size (feasibility, the
stopping quantity and the epsilon-free KKT residual recomputed on the host with numpy, the reported
objective, descent), and against FULL oracle solves of the same seeded problems: C2's runs inside the
test (seconds), those of C3, C4 and C5 (minutes of one core each) are stored under tests/golden/ by
tests/golden/make_full_size_goldens.py, which calls the oracle only.  By the corollary of Theorem 1 both
implementations must reach the global optimum over the box, so the final objective agrees to 1e-8 (fp64
storage) / 1e-4 (fp32 storage) relative and, where the minimiser is unique and well separated from the
bounds (C4, C5), the set of active bounds is identical; C3's objective is convex but not strictly convex
in [p; q], so there the set difference is reported and only bounded.
"""
import json
import os

import numpy as np
import pytest
import torch

import oracle
import paper_2203_16340_amd as L
import workloads
from gpu_helpers import DEV, active_set, host_gradient, host_objective, rel_err

pytestmark = pytest.mark.gpu

CONFIGS = ["C2", "C3", "C4", "C5"]


@pytest.fixture(scope="module", params=CONFIGS)
def full(request):
    name = request.param
    print(f"[full-size] generating {name}", flush=True)
    prob = workloads.config(name)
    s = L.solver_for_problem(prob, DEV)
    print(f"[full-size] {name}: {prob.rows} x {prob.cols} {prob.A.dtype}, a_pass = {s.apass_name}", flush=True)
    yield name, prob, s
    s.close()
    del s, prob
    torch.cuda.empty_cache()


def _golden(name):
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", f"full_size_{name}.json")) as fh:
        return json.load(fh)


def _bitmap(hex_text, n):
    return np.unpackbits(np.frombuffer(bytes.fromhex(hex_text), dtype=np.uint8))[:n].astype(bool)


def _tol(prob):
    return 1e-12 if prob.A.dtype == np.float64 else 1e-5


def _feasible_point(prob, rng, dense):
    n = prob.n
    lo = np.where(np.isfinite(prob.l), prob.l, -1.0)
    hi = np.where(np.isfinite(prob.u), prob.u, lo + 1.0)
    x = lo + (hi - lo) * rng.random(n)
    if not dense:
        keep = np.zeros(n, dtype=bool)
        keep[rng.choice(n, size=64, replace=False)] = True
        x = np.where(keep, x, np.clip(0.0, prob.l, prob.u))
    return x


def test_expected_launch_configuration(full):
    name, prob, s = full
    assert s.apass_name == "fused"


def test_rows_of_the_product_at_a_dense_point(full):
    name, prob, s = full
    rng = np.random.default_rng(77)
    x = _feasible_point(prob, rng, dense=True)
    _, _, row = s.dbg_fg(torch.from_numpy(x).to(DEV), want_rowvec=True)
    row = row.cpu().numpy()
    # first and last rows (workgroup range ends), plus a random sample
    idx = np.unique(np.concatenate([np.arange(8), np.arange(prob.rows - 8, prob.rows),
                                    rng.choice(prob.rows, size=496, replace=False)]))
    sub = oracle.Objective(prob.kind, np.ascontiguousarray(prob.A[idx]), prob.b[idx], prob.lam, prob.mu)
    _, _, row_ref = oracle.fg(sub, x, want_rowvec=True)
    assert rel_err(row[idx], row_ref) <= _tol(prob)
    assert np.all(np.isfinite(row))


def test_objective_rows_and_gradient_entries_at_a_sparse_point(full):
    name, prob, s = full
    rng = np.random.default_rng(78)
    x = _feasible_point(prob, rng, dense=False)
    f, g, row = s.dbg_fg(torch.from_numpy(x).to(DEV), want_rowvec=True)
    g, row = g.cpu().numpy(), row.cpu().numpy()
    cols = prob.cols
    split = prob.kind == workloads.OBJ_LSQ_L1SPLIT
    supp = np.flatnonzero(x[:cols] != 0) if not split else np.flatnonzero((x[:cols] != 0) | (x[cols:] != 0))
    J = np.concatenate([np.arange(4), np.arange(cols - 4, cols), rng.choice(cols, size=56, replace=False)])
    K = np.unique(np.concatenate([supp, J]))
    A_K = np.ascontiguousarray(prob.A[:, K])
    sub = oracle.Objective(prob.kind, A_K, prob.b, prob.lam, prob.mu)
    x_K = np.concatenate([x[K], x[cols + K]]) if split else x[K]
    f_ref, g_ref, row_ref = oracle.fg(sub, x_K, want_rowvec=True)
    tol = _tol(prob)
    if split:
        # entries outside K are zero and contribute lam*0 to the objective
        g_K = np.concatenate([g[K], g[cols + K]])
    else:
        g_K = g[K]
    assert abs(f - f_ref) <= tol * abs(f_ref), (f, f_ref)
    assert rel_err(row, row_ref) <= tol
    assert rel_err(g_K, g_ref) <= tol
    assert np.all(np.isfinite(g))


def test_solve_properties_at_full_size(full):
    name, prob, s = full
    x0 = torch.from_numpy(prob.x0).to(DEV)
    s.set_x(x0)
    f0 = s.info().f
    info = s.solve()                      # the configuration's tolerance: 1e-6 relative
    x = s.x().cpu().numpy()
    assert info.status == L.CONVERGED, info.as_dict()
    assert np.all(x >= prob.l) and np.all(x <= prob.u)
    assert info.f < f0
    assert info.f == pytest.approx(host_objective(prob, x), rel=1e-9)
    g = host_gradient(prob, x)
    g0 = host_gradient(prob, prob.x0)
    free0 = oracle.free_mask(prob.x0, g0, prob.l, prob.u, 1e-10).astype(bool)
    free = oracle.free_mask(x, g, prob.l, prob.u, 1e-10).astype(bool)
    scale = max(1.0, float(np.linalg.norm(g0[free0])))
    slack = 1.5 if prob.A.dtype == np.float64 else 3.0
    assert np.linalg.norm(g[free]) <= slack * 1e-6 * scale
    assert np.abs(x - np.clip(x - g, prob.l, prob.u)).max() <= slack * 1e-6 * scale
    # the solver's gradient (carried by recurrence, refreshed before convergence is declared) is the true one
    assert rel_err(s.g().cpu().numpy(), g) <= (1e-9 if prob.A.dtype == np.float64 else 1e-6)
    print(f"[full-size] {name}: {info.iters} iterations, f = {info.f:.10g}, ||g[S]|| / ||g0[S0]|| = "
          f"{np.linalg.norm(g[free]) / scale:.2e}, {int((~free).sum())} fixed", flush=True)


def _solve_with_the_oracle_now(prob):
    """The same record tests/golden/make_full_size_goldens.py stores, from an oracle solve run inside the test
    (C2: about ten seconds of one core)."""
    eps, tol = 1e-10, 1e-9
    ref = oracle.solve_problem(prob, tol=tol, tol_relative=1, eps=eps)
    active = active_set(prob, ref.x, eps=eps)
    free_idx = np.flatnonzero(~active)
    sample = free_idx[np.unique(np.linspace(0, free_idx.size - 1, min(128, free_idx.size)).astype(np.int64))]
    return dict(rows=prob.rows, cols=prob.cols, n=prob.n, m=prob.m, seed=workloads.CONFIG_SEEDS[prob.name],
                status=int(ref.info.status), iters=int(ref.info.iters), f=float(ref.info.f),
                options=dict(tol=tol, tol_relative=1, eps=eps), n_active=int(active.sum()),
                active_bitmap_hex=np.packbits(active).tobytes().hex(),
                at_upper_bitmap_hex=np.packbits(ref.x >= prob.u - eps).tobytes().hex(),
                x_sample_indices=[int(v) for v in sample], x_sample=[float(v) for v in ref.x[sample]],
                x_norm2=float(np.linalg.norm(ref.x)))


def test_full_size_result_against_a_full_oracle_solve(full):
    """C2-C5 at full size, solved to 1e-9 relative like the oracle run (C2: run here; C3-C5: stored): final objective
    within the benchmark spec's bound, identical active set where the minimiser is unique (C2, C4, C5), the minimiser itself
    on a sample of free variables."""
    name, prob, s0 = full
    gold = _golden(name) if name != "C2" else _solve_with_the_oracle_now(prob)
    assert (gold["rows"], gold["cols"], gold["n"], gold["m"], gold["seed"]) == \
        (prob.rows, prob.cols, prob.n, prob.m, workloads.CONFIG_SEEDS[name])
    assert gold["status"] == oracle.CONVERGED
    opt = gold["options"]
    # a second solver on the matrix already in device memory (the library borrows A and b)
    s = L.Solver(prob.kind, s0._A, s0._b, torch.from_numpy(prob.l).to(DEV), torch.from_numpy(prob.u).to(DEV), prob.m,
                 lam=prob.lam, mu=prob.mu,
                 options=L.default_options(tol=opt["tol"], tol_relative=opt["tol_relative"], eps=opt["eps"], max_iter=1000))
    s.set_x(torch.from_numpy(prob.x0).to(DEV))
    info = s.solve()
    x = s.x().cpu().numpy()
    s.close()
    assert info.status == L.CONVERGED, info.as_dict()
    f_tol = 1e-8 if prob.A.dtype == np.float64 else 1e-4
    assert abs(info.f - gold["f"]) <= f_tol * abs(gold["f"]), (info.f, gold["f"])
    active = active_set(prob, x, eps=opt["eps"])
    gold_active = _bitmap(gold["active_bitmap_hex"], prob.n)
    assert int(gold_active.sum()) == gold["n_active"]
    differ = np.flatnonzero(active != gold_active)
    print(f"[full-size] {name}: {info.iters} iterations (oracle {gold['iters']}), f = {info.f!r} (oracle {gold['f']!r}), "
          f"{int(active.sum())} active (oracle {gold['n_active']}), {differ.size} differ", flush=True)
    idx = np.array(gold["x_sample_indices"])
    x_ref = np.array(gold["x_sample"])
    if name == "C3":
        # convex, not strictly: the set difference is reported; the lasso solution p - q is still unique for a matrix
        # in general position, so only entries whose value is within rounding of the bound may flip
        assert differ.size <= 4, differ
        assert np.all(np.abs(x[differ]) <= 1e-7)
        assert rel_err(x[idx], x_ref) <= 1e-5
    else:
        assert differ.size == 0, (differ, x[differ])
        upper = _bitmap(gold["at_upper_bitmap_hex"], prob.n)
        assert np.array_equal(x >= prob.u - opt["eps"], upper)
        assert rel_err(x[idx], x_ref) <= 1e-6
        assert np.linalg.norm(x) == pytest.approx(gold["x_norm2"], rel=1e-7)
    assert info.iters <= 2 * gold["iters"] + 20
