"""lbfgsb_solve_static: the entry point for callers that cannot allocate.  Its workspace is a fixed array inside the
library instead of the caller's buffer; everything else (kernels, launch geometry, arithmetic order) is what
lbfgsb_create + lbfgsb_set_x + lbfgsb_solve + lbfgsb_get_x run, so the two must agree bit for bit.  Two calls in a
row, the second on a smaller problem (the array still holds the first call's state), then the error paths."""
import numpy as np
import pytest
import torch

import paper_2203_16340_amd as L
import workloads
from gpu_helpers import DEV

pytestmark = pytest.mark.gpu


def _device_problem(prob):
    return tuple(torch.from_numpy(np.ascontiguousarray(a)).to(DEV) for a in (prob.A, prob.b, prob.l, prob.u, prob.x0))


def _reference(prob, dev, **opts):
    A, b, l, u, x0 = dev
    s = L.Solver(prob.kind, A, b, l, u, prob.m, lam=prob.lam, mu=prob.mu, options=L.default_options(**opts))
    s.set_x(x0)
    info = s.solve()
    x = s.x().clone()
    s.close()
    return x, info


def _static(prob, dev, **opts):
    A, b, l, u, x0 = dev
    x = x0.clone()
    info = L.solve_static(prob.kind, A, b, l, u, prob.m, x, lam=prob.lam, mu=prob.mu, options=L.default_options(**opts))
    return x, info


def _same(a, b):
    (xa, ia), (xb, ib) = a, b
    assert torch.equal(xa, xb)
    assert ia.as_dict() == ib.as_dict()


def test_two_calls_in_a_row_match_the_workspace_entry_points_bit_for_bit():
    big = workloads.config("C2", scale=0.1)          # 2000 x 500 fp64 NNLS, m = 10
    small = workloads.config("C1")                   # 200 x 100 fp64 NNLS, m = 5
    logi = workloads.config("C4", scale=0.01)        # 2000 x 20 fp32 logistic, box [-0.5, 0.5]
    cases = ((big, dict(tol=1e-8, tol_relative=1)), (small, dict(tol=1e-8)), (logi, dict(tol=1e-8, tol_relative=1)),
             (big, dict(tol=1e-8, tol_relative=1, a_pass=L.APASS_TWO_PASS)))
    for k, (prob, opts) in enumerate(cases):
        dev = _device_problem(prob)
        ref = _reference(prob, dev, **opts)
        assert ref[1].status == L.CONVERGED and ref[1].iters > 5
        torch.cuda.synchronize()
        free_before, _ = torch.cuda.mem_get_info()
        got = _static(prob, dev, **opts)
        torch.cuda.synchronize()
        free_after, _ = torch.cuda.mem_get_info()
        _same(got, ref)
        if k == 0:
            # the first use of the array in a process makes the runtime load the code object that holds it
            assert free_before - free_after <= L.STATIC_SCRATCH_BYTES + (8 << 20)
        else:
            assert free_after == free_before         # no device memory taken (or given back) by the call
        assert torch.equal(dev[4], torch.from_numpy(prob.x0).to(DEV))   # only x was written


def test_static_entry_point_on_a_stream_of_its_own():
    prob = workloads.config("C5", scale=0.02)        # 2000 x 400 fp32, box [0, 1], m = 20
    dev = _device_problem(prob)
    ref = _reference(prob, dev, tol=1e-8, tol_relative=1)
    st = torch.cuda.Stream(device=DEV)
    with torch.cuda.stream(st):
        got = _static(prob, dev, tol=1e-8, tol_relative=1)
    st.synchronize()
    _same(got, ref)


def test_sizes_beyond_the_fixed_array_and_bad_inputs_are_rejected():
    # 2 m n doubles of pair memory alone exceed the array: n = 220000, m = 10 -> 35 MB
    n = 220000
    A = torch.ones(1, n, dtype=torch.float64, device=DEV)
    b = torch.zeros(1, dtype=torch.float64, device=DEV)
    l = torch.zeros(n, dtype=torch.float64, device=DEV)
    u = torch.ones(n, dtype=torch.float64, device=DEV)
    x = torch.zeros(n, dtype=torch.float64, device=DEV)
    with pytest.raises(L.LbfgsbError) as e:
        L.solve_static(L.OBJ_LSQ, A, b, l, u, 10, x)
    assert e.value.code == L.E_INVALID_ARG and "lbfgsb_solve_static holds" in str(e.value)
    # the same problem goes through lbfgsb_create with a workspace of the caller's
    s = L.Solver(L.OBJ_LSQ, A, b, l, u, 10)
    assert s.workspace.numel() > L.STATIC_SCRATCH_BYTES
    s.close()
    # start point outside the box, crossed bounds: the codes of lbfgsb_set_x / lbfgsb_create
    prob = workloads.config("C1")
    A, b, l, u, x0 = _device_problem(prob)
    bad = x0.clone(); bad[3] = -1.0
    with pytest.raises(L.LbfgsbError) as e:
        L.solve_static(prob.kind, A, b, l, u, prob.m, bad)
    assert e.value.code == L.E_INFEASIBLE_X0
    lo = l.clone(); lo[5] = float("nan")
    with pytest.raises(L.LbfgsbError) as e:
        L.solve_static(prob.kind, A, b, lo, u, prob.m, x0.clone())
    assert e.value.code == L.E_BOUNDS
    # and a good call afterwards still works
    ref = _reference(prob, (A, b, l, u, x0), tol=1e-8)
    _same(_static(prob, (A, b, l, u, x0), tol=1e-8), ref)
