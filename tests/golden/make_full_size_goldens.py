"""Writes tests/golden/full_size_<config>.json: the CPU oracle's result on a benchmark configuration at its
FULL size (same seed, same recipe as everywhere else), solved far past the benchmark's tolerance.

Imports the oracle and the seeded input generators only; nothing here touches the HIP library.  The
expected values are therefore the oracle's own (Algorithm 1 with from-scratch evaluations), and by the
corollary of Theorem 1 (convex objective: the method reaches the global optimum over the box) they are
what any correct implementation must reach: the final objective, and on the strictly convex
configurations the minimiser and its set of active bounds.

    python tests/golden/make_full_size_goldens.py C3 C4 C5        (each config: minutes of one core;
                                                                   C5 holds its 8 GB matrix in memory)

Fields: f (final objective), iters, fevals, status, pg2 (||grad f[S]||_2 at the end), pginf
(||x - P(x - grad f)||_inf), n, n_active (variables within eps of a bound), active_sha256 (SHA-256 of the
sorted active indices as little-endian int64), active_bitmap_hex / at_upper_bitmap_hex (one bit per variable,
numpy.packbits order, as hexadecimal text: which variables sit on a bound, and which of those on the upper one),
x_sample_indices / x_sample (128 evenly spaced free variables and the minimiser there), x_norm2 (||x||_2).
"""
from __future__ import annotations

import hashlib
import json
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import oracle      # noqa: E402
import workloads   # noqa: E402

TOL_RELATIVE = 1e-9     # stop at ||grad f[S]|| <= 1e-9 * max(1, its value at x0)
EPS = 1e-10             # the method's epsilon (Eq. (ws)); also what "on a bound" means below


def active_hash(idx: np.ndarray) -> str:
    return hashlib.sha256(np.sort(idx).astype("<i8").tobytes()).hexdigest()


def solve(name: str) -> dict:
    t0 = time.time()
    prob = workloads.config(name)
    print(f"[{name}] generated {prob.rows} x {prob.cols} {prob.A.dtype} in {time.time() - t0:.1f} s", flush=True)
    obj = oracle.Objective(prob.kind, prob.A, prob.b, prob.lam, prob.mu)
    opts = oracle.default_options(tol=TOL_RELATIVE, tol_relative=1, max_iter=1000, eps=EPS)
    s = oracle.Solver(obj, prob.l, prob.u, prob.x0, prob.m, opts)
    t1 = time.time()
    while s.step() == oracle.RUNNING:
        i = s.info
        print(f"[{name}] it {i.iters:4d}  f = {i.f:.15g}  ||g[S]|| = {i.pg2:.3e}  bt = {i.backtracks}  "
              f"{time.time() - t1:.0f} s", flush=True)
    s.refresh_info()
    info = s.info
    x = s.x
    active = (x <= prob.l + EPS) | (x >= prob.u - EPS)
    free_idx = np.flatnonzero(~active)
    sample = free_idx[np.unique(np.linspace(0, free_idx.size - 1, min(128, free_idx.size)).astype(np.int64))]
    at_upper = x >= prob.u - EPS
    out = dict(
        config=name, seed=workloads.CONFIG_SEEDS[name], rows=prob.rows, cols=prob.cols, dtype=str(prob.A.dtype),
        n=prob.n, m=prob.m, options=dict(tol=TOL_RELATIVE, tol_relative=1, eps=EPS, armijo_c1=opts.armijo_c1,
                                         backtrack=opts.backtrack, max_backtracks=opts.max_backtracks),
        status=int(info.status), iters=int(info.iters), fevals=int(info.fevals), f=float(info.f),
        pg2=float(info.pg2), pginf=float(info.pginf), n_active=int(active.sum()),
        active_sha256=active_hash(np.flatnonzero(active)),
        active_bitmap_hex=np.packbits(active).tobytes().hex(),
        at_upper_bitmap_hex=np.packbits(at_upper).tobytes().hex(),
        x_sample_indices=[int(v) for v in sample], x_sample=[float(v) for v in x[sample]],
        x_norm2=float(np.linalg.norm(x)),
        oracle_seconds=round(time.time() - t1, 1),
    )
    s.close()
    return out


def main(argv):
    names = argv or ["C3", "C4", "C5"]
    for name in names:
        res = solve(name)
        path = os.path.join(HERE, f"full_size_{name}.json")
        with open(path, "w") as fh:
            json.dump(res, fh, indent=1)
            fh.write("\n")
        print(f"[{name}] status {res['status']}, {res['iters']} iterations, f = {res['f']!r}, "
              f"{res['n_active']} of {res['n']} active -> {path}", flush=True)


if __name__ == "__main__":
    main(sys.argv[1:])
