"""ctypes binding of the CPU oracle (oracle/lbfgsb_oracle.c).

TEST INFRASTRUCTURE ONLY.  Only tests, the smoke check and the benchmark's CPU-baseline
leg may import this package; the HIP library and its Python binding never do.

`build()` compiles the C file with gcc into oracle/liblbfgsb_oracle.so; `load()` returns
the ctypes handle (building first when the library is missing or older than its source).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lbfgsb_oracle.c")
_LIB = os.path.join(_HERE, "liblbfgsb_oracle.so")

RUNNING, CONVERGED, MAX_ITER, LINESEARCH_FAILED = 0, 1, 2, 3
LSQ, LSQ_L1SPLIT, LOGISTIC_L2, QP, OT_GAUSS, OT_ENTROPY = 0, 1, 2, 3, 4, 5
F64, F32 = 0, 1


class _Constraints(C.Structure):
    _fields_ = [("n_eq", C.c_int64), ("n_in", C.c_int64), ("C", C.c_void_p), ("d", C.c_void_p),
                ("E", C.c_void_p), ("e", C.c_void_p), ("lam", C.c_void_p), ("mu", C.c_void_p),
                ("rho", C.c_double), ("marginals", C.c_int)]


class _Objective(C.Structure):
    _fields_ = [("kind", C.c_int), ("dtype", C.c_int), ("rows", C.c_int64), ("cols", C.c_int64),
                ("ld", C.c_int64), ("A", C.c_void_p), ("b", C.c_void_p), ("lam", C.c_double),
                ("mu", C.c_double), ("con", C.c_void_p), ("sign", C.c_void_p)]


class AuglagOptions(C.Structure):
    _fields_ = [("rho0", C.c_double), ("ctol", C.c_double), ("max_outer", C.c_int)]


class AuglagInfo(C.Structure):
    _fields_ = [("status", C.c_int), ("outer", C.c_int), ("inner_iters", C.c_int64),
                ("violation", C.c_double), ("rho", C.c_double), ("f", C.c_double), ("L", C.c_double),
                ("pg2", C.c_double)]


class Options(C.Structure):
    _fields_ = [("eps", C.c_double), ("armijo_c1", C.c_double), ("backtrack", C.c_double),
                ("max_backtracks", C.c_int), ("tol", C.c_double), ("tol_relative", C.c_int),
                ("max_iter", C.c_int), ("always_branch2", C.c_int)]


class Info(C.Structure):
    _fields_ = [("status", C.c_int), ("iters", C.c_int64), ("fevals", C.c_int64), ("f", C.c_double),
                ("pg2", C.c_double), ("pginf", C.c_double), ("n_fixed", C.c_int64),
                ("branch", C.c_int), ("backtracks", C.c_int), ("pairs_used", C.c_int),
                ("memory_resets", C.c_int), ("alpha", C.c_double), ("alpha_ub", C.c_double),
                ("gp", C.c_double)]


def build(force: bool = False) -> str:
    """Compile the oracle.  No -ffast-math: the compensated sums rely on IEEE semantics."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        # -mfma: the compensated dot products recover each product's rounding error with
        # fma(); without the flag gcc would call libm's fma() once per matrix element.
        cmd = ["gcc", "-O2", "-std=c11", "-mfma", "-ffp-contract=off", "-fPIC", "-shared", "-Wall",
               "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def load():
    global _lib
    if _lib is None:
        lib = C.CDLL(build())
        dp, u8p = C.c_void_p, C.c_void_p
        lib.orc_num_vars.restype = C.c_int64
        lib.orc_num_vars.argtypes = [C.POINTER(_Objective)]
        lib.orc_fg.restype = C.c_double
        lib.orc_fg.argtypes = [C.POINTER(_Objective), dp, dp, dp]
        lib.orc_delta_f.restype = C.c_double
        lib.orc_delta_f.argtypes = [C.POINTER(_Objective), dp, dp, dp]
        lib.orc_free_mask.restype = None
        lib.orc_free_mask.argtypes = [C.c_int64, dp, dp, dp, dp, C.c_double, u8p]
        lib.orc_two_loop.restype = None
        lib.orc_two_loop.argtypes = [C.c_int64, C.c_int, dp, dp, dp, dp, u8p, C.c_double, dp,
                                     C.POINTER(C.c_int)]
        lib.orc_project_direction.restype = C.c_int
        lib.orc_project_direction.argtypes = [C.c_int64, dp, dp, dp, dp, dp, C.c_double, C.c_int, dp,
                                              C.POINTER(C.c_double)]
        lib.orc_default_options.restype = None
        lib.orc_default_options.argtypes = [C.POINTER(Options)]
        lib.orc_create.restype = C.c_void_p
        lib.orc_create.argtypes = [C.c_int64, C.c_int, dp, dp, dp, C.POINTER(_Objective),
                                   C.POINTER(Options)]
        lib.orc_destroy.restype = None
        lib.orc_destroy.argtypes = [C.c_void_p]
        lib.orc_step.restype = C.c_int
        lib.orc_step.argtypes = [C.c_void_p]
        lib.orc_solve.restype = C.c_int
        lib.orc_solve.argtypes = [C.c_void_p]
        lib.orc_refresh_info.restype = None
        lib.orc_refresh_info.argtypes = [C.c_void_p]
        lib.orc_get_info.restype = None
        lib.orc_get_info.argtypes = [C.c_void_p, C.POINTER(Info)]
        for name in ("orc_x", "orc_g", "orc_d", "orc_p", "orc_mask", "orc_S", "orc_Y", "orc_ynorm2"):
            getattr(lib, name).restype = C.c_void_p
            getattr(lib, name).argtypes = [C.c_void_p]
        lib.orc_npairs.restype = C.c_int
        lib.orc_npairs.argtypes = [C.c_void_p]
        lib.orc_auglag_default_options.restype = None
        lib.orc_auglag_default_options.argtypes = [C.POINTER(AuglagOptions)]
        lib.orc_auglag_solve.restype = C.c_int
        lib.orc_auglag_solve.argtypes = [C.c_int64, C.c_int, dp, dp, dp, C.POINTER(_Objective), C.POINTER(Options),
                                         C.POINTER(AuglagOptions), C.POINTER(AuglagInfo)]
        _lib = lib
    return _lib


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def default_options(**overrides) -> Options:
    o = Options()
    load().orc_default_options(C.byref(o))
    for k, v in overrides.items():
        if not hasattr(o, k):
            raise AttributeError(k)
        setattr(o, k, v)
    return o


class Objective:
    """Keeps the numpy arrays alive next to the C struct that points into them."""

    def __init__(self, kind: int, A: np.ndarray, b: Optional[np.ndarray] = None, lam: float = 0.0, mu: float = 0.0,
                 sign=None):
        if A.dtype not in (np.float64, np.float32) or A.ndim != 2:
            raise TypeError("A must be a 2-d float64 or float32 array")
        if A.strides[1] != A.itemsize or A.strides[0] % A.itemsize:
            A = np.ascontiguousarray(A)
        self.A = A
        self.transport = kind in (OT_GAUSS, OT_ENTROPY)   # A is the cost matrix M, b is not read
        self.b = _f64(b) if b is not None else np.zeros(A.shape[0])
        if self.b.shape != (A.shape[0],):
            raise ValueError("b must have one entry per row of A")
        self.kind = kind
        self.nrow = 0 if self.transport else A.shape[0]   # objective's own entries of the row vector
        self.c = _Objective(kind, F64 if A.dtype == np.float64 else F32, A.shape[0], A.shape[1],
                            A.strides[0] // A.itemsize, _ptr(A), _ptr(self.b), float(lam), float(mu), None, None)
        self.con = None
        self.sign = None
        if sign is not None:
            assert kind == QP
            self.sign = _f64(sign)
            assert self.sign.shape == (A.shape[1],)
            self.c.sign = _ptr(self.sign)
        if kind == QP:
            assert A.shape[0] == A.shape[1], "the quadratic form needs a square (symmetric) matrix"

    def set_constraints(self, C_eq=None, d=None, E_in=None, e=None, lam=None, mu=None, rho: float = 1.0):
        """Attach linear constraints C x = d, E x <= e and a multiplier state (Eq. (augLag)): fg() then
        evaluates the augmented Lagrangian.  The multiplier arrays are kept (and updated in place by
        auglag_solve) as self.lam / self.mu."""
        assert not self.transport, "the transport kinds take set_marginals()"
        cols = self.A.shape[1]
        self.C_eq = _f64(C_eq).reshape(-1, cols) if C_eq is not None else np.zeros((0, cols))
        self.E_in = _f64(E_in).reshape(-1, cols) if E_in is not None else np.zeros((0, cols))
        self.d = _f64(d).reshape(-1) if d is not None else np.zeros(0)
        self.e = _f64(e).reshape(-1) if e is not None else np.zeros(0)
        assert self.d.shape == (self.C_eq.shape[0],) and self.e.shape == (self.E_in.shape[0],)
        self.lam = _f64(lam).copy() if lam is not None else np.zeros(self.C_eq.shape[0])
        self.mu = _f64(mu).copy() if mu is not None else np.zeros(self.E_in.shape[0])
        self.con = _Constraints(self.C_eq.shape[0], self.E_in.shape[0], _ptr(self.C_eq), _ptr(self.d),
                                _ptr(self.E_in), _ptr(self.e), _ptr(self.lam), _ptr(self.mu), float(rho), 0)
        self.c.con = C.cast(C.pointer(self.con), C.c_void_p)
        return self

    def set_marginals(self, u, v, lam=None, rho: float = 1.0):
        """Transport kinds: attach the marginal constraints P 1 = u, P^T 1 = v (rows + cols equality rows, in
        that order) and a multiplier state; fg() then evaluates the augmented Lagrangian of Eq. (augLag)."""
        assert self.transport
        rows, cols = self.A.shape
        self.d = np.concatenate([_f64(u).reshape(-1), _f64(v).reshape(-1)])
        assert self.d.shape == (rows + cols,)
        self.lam = _f64(lam).copy() if lam is not None else np.zeros(rows + cols)
        self.mu = np.zeros(0)
        self.con = _Constraints(rows + cols, 0, None, _ptr(self.d), None, None, _ptr(self.lam), None, float(rho), 1)
        self.c.con = C.cast(C.pointer(self.con), C.c_void_p)
        return self

    @property
    def n(self) -> int:
        return int(load().orc_num_vars(C.byref(self.c)))


def fg(obj: Objective, x, want_rowvec: bool = False):
    """f(x), grad f(x) [, residual or margins (followed by the shifted constraint values when the
    objective carries constraints)]"""
    x = _f64(x)
    assert x.shape == (obj.n,)
    g = np.empty(obj.n)
    ncon = (obj.con.n_eq + obj.con.n_in) if obj.con is not None else 0
    rv = np.empty(obj.nrow + ncon) if want_rowvec else None
    f = load().orc_fg(C.byref(obj.c), _ptr(x), _ptr(g), _ptr(rv))
    return (f, g, rv) if want_rowvec else (f, g)


def f_only(obj: Objective, x) -> float:
    x = _f64(x)
    assert x.shape == (obj.n,)
    return load().orc_fg(C.byref(obj.c), _ptr(x), None, None)


def delta_f(obj: Objective, x, xt, row) -> float:
    """f(xt) - f(x) from the cancellation-free row-wise identity; row = residuals/margins at x."""
    x, xt, row = _f64(x), _f64(xt), _f64(row)
    ncon = (obj.con.n_eq + obj.con.n_in) if obj.con is not None else 0
    assert x.shape == (obj.n,) and xt.shape == (obj.n,) and row.shape == (obj.nrow + ncon,)
    return load().orc_delta_f(C.byref(obj.c), _ptr(x), _ptr(xt), _ptr(row))


def free_mask(x, g, l, u, eps: float) -> np.ndarray:
    x, g, l, u = map(_f64, (x, g, l, u))
    mask = np.empty(x.size, dtype=np.uint8)
    load().orc_free_mask(x.size, _ptr(x), _ptr(g), _ptr(l), _ptr(u), eps, _ptr(mask))
    return mask


def two_loop(S, Y, g, mask, eps: float, ynorm2=None):
    """S, Y: (npairs, n), oldest first.  Returns (d, pairs_used)."""
    g = _f64(g)
    n = g.size
    S = _f64(S).reshape(-1, n)
    Y = _f64(Y).reshape(-1, n)
    npairs = S.shape[0]
    assert Y.shape == S.shape
    if ynorm2 is None:
        ynorm2 = np.einsum("ij,ij->i", Y, Y)
    ynorm2 = _f64(ynorm2)
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    d = np.empty(n)
    used = C.c_int(0)
    load().orc_two_loop(n, npairs, _ptr(S), _ptr(Y), _ptr(ynorm2), _ptr(g), _ptr(mask), eps, _ptr(d),
                        C.byref(used))
    return d, used.value


def project_direction(x, g, d, l, u, eps: float, always_branch2: bool = False):
    """Returns (p, branch, alpha_ub)."""
    x, g, d, l, u = map(_f64, (x, g, d, l, u))
    p = np.empty(x.size)
    ub = C.c_double(0.0)
    br = load().orc_project_direction(x.size, _ptr(x), _ptr(g), _ptr(d), _ptr(l), _ptr(u), eps,
                                      int(always_branch2), _ptr(p), C.byref(ub))
    return p, br, ub.value


@dataclass
class Result:
    x: np.ndarray
    g: np.ndarray
    info: Info


class Solver:
    """Stepwise access to Algorithm 1 so that tests can look at every intermediate vector."""

    def __init__(self, obj: Objective, l, u, x0, m: int, options: Optional[Options] = None):
        self.obj = obj
        self.n = obj.n
        self.m = m
        self._l, self._u, self._x0 = _f64(l), _f64(u), _f64(x0)
        self.options = options if options is not None else default_options()
        self._h = load().orc_create(self.n, m, _ptr(self._l), _ptr(self._u), _ptr(self._x0),
                                    C.byref(obj.c), C.byref(self.options))
        if not self._h:
            raise ValueError("oracle rejected the problem (bad sizes, crossed bounds or infeasible x0)")

    def close(self):
        if self._h:
            load().orc_destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()

    def step(self) -> int:
        return load().orc_step(self._h)

    def solve(self) -> Result:
        load().orc_solve(self._h)
        return Result(self.x, self.g, self.info)

    def refresh_info(self):
        load().orc_refresh_info(self._h)

    @property
    def info(self) -> Info:
        out = Info()
        load().orc_get_info(self._h, C.byref(out))
        return out

    def _vec(self, name: str, count: int, dtype=np.float64) -> np.ndarray:
        addr = getattr(load(), name)(self._h)
        if count == 0:
            return np.empty(0, dtype=dtype)
        buf = (C.c_char * (count * np.dtype(dtype).itemsize)).from_address(addr)
        return np.frombuffer(buf, dtype=dtype, count=count).copy()

    x = property(lambda self: self._vec("orc_x", self.n))
    g = property(lambda self: self._vec("orc_g", self.n))
    d = property(lambda self: self._vec("orc_d", self.n))
    p = property(lambda self: self._vec("orc_p", self.n))
    mask = property(lambda self: self._vec("orc_mask", self.n, np.uint8))
    npairs = property(lambda self: int(load().orc_npairs(self._h)))
    S = property(lambda self: self._vec("orc_S", self.npairs * self.n).reshape(self.npairs, self.n))
    Y = property(lambda self: self._vec("orc_Y", self.npairs * self.n).reshape(self.npairs, self.n))
    ynorm2 = property(lambda self: self._vec("orc_ynorm2", self.npairs))


def solve_problem(prob, **option_overrides) -> Result:
    """Run the oracle on a workloads.Problem."""
    obj = Objective(prob.kind, prob.A, prob.b, prob.lam, prob.mu)
    opts = default_options(tol=prob.tol, tol_relative=int(prob.tol_relative), max_iter=int(getattr(prob, "max_iter", 1000)))
    for k, v in option_overrides.items():
        setattr(opts, k, v)
    s = Solver(obj, prob.l, prob.u, prob.x0, prob.m, opts)
    try:
        return s.solve()
    finally:
        s.close()


def auglag_solve(obj: Objective, l, u, x0, m: int, options: Optional[Options] = None, rho0: float = 1.0,
                 ctol: float = 1e-8, max_outer: int = 100):
    """Algorithm 4 on an objective with constraints attached by set_constraints() / set_marginals().
    Returns (x, lambda, mu, AuglagInfo)."""
    assert obj.con is not None
    x = _f64(x0).copy()
    l, u = _f64(l), _f64(u)
    ao = AuglagOptions(float(rho0), float(ctol), int(max_outer))
    info = AuglagInfo()
    opts = options if options is not None else default_options()
    rc = load().orc_auglag_solve(obj.n, m, _ptr(l), _ptr(u), _ptr(x), C.byref(obj.c), C.byref(opts), C.byref(ao),
                                 C.byref(info))
    if rc != 0:
        raise ValueError("oracle rejected the constrained problem")
    return x, obj.lam.copy(), obj.mu.copy(), info
