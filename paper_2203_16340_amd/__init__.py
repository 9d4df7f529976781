"""Thin Python binding of liblbfgsb (include/lbfgsb.h): argument marshalling only.

Every step of the solver runs in the HIP library; PyTorch is used for device memory and
streams.  There is no CPU fallback: importing the binding's functions without the built
library raises.  Build with `python -m paper_2203_16340_amd.build` (or __graft_entry__.build()).
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblbfgsb.so")

F64, F32 = 0, 1
OBJ_LSQ, OBJ_LSQ_L1SPLIT, OBJ_LOGISTIC_L2, OBJ_QP, OBJ_OT_GAUSS, OBJ_OT_ENTROPY = 0, 1, 2, 3, 4, 5
APASS_AUTO, APASS_TWO_PASS, APASS_FUSED, APASS_RESIDENT = 0, 1, 2, 3
RUNNING, CONVERGED, MAX_ITER, LINESEARCH_FAILED = 0, 1, 2, 3
OK, E_INVALID_ARG, E_BOUNDS, E_INFEASIBLE_X0, E_NONFINITE, E_HIP, E_UNSUPPORTED = 0, -1, -2, -3, -4, -5, -6
MAX_M = 31

EXPORTS = [
    "lbfgsb_last_error", "lbfgsb_default_options", "lbfgsb_workspace_bytes", "lbfgsb_create", "lbfgsb_set_x",
    "lbfgsb_step", "lbfgsb_solve", "lbfgsb_solve_static", "lbfgsb_get_history", "lbfgsb_get_info", "lbfgsb_get_x", "lbfgsb_get_g", "lbfgsb_destroy",
    "lbfgsb_enable_apass_timing", "lbfgsb_apass_timing", "lbfgsb_apass_name", "lbfgsb_dbg_fg",
    "lbfgsb_dbg_free_mask", "lbfgsb_dbg_two_loop", "lbfgsb_dbg_project_direction",
    "lbfgsb_auglag_default_options", "lbfgsb_auglag_workspace_bytes", "lbfgsb_auglag_create", "lbfgsb_auglag_solve",
    "lbfgsb_auglag_get_x", "lbfgsb_auglag_get_lambda", "lbfgsb_auglag_inner", "lbfgsb_auglag_destroy",
    "lbfgsb_auglag_rows_workspace_bytes", "lbfgsb_auglag_create_rows",
    "lbfgsb_auglag_marginals_workspace_bytes", "lbfgsb_auglag_create_marginals",
]


class Objective(C.Structure):
    _fields_ = [("kind", C.c_int), ("dtype", C.c_int), ("rows", C.c_int64), ("cols", C.c_int64),
                ("ld", C.c_int64), ("A", C.c_void_p), ("b", C.c_void_p), ("lam", C.c_double),
                ("mu", C.c_double), ("row_weight", C.c_void_p), ("sign", C.c_void_p), ("n_extra", C.c_int64),
                ("extra_rows", C.c_void_p), ("extra_target", C.c_void_p), ("extra_weight", C.c_void_p)]


class AuglagOptions(C.Structure):
    _fields_ = [("rho0", C.c_double), ("ctol", C.c_double), ("max_outer", C.c_int)]


class AuglagInfo(C.Structure):
    _fields_ = [("status", C.c_int), ("outer", C.c_int), ("inner_iters", C.c_int64), ("violation", C.c_double),
                ("rho", C.c_double), ("f", C.c_double), ("L", C.c_double), ("pg2", C.c_double)]

    def as_dict(self) -> dict:
        return {name: getattr(self, name) for name, _ in self._fields_}


class Options(C.Structure):
    _fields_ = [("eps", C.c_double), ("armijo_c1", C.c_double), ("backtrack", C.c_double),
                ("max_backtracks", C.c_int), ("tol", C.c_double), ("tol_relative", C.c_int),
                ("max_iter", C.c_int), ("refresh_every", C.c_int), ("poll_every", C.c_int),
                ("a_pass", C.c_int)]


class Info(C.Structure):
    _fields_ = [("status", C.c_int), ("iters", C.c_int64), ("fevals", C.c_int64), ("f", C.c_double),
                ("pg2", C.c_double), ("pginf", C.c_double), ("n_fixed", C.c_int64), ("branch", C.c_int),
                ("backtracks", C.c_int), ("pairs_used", C.c_int), ("memory_resets", C.c_int),
                ("alpha", C.c_double), ("alpha_ub", C.c_double), ("gp", C.c_double)]

    def as_dict(self) -> dict:
        return {name: getattr(self, name) for name, _ in self._fields_}


HISTORY_CAPACITY = 256


class IterRecord(C.Structure):
    _fields_ = [("iter", C.c_int64), ("f", C.c_double), ("pg2", C.c_double), ("pginf", C.c_double),
                ("n_fixed", C.c_int64), ("alpha", C.c_double), ("alpha_ub", C.c_double), ("gp", C.c_double),
                ("branch", C.c_int), ("backtracks", C.c_int), ("pairs_used", C.c_int), ("memory_resets", C.c_int)]

    def as_dict(self) -> dict:
        return {name: getattr(self, name) for name, _ in self._fields_}


class LbfgsbError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"liblbfgsb error {code}: {message}")
        self.code = code


_lib = None


def lib():
    """The loaded C-ABI library.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2203_16340_amd.build`; "
                               "there is no fallback path")
        L = C.CDLL(LIB_PATH)
        vp, i64, dbl = C.c_void_p, C.c_int64, C.c_double
        L.lbfgsb_last_error.restype = C.c_char_p
        L.lbfgsb_last_error.argtypes = []
        L.lbfgsb_default_options.restype = None
        L.lbfgsb_default_options.argtypes = [C.POINTER(Options)]
        L.lbfgsb_workspace_bytes.restype = C.c_size_t
        L.lbfgsb_workspace_bytes.argtypes = [i64, C.c_int, C.POINTER(Objective), C.POINTER(Options)]
        L.lbfgsb_create.restype = C.c_int
        L.lbfgsb_create.argtypes = [C.POINTER(vp), i64, C.c_int, vp, vp, C.POINTER(Objective), C.POINTER(Options),
                                    vp, C.c_size_t, vp]
        L.lbfgsb_set_x.restype = C.c_int
        L.lbfgsb_set_x.argtypes = [vp, vp]
        L.lbfgsb_step.restype = C.c_int
        L.lbfgsb_step.argtypes = [vp, C.POINTER(Info)]
        L.lbfgsb_solve.restype = C.c_int
        L.lbfgsb_solve.argtypes = [vp, C.POINTER(Info)]
        L.lbfgsb_solve_static.restype = C.c_int
        L.lbfgsb_solve_static.argtypes = [i64, C.c_int, vp, vp, C.POINTER(Objective), C.POINTER(Options), vp,
                                          C.POINTER(Info), vp]
        L.lbfgsb_get_info.restype = C.c_int
        L.lbfgsb_get_info.argtypes = [vp, C.POINTER(Info)]
        L.lbfgsb_get_history.restype = C.c_int
        L.lbfgsb_get_history.argtypes = [vp, C.POINTER(IterRecord), C.c_int, C.POINTER(C.c_int)]
        L.lbfgsb_get_x.restype = C.c_int
        L.lbfgsb_get_x.argtypes = [vp, vp]
        L.lbfgsb_get_g.restype = C.c_int
        L.lbfgsb_get_g.argtypes = [vp, vp]
        L.lbfgsb_destroy.restype = None
        L.lbfgsb_destroy.argtypes = [vp]
        L.lbfgsb_enable_apass_timing.restype = C.c_int
        L.lbfgsb_enable_apass_timing.argtypes = [vp, C.c_int]
        L.lbfgsb_apass_timing.restype = C.c_int
        L.lbfgsb_apass_timing.argtypes = [vp, C.POINTER(i64), C.POINTER(dbl), C.POINTER(dbl)]
        L.lbfgsb_apass_name.restype = C.c_char_p
        L.lbfgsb_apass_name.argtypes = [vp]
        L.lbfgsb_dbg_fg.restype = C.c_int
        L.lbfgsb_dbg_fg.argtypes = [vp, vp, C.POINTER(dbl), vp, vp]
        L.lbfgsb_dbg_free_mask.restype = C.c_int
        L.lbfgsb_dbg_free_mask.argtypes = [vp, vp, vp, vp]
        L.lbfgsb_dbg_two_loop.restype = C.c_int
        L.lbfgsb_dbg_two_loop.argtypes = [vp, vp, vp, vp, C.c_int, vp, vp, vp, C.POINTER(C.c_int)]
        L.lbfgsb_dbg_project_direction.restype = C.c_int
        L.lbfgsb_dbg_project_direction.argtypes = [vp, vp, vp, vp, vp, C.POINTER(C.c_int), C.POINTER(dbl)]
        L.lbfgsb_auglag_default_options.restype = None
        L.lbfgsb_auglag_default_options.argtypes = [C.POINTER(AuglagOptions)]
        L.lbfgsb_auglag_workspace_bytes.restype = C.c_size_t
        L.lbfgsb_auglag_workspace_bytes.argtypes = [i64, C.c_int, C.POINTER(Objective), i64, C.POINTER(Options)]
        L.lbfgsb_auglag_create.restype = C.c_int
        L.lbfgsb_auglag_create.argtypes = [C.POINTER(vp), i64, C.c_int, vp, vp, C.POINTER(Objective), i64,
                                           C.POINTER(Options), C.POINTER(AuglagOptions), vp, C.c_size_t, vp]
        L.lbfgsb_auglag_rows_workspace_bytes.restype = C.c_size_t
        L.lbfgsb_auglag_rows_workspace_bytes.argtypes = [i64, C.c_int, C.POINTER(Objective), i64, C.POINTER(Options)]
        L.lbfgsb_auglag_create_rows.restype = C.c_int
        L.lbfgsb_auglag_create_rows.argtypes = [C.POINTER(vp), i64, C.c_int, vp, vp, C.POINTER(Objective), i64, vp, vp,
                                                C.POINTER(Options), C.POINTER(AuglagOptions), vp, C.c_size_t, vp]
        L.lbfgsb_auglag_marginals_workspace_bytes.restype = C.c_size_t
        L.lbfgsb_auglag_marginals_workspace_bytes.argtypes = [C.c_int, C.POINTER(Objective), C.POINTER(Options)]
        L.lbfgsb_auglag_create_marginals.restype = C.c_int
        L.lbfgsb_auglag_create_marginals.argtypes = [C.POINTER(vp), C.c_int, vp, vp, C.POINTER(Objective), vp,
                                                     C.POINTER(Options), C.POINTER(AuglagOptions), vp, C.c_size_t, vp]
        L.lbfgsb_auglag_solve.restype = C.c_int
        L.lbfgsb_auglag_solve.argtypes = [vp, vp, C.POINTER(AuglagInfo)]
        L.lbfgsb_auglag_get_x.restype = C.c_int
        L.lbfgsb_auglag_get_x.argtypes = [vp, vp]
        L.lbfgsb_auglag_get_lambda.restype = C.c_int
        L.lbfgsb_auglag_get_lambda.argtypes = [vp, vp]
        L.lbfgsb_auglag_inner.restype = vp
        L.lbfgsb_auglag_inner.argtypes = [vp]
        L.lbfgsb_auglag_destroy.restype = None
        L.lbfgsb_auglag_destroy.argtypes = [vp]
        _lib = L
    return _lib


def _check(rc: int) -> None:
    if rc != OK:
        raise LbfgsbError(rc, lib().lbfgsb_last_error().decode())


def default_options(**overrides) -> Options:
    o = Options()
    lib().lbfgsb_default_options(C.byref(o))
    for k, v in overrides.items():
        if not hasattr(o, k):
            raise AttributeError(k)
        setattr(o, k, v)
    return o


def _dev_f64(t, name: str, numel: Optional[int] = None):
    import torch
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.float64 and t.is_contiguous()):
        raise TypeError(f"{name} must be a contiguous float64 tensor on the GPU")
    if numel is not None and t.numel() != numel:
        raise ValueError(f"{name} must have {numel} entries, got {t.numel()}")
    return t


class Solver:
    """lbfgsb_create / lbfgsb_set_x / lbfgsb_step / lbfgsb_solve / lbfgsb_destroy on torch tensors.

    A: (rows, cols) float64 or float32 CUDA tensor with unit column stride; b, l, u: float64 CUDA
    tensors.  The solver keeps references to A and b (the library borrows them) and owns its
    workspace tensor.  All work runs on torch's current stream at construction time.
    """

    def __init__(self, kind: int, A, b, l, u, m: int, *, lam: float = 0.0, mu: float = 0.0,
                 options: Optional[Options] = None, row_weight=None, sign=None, extra=None):
        import torch
        if not (isinstance(A, torch.Tensor) and A.is_cuda and A.dim() == 2 and A.stride(1) == 1
                and A.dtype in (torch.float64, torch.float32)):
            raise TypeError("A must be a 2-d float64/float32 CUDA tensor with unit column stride")
        rows, cols = A.shape
        transport = kind in (OBJ_OT_GAUSS, OBJ_OT_ENTROPY)   # A = cost matrix; b, row_weight: rows + cols marginal terms
        self.n = rows * cols if transport else (2 * cols if kind == OBJ_LSQ_L1SPLIT else cols)
        self.rows, self.cols, self.m, self.kind = rows, cols, m, kind
        self.row_entries = rows + cols if transport else rows
        self._A = A
        self._b = _dev_f64(b, "b", self.row_entries) if (b is not None or not transport) else None
        if kind == OBJ_QP and rows != cols:
            raise ValueError("the quadratic form needs a square matrix")
        _dev_f64(l, "l", self.n)
        _dev_f64(u, "u", self.n)
        self.device = A.device
        self.options = options if options is not None else default_options()
        self._w = _dev_f64(row_weight, "row_weight", self.row_entries) if row_weight is not None else None
        self._sign = _dev_f64(sign, "sign", self.n) if sign is not None else None
        # extra = (rows E: (n_extra, n), targets: n_extra, weights: n_extra or None), float64 CUDA tensors
        self._extra = extra
        n_extra = 0 if extra is None else int(extra[0].shape[0])
        if extra is not None:
            _dev_f64(extra[0], "extra rows", n_extra * self.n)
            _dev_f64(extra[1], "extra targets", n_extra)
            if extra[2] is not None:
                _dev_f64(extra[2], "extra weights", n_extra)
        self._obj = Objective(kind, F64 if A.dtype == torch.float64 else F32, rows, cols,
                              A.stride(0) if rows > 1 else cols, A.data_ptr(),
                              self._b.data_ptr() if self._b is not None else None, float(lam), float(mu),
                              self._w.data_ptr() if self._w is not None else None,
                              self._sign.data_ptr() if self._sign is not None else None, n_extra,
                              extra[0].data_ptr() if n_extra else None, extra[1].data_ptr() if n_extra else None,
                              extra[2].data_ptr() if n_extra and extra[2] is not None else None)
        self._h = C.c_void_p()
        with torch.cuda.device(self.device):
            nbytes = lib().lbfgsb_workspace_bytes(self.n, m, C.byref(self._obj), C.byref(self.options))
            if nbytes == 0:
                raise LbfgsbError(E_INVALID_ARG, lib().lbfgsb_last_error().decode())
            self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
            self._stream = torch.cuda.current_stream(self.device)
            _check(lib().lbfgsb_create(C.byref(self._h), self.n, m, l.data_ptr(), u.data_ptr(), C.byref(self._obj),
                                       C.byref(self.options), self.workspace.data_ptr(), nbytes,
                                       C.c_void_p(self._stream.cuda_stream)))

    # -- lifetime
    def close(self) -> None:
        if getattr(self, "_h", None) is not None and self._h:
            lib().lbfgsb_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    # -- the path
    def set_x(self, x0) -> None:
        _check(lib().lbfgsb_set_x(self._h, _dev_f64(x0, "x0", self.n).data_ptr()))

    def step(self, want_info: bool = True) -> Optional[Info]:
        if want_info:
            info = Info()
            _check(lib().lbfgsb_step(self._h, C.byref(info)))
            return info
        _check(lib().lbfgsb_step(self._h, None))
        return None

    def solve(self) -> Info:
        info = Info()
        _check(lib().lbfgsb_solve(self._h, C.byref(info)))
        return info

    def info(self) -> Info:
        info = Info()
        _check(lib().lbfgsb_get_info(self._h, C.byref(info)))
        return info

    def history(self, capacity: int = HISTORY_CAPACITY):
        """The most recent per-iteration records (oldest first), as a list of IterRecord."""
        buf = (IterRecord * max(1, capacity))()
        cnt = C.c_int(0)
        _check(lib().lbfgsb_get_history(self._h, buf, int(capacity), C.byref(cnt)))
        return [buf[k] for k in range(cnt.value)]

    def _copy_out(self, getter, numel: int):
        """A new tensor filled by a library copy that runs on the SOLVER's stream (the one current when it was
        created).  The tensor is allocated under that stream, and a caller on another stream is made to wait for
        the copy, so the result is safe to use wherever this returns."""
        import torch
        with torch.cuda.stream(self._stream):
            out = torch.empty(numel, dtype=torch.float64, device=self.device)
            _check(getter(self._h, out.data_ptr()))
        cur = torch.cuda.current_stream(self.device)
        if cur != self._stream:
            cur.wait_stream(self._stream)
            out.record_stream(cur)
        return out

    def x(self):
        return self._copy_out(lib().lbfgsb_get_x, self.n)

    def g(self):
        return self._copy_out(lib().lbfgsb_get_g, self.n)

    # -- timing of the A pass
    def enable_apass_timing(self, mode: int = 2) -> None:
        """0 = pause, 1 = resume, 2 = discard the records and start"""
        _check(lib().lbfgsb_enable_apass_timing(self._h, int(mode)))

    def apass_timing(self):
        """(launches timed, total milliseconds, bytes of A one launch reads)"""
        cnt, ms, by = C.c_int64(0), C.c_double(0.0), C.c_double(0.0)
        _check(lib().lbfgsb_apass_timing(self._h, C.byref(cnt), C.byref(ms), C.byref(by)))
        return cnt.value, ms.value, by.value

    @property
    def apass_name(self) -> str:
        return lib().lbfgsb_apass_name(self._h).decode()

    # -- primitive-level hooks
    def dbg_fg(self, x, want_rowvec: bool = False):
        import torch
        g = torch.empty(self.n, dtype=torch.float64, device=self.device)
        row = torch.empty(self.row_entries, dtype=torch.float64, device=self.device) if want_rowvec else None
        f = C.c_double(0.0)
        _check(lib().lbfgsb_dbg_fg(self._h, _dev_f64(x, "x", self.n).data_ptr(), C.byref(f), g.data_ptr(),
                                   row.data_ptr() if row is not None else None))
        return (f.value, g, row) if want_rowvec else (f.value, g)

    def dbg_free_mask(self, x, g):
        import torch
        mask = torch.empty(self.n, dtype=torch.uint8, device=self.device)
        _check(lib().lbfgsb_dbg_free_mask(self._h, _dev_f64(x, "x", self.n).data_ptr(),
                                          _dev_f64(g, "g", self.n).data_ptr(), mask.data_ptr()))
        return mask

    def dbg_two_loop(self, S, Y, ynorm2, g, mask):
        import torch
        npairs = 0 if S is None else S.shape[0]
        d = torch.empty(self.n, dtype=torch.float64, device=self.device)
        used = C.c_int(0)
        if not (mask.is_cuda and mask.dtype == torch.uint8 and mask.is_contiguous() and mask.numel() == self.n):
            raise TypeError("mask must be a contiguous uint8 CUDA tensor with n entries")
        sp = _dev_f64(S, "S", npairs * self.n).data_ptr() if npairs else None
        yp = _dev_f64(Y, "Y", npairs * self.n).data_ptr() if npairs else None
        np_ = _dev_f64(ynorm2, "ynorm2", npairs).data_ptr() if npairs else None
        _check(lib().lbfgsb_dbg_two_loop(self._h, sp, yp, np_, npairs, _dev_f64(g, "g", self.n).data_ptr(),
                                         mask.data_ptr(), d.data_ptr(), C.byref(used)))
        return d, used.value

    def dbg_project_direction(self, x, g, d):
        import torch
        p = torch.empty(self.n, dtype=torch.float64, device=self.device)
        br, ub = C.c_int(0), C.c_double(0.0)
        _check(lib().lbfgsb_dbg_project_direction(self._h, _dev_f64(x, "x", self.n).data_ptr(),
                                                  _dev_f64(g, "g", self.n).data_ptr(),
                                                  _dev_f64(d, "d", self.n).data_ptr(), p.data_ptr(), C.byref(br),
                                                  C.byref(ub)))
        return p, br.value, ub.value


class Auglag:
    """lbfgsb_auglag_*: Algorithm 4 for  min 0.5||A x - b||^2  s.t.  C x = d, l <= x <= u.

    A_stacked: (data rows + n_eq, cols) CUDA tensor holding [A; C]; b_stacked: [b; d] (float64 CUDA)."""

    def __init__(self, A_stacked, b_stacked, n_eq: int, l, u, m: int, *, options: Optional[Options] = None,
                 rho0: float = 1.0, ctol: float = 1e-8, max_outer: int = 100):
        import torch
        A = A_stacked
        if not (isinstance(A, torch.Tensor) and A.is_cuda and A.dim() == 2 and A.stride(1) == 1
                and A.dtype in (torch.float64, torch.float32)):
            raise TypeError("A_stacked must be a 2-d float64/float32 CUDA tensor with unit column stride")
        rows, cols = A.shape
        self.n, self.n_eq, self.m = cols, int(n_eq), m
        self._A, self._b = A, _dev_f64(b_stacked, "b_stacked", rows)
        _dev_f64(l, "l", cols)
        _dev_f64(u, "u", cols)
        self.device = A.device
        self.options = options if options is not None else default_options()
        self.al_options = AuglagOptions(float(rho0), float(ctol), int(max_outer))
        self._obj = Objective(OBJ_LSQ, F64 if A.dtype == torch.float64 else F32, rows, cols,
                              A.stride(0) if rows > 1 else cols, A.data_ptr(), self._b.data_ptr(), 0.0, 0.0, None, None, 0,
                              None, None, None)
        self._h = C.c_void_p()
        with torch.cuda.device(self.device):
            nbytes = lib().lbfgsb_auglag_workspace_bytes(self.n, m, C.byref(self._obj), self.n_eq, C.byref(self.options))
            if nbytes == 0:
                raise LbfgsbError(E_INVALID_ARG, lib().lbfgsb_last_error().decode())
            self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
            self._stream = torch.cuda.current_stream(self.device)
            _check(lib().lbfgsb_auglag_create(C.byref(self._h), self.n, m, l.data_ptr(), u.data_ptr(),
                                              C.byref(self._obj), self.n_eq, C.byref(self.options),
                                              C.byref(self.al_options), self.workspace.data_ptr(), nbytes,
                                              C.c_void_p(self._stream.cuda_stream)))

    def close(self) -> None:
        if getattr(self, "_h", None) is not None and self._h:
            lib().lbfgsb_auglag_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def solve(self, x0) -> AuglagInfo:
        info = AuglagInfo()
        _check(lib().lbfgsb_auglag_solve(self._h, _dev_f64(x0, "x0", self.n).data_ptr(), C.byref(info)))
        return info

    def x(self):
        return Solver._copy_out(self, lib().lbfgsb_auglag_get_x, self.n)

    def lam(self):
        return Solver._copy_out(self, lib().lbfgsb_auglag_get_lambda, max(self.n_eq, 1))[:self.n_eq]

    def inner_apass_timing(self, mode: Optional[int] = None):
        """mode given: lbfgsb_enable_apass_timing on the inner solver; else its (launches, ms, bytes per launch)"""
        h = lib().lbfgsb_auglag_inner(self._h)
        if mode is not None:
            _check(lib().lbfgsb_enable_apass_timing(h, int(mode)))
            return None
        cnt, ms, by = C.c_int64(0), C.c_double(0.0), C.c_double(0.0)
        _check(lib().lbfgsb_apass_timing(h, C.byref(cnt), C.byref(ms), C.byref(by)))
        return cnt.value, ms.value, by.value


def stack_constraints(A, b, C_eq, d, E_in, e, l, u, x0):
    """Host-side layout of a linearly constrained least-squares problem  min 0.5||A x - b||^2  s.t.  C x = d,
    E x <= e, l <= x <= u  as lbfgsb_auglag_create takes it (numpy arrays in, numpy arrays out; no solver arithmetic):
    equality rows appended to A, and one slack column s_r >= 0 per inequality row so that E x + s = e is an equality
    too (minimising the augmented Lagrangian of Eq. (augLag) over s_r gives exactly its (.)_+ term).  Variables
    [x; s], rows [A 0; C 0; E I], targets [b; d; e], bounds [l; 0] <= [x; s] <= [u; inf], start [x0; max(e - E x0, 0)].
    Returns (A_stacked, b_stacked, n_eq_total, l, u, x0)."""
    import math
    import numpy as np
    n, ne, ni = A.shape[1], C_eq.shape[0], E_in.shape[0]
    top = np.hstack([A, np.zeros((A.shape[0], ni), dtype=A.dtype)])
    mid = np.hstack([C_eq.astype(A.dtype), np.zeros((ne, ni), dtype=A.dtype)])
    bot = np.hstack([E_in.astype(A.dtype), np.eye(ni, dtype=A.dtype)])
    A_s = np.ascontiguousarray(np.vstack([top, mid, bot]))
    b_s = np.concatenate([b, d, e])
    l_s = np.concatenate([l, np.zeros(ni)])
    u_s = np.concatenate([u, np.full(ni, math.inf)])
    s0 = np.maximum(e - E_in @ x0, 0.0) if ni else np.zeros(0)
    return A_s, b_s, ne + ni, l_s, u_s, np.concatenate([x0, s0])


class AuglagRows(Auglag):
    """lbfgsb_auglag_create_rows: Algorithm 4 with the constraint rows C x = d passed separately, on top of a
    quadratic objective kind given as it is (e.g. OBJ_QP with the kernel matrix for the dual SVM)."""

    def __init__(self, kind: int, A, b, C_rows, d, l, u, m: int, *, sign=None, lam: float = 0.0,
                 options: Optional[Options] = None, rho0: float = 1.0, ctol: float = 1e-8, max_outer: int = 100):
        import torch
        if not (isinstance(A, torch.Tensor) and A.is_cuda and A.dim() == 2 and A.stride(1) == 1
                and A.dtype in (torch.float64, torch.float32)):
            raise TypeError("A must be a 2-d float64/float32 CUDA tensor with unit column stride")
        rows, cols = A.shape
        self.n = 2 * cols if kind == OBJ_LSQ_L1SPLIT else cols
        self.n_eq, self.m = int(C_rows.shape[0]), m
        self._A, self._b = A, _dev_f64(b, "b", rows)
        self._C = _dev_f64(C_rows, "C", self.n_eq * self.n)
        self._d = _dev_f64(d, "d", self.n_eq)
        self._sign = _dev_f64(sign, "sign", self.n) if sign is not None else None
        _dev_f64(l, "l", self.n)
        _dev_f64(u, "u", self.n)
        self.device = A.device
        self.options = options if options is not None else default_options()
        self.al_options = AuglagOptions(float(rho0), float(ctol), int(max_outer))
        self._obj = Objective(kind, F64 if A.dtype == torch.float64 else F32, rows, cols,
                              A.stride(0) if rows > 1 else cols, A.data_ptr(), self._b.data_ptr(), float(lam), 0.0, None,
                              self._sign.data_ptr() if self._sign is not None else None, 0, None, None, None)
        self._h = C.c_void_p()
        with torch.cuda.device(self.device):
            nbytes = lib().lbfgsb_auglag_rows_workspace_bytes(self.n, m, C.byref(self._obj), self.n_eq,
                                                              C.byref(self.options))
            if nbytes == 0:
                raise LbfgsbError(E_INVALID_ARG, lib().lbfgsb_last_error().decode())
            self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
            self._stream = torch.cuda.current_stream(self.device)
            _check(lib().lbfgsb_auglag_create_rows(C.byref(self._h), self.n, m, l.data_ptr(), u.data_ptr(),
                                                   C.byref(self._obj), self.n_eq,
                                                   self._C.data_ptr() if self.n_eq else None,
                                                   self._d.data_ptr() if self.n_eq else None, C.byref(self.options),
                                                   C.byref(self.al_options), self.workspace.data_ptr(), nbytes,
                                                   C.c_void_p(self._stream.cuda_stream)))


class AuglagMarginals(Auglag):
    """lbfgsb_auglag_create_marginals: Algorithm 4 for  min <M,P> + lam r(P)  s.t.  P 1 = u, P^T 1 = v, l <= P <= ub
    (kind OBJ_OT_GAUSS or OBJ_OT_ENTROPY).  M: (rows, cols) CUDA tensor; marginals: [u; v] (float64 CUDA);
    l, ub and x0: rows*cols entries, row-major."""

    def __init__(self, kind: int, M, marginals, l, u, m: int, *, lam: float, options: Optional[Options] = None,
                 rho0: float = 1.0, ctol: float = 1e-8, max_outer: int = 100):
        import torch
        if not (isinstance(M, torch.Tensor) and M.is_cuda and M.dim() == 2 and M.stride(1) == 1
                and M.dtype in (torch.float64, torch.float32)):
            raise TypeError("M must be a 2-d float64/float32 CUDA tensor with unit column stride")
        rows, cols = M.shape
        self.n, self.n_eq, self.m = rows * cols, rows + cols, m
        self._A = M
        self._d = _dev_f64(marginals, "marginals", rows + cols)
        _dev_f64(l, "l", self.n)
        _dev_f64(u, "u", self.n)
        self.device = M.device
        self.options = options if options is not None else default_options()
        self.al_options = AuglagOptions(float(rho0), float(ctol), int(max_outer))
        self._obj = Objective(kind, F64 if M.dtype == torch.float64 else F32, rows, cols,
                              M.stride(0) if rows > 1 else cols, M.data_ptr(), None, float(lam), 0.0, None, None, 0,
                              None, None, None)
        self._h = C.c_void_p()
        with torch.cuda.device(self.device):
            nbytes = lib().lbfgsb_auglag_marginals_workspace_bytes(m, C.byref(self._obj), C.byref(self.options))
            if nbytes == 0:
                raise LbfgsbError(E_INVALID_ARG, lib().lbfgsb_last_error().decode())
            self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
            self._stream = torch.cuda.current_stream(self.device)
            _check(lib().lbfgsb_auglag_create_marginals(C.byref(self._h), m, l.data_ptr(), u.data_ptr(),
                                                        C.byref(self._obj), self._d.data_ptr(), C.byref(self.options),
                                                        C.byref(self.al_options), self.workspace.data_ptr(), nbytes,
                                                        C.c_void_p(self._stream.cuda_stream)))


STATIC_SCRATCH_BYTES = 32 << 20


def solve_static(kind: int, A, b, l, u, m: int, x, *, lam: float = 0.0, mu: float = 0.0,
                 options: Optional[Options] = None) -> Info:
    """lbfgsb_solve_static: the whole solve in one call that allocates nothing (the workspace is a fixed array inside
    the library).  x: float64 CUDA tensor, in: the start point, out: the result (overwritten in place).  Runs on
    torch's current stream; no tensor is created here either."""
    import torch
    if not (isinstance(A, torch.Tensor) and A.is_cuda and A.dim() == 2 and A.stride(1) == 1
            and A.dtype in (torch.float64, torch.float32)):
        raise TypeError("A must be a 2-d float64/float32 CUDA tensor with unit column stride")
    rows, cols = A.shape
    n = 2 * cols if kind == OBJ_LSQ_L1SPLIT else cols
    _dev_f64(b, "b", rows)
    _dev_f64(l, "l", n)
    _dev_f64(u, "u", n)
    _dev_f64(x, "x", n)
    opts = options if options is not None else default_options()
    obj = Objective(kind, F64 if A.dtype == torch.float64 else F32, rows, cols, A.stride(0) if rows > 1 else cols,
                    A.data_ptr(), b.data_ptr(), float(lam), float(mu), None, None, 0, None, None, None)
    info = Info()
    with torch.cuda.device(A.device):
        stream = torch.cuda.current_stream(A.device)
        _check(lib().lbfgsb_solve_static(n, m, l.data_ptr(), u.data_ptr(), C.byref(obj), C.byref(opts), x.data_ptr(),
                                         C.byref(info), C.c_void_p(stream.cuda_stream)))
    return info


def solver_for_problem(prob, device="cuda:0", **option_overrides) -> Solver:
    """Uploads a workloads.Problem and creates a solver positioned at its x0."""
    import torch
    dev = torch.device(device)
    A = torch.from_numpy(prob.A).to(dev)
    b = torch.from_numpy(prob.b).to(dev)
    l = torch.from_numpy(prob.l).to(dev)
    u = torch.from_numpy(prob.u).to(dev)
    opts = default_options(tol=prob.tol, tol_relative=int(prob.tol_relative), max_iter=int(getattr(prob, "max_iter", 1000)))
    for k, v in option_overrides.items():
        if not hasattr(opts, k):
            raise AttributeError(k)
        setattr(opts, k, v)
    s = Solver(prob.kind, A, b, l, u, prob.m, lam=prob.lam, mu=prob.mu, options=opts)
    s.set_x(torch.from_numpy(prob.x0).to(dev))
    return s
