"""Seeded synthetic inputs for the box-constrained solver: the five benchmark
configurations and scaled-down relatives of them.

This module is shared by the CPU oracle's tests and by the HIP path's tests and
benchmark.  It only draws random numbers and assembles arrays; it contains none of
the solver's arithmetic beyond what is needed to *define* the data (b = A x* + noise,
labels = sign(X w* + noise), lambda = 0.1 * ||A^T b||_inf).

Draw order, fixed for reproducibility: matrix, support of the ground truth, its
non-zero values, noise.  The matrix is drawn row-chunk by row-chunk directly in its
storage dtype so that the 8 GB configuration never needs an fp64 temporary.

The NNLS family follows the paper's experiment (ii) of its non-negative least squares
section (tall Gaussian design, sparse non-negative ground truth, small Gaussian
noise); `paper_nnls_i` / `paper_nnls_ii` reproduce the two recipes of that section
with their printed scalings.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

OBJ_LSQ = 0          # 0.5*||A x - b||^2,                                   n = cols
OBJ_LSQ_L1SPLIT = 1  # 0.5*||A(p-q) - b||^2 + lam*sum(p+q), x = [p; q],     n = 2*cols
OBJ_LOGISTIC_L2 = 2  # (1/rows)*sum softplus(-y_i * X_i.w) + mu/2*||w||^2,  n = cols


@dataclass
class Problem:
    name: str
    kind: int
    A: np.ndarray            # rows x cols, C-contiguous, float64 or float32
    b: np.ndarray            # rows, float64 (targets, or labels in {-1,+1})
    l: np.ndarray            # n, float64 (may hold -inf)
    u: np.ndarray            # n, float64 (may hold +inf)
    x0: np.ndarray           # n, float64, feasible
    m: int                   # number of stored curvature pairs
    lam: float = 0.0
    mu: float = 0.0
    tol: float = 1e-8
    tol_relative: bool = False
    x_true: Optional[np.ndarray] = None
    meta: dict = field(default_factory=dict)
    max_iter: int = 1000

    @property
    def rows(self) -> int:
        return self.A.shape[0]

    @property
    def cols(self) -> int:
        return self.A.shape[1]

    @property
    def n(self) -> int:
        return 2 * self.cols if self.kind == OBJ_LSQ_L1SPLIT else self.cols


def _normal_matrix(rng: np.random.Generator, rows: int, cols: int, dtype, scale: float = 1.0,
                   out: Optional[np.ndarray] = None) -> np.ndarray:
    """rows x cols iid N(0, scale^2) in `dtype`, drawn in row chunks of <= 64 MiB."""
    A = out if out is not None else np.empty((rows, cols), dtype=dtype)
    chunk = max(1, (64 << 20) // (cols * A.itemsize))
    for r0 in range(0, rows, chunk):
        r1 = min(rows, r0 + chunk)
        blk = rng.standard_normal((r1 - r0, cols), dtype=A.dtype)
        if scale != 1.0:
            blk *= A.dtype.type(scale)
        A[r0:r1] = blk
    return A


def _matvec(A: np.ndarray, x: np.ndarray) -> np.ndarray:
    """A @ x accumulated in float64, in row chunks (data definition, not solver code)."""
    rows, cols = A.shape
    out = np.empty(rows, dtype=np.float64)
    chunk = max(1, (256 << 20) // (cols * 8))
    nz = np.flatnonzero(x)
    xs = x[nz]
    for r0 in range(0, rows, chunk):
        r1 = min(rows, r0 + chunk)
        out[r0:r1] = A[r0:r1][:, nz].astype(np.float64) @ xs
    return out


def _rmatvec(A: np.ndarray, v: np.ndarray) -> np.ndarray:
    rows, cols = A.shape
    out = np.zeros(cols, dtype=np.float64)
    chunk = max(1, (256 << 20) // (cols * 8))
    for r0 in range(0, rows, chunk):
        r1 = min(rows, r0 + chunk)
        out += v[r0:r1] @ A[r0:r1].astype(np.float64)
    return out


def nnls(rows: int, cols: int, *, seed: int, dtype=np.float64, zero_frac: float, nonzero: str,
         noise: float = 0.01, upper: float = math.inf, m: int = 10, name: str = "nnls",
         tol: float = 1e-8, tol_relative: bool = False, a_out: Optional[np.ndarray] = None) -> Problem:
    """min 0.5*||A x - b||^2  s.t. 0 <= x <= upper.  A iid N(0,1); x* has round(zero_frac*cols)
    zeros on a uniformly random support complement; non-zeros |N(0,1)| ("absnormal") or
    U(0,1) ("uniform"); b = A x* + noise*N(0,1)."""
    rng = np.random.default_rng(seed)
    A = _normal_matrix(rng, rows, cols, np.dtype(dtype), out=a_out)
    n_zero = int(round(zero_frac * cols))
    perm = rng.permutation(cols)
    support = np.sort(perm[n_zero:])
    x_true = np.zeros(cols)
    if nonzero == "absnormal":
        x_true[support] = np.abs(rng.standard_normal(support.size))
    elif nonzero == "uniform":
        x_true[support] = rng.random(support.size)
    else:
        raise ValueError(nonzero)
    b = _matvec(A, x_true) + noise * rng.standard_normal(rows)
    return Problem(name=name, kind=OBJ_LSQ, A=A, b=b, l=np.zeros(cols), u=np.full(cols, upper),
                   x0=np.zeros(cols), m=m, tol=tol, tol_relative=tol_relative, x_true=x_true,
                   meta=dict(seed=seed, zero_frac=zero_frac, nonzero=nonzero, noise=noise))


def l1_split(rows: int, cols: int, *, seed: int, nnz_frac: float = 0.01, noise: float = 0.01,
             lam_frac: float = 0.1, m: int = 10, name: str = "l1split", tol: float = 1e-8,
             tol_relative: bool = False) -> Problem:
    """L1-regularised least squares written as a box problem through x = p - q, p, q >= 0:
    min 0.5*||A(p-q) - b||^2 + lam*sum(p+q).  A iid N(0,1)/sqrt(rows); x* has
    round(nnz_frac*cols) N(0,1) non-zeros; b = A x* + noise*N(0,1);
    lam = lam_frac*||A^T b||_inf."""
    rng = np.random.default_rng(seed)
    A = _normal_matrix(rng, rows, cols, np.dtype(np.float64), scale=1.0 / math.sqrt(rows))
    nnz = int(round(nnz_frac * cols))
    support = np.sort(rng.permutation(cols)[:nnz])
    x_true = np.zeros(cols)
    x_true[support] = rng.standard_normal(nnz)
    b = _matvec(A, x_true) + noise * rng.standard_normal(rows)
    lam = lam_frac * float(np.max(np.abs(_rmatvec(A, b))))
    n = 2 * cols
    return Problem(name=name, kind=OBJ_LSQ_L1SPLIT, A=A, b=b, l=np.zeros(n), u=np.full(n, math.inf),
                   x0=np.zeros(n), m=m, lam=lam, tol=tol, tol_relative=tol_relative, x_true=x_true,
                   meta=dict(seed=seed, nnz_frac=nnz_frac, noise=noise, lam_frac=lam_frac))


def logistic(rows: int, cols: int, *, seed: int, dtype=np.float32, label_noise: float = 0.5,
             mu: float = 1e-3, bound: float = 0.5, m: int = 10, name: str = "logistic",
             tol: float = 1e-8, tol_relative: bool = False, feature_scale: float = 1.0,
             column_spread: float = 0.0, random_start: bool = False) -> Problem:
    """Box-constrained L2-regularised logistic regression:
    min (1/rows)*sum_i softplus(-y_i * X_i.w) + mu/2*||w||^2  s.t. -bound <= w <= bound.
    X iid N(0,1); w* N(0,1); y = sign(X w* + label_noise*N(0,1)) in {-1,+1}.

    Badly scaled variants (for the line search: unit steps overshoot and have to be halved): after the labels
    are fixed, column j of X is multiplied by feature_scale * 10^(column_spread * U(-1,1)); random_start
    draws x0 uniformly in the box instead of 0.  With the defaults nothing more is drawn and X is untouched."""
    rng = np.random.default_rng(seed)
    X = _normal_matrix(rng, rows, cols, np.dtype(dtype))
    w_true = rng.standard_normal(cols)
    score = _matvec(X, w_true) + label_noise * rng.standard_normal(rows)
    y = np.where(score >= 0.0, 1.0, -1.0)
    x0 = np.zeros(cols)
    if feature_scale != 1.0 or column_spread != 0.0:
        col_scale = feature_scale * 10.0 ** (column_spread * rng.uniform(-1.0, 1.0, cols))
        X *= col_scale.astype(X.dtype)[None, :]
    if random_start:
        x0 = rng.uniform(-bound, bound, cols)
    return Problem(name=name, kind=OBJ_LOGISTIC_L2, A=X, b=y, l=np.full(cols, -bound),
                   u=np.full(cols, bound), x0=x0, m=m, mu=mu, tol=tol,
                   tol_relative=tol_relative, x_true=w_true,
                   meta=dict(seed=seed, label_noise=label_noise, bound=bound, feature_scale=feature_scale,
                             column_spread=column_spread, random_start=random_start))


def spectrum_lsq(rows: int, cols: int, *, seed: int, sigma_min: float, sigma_max: float, lower: float = -math.inf,
                 m: int = 5, name: str = "spectrum_lsq") -> Problem:
    """Least squares with a prescribed spectrum: A = U diag(sigma) V^T with U (rows x cols) and V (cols x cols)
    orthonormal (QR of Gaussian matrices) and sigma log-uniform in [sigma_min, sigma_max]; b = 5*N(0,1).
    With sigma_max^2 < 2 a unit steepest-descent step always satisfies the Armijo condition while unit
    quasi-Newton steps sometimes do not, which is what the tests of an exhausted line search need.
    Draw order: U's Gaussian, V's Gaussian, sigma, b."""
    rng = np.random.default_rng(seed)
    U, _ = np.linalg.qr(rng.standard_normal((rows, cols)))
    V, _ = np.linalg.qr(rng.standard_normal((cols, cols)))
    sigma = np.exp(rng.uniform(math.log(sigma_min), math.log(sigma_max), cols))
    A = np.ascontiguousarray((U * sigma) @ V.T)
    b = 5.0 * rng.standard_normal(rows)
    return Problem(name=name, kind=OBJ_LSQ, A=A, b=b, l=np.full(cols, lower), u=np.full(cols, math.inf),
                   x0=np.zeros(cols) if lower <= 0.0 else np.full(cols, lower), m=m, tol=1e-9,
                   meta=dict(seed=seed, sigma_min=sigma_min, sigma_max=sigma_max))


def paper_nnls_i(t: float, *, seed: int, m: int = 10) -> Problem:
    """The paper's NNLS experiment (i): A in R^{2000t x 6000t} with U(0,1) entries, x with
    N(0,1) non-zeros at sparsity 0.01, y = sqrt(0.003)*A x + 0.003*z."""
    rows, cols = int(round(2000 * t)), int(round(6000 * t))
    rng = np.random.default_rng(seed)
    A = rng.random((rows, cols))
    nnz = max(1, int(round(0.01 * cols)))
    support = np.sort(rng.permutation(cols)[:nnz])
    x_true = np.zeros(cols)
    x_true[support] = rng.standard_normal(nnz)
    b = math.sqrt(0.003) * _matvec(A, x_true) + 0.003 * rng.standard_normal(rows)
    return Problem(name=f"paper_nnls_i_t{t}", kind=OBJ_LSQ, A=A, b=b, l=np.zeros(cols),
                   u=np.full(cols, math.inf), x0=np.zeros(cols), m=m, tol=1e-6, tol_relative=True,
                   x_true=x_true, meta=dict(seed=seed, t=t))


def paper_nnls_ii(t: float, *, seed: int, m: int = 10) -> Problem:
    """The paper's NNLS experiment (ii): A in R^{6000t x 3000t} Gaussian, x at sparsity 0.1
    (taken as 10 % non-zeros, |N(0,1)|), y = sqrt(1/6000)*A x + 0.003*z."""
    rows, cols = int(round(6000 * t)), int(round(3000 * t))
    rng = np.random.default_rng(seed)
    A = _normal_matrix(rng, rows, cols, np.dtype(np.float64))
    nnz = max(1, int(round(0.1 * cols)))
    support = np.sort(rng.permutation(cols)[:nnz])
    x_true = np.zeros(cols)
    x_true[support] = np.abs(rng.standard_normal(nnz))
    b = math.sqrt(1.0 / 6000.0) * _matvec(A, x_true) + 0.003 * rng.standard_normal(rows)
    return Problem(name=f"paper_nnls_ii_t{t}", kind=OBJ_LSQ, A=A, b=b, l=np.zeros(cols),
                   u=np.full(cols, math.inf), x0=np.zeros(cols), m=m, tol=1e-6, tol_relative=True,
                   x_true=x_true, meta=dict(seed=seed, t=t))


# ---- the five benchmark configurations -------------------------------------------------------

CONFIG_SEEDS = {"C1": 1001, "C2": 1002, "C3": 1003, "C4": 1004, "C5": 1005}


def config(name: str, *, scale: float = 1.0, a_out: Optional[np.ndarray] = None) -> Problem:
    """C1..C5 at full size (scale=1) or with both matrix dimensions multiplied by `scale`
    (same seed, same recipe) for parity cases the CPU oracle finishes in seconds."""
    def dim(v: int) -> int:
        return max(4, int(round(v * scale)))
    seed = CONFIG_SEEDS.get(name, 0)
    if name == "C1":
        return nnls(dim(200), dim(100), seed=seed, zero_frac=0.5, nonzero="absnormal", m=5,
                    name="C1", tol=1e-8, tol_relative=False)
    if name == "C2":
        return nnls(dim(20000), dim(5000), seed=seed, zero_frac=0.8, nonzero="uniform", m=10,
                    name="C2", tol=1e-6, tol_relative=True, a_out=a_out)
    if name == "C3":
        return l1_split(dim(10000), dim(20000), seed=seed, nnz_frac=0.01, m=10, name="C3",
                        tol=1e-6, tol_relative=True)
    if name == "C4":
        return logistic(dim(200000), dim(2000), seed=seed, dtype=np.float32, m=10, name="C4",
                        tol=1e-6, tol_relative=True)
    if name == "C5":
        return nnls(dim(100000), dim(20000), seed=seed, dtype=np.float32, zero_frac=0.9,
                    nonzero="uniform", upper=1.0, m=20, name="C5", tol=1e-6, tol_relative=True,
                    a_out=a_out)
    # the paper's own NNLS recipes (section "Experiments"); `scale` multiplies the paper's parameter t.
    # The paper's tables index instances by a "size" it does not define; the t values here make
    # rows + cols equal to the largest size of each table (11600 and 44400), P2b makes rows equal to it.
    if name == "P1":
        p = paper_nnls_i(1.45 * scale, seed=2001)            # 2900 x 8700, U(0,1) entries, singular Gram matrix
        p.max_iter = 200000                                  # non-isotropic rows: thousands of iterations
    elif name == "P2":
        p = paper_nnls_ii(44400.0 / 9000.0 * scale, seed=2002)   # 29600 x 14800 Gaussian
    elif name == "P2b":
        p = paper_nnls_ii(7.4 * scale, seed=2003)            # 44400 x 22200 Gaussian (7.9 GB): wider than the fused pass takes
    else:
        raise KeyError(name)
    p.name = name
    return p


# ---- linearly constrained least squares (for the augmented Lagrangian algorithm) ---------------

@dataclass
class ConstrainedProblem:
    """min 0.5*||A x - b||^2  s.t.  C x = d,  E x <= e,  l <= x <= u."""
    name: str
    A: np.ndarray
    b: np.ndarray
    C: np.ndarray            # n_eq x cols
    d: np.ndarray
    E: np.ndarray            # n_in x cols
    e: np.ndarray
    l: np.ndarray
    u: np.ndarray
    x0: np.ndarray
    m: int
    x_true: Optional[np.ndarray] = None

    @property
    def rows(self) -> int:
        return self.A.shape[0]

    @property
    def cols(self) -> int:
        return self.A.shape[1]


def simplex_lsq(rows: int, cols: int, *, seed: int, dtype=np.float64, noise: float = 0.01, budget: float = 1.0,
                m: int = 10) -> ConstrainedProblem:
    """The example problem of the paper's section "Complete Framework": least squares subject to
    sum(x) = budget, x >= 0.  A iid N(0,1); x* = budget * (sparse point of the simplex: 10 % non-zeros with
    Dirichlet(1) weights); b = A x* + noise*N(0,1)."""
    rng = np.random.default_rng(seed)
    A = _normal_matrix(rng, rows, cols, np.dtype(dtype))
    k = max(1, cols // 10)
    support = np.sort(rng.permutation(cols)[:k])
    x_true = np.zeros(cols)
    x_true[support] = budget * rng.dirichlet(np.ones(k))
    b = _matvec(A, x_true) + noise * rng.standard_normal(rows)
    return ConstrainedProblem(name="simplex_lsq", A=A, b=b, C=np.ones((1, cols)), d=np.array([budget]),
                              E=np.zeros((0, cols)), e=np.zeros(0), l=np.zeros(cols), u=np.full(cols, math.inf),
                              x0=np.zeros(cols), m=m, x_true=x_true)


def constrained_lsq(rows: int, cols: int, n_eq: int, n_in: int, *, seed: int, lower: float = 0.0, upper: float = 1.0,
                    m: int = 10) -> ConstrainedProblem:
    """Random linear constraints around a feasible point: A, C, E iid N(0,1) (C, E scaled by 1/sqrt(cols)),
    x_feas ~ U(lower, upper), d = C x_feas, e = E x_feas + U(0, 0.5), b = A x_any + N(0,1) with x_any ~ N(0,1)."""
    rng = np.random.default_rng(seed)
    A = _normal_matrix(rng, rows, cols, np.dtype(np.float64))
    C = rng.standard_normal((n_eq, cols)) / math.sqrt(cols)
    E = rng.standard_normal((n_in, cols)) / math.sqrt(cols)
    x_feas = lower + (upper - lower) * rng.random(cols)
    d = C @ x_feas
    e = E @ x_feas + 0.5 * rng.random(n_in)
    b = _matvec(A, rng.standard_normal(cols)) + rng.standard_normal(rows)
    x0 = np.clip(np.zeros(cols), lower, upper)
    return ConstrainedProblem(name="constrained_lsq", A=A, b=b, C=C, d=d, E=E, e=e, l=np.full(cols, lower),
                              u=np.full(cols, upper), x0=x0, m=m, x_true=x_feas)


def constrained_config(name: str, *, scale: float = 1.0) -> ConstrainedProblem:
    """AL2: the C2 recipe (NNLS 20000 x 5000 fp64, same seed) with the budget constraint sum(x) = sum(x*)."""
    if name != "AL2":
        raise KeyError(name)
    base = config("C2", scale=scale)
    cols = base.cols
    return ConstrainedProblem(name="AL2", A=base.A, b=base.b, C=np.ones((1, cols)), d=np.array([base.x_true.sum()]),
                              E=np.zeros((0, cols)), e=np.zeros(0), l=base.l, u=base.u, x0=base.x0, m=base.m,
                              x_true=base.x_true)


# ---- dual SVM (quadratic form with one equality constraint) -------------------------------------

@dataclass
class SvmProblem:
    """min 0.5*(a.y)^T K (a.y) - sum(a)  s.t.  y^T a = 0,  0 <= a <= c   (the paper's section "Dual SVM")."""
    name: str
    K: np.ndarray            # n x n Gaussian kernel matrix
    y: np.ndarray            # labels in {-1, +1}
    c: float
    m: int
    X: Optional[np.ndarray] = None

    @property
    def n(self) -> int:
        return self.K.shape[0]


def svm_dual(n: int, dim: int = 20, *, seed: int, gamma: float = 1.0, c: float = 1.0, separation: float = 1.0,
             dtype=np.float64, m: int = 10) -> SvmProblem:
    """Two Gaussian classes in `dim` dimensions (identity covariance scaled by 1/dim, means +-separation/2 along a
    random unit direction), labels alternating; K_ij = exp(-gamma*||x_i - x_j||^2) as in the paper (gamma = 1,
    c = 1), built in row chunks."""
    rng = np.random.default_rng(seed)
    y = np.where(np.arange(n) % 2 == 0, 1.0, -1.0)
    direction = rng.standard_normal(dim)
    direction /= np.linalg.norm(direction)
    X = rng.standard_normal((n, dim)) / math.sqrt(dim) + 0.5 * separation * y[:, None] * direction[None, :]
    sq = (X * X).sum(1)
    K = np.empty((n, n), dtype=dtype)
    chunk = max(1, (128 << 20) // (n * 8))
    for r0 in range(0, n, chunk):
        r1 = min(n, r0 + chunk)
        d2 = sq[r0:r1, None] + sq[None, :] - 2.0 * (X[r0:r1] @ X.T)
        np.maximum(d2, 0.0, out=d2)
        K[r0:r1] = np.exp(-gamma * d2)
    K = 0.5 * (K + K.T) if n <= 4096 else K                  # exact symmetry (large n: symmetric up to rounding of the products)
    return SvmProblem(name="svm_dual", K=K, y=y, c=c, m=m, X=X)


# ---- joint probability distribution (regularised optimal transport) -----------------------------

OBJ_OT_GAUSS = 4     # <M,P> + lam/2*sum(P^2)        over the rows x cols matrix P (row-major), n = rows*cols
OBJ_OT_ENTROPY = 5   # <M,P> + lam*sum(P log P)


@dataclass
class TransportProblem:
    """min <M,P> + lam*r(P)  s.t.  P 1 = u,  P^T 1 = v,  P >= lower   (the paper's section "Joint Probability
    Distribution"); r the Gaussian (0.5*sum P^2) or the entropy (sum P log P) regulariser."""
    name: str
    kind: int                # OBJ_OT_GAUSS / OBJ_OT_ENTROPY
    M: np.ndarray            # rows x cols cost matrix
    u: np.ndarray            # rows, sums to one
    v: np.ndarray            # cols, sums to one
    lam: float
    lower: float             # 0 for the Gaussian regulariser; a tiny positive number for the entropy (log P)
    m: int

    @property
    def rows(self) -> int:
        return self.M.shape[0]

    @property
    def cols(self) -> int:
        return self.M.shape[1]

    @property
    def n(self) -> int:
        return self.M.size

    @property
    def l(self) -> np.ndarray:
        return np.full(self.n, self.lower)

    @property
    def ub(self) -> np.ndarray:
        return np.full(self.n, math.inf)

    @property
    def x0(self) -> np.ndarray:
        return np.full(self.n, self.lower)     # Algorithm 4's x^0 = 0, moved onto the lower bound


def _gauss_pdf(t, mean, sd):
    return np.exp(-0.5 * ((t - mean) / sd) ** 2) / (sd * math.sqrt(2.0 * math.pi))


def joint_probability(size: int, *, dataset: int = 1, reg: str = "gauss", seed: int = 0, lam: float = 0.5,
                      dtype=np.float64, m: int = 10, lower: Optional[float] = None) -> TransportProblem:
    """The two synthetic families of the paper's joint-probability experiment, lambda = 1/2.
    dataset 1 (rows = cols = size): on the grid t_k = (k + 0.5)/size, u = a Gaussian N(0.5, 0.12^2) and
      v = an equal mixture of N(0.3, 0.06^2) and N(0.7, 0.08^2), both discretised (density at the grid points,
      normalised to sum one); cost M = u u^T.  (The paper names the shapes, not their parameters.)  No random draw.
    dataset 2 (rows = 2*size, cols = size): u, v ~ U(0,1) normalised to sum one, M ~ U(0,1) entrywise.
      Draw order: u, v, M (row chunks)."""
    kind = {"gauss": OBJ_OT_GAUSS, "entropy": OBJ_OT_ENTROPY}[reg]
    if dataset == 1:
        t = (np.arange(size) + 0.5) / size
        u = _gauss_pdf(t, 0.5, 0.12)
        v = 0.5 * _gauss_pdf(t, 0.3, 0.06) + 0.5 * _gauss_pdf(t, 0.7, 0.08)
        u /= u.sum()
        v /= v.sum()
        M = np.ascontiguousarray(np.outer(u, u).astype(dtype))
    elif dataset == 2:
        rng = np.random.default_rng(seed)
        rows, cols = 2 * size, size
        u = rng.random(rows)
        v = rng.random(cols)
        u /= u.sum()
        v /= v.sum()
        M = np.empty((rows, cols), dtype=dtype)
        chunk = max(1, (64 << 20) // (cols * 8))
        for r0 in range(0, rows, chunk):
            r1 = min(rows, r0 + chunk)
            M[r0:r1] = rng.random((r1 - r0, cols)).astype(dtype)
    else:
        raise KeyError(dataset)
    if lower is None:
        lower = 0.0 if kind == OBJ_OT_GAUSS else 1e-30
    return TransportProblem(name=f"jp{dataset}_{reg}_{size}", kind=kind, M=M, u=u, v=v, lam=lam, lower=lower, m=m)
