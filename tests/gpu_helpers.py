"""Helpers shared by the GPU parity tests (no solver arithmetic of the HIP path lives here)."""
import numpy as np
import torch

import paper_2203_16340_amd as L
import workloads

DEV = "cuda:0"


def to_dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def rel_err(got, ref):
    """normwise relative error ||got - ref||_2 / max(||ref||_2, tiny)"""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300))


def make_solver(kind, A, b, l, u, m, lam=0.0, mu=0.0, **opts):
    return L.Solver(kind, to_dev(A) if isinstance(A, np.ndarray) else A, to_dev(b), to_dev(l), to_dev(u), m,
                    lam=lam, mu=mu, options=L.default_options(**opts))


def host_matvec(A, v, chunk_bytes=512 << 20):
    """A @ v with fp64 accumulation for fp32 or fp64 A, in row chunks."""
    rows, cols = A.shape
    out = np.empty(rows)
    step = max(1, chunk_bytes // (cols * 8))
    for r0 in range(0, rows, step):
        out[r0:r0 + step] = A[r0:r0 + step].astype(np.float64, copy=False) @ v
    return out


def host_rmatvec(A, w, chunk_bytes=512 << 20):
    rows, cols = A.shape
    out = np.zeros(cols)
    step = max(1, chunk_bytes // (cols * 8))
    for r0 in range(0, rows, step):
        out += w[r0:r0 + step] @ A[r0:r0 + step].astype(np.float64, copy=False)
    return out


def host_gradient(prob, x):
    """grad f(x) recomputed on the host in fp64 with numpy (independent of both implementations)."""
    if prob.kind == workloads.OBJ_LSQ:
        return host_rmatvec(prob.A, host_matvec(prob.A, x) - prob.b)
    if prob.kind == workloads.OBJ_LSQ_L1SPLIT:
        c = prob.cols
        w = host_rmatvec(prob.A, host_matvec(prob.A, x[:c] - x[c:]) - prob.b)
        return np.concatenate([w + prob.lam, -w + prob.lam])
    from scipy.special import expit
    z = host_matvec(prob.A, x)
    return -host_rmatvec(prob.A, prob.b * expit(-prob.b * z)) / prob.rows + prob.mu * x


def host_objective(prob, x):
    if prob.kind == workloads.OBJ_LSQ:
        r = host_matvec(prob.A, x) - prob.b
        return 0.5 * r @ r
    if prob.kind == workloads.OBJ_LSQ_L1SPLIT:
        c = prob.cols
        r = host_matvec(prob.A, x[:c] - x[c:]) - prob.b
        return 0.5 * r @ r + prob.lam * x.sum()
    from scipy.special import log_expit
    return -log_expit(prob.b * host_matvec(prob.A, x)).sum() / prob.rows + 0.5 * prob.mu * x @ x


def kkt_residual(prob, x, g=None):
    """||x - P(x - g)||_inf with g recomputed on the host; also checks feasibility."""
    assert np.all(x >= prob.l) and np.all(x <= prob.u), "iterate left the box"
    if g is None:
        g = host_gradient(prob, x)
    return float(np.abs(x - np.clip(x - g, prob.l, prob.u)).max()), g


def active_set(prob, x, eps=1e-10):
    return (x <= prob.l + eps) | (x >= prob.u - eps)
