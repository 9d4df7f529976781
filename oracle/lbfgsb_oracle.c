/*
 * CPU oracle for the modified L-BFGS-B method (box-constrained quasi-Newton without the
 * Cauchy-point search).  TEST INFRASTRUCTURE ONLY: plain, single-threaded, fp64, slow.
 * It shares no code with the HIP library and must never be called from the product path.
 *
 * What it follows, in the paper's notation:
 *   - Algorithm 1 (main loop)                               -> orc_step / orc_solve
 *   - Eq. (ws), the working set S^k of free variables       -> orc_free_mask
 *   - Algorithm 3 (modified two-loop recursion, appendix)   -> orc_two_loop
 *   - Algorithm 2 (projectDirection)                        -> orc_project_direction
 *   - backtracking Armijo line search (Section "Algorithm") -> line_search
 *   - objectives: the NNLS section's least-squares objective (scaled by 1/2), its
 *     L1-regularised variant split into x = p - q, and the regularised empirical
 *     logistic risk of the fairness section restricted to a box       -> orc_fg
 *   - the dual SVM objective of the section "Dual SVM", 0.5 (a.y)^T K (a.y) - sum(a), as the
 *     quadratic form ORC_QP                                           -> orc_fg
 *   - Eq. (augLag) and Algorithm 4 (augmented Lagrangian algorithm, section "Complete
 *     Framework" and appendix) for LINEAR constraints h(x) = C x - d = 0 and
 *     g(x) = E x - e <= 0 on top of the least-squares or quadratic-form objective
 *                                                                     -> orc_fg, orc_auglag_solve
 *   - the regularised optimal-transport objective of the section "Joint Probability
 *     Distribution", <M,P> + lambda r(P) over a matrix P >= 0 stored row by row, r the Gaussian
 *     (0.5 sum P^2) or the entropy (sum P log P) regulariser, with the marginal constraints
 *     P 1 = u, P^T 1 = v as the equality constraints of Algorithm 4      -> orc_fg, orc_auglag_solve
 *
 * Nothing here is blocked, fused or reordered: every objective value and gradient is
 * evaluated from scratch at every trial point, the two-loop recursion is the literal
 * sequence of dot products and axpys.  All sums are Neumaier-compensated so that the
 * oracle's own rounding is negligible next to that of the code it checks.
 *
 * Readings taken where the paper gives no value or is ambiguous (each one is also an
 * option or a comment at the place it is used):
 *   - one epsilon for Eq. (ws), Algorithm 2 and the curvature gate of Algorithm 3;
 *     convergence uses a separate tolerance on ||grad f(x^k)[S^k]||_2;
 *   - ||y^i||^2 in Algorithm 3 is the full-vector norm, as printed (no [S^k]);
 *   - the gate is the strict '>' of the algorithm listing;
 *   - d[S] = -q for the q Algorithm 3 returns;
 *   - with fewer than m pairs only the stored ones are visited; with none d = -g[S];
 *   - every pair is stored; the gate alone decides whether it is used;
 *   - step-length bound: 1 in the projection branch, the largest feasible step in the
 *     other branch; the first trial step is min(1, bound);
 *   - Armijo constant 1e-4 and halving are defaults of the options struct;
 *   - the Armijo inequality f(x + alpha p) <= f(x) + c1 alpha <grad f, p> is tested as
 *     [f(x_t) - f(x)] <= c1 alpha <grad f, p>, where the bracket is summed row by row from
 *     the identity  loss_r(x_t) - loss_r(x)  written in terms of (A (x_t - x))_r, and
 *     A (x_t - x) is a from-scratch product with the difference of the two points
 *     (orc_delta_f).  It is the same inequality, evaluated without cancellation:
 *     differencing two rounded objective values stalls the iteration at
 *     ||g|| ~ sqrt(ulp(f) * L), above the 1e-8 that the small NNLS case asks for.  f(x_t)
 *     itself is still evaluated from scratch at every trial (reported, finiteness check);
 *   - x + alpha p is clamped to the box (an exact no-op in exact arithmetic);
 *   - when backtracking is exhausted the pair memory is cleared and the iteration is
 *     redone once from the steepest-descent direction; if that fails too the solver
 *     stops with ORC_LINESEARCH_FAILED.
 *
 *   - Algorithm 4 says "update rho" and "until convergence" without formulas; the text says
 *     rho is doubled when the infinity norm of the constraint violation is not halved in an
 *     iteration.  Taken here: violation = max(||h(x)||_inf, ||max(g(x), 0)||_inf); the first
 *     iteration compares with the violation at x^0; the loop stops when the violation is at most
 *     ctol and the inner solve converged (or after max_outer iterations); every inner solve is
 *     warm-started at the previous x with an empty pair memory and run to the box solver's own
 *     tolerance; x^0 is the caller's (the listing's x^0 = 0 when that is feasible).
 *   - Joint probability: the paper names the regularisers without formulas.  Taken here: Gaussian
 *     r(P) = 0.5 sum P_ij^2, entropy r(P) = sum P_ij log P_ij (the negative entropy) with 0 log 0 = 0.
 *     The entropy's gradient log P + 1 is -inf at P = 0, so callers give it a (tiny) positive lower bound
 *     and start there; the oracle itself only evaluates what it is given.
 *
 * Parity pins (tests/test_oracle_*.py): KKT at the returned point, numpy lstsq when no
 * bound is active, brute-force active-set enumeration, scipy nnls / lsq_linear /
 * L-BFGS-B minimisers, dense BFGS-matrix construction for Algorithm 3, truth tables for
 * Eq. (ws) and Algorithm 2, finite differences for the gradients; for the transport kinds the same
 * objective written as the generic quadratic form with a dense 0/1 constraint matrix, entrywise closed
 * forms, the closed-form couplings for zero cost, the dual structure of the solution and scipy's SLSQP
 * (tests/test_oracle_transport.py).  The exhausted-line-search branch of orc_step (memory cleared, one
 * retry from steepest descent, then ORC_LINESEARCH_FAILED) is pinned by hand-worked two-variable
 * quadratics whose directions and Armijo decisions are re-derived in rational arithmetic from the dense
 * BFGS matrix (tests/test_oracle_linesearch_exhausted.py).  The individual
 * trajectory (iterates, step lengths) is parity unpinned: the paper prints no worked
 * example and none of the constants above.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_LSQ = 0, ORC_LSQ_L1SPLIT = 1, ORC_LOGISTIC_L2 = 2, ORC_QP = 3, ORC_OT_GAUSS = 4, ORC_OT_ENTROPY = 5 };
enum { ORC_F64 = 0, ORC_F32 = 1 };
enum { ORC_RUNNING = 0, ORC_CONVERGED = 1, ORC_MAX_ITER = 2, ORC_LINESEARCH_FAILED = 3 };

/* Linear constraints and the multiplier state of Eq. (augLag):
 *   h(x) = C x - d = 0 (n_eq rows),  g(x) = E x - e <= 0 (n_in rows),  C and E row-major with
 *   `cols` columns.  When an objective carries one of these, orc_fg evaluates
 *   L(x, lambda, mu, rho) = f(x) + rho/2 ||h(x) + lambda/rho||^2 + rho/2 ||(g(x) + mu/rho)_+||^2. */
typedef struct {
    int64_t n_eq, n_in;
    const double *C, *d, *E, *e;
    double *lambda, *mu;   /* n_eq / n_in entries, updated by orc_auglag_solve */
    double rho;
    int marginals;         /* transport kinds: the n_eq = rows + cols equality constraints are the marginals
                              P 1 = d[0..rows), P^T 1 = d[rows..rows+cols) of the rows x cols matrix x; C is not read */
} orc_constraints;

typedef struct {
    int kind, dtype;
    int64_t rows, cols, ld;
    const void* A;     /* row-major rows x cols, leading dimension ld */
    const double* b;   /* targets (least squares) or labels in {-1,+1} (logistic) */
    double lambda, mu;
    const orc_constraints* con;   /* NULL: no constraints besides the box (otherwise: ORC_LSQ, ORC_QP, transport kinds) */
    const double* sign;           /* ORC_QP: f = 0.5 (s.x)^T A (s.x) + b^T x with A symmetric (rows = cols), s = sign
                                     (NULL = ones); with A a kernel matrix, s the labels and b = -1 this is the dual
                                     SVM objective of the paper's section "Dual SVM" */
    /* ORC_OT_GAUSS / ORC_OT_ENTROPY: A is the rows x cols cost matrix M, the variable is the rows x cols matrix P
     * (row-major, n = rows*cols), f = sum M_ij P_ij + lambda sum phi(P_ij), phi(p) = p^2/2 or p log p (0 at p = 0);
     * b is not read */
} orc_objective;

typedef struct {
    double eps;
    double armijo_c1;
    double backtrack;
    int max_backtracks;
    double tol;
    int tol_relative;
    int max_iter;
    int always_branch2;   /* skip the projection branch of Algorithm 2 (remark after the corollary) */
} orc_options;

typedef struct {
    int status;
    int64_t iters, fevals;
    double f, pg2, pginf;
    int64_t n_fixed;
    /* diagnostics of the last completed iteration */
    int branch;            /* 1 = projection branch, 2 = masked quasi-Newton direction */
    int backtracks;
    int pairs_used;
    int memory_resets;
    double alpha, alpha_ub, gp;
} orc_info;

/* ---- compensated summation ------------------------------------------------------------- */

typedef struct { double s, c; } nsum;

static inline void ns_add(nsum* a, double v) {
    double t = a->s + v;
    if (fabs(a->s) >= fabs(v)) a->c += (a->s - t) + v;
    else a->c += (v - t) + a->s;
    a->s = t;
}
static inline double ns_val(const nsum* a) { return a->s + a->c; }

/* adds the exact product a*b (rounded product plus its fma-recovered error) */
static inline void ns_add_prod(nsum* acc, double a, double b) {
    double p = a * b;
    double e = fma(a, b, -p);
    ns_add(acc, p);
    acc->c += e;
}

static double dot_masked(int64_t n, const double* a, const double* b, const uint8_t* mask) {
    nsum acc = {0.0, 0.0};
    for (int64_t i = 0; i < n; ++i)
        if (!mask || mask[i]) ns_add_prod(&acc, a[i], b[i]);
    return ns_val(&acc);
}

static inline double a_at(const orc_objective* o, int64_t r, int64_t c) {
    return o->dtype == ORC_F64 ? ((const double*)o->A)[r * o->ld + c]
                               : (double)((const float*)o->A)[r * o->ld + c];
}

static inline double softplus(double t) { return (t > 0.0 ? t : 0.0) + log1p(exp(-fabs(t))); }
static inline double sigmoid(double t) {
    if (t >= 0.0) return 1.0 / (1.0 + exp(-t));
    double e = exp(t);
    return e / (1.0 + e);
}

/* ---- objectives -------------------------------------------------------------------------- */

static inline int is_transport(const orc_objective* o) { return o->kind == ORC_OT_GAUSS || o->kind == ORC_OT_ENTROPY; }

int64_t orc_num_vars(const orc_objective* o) {
    if (is_transport(o)) return o->rows * o->cols;
    return o->kind == ORC_LSQ_L1SPLIT ? 2 * o->cols : o->cols;
}

/* entries of the row vector that belong to the objective itself (the constraint values follow them) */
static inline int64_t obj_rows(const orc_objective* o) { return is_transport(o) ? 0 : o->rows; }

/* (row r of the constraint matrix) . z: a dense row of C or E; or, for the marginal constraints, the sum
 * of row r of the rows x cols matrix z (r < rows) or of its column r - rows */
static double con_dot(const orc_constraints* k, const orc_objective* o, int64_t r, const double* z) {
    nsum acc = {0.0, 0.0};
    if (k->marginals) {
        if (r < o->rows) for (int64_t j = 0; j < o->cols; ++j) ns_add(&acc, z[r * o->cols + j]);
        else for (int64_t i = 0; i < o->rows; ++i) ns_add(&acc, z[i * o->cols + (r - o->rows)]);
    } else {
        const double* crow = r < k->n_eq ? k->C + r * o->cols : k->E + (r - k->n_eq) * o->cols;
        for (int64_t c = 0; c < o->cols; ++c) ns_add_prod(&acc, crow[c], z[c]);
    }
    return ns_val(&acc);
}

/* g += coef * (row r of the constraint matrix) */
static void con_axpy(const orc_constraints* k, const orc_objective* o, int64_t r, double coef, double* g) {
    if (k->marginals) {
        if (r < o->rows) for (int64_t j = 0; j < o->cols; ++j) g[r * o->cols + j] += coef;
        else for (int64_t i = 0; i < o->rows; ++i) g[i * o->cols + (r - o->rows)] += coef;
    } else {
        const double* crow = r < k->n_eq ? k->C + r * o->cols : k->E + (r - k->n_eq) * o->cols;
        for (int64_t c = 0; c < o->cols; ++c) g[c] += coef * crow[c];
    }
}

/* Eq. (augLag): the two penalty terms at x (returned), their gradients C^T rho (h + lambda/rho) and
 * E^T rho (g + mu/rho)_+ added to g (if given), and the shifted constraint values h + lambda/rho,
 * g + mu/rho written to shifted[0 .. n_eq + n_in) (if given) */
static double penalty_terms(const orc_objective* o, const double* x, double* g, double* shifted) {
    const orc_constraints* k = o->con;
    nsum pen = {0.0, 0.0};
    for (int64_t r = 0; r < k->n_eq + k->n_in; ++r) {
        const int eq = r < k->n_eq;
        double a = eq ? con_dot(k, o, r, x) - k->d[r] + k->lambda[r] / k->rho
                      : con_dot(k, o, r, x) - k->e[r - k->n_eq] + k->mu[r - k->n_eq] / k->rho;
        if (shifted) shifted[r] = a;
        double act = eq ? a : (a > 0.0 ? a : 0.0);
        ns_add(&pen, 0.5 * k->rho * act * act);
        if (g) con_axpy(k, o, r, k->rho * act, g);
    }
    return ns_val(&pen);
}

/* change of the penalty terms from x to xt, without cancellation; shifted = the values penalty_terms left at x:
 *   rho/2 [(a + da)^2 - a^2] = rho da (a + da/2) for an equality row;
 *   rho/2 [(a + da)_+^2 - a_+^2] = rho/2 (p1 - p0)(p1 + p0) for an inequality row */
static double penalty_delta(const orc_objective* o, const double* x, const double* xt, const double* shifted) {
    const orc_constraints* k = o->con;
    const int64_t n = orc_num_vars(o);
    double* dx = (double*)malloc(sizeof(double) * (size_t)n);
    for (int64_t i = 0; i < n; ++i) dx[i] = xt[i] - x[i];
    nsum acc = {0.0, 0.0};
    for (int64_t r = 0; r < k->n_eq + k->n_in; ++r) {
        double da = con_dot(k, o, r, dx), a = shifted[r];
        if (r < k->n_eq) {
            ns_add_prod(&acc, k->rho * da, a + 0.5 * da);
        } else {
            double p0 = a > 0.0 ? a : 0.0, p1 = a + da > 0.0 ? a + da : 0.0;
            ns_add_prod(&acc, 0.5 * k->rho * (p1 - p0), p1 + p0);
        }
    }
    free(dx);
    return ns_val(&acc);
}

/* the transport objective <M,P> + lambda sum phi(P_ij) and its gradient M + lambda phi'(P) */
static double transport_fg(const orc_objective* o, const double* x, double* g) {
    nsum fsum = {0.0, 0.0};
    for (int64_t i = 0; i < o->rows; ++i)
        for (int64_t j = 0; j < o->cols; ++j) {
            const double p = x[i * o->cols + j], mij = a_at(o, i, j);
            ns_add_prod(&fsum, mij, p);
            if (o->kind == ORC_OT_GAUSS) {
                ns_add_prod(&fsum, 0.5 * o->lambda * p, p);
                if (g) g[i * o->cols + j] = mij + o->lambda * p;
            } else {
                if (p > 0.0) ns_add_prod(&fsum, o->lambda * p, log(p));
                if (g) g[i * o->cols + j] = mij + o->lambda * (log(p) + 1.0);
            }
        }
    return ns_val(&fsum);
}

/* f(x); if g != NULL also grad f(x); if rowvec != NULL it receives the residual A v - b
 * (least squares) or the margins X w (logistic), one entry per row. */
double orc_fg(const orc_objective* o, const double* x, double* g, double* rowvec) {
    const int64_t rows = o->rows, cols = o->cols;
    if (is_transport(o)) {
        double f = transport_fg(o, x, g);
        if (o->con) f += penalty_terms(o, x, g, rowvec);
        return f;
    }
    double* v = (double*)malloc(sizeof(double) * (size_t)cols);   /* the vector A multiplies */
    double* psi = (double*)malloc(sizeof(double) * (size_t)(rows > 0 ? rows : 1));
    for (int64_t c = 0; c < cols; ++c)
        v[c] = o->kind == ORC_LSQ_L1SPLIT ? x[c] - x[cols + c]
             : (o->kind == ORC_QP && o->sign) ? o->sign[c] * x[c] : x[c];

    nsum fsum = {0.0, 0.0};
    for (int64_t r = 0; r < rows; ++r) {
        nsum acc = {0.0, 0.0};
        for (int64_t c = 0; c < cols; ++c) ns_add_prod(&acc, a_at(o, r, c), v[c]);
        double z = ns_val(&acc);
        if (o->kind == ORC_LOGISTIC_L2) {
            double yr = o->b[r];
            ns_add(&fsum, softplus(-yr * z));
            psi[r] = -yr * sigmoid(-yr * z);
            if (rowvec) rowvec[r] = z;
        } else if (o->kind == ORC_QP) {
            /* z = (A v)_r: f gets 0.5 v_r z + b_r x_r, the gradient entry is s_r z + b_r */
            ns_add_prod(&fsum, 0.5 * v[r], z);
            ns_add_prod(&fsum, o->b[r], x[r]);
            psi[r] = z;
            if (rowvec) rowvec[r] = z;
        } else {
            double res = z - o->b[r];
            ns_add(&fsum, 0.5 * res * res);
            psi[r] = res;
            if (rowvec) rowvec[r] = res;
        }
    }
    double f = ns_val(&fsum);
    if (o->kind == ORC_LOGISTIC_L2) {
        f /= (double)rows;
        f += 0.5 * o->mu * dot_masked(cols, x, x, NULL);
    } else if (o->kind == ORC_LSQ_L1SPLIT) {
        nsum l1 = {0.0, 0.0};
        for (int64_t i = 0; i < 2 * cols; ++i) ns_add(&l1, x[i]);
        f += o->lambda * ns_val(&l1);
    }

    if (g && o->kind == ORC_QP) {
        for (int64_t c = 0; c < cols; ++c) g[c] = (o->sign ? o->sign[c] : 1.0) * psi[c] + o->b[c];
    } else if (g) {
        /* w = A^T psi, column by column as the definition says */
        nsum* acc = (nsum*)calloc((size_t)cols, sizeof(nsum));
        for (int64_t r = 0; r < rows; ++r)
            for (int64_t c = 0; c < cols; ++c) ns_add_prod(&acc[c], a_at(o, r, c), psi[r]);
        for (int64_t c = 0; c < cols; ++c) {
            double w = ns_val(&acc[c]);
            if (o->kind == ORC_LSQ) g[c] = w;
            else if (o->kind == ORC_LSQ_L1SPLIT) { g[c] = w + o->lambda; g[cols + c] = -w + o->lambda; }
            else g[c] = w / (double)rows + o->mu * x[c];
        }
        free(acc);
    }
    if (o->con && (o->kind == ORC_LSQ || o->kind == ORC_QP))
        f += penalty_terms(o, x, g, rowvec ? rowvec + rows : NULL);   /* after the rows of A in rowvec */
    free(v);
    free(psi);
    return f;
}

/* f(xt) - f(x) without cancellation.  row = residuals (least squares) or margins
 * (logistic) at x, as orc_fg produced them.  With dz = A (vt - v) computed from scratch:
 *   least squares:  0.5*(res+dz)^2 - 0.5*res^2 = dz*(res + 0.5*dz)
 *   logistic:       softplus(a+da) - softplus(a) = log(1 + sigmoid(a)*expm1(da)),
 *                   a = -y*z, da = -y*dz (evaluated as log1p(.) or, where sigmoid(a)*expm1(da) comes close
 *                   to -1, as log(sigmoid(-a) + sigmoid(a)*exp(da)): no difference of nearly equal numbers
 *                   in either regime)
 * plus the difference of the separable terms (lambda*sum x, mu/2*||x||^2). */
double orc_delta_f(const orc_objective* o, const double* x, const double* xt, const double* row) {
    const int64_t rows = o->rows, cols = o->cols, n = orc_num_vars(o);
    if (is_transport(o)) {
        /* entry by entry, dp = pt - p:  M dp;  Gaussian: (pt^2 - p^2)/2 = dp (p + dp/2);
         * entropy: pt log pt - p log p = dp log pt + p log(pt/p) when both are positive and |dp| <= p/2 */
        nsum acc = {0.0, 0.0};
        for (int64_t i = 0; i < rows; ++i)
            for (int64_t j = 0; j < cols; ++j) {
                const double p = x[i * cols + j], pt = xt[i * cols + j], dp = pt - p;
                ns_add_prod(&acc, a_at(o, i, j), dp);
                if (o->kind == ORC_OT_GAUSS) {
                    ns_add_prod(&acc, o->lambda * dp, p + 0.5 * dp);
                } else {
                    if (p > 0.0 && pt > 0.0 && fabs(dp) <= 0.5 * p) {
                        ns_add_prod(&acc, o->lambda * dp, log(pt));
                        ns_add_prod(&acc, o->lambda * p, log1p(dp / p));
                    } else if (p > 0.0 && pt > 0.0) {
                        /* a large relative change: the two values differ enough to be subtracted directly (and
                         * the split form would add +-huge terms, or log(0) once dp/p rounds to -1) */
                        ns_add_prod(&acc, o->lambda * pt, log(pt));
                        ns_add_prod(&acc, -o->lambda * p, log(p));
                    } else if (pt > 0.0) {
                        ns_add_prod(&acc, o->lambda * pt, log(pt));     /* p = 0 */
                    } else if (p > 0.0) {
                        ns_add_prod(&acc, -o->lambda * p, log(p));      /* pt = 0 */
                    }
                }
            }
        double df = ns_val(&acc);
        if (o->con) df += penalty_delta(o, x, xt, row);
        return df;
    }
    double* dv = (double*)malloc(sizeof(double) * (size_t)cols);
    for (int64_t c = 0; c < cols; ++c)
        dv[c] = o->kind == ORC_LSQ_L1SPLIT ? (xt[c] - x[c]) - (xt[cols + c] - x[cols + c])
              : (o->kind == ORC_QP && o->sign) ? o->sign[c] * (xt[c] - x[c]) : xt[c] - x[c];
    nsum acc = {0.0, 0.0};
    for (int64_t r = 0; r < rows; ++r) {
        nsum dacc = {0.0, 0.0};
        for (int64_t c = 0; c < cols; ++c) ns_add_prod(&dacc, a_at(o, r, c), dv[c]);
        double dz = ns_val(&dacc);
        if (o->kind == ORC_LOGISTIC_L2) {
            double a = -o->b[r] * row[r], da = -o->b[r] * dz;
            if (fabs(da) < 30.0) {
                /* log(1 + sigmoid(a) (e^da - 1)): log1p of the product while that is not close to -1; otherwise
                 * (a saturated margin that the step undoes: sigmoid(a) ~ 1, e^da ~ 0) the same number written as
                 * log(sigmoid(-a) + sigmoid(a) e^da), a sum of two positive terms */
                double u = sigmoid(a) * expm1(da);
                ns_add(&acc, u > -0.5 ? log1p(u) : log(sigmoid(-a) + sigmoid(a) * exp(da)));
            } else {
                ns_add(&acc, softplus(a + da) - softplus(a));
            }
        } else if (o->kind == ORC_QP) {
            /* 0.5 (v+dv)^T A (v+dv) - 0.5 v^T A v = dv^T (A v) + 0.5 dv^T (A dv) (A symmetric), plus b^T dx */
            ns_add_prod(&acc, dv[r], row[r] + 0.5 * dz);
            ns_add_prod(&acc, o->b[r], xt[r] - x[r]);
        } else {
            ns_add_prod(&acc, dz, row[r] + 0.5 * dz);
        }
    }
    free(dv);
    double df = ns_val(&acc);
    if (o->con && (o->kind == ORC_LSQ || o->kind == ORC_QP)) df += penalty_delta(o, x, xt, row + rows);
    if (o->kind == ORC_LOGISTIC_L2) {
        nsum reg = {0.0, 0.0};
        for (int64_t i = 0; i < n; ++i) ns_add_prod(&reg, xt[i] - x[i], xt[i] + x[i]);
        df = df / (double)rows + 0.5 * o->mu * ns_val(&reg);
    } else if (o->kind == ORC_LSQ_L1SPLIT) {
        nsum l1 = {0.0, 0.0};
        for (int64_t i = 0; i < n; ++i) ns_add(&l1, xt[i] - x[i]);
        df += o->lambda * ns_val(&l1);
    }
    return df;
}

/* ---- Eq. (ws): mask[i] = 1 for free variables, 0 for fixed ones -------------------------- */

void orc_free_mask(int64_t n, const double* x, const double* g, const double* l, const double* u,
                   double eps, uint8_t* mask) {
    for (int64_t i = 0; i < n; ++i) {
        int at_lower = (x[i] <= l[i] + eps) && (g[i] >= 0.0);
        int at_upper = (x[i] >= u[i] - eps) && (g[i] <= 0.0);
        mask[i] = (at_lower || at_upper) ? 0 : 1;
    }
}

/* ---- Algorithm 3: modified two-loop recursion -------------------------------------------
 * S, Y: npairs x n, oldest pair first, newest last.  ynorm2[i] = ||y^i||^2 over the full
 * vector.  Returns d with d[S^k] = -q, d elsewhere = 0; *pairs_used counts pairs that
 * passed the curvature gate. */
void orc_two_loop(int64_t n, int npairs, const double* S, const double* Y, const double* ynorm2,
                  const double* g, const uint8_t* mask, double eps, double* d, int* pairs_used) {
    double* q = (double*)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
    double* rho = (double*)malloc(sizeof(double) * (size_t)(npairs > 0 ? npairs : 1));
    double* alpha = (double*)malloc(sizeof(double) * (size_t)(npairs > 0 ? npairs : 1));
    int* pass = (int*)malloc(sizeof(int) * (size_t)(npairs > 0 ? npairs : 1));
    int used = 0;

    for (int64_t e = 0; e < n; ++e) q[e] = mask[e] ? g[e] : 0.0;

    for (int i = npairs - 1; i >= 0; --i) {
        const double* s = S + (size_t)i * n;
        const double* y = Y + (size_t)i * n;
        rho[i] = dot_masked(n, s, y, mask);
        pass[i] = rho[i] > eps * ynorm2[i];
        if (pass[i]) {
            ++used;
            alpha[i] = dot_masked(n, s, q, mask) / rho[i];
            for (int64_t e = 0; e < n; ++e)
                if (mask[e]) q[e] -= alpha[i] * y[e];
        }
    }
    if (npairs > 0 && pass[npairs - 1]) {
        double scale = rho[npairs - 1] / ynorm2[npairs - 1];
        for (int64_t e = 0; e < n; ++e) q[e] *= scale;
    }
    for (int i = 0; i < npairs; ++i) {
        if (!pass[i]) continue;
        const double* s = S + (size_t)i * n;
        const double* y = Y + (size_t)i * n;
        double beta = dot_masked(n, y, q, mask) / rho[i];
        for (int64_t e = 0; e < n; ++e)
            if (mask[e]) q[e] += (alpha[i] - beta) * s[e];
    }
    for (int64_t e = 0; e < n; ++e) d[e] = mask[e] ? -q[e] : 0.0;
    if (pairs_used) *pairs_used = used;
    free(q); free(rho); free(alpha); free(pass);
}

/* ---- Algorithm 2: projectDirection ------------------------------------------------------
 * Returns the branch taken (1 or 2), writes p and the step-length bound. */
static inline double clampd(double v, double lo, double hi) { return v < lo ? lo : (v > hi ? hi : v); }

int orc_project_direction(int64_t n, const double* x, const double* g, const double* d,
                          const double* l, const double* u, double eps, int always_branch2,
                          double* p, double* alpha_ub) {
    nsum pg = {0.0, 0.0}, pp = {0.0, 0.0};
    for (int64_t i = 0; i < n; ++i) {
        double z = clampd(x[i] + d[i], l[i], u[i]);
        p[i] = z - x[i];
        ns_add(&pg, p[i] * g[i]);
        ns_add(&pp, p[i] * p[i]);
    }
    double pgv = ns_val(&pg), ppv = ns_val(&pp);
    if (!always_branch2 && pgv <= -eps * ppv && ppv >= eps) {
        *alpha_ub = 1.0;
        return 1;
    }
    double ub = INFINITY;
    for (int64_t i = 0; i < n; ++i) {
        double pi = d[i];
        if (d[i] < 0.0 && x[i] <= l[i] + eps) pi = 0.0;
        if (d[i] > 0.0 && x[i] >= u[i] - eps) pi = 0.0;
        p[i] = pi;
        if (pi > 0.0) { double a = (u[i] - x[i]) / pi; if (a < ub) ub = a; }
        else if (pi < 0.0) { double a = (l[i] - x[i]) / pi; if (a < ub) ub = a; }
    }
    *alpha_ub = ub;
    return 2;
}

/* ---- solver state (Algorithm 1) ---------------------------------------------------------- */

typedef struct {
    int64_t n;
    int m;
    orc_objective obj;
    orc_options opt;
    double *l, *u, *x, *g, *d, *p, *xt, *gt;
    double *row;              /* residuals (margins) at x */
    uint8_t* mask;
    double *S, *Y, *ynorm2;   /* oldest first */
    int npairs;
    double f;
    double tol_abs;           /* resolved at the first iteration when tol_relative is set */
    int tol_resolved;
    orc_info info;
} orc_solver;

void orc_default_options(orc_options* o) {
    o->eps = 1e-10;
    o->armijo_c1 = 1e-4;
    o->backtrack = 0.5;
    o->max_backtracks = 60;
    o->tol = 1e-8;
    o->tol_relative = 0;
    o->max_iter = 1000;
    o->always_branch2 = 0;
}

void orc_destroy(orc_solver* s) {
    if (!s) return;
    free(s->l); free(s->u); free(s->x); free(s->g); free(s->d); free(s->p); free(s->xt); free(s->gt);
    free(s->row);
    free(s->mask); free(s->S); free(s->Y); free(s->ynorm2);
    free(s);
}

/* Returns NULL when the arguments are invalid, bounds cross, or x0 is infeasible
 * (Algorithm 1 requires l <= x^0 <= u). */
orc_solver* orc_create(int64_t n, int m, const double* l, const double* u, const double* x0,
                       const orc_objective* obj, const orc_options* opt) {
    if (n <= 0 || m <= 0 || !l || !u || !x0 || !obj || orc_num_vars(obj) != n) return NULL;
    for (int64_t i = 0; i < n; ++i)
        if (!(l[i] <= u[i]) || !(x0[i] >= l[i]) || !(x0[i] <= u[i])) return NULL;
    orc_solver* s = (orc_solver*)calloc(1, sizeof(orc_solver));
    s->n = n; s->m = m; s->obj = *obj;
    if (opt) s->opt = *opt; else orc_default_options(&s->opt);
    size_t nb = sizeof(double) * (size_t)n;
    s->l = (double*)malloc(nb); s->u = (double*)malloc(nb); s->x = (double*)malloc(nb);
    s->g = (double*)malloc(nb); s->d = (double*)malloc(nb); s->p = (double*)malloc(nb);
    s->xt = (double*)malloc(nb); s->gt = (double*)malloc(nb);
    s->mask = (uint8_t*)malloc((size_t)n);
    s->row = (double*)malloc(sizeof(double) * (size_t)(obj_rows(obj) + (obj->con ? obj->con->n_eq + obj->con->n_in : 0) + 1));
    s->S = (double*)malloc(nb * (size_t)m); s->Y = (double*)malloc(nb * (size_t)m);
    s->ynorm2 = (double*)malloc(sizeof(double) * (size_t)m);
    memcpy(s->l, l, nb); memcpy(s->u, u, nb); memcpy(s->x, x0, nb);
    s->npairs = 0;
    s->f = orc_fg(&s->obj, s->x, s->g, s->row);
    s->info.status = ORC_RUNNING;
    s->info.fevals = 1;
    s->info.f = s->f;
    return s;
}

static void kkt_measures(orc_solver* s) {
    /* ||g[S^k]||_2 (the stopping quantity) and ||x - P(x - g)||_inf (epsilon-free KKT residual) */
    int64_t fixed = 0;
    double pginf = 0.0;
    for (int64_t i = 0; i < s->n; ++i) {
        if (!s->mask[i]) ++fixed;
        double r = fabs(s->x[i] - clampd(s->x[i] - s->g[i], s->l[i], s->u[i]));
        if (r > pginf) pginf = r;
    }
    s->info.pg2 = sqrt(dot_masked(s->n, s->g, s->g, s->mask));
    s->info.pginf = pginf;
    s->info.n_fixed = fixed;
    s->info.f = s->f;
}

/* backtracking Armijo search along p from x; on success xt holds the accepted point and
 * *f_new its objective value.  Every trial evaluates f from scratch. */
static int line_search(orc_solver* s, double gp, double alpha_ub, double* alpha_out, double* f_new,
                       int* backtracks) {
    double alpha = alpha_ub < 1.0 ? alpha_ub : 1.0;
    for (int t = 0; t <= s->opt.max_backtracks; ++t) {
        for (int64_t i = 0; i < s->n; ++i)
            s->xt[i] = clampd(s->x[i] + alpha * s->p[i], s->l[i], s->u[i]);
        double ft = orc_fg(&s->obj, s->xt, NULL, NULL);
        s->info.fevals++;
        double df = orc_delta_f(&s->obj, s->x, s->xt, s->row);
        if (isfinite(ft) && isfinite(df) && df <= s->opt.armijo_c1 * alpha * gp) {
            *alpha_out = alpha; *f_new = ft; *backtracks = t;
            return 1;
        }
        alpha *= s->opt.backtrack;
    }
    return 0;
}

/* One iteration of Algorithm 1.  Returns the status after it. */
int orc_step(orc_solver* s) {
    if (s->info.status != ORC_RUNNING) return s->info.status;
    const int64_t n = s->n;

    orc_free_mask(n, s->x, s->g, s->l, s->u, s->opt.eps, s->mask);
    kkt_measures(s);
    if (!s->tol_resolved) {
        s->tol_abs = s->opt.tol_relative ? s->opt.tol * fmax(1.0, s->info.pg2) : s->opt.tol;
        s->tol_resolved = 1;
    }
    if (s->info.pg2 <= s->tol_abs) return s->info.status = ORC_CONVERGED;
    if (s->info.iters >= s->opt.max_iter) return s->info.status = ORC_MAX_ITER;

    for (int attempt = 0; attempt < 2; ++attempt) {
        int used = 0;
        orc_two_loop(n, s->npairs, s->S, s->Y, s->ynorm2, s->g, s->mask, s->opt.eps, s->d, &used);
        double alpha_ub;
        int branch = orc_project_direction(n, s->x, s->g, s->d, s->l, s->u, s->opt.eps,
                                           s->opt.always_branch2, s->p, &alpha_ub);
        double gp = dot_masked(n, s->g, s->p, NULL);
        double alpha, f_new;
        int bt;
        if (line_search(s, gp, alpha_ub, &alpha, &f_new, &bt)) {
            orc_fg(&s->obj, s->xt, s->gt, s->row);      /* gradient at the new point, from scratch */
            s->info.fevals++;
            if (s->npairs == s->m) {                    /* evict the oldest pair */
                memmove(s->S, s->S + n, sizeof(double) * (size_t)n * (size_t)(s->m - 1));
                memmove(s->Y, s->Y + n, sizeof(double) * (size_t)n * (size_t)(s->m - 1));
                memmove(s->ynorm2, s->ynorm2 + 1, sizeof(double) * (size_t)(s->m - 1));
                s->npairs--;
            }
            double* sn = s->S + (size_t)s->npairs * n;
            double* yn = s->Y + (size_t)s->npairs * n;
            for (int64_t i = 0; i < n; ++i) { sn[i] = s->xt[i] - s->x[i]; yn[i] = s->gt[i] - s->g[i]; }
            s->ynorm2[s->npairs] = dot_masked(n, yn, yn, NULL);
            s->npairs++;
            memcpy(s->x, s->xt, sizeof(double) * (size_t)n);
            memcpy(s->g, s->gt, sizeof(double) * (size_t)n);
            s->f = f_new;
            s->info.f = f_new;
            s->info.iters++;
            s->info.branch = branch; s->info.backtracks = bt; s->info.pairs_used = used;
            s->info.alpha = alpha; s->info.alpha_ub = alpha_ub; s->info.gp = gp;
            return ORC_RUNNING;
        }
        if (s->npairs == 0) break;
        s->npairs = 0;                                  /* clear the memory, retry once */
        s->info.memory_resets++;
    }
    return s->info.status = ORC_LINESEARCH_FAILED;
}

int orc_solve(orc_solver* s) {
    while (orc_step(s) == ORC_RUNNING) {}
    return s->info.status;
}

/* Re-evaluates the mask and the KKT measures at the current point without stepping
 * (used after the last iteration so that info describes the returned x). */
void orc_refresh_info(orc_solver* s) {
    orc_free_mask(s->n, s->x, s->g, s->l, s->u, s->opt.eps, s->mask);
    kkt_measures(s);
}

void orc_get_info(const orc_solver* s, orc_info* out) { *out = s->info; }
const double* orc_x(const orc_solver* s) { return s->x; }
const double* orc_g(const orc_solver* s) { return s->g; }
const double* orc_d(const orc_solver* s) { return s->d; }
const double* orc_p(const orc_solver* s) { return s->p; }
const uint8_t* orc_mask(const orc_solver* s) { return s->mask; }
const double* orc_S(const orc_solver* s) { return s->S; }
const double* orc_Y(const orc_solver* s) { return s->Y; }
const double* orc_ynorm2(const orc_solver* s) { return s->ynorm2; }
int orc_npairs(const orc_solver* s) { return s->npairs; }

/* ---- Algorithm 4: augmented Lagrangian algorithm ------------------------------------------ */

typedef struct {
    double rho0;        /* initial rho (the listing: 1) */
    double ctol;        /* stop when the constraint violation is at most this and the inner solve converged */
    int max_outer;
} orc_auglag_options;

typedef struct {
    int status;             /* ORC_CONVERGED, ORC_MAX_ITER (outer limit) or the inner solver's failure status */
    int outer;              /* outer iterations done */
    int64_t inner_iters;    /* box-solver iterations, all outer iterations together */
    double violation;       /* max(||h(x)||_inf, ||max(g(x), 0)||_inf) at the returned x */
    double rho;
    double f;               /* objective without the penalty terms */
    double L;               /* augmented Lagrangian at the returned x with the multipliers it was minimised for */
    double pg2;             /* the last inner solve's stopping quantity */
} orc_auglag_info;

void orc_auglag_default_options(orc_auglag_options* o) {
    o->rho0 = 1.0;
    o->ctol = 1e-8;
    o->max_outer = 100;
}

/* h = C x - d and g = E x - e at x; returns max(||h||_inf, ||max(g, 0)||_inf) */
static double constraint_values(const orc_objective* o, const double* x, double* h, double* g) {
    const orc_constraints* k = o->con;
    double viol = 0.0;
    for (int64_t r = 0; r < k->n_eq + k->n_in; ++r) {
        if (r < k->n_eq) {
            h[r] = con_dot(k, o, r, x) - k->d[r];
            if (fabs(h[r]) > viol) viol = fabs(h[r]);
        } else {
            g[r - k->n_eq] = con_dot(k, o, r, x) - k->e[r - k->n_eq];
            if (g[r - k->n_eq] > viol) viol = g[r - k->n_eq];
        }
    }
    return viol;
}

/* Algorithm 4 on a least-squares, quadratic-form or transport objective that carries constraints (obj->con; its lambda and mu arrays are
 * the multiplier state: set to zero here, updated in place, returned).  x: in = x^0 (feasible for the
 * box), out = the result. */
int orc_auglag_solve(int64_t n, int m, const double* l, const double* u, double* x, const orc_objective* obj,
                     const orc_options* opt, const orc_auglag_options* aopt, orc_auglag_info* info) {
    memset(info, 0, sizeof *info);
    if (!obj || (obj->kind != ORC_LSQ && obj->kind != ORC_QP && !is_transport(obj)) || !obj->con ||
        n != orc_num_vars(obj))
        return -1;
    if (obj->con->marginals && (!is_transport(obj) || obj->con->n_eq != obj->rows + obj->cols || obj->con->n_in != 0))
        return -1;
    orc_constraints* k = (orc_constraints*)obj->con;   /* the multiplier state is the caller's, mutable */
    orc_auglag_options ao;
    if (aopt) ao = *aopt; else orc_auglag_default_options(&ao);
    double* h = (double*)malloc(sizeof(double) * (size_t)(k->n_eq + 1));
    double* g = (double*)malloc(sizeof(double) * (size_t)(k->n_in + 1));
    for (int64_t r = 0; r < k->n_eq; ++r) k->lambda[r] = 0.0;
    for (int64_t r = 0; r < k->n_in; ++r) k->mu[r] = 0.0;
    k->rho = ao.rho0;
    double viol_prev = constraint_values(obj, x, h, g);
    info->status = ORC_MAX_ITER;
    info->violation = viol_prev;
    for (int it = 0; it < ao.max_outer; ++it) {
        /* x^{k+1} = argmin over the box of L(., lambda^k, mu^k, rho) by Algorithm 1 */
        orc_solver* s = orc_create(n, m, l, u, x, obj, opt);
        if (!s) { free(h); free(g); return -1; }
        int st = orc_solve(s);
        memcpy(x, s->x, sizeof(double) * (size_t)n);
        info->inner_iters += s->info.iters;
        info->L = s->f;
        info->pg2 = s->info.pg2;
        orc_destroy(s);
        info->outer = it + 1;
        if (st == ORC_LINESEARCH_FAILED) { info->status = st; break; }
        /* lambda^{k+1} = lambda^k + rho h(x^{k+1});  mu^{k+1} = (mu^k + rho g(x^{k+1}))_+ */
        double viol = constraint_values(obj, x, h, g);
        for (int64_t r = 0; r < k->n_eq; ++r) k->lambda[r] += k->rho * h[r];
        for (int64_t r = 0; r < k->n_in; ++r) {
            double v = k->mu[r] + k->rho * g[r];
            k->mu[r] = v > 0.0 ? v : 0.0;
        }
        info->violation = viol;
        if (viol <= ao.ctol && st == ORC_CONVERGED) { info->status = ORC_CONVERGED; break; }
        /* rho is doubled when the violation was not halved in this iteration */
        if (viol > 0.5 * viol_prev) k->rho *= 2.0;
        viol_prev = viol;
    }
    info->rho = k->rho;
    {
        orc_objective plain = *obj;
        plain.con = NULL;
        info->f = orc_fg(&plain, x, NULL, NULL);
    }
    free(h); free(g);
    return 0;
}
