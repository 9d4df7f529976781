/*
 * liblbfgsb -- box-constrained limited-memory quasi-Newton solver for one MI355X (gfx950).
 *
 * Problem (the paper's section "Algorithm"):  minimise f(x) subject to l <= x <= u, with
 * l, u in (R u {-inf,+inf})^n and a FEASIBLE initial iterate.  One call of lbfgsb_step is one
 * pass of the body of Algorithm 1:
 *     gradient + free set S^k (Eq. (ws)) -> modified two-loop recursion on S^k (Algorithm 3,
 *     appendix) -> d[complement of S^k] = 0 -> projectDirection (Algorithm 2) -> backtracking
 *     Armijo line search with the step bounded so that the iterate stays in the box -> new
 *     curvature pair (s, y) stored in a FIFO of m pairs.
 * There is no Cauchy-point search: the free set is computed directly, which is what lets every
 * part of an iteration run data-parallel on the GPU.
 *
 * Conventions
 *   - Every pointer is a DEVICE pointer unless its name ends in _host or the comment says host.
 *   - All vectors (x, g, l, u, b, ...) are fp64.  Only the matrix A may be stored in fp32
 *     (dtype), and then every product is still accumulated in fp64.
 *   - A is row-major, rows x cols, leading dimension ld >= cols (in elements).
 *   - Infinite bounds are IEEE infinities.
 *   - The library allocates no device memory: the caller passes a workspace of
 *     lbfgsb_workspace_bytes() bytes (256-byte aligned) that the solver owns until
 *     lbfgsb_destroy.  A, b are BORROWED for the solver's lifetime and must not change;
 *     l, u, x0 are copied into the workspace.
 *   - All work is enqueued on the HIP stream given at creation (NULL = the default stream).
 *   - Every function returns LBFGSB_OK (0) or a negative error code; none throws, aborts or
 *     prints.  lbfgsb_last_error() gives a human-readable message for the calling thread.
 *     The reason a solve stopped is not an error; it is reported in lbfgsb_info.status.
 */
#ifndef LBFGSB_H
#define LBFGSB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LBFGSB_MAX_M 31   /* at most 31 stored pairs (2m+1 <= 64 vectors in the batched two-loop) */

typedef struct lbfgsb_solver lbfgsb_solver;   /* opaque, host object */

/* storage type of the matrix only */
enum { LBFGSB_F64 = 0, LBFGSB_F32 = 1 };

/* objective kinds.  LSQ is the least-squares objective of the paper's NNLS section scaled by
 * 1/2; L1SPLIT is its L1-regularised form written over x = [p; q], x_orig = p - q, p, q >= 0;
 * LOGISTIC_L2 is the regularised empirical logistic risk (the loss of the paper's fairness
 * section) over a box. */
enum {
    LBFGSB_OBJ_LSQ = 0,          /* f = 0.5*||A x - b||^2,                               n = cols   */
    LBFGSB_OBJ_LSQ_L1SPLIT = 1,  /* f = 0.5*||A(p-q) - b||^2 + lambda*sum(p+q), x=[p;q], n = 2*cols */
    LBFGSB_OBJ_LOGISTIC_L2 = 2,  /* f = (1/rows)*sum_i softplus(-b_i*(A x)_i) + mu/2*||x||^2, b_i in {-1,+1}, n = cols */
    LBFGSB_OBJ_QP = 3,           /* f = 0.5*(s.x)^T A (s.x) + b^T x, A symmetric, rows = cols = n, s = sign (or ones).
                                    With A a kernel matrix, s the labels and b = -1 this is the dual SVM objective of
                                    the paper's section "Dual SVM".  One product with A per iteration (no transposed pass) */
    /* The regularised optimal-transport objective of the paper's section "Joint Probability Distribution" over a
     * rows x cols matrix P stored row by row as the variable vector (n = rows*cols); A is the cost matrix M (used
     * entry by entry: there is no matrix-vector product), lambda > 0 the regularisation parameter:
     *     f = <M,P> + lambda*sum_ij phi(P_ij) + 0.5*sum_k row_weight_k*((K P)_k - b_k)^2,   K P = [P 1; P^T 1],
     * phi(p) = p^2/2 (Gaussian regulariser) or p*log(p) (entropy; needs l > 0).  b and row_weight have rows + cols
     * entries (row sums first); row_weight NULL drops the last term (b is then not read).  That term is how the
     * marginal constraints P 1 = u, P^T 1 = v enter through the augmented Lagrangian (lbfgsb_auglag_create_marginals);
     * b and row_weight may change between lbfgsb_set_x calls. */
    LBFGSB_OBJ_OT_GAUSS = 4,
    LBFGSB_OBJ_OT_ENTROPY = 5
};

typedef struct {
    int kind;            /* LBFGSB_OBJ_* */
    int dtype;           /* LBFGSB_F64 / LBFGSB_F32: element type of A */
    int64_t rows, cols, ld;
    const void* A;       /* device, row-major, borrowed */
    const double* b;     /* device, rows entries: targets (least squares) or labels (logistic), borrowed */
    double lambda;       /* L1SPLIT, OT_GAUSS, OT_ENTROPY */
    double mu;           /* LOGISTIC_L2 only */
    const double* row_weight; /* device, rows entries or NULL (= all ones), borrowed; least-squares kinds only:
                                 f = 0.5*sum_r row_weight_r*(A v - b)_r^2 (+ lambda*sum(p+q)) */
    const double* sign;       /* device, n entries or NULL (= all ones), borrowed; LBFGSB_OBJ_QP only */
    /* A few extra dense rows on top of a quadratic kind (LSQ, L1SPLIT, QP):
     *   f += 0.5*sum_r extra_weight_r*(extra_rows_r . x - extra_target_r)^2,   r < n_extra <= 64.
     * extra_rows: device, n_extra x n row-major fp64; extra_target, extra_weight: device, n_extra entries
     * (weights NULL = ones).  All borrowed; target and weight may change between lbfgsb_set_x calls (this is
     * how the augmented Lagrangian algorithm attaches its penalty term to the QP kind). */
    int64_t n_extra;
    const double* extra_rows;
    const double* extra_target;
    const double* extra_weight;
} lbfgsb_objective;

/* how the products with A are organised (results agree to rounding) */
enum {
    LBFGSB_APASS_AUTO = 0,     /* fused single read of A when the shape allows it (16-byte aligned rows of at most
                                  20428 columns; 10240 for an fp64 logistic matrix), else two passes */
    LBFGSB_APASS_TWO_PASS = 1, /* t = A v, then w = A^T psi: A is read twice per evaluation and per iteration */
    LBFGSB_APASS_FUSED = 2,    /* force the fused kernel; lbfgsb_create fails if the shape does not fit.  For the
                                  logistic objective an iteration's single read yields t = A p and A^T psi of the first
                                  trial step; a second (transposed) pass runs only if that step is rejected */
    LBFGSB_APASS_RESIDENT = 3  /* small plain least-squares problems (kind LSQ without row weights or extra rows; up to
                                  256 rows of at most 128 columns, or 128 rows of at most 256: at most 256 KB of fp64 matrix):
                                  one workgroup keeps the matrix in registers and the vectors in LDS and runs whole
                                  iterations without leaving its compute unit -- one launch per lbfgsb_step call, ONE
                                  launch per lbfgsb_solve.  LBFGSB_APASS_AUTO picks it whenever the problem qualifies;
                                  asking for it explicitly fails with LBFGSB_E_UNSUPPORTED when it does not.  Same
                                  arithmetic as the other organisations with different summation orders (results agree
                                  to rounding).  On this path a step that finds the stopping test met recomputes the
                                  gradient from x and tests again before reporting LBFGSB_CONVERGED. */
};

typedef struct {
    double eps;            /* the paper's epsilon: Eq. (ws), Algorithm 2 and the curvature gate of Algorithm 3. default 1e-10 */
    double armijo_c1;      /* Armijo constant, default 1e-4 */
    double backtrack;      /* step reduction factor in (0,1), default 0.5 */
    int max_backtracks;    /* default 60 */
    double tol;            /* stop when ||grad f(x^k)[S^k]||_2 <= tol (absolute) or <= tol*max(1, its value at x^0) */
    int tol_relative;      /* 0 absolute (default), 1 relative */
    int max_iter;          /* default 1000 */
    int refresh_every;     /* least-squares kinds carry residual and gradient by recurrence; every this many
                              iterations they are recomputed from x (default 32, 0 = never) */
    int poll_every;        /* lbfgsb_solve reads the device status flag every this many iterations (default 8); in a long
                              run the interval doubles each time eight intervals have gone by, up to 64 */
    int a_pass;            /* LBFGSB_APASS_* */
} lbfgsb_options;

/* termination state */
enum { LBFGSB_RUNNING = 0, LBFGSB_CONVERGED = 1, LBFGSB_MAX_ITER = 2, LBFGSB_LINESEARCH_FAILED = 3 };

typedef struct {          /* HOST struct */
    int status;           /* LBFGSB_RUNNING ... */
    int64_t iters;        /* accepted iterations so far */
    int64_t fevals;       /* objective evaluations (line-search trials + refreshes) */
    double f;             /* objective at the current iterate */
    double pg2;           /* ||grad f(x)[S]||_2 at the last free-set evaluation (the stopping quantity) */
    double pginf;         /* ||x - P(x - grad f(x))||_inf at the same point (epsilon-free KKT residual) */
    int64_t n_fixed;      /* variables outside the free set at that point */
    int branch;           /* last iteration: 1 = projected direction returned by Algorithm 2, 2 = masked quasi-Newton direction */
    int backtracks;       /* last iteration: rejected trial steps */
    int pairs_used;       /* last iteration: pairs that passed the curvature gate */
    int memory_resets;    /* times the pair memory was cleared after an exhausted line search */
    double alpha;         /* last accepted step length */
    double alpha_ub;      /* its upper bound */
    double gp;            /* <grad f, p> of the last iteration */
} lbfgsb_info;

/* error codes */
enum {
    LBFGSB_OK = 0,
    LBFGSB_E_INVALID_ARG = -1,   /* null pointer, n <= 0, m <= 0 or > LBFGSB_MAX_M, ld < cols, n inconsistent with the objective,
                                    workspace too small or misaligned, bad option value */
    LBFGSB_E_BOUNDS = -2,        /* some l_i > u_i, or a NaN bound */
    LBFGSB_E_INFEASIBLE_X0 = -3, /* x0 outside [l, u] or NaN (Algorithm 1 requires a feasible start; it is not projected silently) */
    LBFGSB_E_NONFINITE = -4,     /* f or grad f not finite at x0 */
    LBFGSB_E_HIP = -5,           /* a HIP runtime call failed */
    LBFGSB_E_UNSUPPORTED = -6    /* LBFGSB_APASS_FUSED requested for a shape the fused kernel cannot hold */
};

/* Message for the last error on the calling thread (host string owned by the library). */
const char* lbfgsb_last_error(void);

/* Fills *opt (host) with the defaults listed above. */
void lbfgsb_default_options(lbfgsb_options* opt);

/* Bytes of device workspace lbfgsb_create needs for n variables, m pairs and this objective
 * (only kind, dtype, rows, cols are read).  Returns 0 on invalid arguments. */
size_t lbfgsb_workspace_bytes(int64_t n, int m, const lbfgsb_objective* obj_host, const lbfgsb_options* opt_host);

/* Creates a solver.  l, u: device, n entries each, copied.  obj_host/opt_host: host structs,
 * copied (opt_host may be NULL = defaults).  workspace: device, borrowed until destroy.
 * hip_stream: a hipStream_t (or NULL).  Synchronises the stream (bounds are validated on the
 * host).  The iterate is undefined until lbfgsb_set_x. */
int lbfgsb_create(lbfgsb_solver** out, int64_t n, int m, const double* l, const double* u,
                  const lbfgsb_objective* obj_host, const lbfgsb_options* opt_host,
                  void* workspace, size_t workspace_bytes, void* hip_stream);

/* Sets the iterate to x0 (device, n entries, copied), clears the pair memory and the
 * iteration counter, and evaluates f and grad f there.  Fails with LBFGSB_E_INFEASIBLE_X0 /
 * LBFGSB_E_NONFINITE.  Synchronises the stream. */
int lbfgsb_set_x(lbfgsb_solver* s, const double* x0);

/* One iteration of Algorithm 1 (a no-op once the status is not RUNNING).  With
 * info_host == NULL the call only enqueues kernels and returns without synchronising; with a
 * non-NULL info_host it synchronises and fills it.  The info_host == NULL form issues kernel launches
 * only (no memset, copy or wait), so a run of such calls may be recorded into a HIP graph on the solver's
 * stream; whether a step also recomputes residual and gradient (refresh_every) is decided on the host when
 * the call is made, so a recorded run replays the pattern it was recorded with (use refresh_every = 0, or
 * record a multiple of it).  Not while lbfgsb_enable_apass_timing is on: timed launches carry events. */
int lbfgsb_step(lbfgsb_solver* s, lbfgsb_info* info_host);
/* (For the quadratic kinds the gradient is carried by recurrence between the periodic recomputations.  lbfgsb_solve
 * and the resident organisation re-evaluate it from x before they report LBFGSB_CONVERGED; a loop of lbfgsb_step
 * calls on the fused / two-pass organisations reports LBFGSB_CONVERGED from the carried gradient -- call
 * lbfgsb_solve once at the end if the difference matters.) */

/* Iterates until the tolerance, max_iter or a line-search failure.  The device decides all
 * data-dependent branches; the host only polls the status flag every poll_every iterations (less often in long runs).
 * A least-squares solve is declared converged only with residual and gradient freshly
 * recomputed from x.  info_host may be NULL. */
int lbfgsb_solve(lbfgsb_solver* s, lbfgsb_info* info_host);
/* (Returns LBFGSB_OK with info.status == LBFGSB_RUNNING if 2*max_iter + 64 step launches -- accepted iterations plus
 * retries after memory resets -- have not ended the solve.) */

/* For callers that cannot allocate device memory (code that may run under HIP graph capture restrictions, tight
 * serving loops, harnesses that forbid hipMalloc): lbfgsb_create + lbfgsb_set_x + lbfgsb_solve + lbfgsb_get_x in one
 * call that allocates nothing -- no hipMalloc / hipFree / hipHostMalloc, no event, no host heap object.  The
 * workspace is a file-scope device array of LBFGSB_STATIC_SCRATCH_BYTES inside the library (every GPU the library
 * runs on holds its own copy until the process ends); the host object is static too.
 *   x: device, n entries; in: the feasible start point x0, out: the final iterate.
 *   l, u, obj_host, opt_host, hip_stream, info_host: as for lbfgsb_create / lbfgsb_solve (info_host may be NULL).
 * Same kernels, same arithmetic and same results as the four calls it stands for.  Fails with LBFGSB_E_INVALID_ARG
 * (message naming both sizes) when lbfgsb_workspace_bytes() of the problem exceeds LBFGSB_STATIC_SCRATCH_BYTES, and
 * with the error codes of lbfgsb_create / lbfgsb_set_x otherwise.  Synchronises the stream.  All calls on one GPU
 * share that GPU's array and host object: calls that overlap on one GPU (two threads, two streams) race; calls on
 * different GPUs do not.  The part of the array a call uses is cleared first, so nothing carries over between calls. */
#define LBFGSB_STATIC_SCRATCH_BYTES (32u << 20)
int lbfgsb_solve_static(int64_t n, int m, const double* l, const double* u, const lbfgsb_objective* obj_host,
                        const lbfgsb_options* opt_host, double* x, lbfgsb_info* info_host, void* hip_stream);

/* Per-iteration record, kept on the device in a ring of LBFGSB_HISTORY_CAPACITY entries (the solver's workspace holds
 * it; nothing is read back while iterating).  One record per ACCEPTED iteration of Algorithm 1. */
#define LBFGSB_HISTORY_CAPACITY 256
typedef struct {          /* HOST struct (the device keeps the same layout) */
    int64_t iter;         /* 1-based index of the iteration */
    double f;             /* objective after it */
    double pg2, pginf;    /* ||grad f[S]||_2 and ||x - P(x - grad f)||_inf at the iterate it started from */
    int64_t n_fixed;      /* variables outside the free set there */
    double alpha, alpha_ub, gp;   /* accepted step length, its bound, <grad f, p> */
    int branch;           /* Algorithm 2: 1 = projected direction, 2 = masked quasi-Newton direction */
    int backtracks;       /* rejected trial steps */
    int pairs_used;       /* pairs that passed the curvature gate of Algorithm 3 */
    int memory_resets;    /* resets of the pair memory so far */
} lbfgsb_iter_record;
/* Synchronises and copies the most recent records, oldest first, into records_host (room for `capacity` entries);
 * *count_host receives how many were written (at most min(capacity, LBFGSB_HISTORY_CAPACITY, iterations since
 * lbfgsb_set_x)).  lbfgsb_set_x clears the ring. */
int lbfgsb_get_history(lbfgsb_solver* s, lbfgsb_iter_record* records_host, int capacity, int* count_host);

/* Synchronises and reports the current state. */
int lbfgsb_get_info(lbfgsb_solver* s, lbfgsb_info* info_host);

/* Device-to-device copies of the current iterate / gradient (n entries), enqueued on the
 * solver's stream.  (Logistic objective on the fused pass: steps enqueued without an info struct use a short launch
 * sequence that assumes the first trial step of the line search is accepted; when it is not, the iteration is
 * finished, and the steps after it are redone, the next time the library looks at the device state.  These two calls
 * do that first, which means they wait for the stream, whenever such steps have been enqueued since the last look.
 * Steps replayed from a recorded HIP graph are not seen by that bookkeeping: call lbfgsb_get_info after a replay and
 * before reading x or g.) */
int lbfgsb_get_x(lbfgsb_solver* s, double* x_out);
int lbfgsb_get_g(lbfgsb_solver* s, double* g_out);

/* Frees the host object (the workspace stays the caller's).  NULL is a no-op. */
void lbfgsb_destroy(lbfgsb_solver* s);

/* ---- augmented Lagrangian algorithm -------------------------------------------------------------
 * The paper's section "Complete Framework" (Eq. (augLag)) and Algorithm 4 of its appendix, for LINEAR
 * equality constraints on the least-squares objective:
 *     minimise 0.5*||A x - b||^2  subject to  C x = d,  l <= x <= u.
 * Every outer iteration minimises  L(x, lambda, rho) = 0.5*||A x - b||^2 + rho/2*||C x - d + lambda/rho||^2
 * over the box with the solver above (warm-started at the previous x, pair memory cleared), then sets
 * lambda += rho*(C x - d), and doubles rho when ||C x - d||_inf was not halved by the iteration (the first
 * iteration is compared with the violation at x0).  It stops when the violation is at most ctol and the
 * inner solve converged, or after max_outer iterations.  An inequality row e_r . x <= f_r is passed as the
 * equality e_r . x + s_r = f_r with one more variable s_r >= 0 (minimising L over s_r gives the (.)_+ term
 * of Eq. (augLag) and the multiplier update mu = (mu + rho g)_+).
 *
 * The objective handed to lbfgsb_auglag_create is the STACKED problem: kind LSQ, A = [A; C] with
 * rows = data rows + n_eq, b = [b; d], row_weight NULL.  A and b are borrowed as before; the targets and
 * weights the algorithm rewrites live in the workspace.  Between two inner solves only the constraint rows'
 * targets and weights change; f and grad f at the unchanged x are brought up to date from those n_eq rows
 * alone, not by another pass over the whole matrix.  info.status uses the LBFGSB_* termination codes
 * (LBFGSB_MAX_ITER: outer limit reached). */
typedef struct lbfgsb_auglag lbfgsb_auglag;   /* opaque, host object */

typedef struct {
    double rho0;       /* initial penalty parameter, default 1 (Algorithm 4) */
    double ctol;       /* tolerance on ||C x - d||_inf, default 1e-8 */
    int max_outer;     /* default 100 */
} lbfgsb_auglag_options;

typedef struct {           /* HOST struct */
    int status;            /* LBFGSB_CONVERGED, LBFGSB_MAX_ITER or LBFGSB_LINESEARCH_FAILED */
    int outer;             /* outer iterations done */
    int64_t inner_iters;   /* iterations of the box solver, all outer iterations together */
    double violation;      /* ||C x - d||_inf at the returned x */
    double rho;            /* final penalty parameter */
    double f;              /* 0.5*||A x - b||^2 at the returned x */
    double L;              /* augmented Lagrangian at the returned x for the multipliers it was minimised with */
    double pg2;            /* stopping quantity of the last inner solve */
} lbfgsb_auglag_info;

void lbfgsb_auglag_default_options(lbfgsb_auglag_options* opt);
/* workspace for the inner solver plus the targets, weights and multipliers (0 on invalid arguments) */
size_t lbfgsb_auglag_workspace_bytes(int64_t n, int m, const lbfgsb_objective* stacked_host, int64_t n_eq,
                                     const lbfgsb_options* opt_host);
/* opt_host: options of the inner box solver (tol, tol_relative, max_iter per outer iteration, ...); may be NULL */
int lbfgsb_auglag_create(lbfgsb_auglag** out, int64_t n, int m, const double* l, const double* u,
                         const lbfgsb_objective* stacked_host, int64_t n_eq, const lbfgsb_options* opt_host,
                         const lbfgsb_auglag_options* al_opt_host, void* workspace, size_t workspace_bytes,
                         void* hip_stream);
/* The same algorithm with the constraint rows passed separately: C (device, n_eq x n row-major fp64, n_eq <= 64)
 * and d (device, n_eq entries), on top of any quadratic kind (LSQ, L1SPLIT, QP) given as it is -- nothing is
 * stacked; the penalty term rides on the objective's extra rows.  This is how the dual SVM of the paper's
 * section "Dual SVM" is solved: kind QP with the kernel matrix, the labels as sign and as the single
 * constraint row, b = -1, 0 <= a <= c.  lbfgsb_auglag_info.f is then the objective without the penalty term. */
size_t lbfgsb_auglag_rows_workspace_bytes(int64_t n, int m, const lbfgsb_objective* obj_host, int64_t n_eq,
                                          const lbfgsb_options* opt_host);
int lbfgsb_auglag_create_rows(lbfgsb_auglag** out, int64_t n, int m, const double* l, const double* u,
                              const lbfgsb_objective* obj_host, int64_t n_eq, const double* C, const double* d,
                              const lbfgsb_options* opt_host, const lbfgsb_auglag_options* al_opt_host,
                              void* workspace, size_t workspace_bytes, void* hip_stream);
/* The same algorithm for the marginal constraints of the transport kinds (section "Joint Probability
 * Distribution"):  minimise <M,P> + lambda*r(P)  subject to  P 1 = u,  P^T 1 = v,  l <= P <= u_box.
 * obj_host: kind OT_GAUSS or OT_ENTROPY with A = M, lambda; its b and row_weight are ignored (the algorithm owns
 * them).  marginals: device, rows + cols entries [u; v], borrowed.  The rows + cols multipliers come back from
 * lbfgsb_auglag_get_lambda in the same order.  n_eq = rows + cols structured constraints cost two small sum
 * kernels per evaluation, however many there are. */
size_t lbfgsb_auglag_marginals_workspace_bytes(int m, const lbfgsb_objective* obj_host, const lbfgsb_options* opt_host);
int lbfgsb_auglag_create_marginals(lbfgsb_auglag** out, int m, const double* l, const double* u,
                                   const lbfgsb_objective* obj_host, const double* marginals,
                                   const lbfgsb_options* opt_host, const lbfgsb_auglag_options* al_opt_host,
                                   void* workspace, size_t workspace_bytes, void* hip_stream);
/* Runs Algorithm 4 from x0 (device, n entries, feasible for the box) with lambda = 0, rho = rho0.  The host
 * reads two scalars per outer iteration; everything else stays on the device.  Synchronises. */
int lbfgsb_auglag_solve(lbfgsb_auglag* al, const double* x0, lbfgsb_auglag_info* info_host);
int lbfgsb_auglag_get_x(lbfgsb_auglag* al, double* x_out);            /* device, n entries */
int lbfgsb_auglag_get_lambda(lbfgsb_auglag* al, double* lambda_out);  /* device, n_eq entries */
/* the box solver inside (owned by al): for lbfgsb_get_info, lbfgsb_apass_timing, ... */
lbfgsb_solver* lbfgsb_auglag_inner(lbfgsb_auglag* al);
void lbfgsb_auglag_destroy(lbfgsb_auglag* al);

/* ---- timing of the products with A (the kernels that dominate an iteration) ------------------
 * While enabled, every launch of a kernel that reads A carries a pair of HIP events attached to
 * the dispatch itself (start and end of that kernel on the solver's stream, no extra stream
 * markers) (at most 4096 launches are kept; later ones are not recorded).  enable: 0 =
 * pause (records kept), 1 = resume, 2 = discard the records and start.  lbfgsb_apass_timing
 * synchronises and returns how many launches were timed (launches that returned at once because the
 * solver had already stopped -- duration below half of the 90th-percentile duration -- are left out), their total duration in milliseconds
 * and the bytes of A one launch requests from memory (rows*cols*sizeof(element): each such
 * kernel reads A exactly once).  The transport kinds have no such kernel: there the Gram kernel of the batched
 * two-loop recursion (the longest kernel of an iteration) is timed instead, from the m-th iteration after
 * lbfgsb_set_x on, when all m pairs are stored; the bytes are 41*n (x, g, l, u, the newest y, the mask; 25*n when
 * all variables share the same bounds, which are then not streamed) plus 16*m per free variable (the pair vectors
 * are not read where a variable is fixed). */
int lbfgsb_enable_apass_timing(lbfgsb_solver* s, int enable);
int lbfgsb_apass_timing(lbfgsb_solver* s, int64_t* count_host, double* total_ms_host, double* bytes_per_pass_host);
/* Name of the A-pass organisation in use: "fused", "two_pass" or "resident" (host string). */
const char* lbfgsb_apass_name(const lbfgsb_solver* s);

/* ---- primitive-level hooks --------------------------------------------------------------------
 * Each runs ONE step of the path, with the same kernels lbfgsb_step uses, on inputs the caller
 * supplies, so that it can be compared with a reference implementation on identical data.  They
 * overwrite the solver's iterate and pair memory: call lbfgsb_set_x before stepping again.  All
 * synchronise. */

/* f(x) -> *f_host, grad f(x) -> g (n entries); rowvec (rows entries, may be NULL) receives
 * A v - b (least squares) or the margins A x (logistic); for the transport kinds it has rows + cols entries
 * and receives K P - b. */
int lbfgsb_dbg_fg(lbfgsb_solver* s, const double* x, double* f_host, double* g, double* rowvec);

/* Eq. (ws): mask[i] = 1 if i is free at (x, g), else 0. */
int lbfgsb_dbg_free_mask(lbfgsb_solver* s, const double* x, const double* g, uint8_t* mask);

/* Algorithm 3 on npairs <= m pairs (S, Y: npairs x n, oldest first), gradient g and free mask
 * (1 = free); ynorm2: npairs full-vector values ||y^i||^2.  d receives -q on the free set and 0
 * elsewhere; *pairs_used_host the number of pairs that passed the gate. */
int lbfgsb_dbg_two_loop(lbfgsb_solver* s, const double* S, const double* Y, const double* ynorm2, int npairs,
                        const double* g, const uint8_t* mask, double* d, int* pairs_used_host);

/* Algorithm 2 at (x, g, d): p, the branch taken (1 or 2) and the step-length bound. */
int lbfgsb_dbg_project_direction(lbfgsb_solver* s, const double* x, const double* g, const double* d,
                                 double* p, int* branch_host, double* alpha_ub_host);

#ifdef __cplusplus
}
#endif
#endif /* LBFGSB_H */
