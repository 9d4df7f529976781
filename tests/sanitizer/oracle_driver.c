/*
 * Runs the CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer: the oracle's source is compiled INTO this
 * program with -fsanitize=address,undefined, and the program drives every entry point on small seeded problems
 * (all objective kinds, both storage types, the augmented Lagrangian algorithm, the marginal constraints, an
 * exhausted line search) and checks a few invariants of the results.  A memory error or undefined behaviour aborts
 * the program; a failed check makes it exit with status 1.  Test infrastructure only (tests/test_sanitizers.py).
 */
#include "../../oracle/lbfgsb_oracle.c"

#include <stdio.h>

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static double uniform01(void) {                 /* xorshift64*: enough for test data */
    rng_state ^= rng_state >> 12; rng_state ^= rng_state << 25; rng_state ^= rng_state >> 27;
    return (double)((rng_state * 0x2545F4914F6CDD1Dull) >> 11) / 9007199254740992.0;
}
static double normalish(void) { double s = 0.0; for (int k = 0; k < 12; ++k) s += uniform01(); return s - 6.0; }

static int failures = 0;
#define CHECK(cond) do { if (!(cond)) { fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); ++failures; } } while (0)

static double kkt_residual(int64_t n, const double* x, const double* g, const double* l, const double* u) {
    double r = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        double v = fabs(x[i] - clampd(x[i] - g[i], l[i], u[i]));
        if (v > r) r = v;
    }
    return r;
}

static void solve_kind(int kind, int dtype, int64_t rows, int64_t cols, int m) {
    const int64_t ld = cols + 3;                /* a padded leading dimension */
    double* Ad = (double*)malloc(sizeof(double) * (size_t)(rows * ld));
    float* Af = (float*)malloc(sizeof(float) * (size_t)(rows * ld));
    double* b = (double*)malloc(sizeof(double) * (size_t)rows);
    for (int64_t i = 0; i < rows * ld; ++i) { Ad[i] = normalish(); Af[i] = (float)Ad[i]; }
    if (kind == ORC_QP) {                       /* symmetric positive definite: A = B^T B / rows + I */
        for (int64_t i = 0; i < cols; ++i)
            for (int64_t j = 0; j <= i; ++j) {
                double s = i == j ? 1.0 : 0.0;
                for (int64_t k = 0; k < cols; ++k) s += Ad[k * ld + i] * Ad[k * ld + j] / (double)cols;
                Af[i * ld + j] = Af[j * ld + i] = (float)s;
            }
        for (int64_t i = 0; i < cols; ++i) for (int64_t j = 0; j < cols; ++j) Ad[i * ld + j] = Af[i * ld + j];
    }
    for (int64_t r = 0; r < rows; ++r) b[r] = kind == ORC_LOGISTIC_L2 ? (uniform01() < 0.5 ? -1.0 : 1.0) : normalish();
    orc_objective o;
    memset(&o, 0, sizeof o);
    o.kind = kind; o.dtype = dtype; o.rows = rows; o.cols = cols; o.ld = ld;
    o.A = dtype == ORC_F64 ? (const void*)Ad : (const void*)Af; o.b = b; o.lambda = 0.3; o.mu = 1e-2;
    const int64_t n = orc_num_vars(&o);
    double* l = (double*)malloc(sizeof(double) * (size_t)n);
    double* u = (double*)malloc(sizeof(double) * (size_t)n);
    double* x0 = (double*)malloc(sizeof(double) * (size_t)n);
    for (int64_t i = 0; i < n; ++i) {
        l[i] = kind == ORC_LSQ_L1SPLIT ? 0.0 : (i % 5 == 0 ? -INFINITY : -0.4);
        u[i] = kind == ORC_LSQ_L1SPLIT ? INFINITY : (i % 7 == 0 ? INFINITY : 0.6);
        x0[i] = 0.0;
    }
    orc_options opt;
    orc_default_options(&opt);
    opt.tol = 1e-7; opt.max_iter = 400;
    orc_solver* s = orc_create(n, m, l, u, x0, &o, &opt);
    CHECK(s != NULL);
    if (s) {
        double f_prev = s->f;
        while (orc_step(s) == ORC_RUNNING) { CHECK(s->f <= f_prev + 1e-12 * fabs(f_prev)); f_prev = s->f; }
        orc_refresh_info(s);
        orc_info info;
        orc_get_info(s, &info);
        CHECK(info.status == ORC_CONVERGED);
        CHECK(kkt_residual(n, orc_x(s), orc_g(s), l, u) <= 1e-5);
        for (int64_t i = 0; i < n; ++i) CHECK(orc_x(s)[i] >= l[i] && orc_x(s)[i] <= u[i]);
        CHECK(orc_npairs(s) <= m && orc_S(s) && orc_Y(s) && orc_ynorm2(s) && orc_d(s) && orc_p(s) && orc_mask(s));
        orc_destroy(s);
    }
    x0[1] = -7.0;                                /* infeasible start: refused, nothing allocated is left behind */
    CHECK(orc_create(n, m, l, u, x0, &o, &opt) == NULL);
    x0[1] = 0.0; l[1] = 2.0; u[1] = 1.0;         /* crossed bounds */
    CHECK(orc_create(n, m, l, u, x0, &o, &opt) == NULL);
    free(Ad); free(Af); free(b); free(l); free(u); free(x0);
}

/* the hand-worked exhausted searches of tests/test_oracle_linesearch_exhausted.py */
static void exhausted_search(void) {
    const double A[4] = {2.0, 0.0, 0.0, 1.0}, b[2] = {-0.125, -4.0};
    const double l[2] = {-INFINITY, -INFINITY}, u[2] = {INFINITY, INFINITY}, x0[2] = {0.0, 0.0};
    orc_objective o;
    memset(&o, 0, sizeof o);
    o.kind = ORC_LSQ; o.dtype = ORC_F64; o.rows = 2; o.cols = 2; o.ld = 2; o.A = A; o.b = b;
    orc_options opt;
    orc_default_options(&opt);
    opt.max_backtracks = 0; opt.tol = 1e-12;
    orc_solver* s = orc_create(2, 3, l, u, x0, &o, &opt);
    CHECK(s != NULL);
    CHECK(orc_step(s) == ORC_RUNNING);
    CHECK(orc_x(s)[0] == -0.25 && orc_x(s)[1] == -4.0);
    CHECK(orc_step(s) == ORC_LINESEARCH_FAILED);
    orc_info info;
    orc_get_info(s, &info);
    CHECK(info.memory_resets == 1 && info.iters == 1 && orc_npairs(s) == 0);
    CHECK(orc_x(s)[0] == -0.25 && orc_x(s)[1] == -4.0);
    orc_destroy(s);
}

/* min 0.5 ||A x - b||^2 s.t. sum x = 1, x >= 0, and one inequality row, through Algorithm 4 */
static void auglag_dense(void) {
    enum { R = 30, N = 8 };
    double A[R * N], b[R], C[N], d[1] = {1.0}, E[N], e[1] = {0.3}, lam[1], mu[1], l[N], u[N], x[N];
    for (int i = 0; i < R * N; ++i) A[i] = normalish();
    for (int i = 0; i < R; ++i) b[i] = normalish();
    for (int i = 0; i < N; ++i) { C[i] = 1.0; E[i] = i == 0 ? 1.0 : 0.0; l[i] = 0.0; u[i] = INFINITY; x[i] = 0.0; }
    orc_constraints k;
    memset(&k, 0, sizeof k);
    k.n_eq = 1; k.n_in = 1; k.C = C; k.d = d; k.E = E; k.e = e; k.lambda = lam; k.mu = mu; k.rho = 1.0;
    orc_objective o;
    memset(&o, 0, sizeof o);
    o.kind = ORC_LSQ; o.dtype = ORC_F64; o.rows = R; o.cols = N; o.ld = N; o.A = A; o.b = b; o.con = &k;
    orc_options opt;
    orc_default_options(&opt);
    opt.tol = 1e-9;
    orc_auglag_options ao;
    orc_auglag_default_options(&ao);
    orc_auglag_info info;
    CHECK(orc_auglag_solve(N, 5, l, u, x, &o, &opt, &ao, &info) == 0);
    CHECK(info.status == ORC_CONVERGED);
    double sum = 0.0;
    for (int i = 0; i < N; ++i) { sum += x[i]; CHECK(x[i] >= 0.0); }
    CHECK(fabs(sum - 1.0) <= 1e-7 && x[0] <= 0.3 + 1e-7);
}

/* regularised transport with the marginal constraints, both regularisers */
static void transport(int kind) {
    enum { R = 6, Cn = 5 };
    double M[R * Cn], d[R + Cn], lam[R + Cn], l[R * Cn], u[R * Cn], x[R * Cn];
    for (int i = 0; i < R * Cn; ++i) { M[i] = uniform01(); l[i] = kind == ORC_OT_ENTROPY ? 1e-30 : 0.0; u[i] = INFINITY; x[i] = l[i]; }
    for (int i = 0; i < R; ++i) d[i] = 1.0 / R;
    for (int j = 0; j < Cn; ++j) d[R + j] = 1.0 / Cn;
    orc_constraints k;
    memset(&k, 0, sizeof k);
    k.n_eq = R + Cn; k.d = d; k.lambda = lam; k.rho = 1.0; k.marginals = 1;
    orc_objective o;
    memset(&o, 0, sizeof o);
    o.kind = kind; o.dtype = ORC_F64; o.rows = R; o.cols = Cn; o.ld = Cn; o.A = M; o.lambda = 0.5; o.con = &k;
    orc_options opt;
    orc_default_options(&opt);
    opt.tol = 1e-7; opt.eps = kind == ORC_OT_ENTROPY ? 1e-20 : 1e-10; opt.max_iter = 2000;
    orc_auglag_options ao;
    orc_auglag_default_options(&ao);
    ao.ctol = 1e-6;
    orc_auglag_info info;
    CHECK(orc_auglag_solve(R * Cn, 5, l, u, x, &o, &opt, &ao, &info) == 0);
    CHECK(info.status == ORC_CONVERGED && info.violation <= 1e-6);
    for (int i = 0; i < R; ++i) { double s = 0.0; for (int j = 0; j < Cn; ++j) s += x[i * Cn + j]; CHECK(fabs(s - d[i]) <= 1e-5); }
}

static void primitives(void) {
    enum { N = 9 };
    double x[N], g[N], l[N], u[N], d[N], p[N], S[2 * N], Y[2 * N], yn[2];
    uint8_t mask[N];
    for (int i = 0; i < N; ++i) { x[i] = uniform01(); g[i] = normalish(); l[i] = i % 3 ? 0.0 : -INFINITY; u[i] = i % 2 ? 1.0 : INFINITY; }
    x[1] = 0.0; x[3] = 1.0;
    orc_free_mask(N, x, g, l, u, 1e-10, mask);
    for (int i = 0; i < 2 * N; ++i) { S[i] = normalish(); Y[i] = S[i] * (1.0 + uniform01()); }
    for (int k = 0; k < 2; ++k) { yn[k] = 0.0; for (int i = 0; i < N; ++i) yn[k] += Y[k * N + i] * Y[k * N + i]; }
    int used = -1;
    orc_two_loop(N, 2, S, Y, yn, g, mask, 1e-10, d, &used);
    CHECK(used >= 0 && used <= 2);
    orc_two_loop(N, 0, NULL, NULL, NULL, g, mask, 1e-10, d, &used);    /* empty memory: d = -g on the free set */
    for (int i = 0; i < N; ++i) CHECK(d[i] == (mask[i] ? -g[i] : 0.0));
    double ub = 0.0;
    int br = orc_project_direction(N, x, g, d, l, u, 1e-10, 0, p, &ub);
    CHECK((br == 1 || br == 2) && ub > 0.0);
    br = orc_project_direction(N, x, g, d, l, u, 1e-10, 1, p, &ub);
    CHECK(br == 2);
}

int main(void) {
    primitives();
    exhausted_search();
    const int kinds[4] = {ORC_LSQ, ORC_LSQ_L1SPLIT, ORC_LOGISTIC_L2, ORC_QP};
    for (int k = 0; k < 4; ++k)
        for (int dt = 0; dt < 2; ++dt)
            solve_kind(kinds[k], dt, kinds[k] == ORC_QP ? 11 : 40, 11, 4);
    solve_kind(ORC_LSQ, ORC_F64, 7, 13, 1);       /* more columns than rows, a single stored pair */
    auglag_dense();
    transport(ORC_OT_GAUSS);
    transport(ORC_OT_ENTROPY);
    if (failures) { fprintf(stderr, "%d check(s) failed\n", failures); return 1; }
    printf("oracle under the sanitizers: all checks passed\n");
    return 0;
}
