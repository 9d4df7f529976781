// Runs the host side of the C-ABI library (argument validation, workspace sizing, error reporting) under
// AddressSanitizer and UndefinedBehaviorSanitizer: the library's sources are compiled into this program with the host
// pass instrumented (tests/test_sanitizers.py).  Every call here is refused, or answered, before any device work, so
// the program needs no GPU.  A memory error or undefined behaviour aborts it; a wrong answer makes it exit with 1.
#include <cstdio>
#include <cstring>

#include "lbfgsb.h"

static int failures = 0;
#define CHECK(cond) do { if (!(cond)) { std::fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); ++failures; } } while (0)

static lbfgsb_objective objective(int kind, int64_t rows, int64_t cols) {
    lbfgsb_objective o;
    std::memset(&o, 0, sizeof o);
    o.kind = kind; o.dtype = LBFGSB_F64; o.rows = rows; o.cols = cols; o.ld = cols;
    o.A = (const void*)0x100000; o.b = (const double*)0x200000; o.lambda = 0.5; o.mu = 1e-3;
    return o;
}

int main() {
    lbfgsb_options opt;
    lbfgsb_default_options(&opt);
    lbfgsb_default_options(nullptr);
    CHECK(opt.eps == 1e-10 && opt.max_backtracks == 60 && opt.a_pass == LBFGSB_APASS_AUTO);
    double* const L = (double*)0x300000;
    double* const U = (double*)0x400000;
    void* const W = (void*)0x1000000;
    lbfgsb_solver* s = (lbfgsb_solver*)0x1;

    for (int kind = LBFGSB_OBJ_LSQ; kind <= LBFGSB_OBJ_OT_ENTROPY; ++kind) {
        const bool ot = kind >= LBFGSB_OBJ_OT_GAUSS;
        lbfgsb_objective o = objective(kind, kind == LBFGSB_OBJ_QP ? 96 : 300, 96);
        const int64_t n = ot ? o.rows * o.cols : (kind == LBFGSB_OBJ_LSQ_L1SPLIT ? 192 : 96);
        const size_t need = lbfgsb_workspace_bytes(n, 7, &o, &opt);
        CHECK(need > 0 && need % 256 == 0);
        CHECK(lbfgsb_workspace_bytes(n + 1, 7, &o, &opt) == 0);
        CHECK(lbfgsb_workspace_bytes(n, 0, &o, &opt) == 0 && lbfgsb_workspace_bytes(n, LBFGSB_MAX_M + 1, &o, &opt) == 0);
        CHECK(lbfgsb_create(&s, n, 7, L, U, &o, &opt, W, need - 1, nullptr) == LBFGSB_E_INVALID_ARG && s == nullptr);
        CHECK(std::strstr(lbfgsb_last_error(), "too small") != nullptr);
        CHECK(lbfgsb_create(&s, n, 7, L, U, &o, &opt, (char*)W + 8, need, nullptr) == LBFGSB_E_INVALID_ARG);
        CHECK(lbfgsb_create(&s, n, 7, nullptr, U, &o, &opt, W, need, nullptr) == LBFGSB_E_INVALID_ARG);
        CHECK(lbfgsb_create(nullptr, n, 7, L, U, &o, &opt, W, need, nullptr) == LBFGSB_E_INVALID_ARG);
        lbfgsb_objective bad = o;
        bad.ld = o.cols - 1;
        CHECK(lbfgsb_create(&s, n, 7, L, U, &bad, &opt, W, need, nullptr) == LBFGSB_E_INVALID_ARG);
        bad = o; bad.A = nullptr;
        CHECK(lbfgsb_create(&s, n, 7, L, U, &bad, &opt, W, need, nullptr) == LBFGSB_E_INVALID_ARG);
        bad = o; bad.dtype = 7;
        CHECK(lbfgsb_create(&s, n, 7, L, U, &bad, &opt, W, need, nullptr) == LBFGSB_E_INVALID_ARG);
        lbfgsb_options bo = opt;
        bo.backtrack = 1.5;
        CHECK(lbfgsb_create(&s, n, 7, L, U, &o, &bo, W, need, nullptr) == LBFGSB_E_INVALID_ARG);
        bo = opt; bo.a_pass = 17;
        CHECK(lbfgsb_create(&s, n, 7, L, U, &o, &bo, W, need, nullptr) == LBFGSB_E_INVALID_ARG);
    }
    lbfgsb_objective unknown = objective(42, 10, 10);
    CHECK(lbfgsb_workspace_bytes(10, 3, &unknown, &opt) == 0 && lbfgsb_workspace_bytes(10, 3, nullptr, &opt) == 0);
    lbfgsb_objective rect = objective(LBFGSB_OBJ_QP, 20, 10);
    CHECK(lbfgsb_workspace_bytes(10, 3, &rect, &opt) == 0);

    lbfgsb_info info;
    CHECK(lbfgsb_step(nullptr, &info) == LBFGSB_E_INVALID_ARG && lbfgsb_solve(nullptr, &info) == LBFGSB_E_INVALID_ARG);
    CHECK(lbfgsb_set_x(nullptr, L) == LBFGSB_E_INVALID_ARG && lbfgsb_get_x(nullptr, L) == LBFGSB_E_INVALID_ARG);
    CHECK(lbfgsb_get_g(nullptr, L) == LBFGSB_E_INVALID_ARG && lbfgsb_get_info(nullptr, &info) == LBFGSB_E_INVALID_ARG);
    CHECK(lbfgsb_enable_apass_timing(nullptr, 1) == LBFGSB_E_INVALID_ARG);
    CHECK(std::strcmp(lbfgsb_apass_name(nullptr), "two_pass") == 0);
    lbfgsb_destroy(nullptr);
    lbfgsb_objective lsq = objective(LBFGSB_OBJ_LSQ, 300, 96);
    CHECK(lbfgsb_solve_static(96, 7, L, U, &lsq, &opt, nullptr, &info, nullptr) == LBFGSB_E_INVALID_ARG);

    lbfgsb_auglag_options ao;
    lbfgsb_auglag_default_options(&ao);
    CHECK(ao.rho0 == 1.0 && ao.max_outer == 100);
    lbfgsb_auglag* al = nullptr;
    CHECK(lbfgsb_auglag_workspace_bytes(96, 7, &lsq, 3, &opt) > lbfgsb_workspace_bytes(96, 7, &lsq, &opt));
    CHECK(lbfgsb_auglag_workspace_bytes(96, 7, &lsq, 300, &opt) == 0);
    CHECK(lbfgsb_auglag_create(&al, 96, 7, L, U, &lsq, -1, &opt, &ao, W, 1 << 24, nullptr) == LBFGSB_E_INVALID_ARG);
    CHECK(lbfgsb_auglag_rows_workspace_bytes(96, 7, &lsq, 65, &opt) == 0);
    CHECK(lbfgsb_auglag_solve(nullptr, nullptr, nullptr) == LBFGSB_E_INVALID_ARG);
    CHECK(lbfgsb_auglag_inner(nullptr) == nullptr);
    lbfgsb_auglag_destroy(nullptr);

    if (failures) { std::fprintf(stderr, "%d check(s) failed\n", failures); return 1; }
    std::printf("library boundary under the sanitizers: all checks passed\n");
    return 0;
}
