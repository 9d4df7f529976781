// C-ABI layer of liblbfgsb: argument checks, workspace layout, the fixed kernel sequence of one
// iteration of Algorithm 1, the polling loop of lbfgsb_solve and the primitive-level hooks.
// No solver arithmetic happens on the host.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "common.h"

using namespace lb;

namespace {

thread_local std::string g_err;

int fail(int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

#define HIP_TRY(expr)                                                                           \
    do {                                                                                        \
        hipError_t e_ = (expr);                                                                 \
        if (e_ != hipSuccess) return fail(LBFGSB_E_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

constexpr int kMaxTimed = 4096;

size_t align_up(size_t v) { return (v + 255) & ~(size_t)255; }

}  // namespace

// Workspace of lbfgsb_solve_static, for callers that cannot allocate.  In host code this name is only a stand-in
// for the symbol: the device address comes from hipGetSymbolAddress, once per device (static_slot()), and that
// address is what every kernel argument, fill and copy uses.
// (No `used` attribute: it keeps the symbol local in the code object, and the runtime, which finds a device variable
// by name among the code object's global symbols, then aborts in hipGetSymbolAddress.  The host code's use of the
// variable is what makes the compiler export it.)
static __device__ __align__(256) unsigned char scratch[LBFGSB_STATIC_SCRATCH_BYTES];

struct lbfgsb_solver {
    Dims dm;
    Opts op;
    lbfgsb_options options;
    lbfgsb_objective obj;
    Geometry ge;
    Buffers bf;
    hipStream_t stream;
    Scal* h_scal;            // host copy (pinned, allocated by lbfgsb_create)
    bool owns_h_scal;
    int use_fused;
    int use_resident;        // small least squares: whole iterations in one resident workgroup
    // logistic objective on the fused pass: steps still to be enqueued with the full launch sequence (after a
    // rejected first trial step), and short-sequence steps enqueued since the host last looked at the scalar block
    int logi_full_left;
    int short_steps_unseen;
    bool short_ok;           // the short sequence is available (the pass has the LDS for its per-row numbers)
    bool commit_needed;      // resident solver: a kernel of the multi-kernel path may have left an update pending
    // Called by lbfgsb_solve after it has enqueued the re-evaluation that confirms convergence and before it waits for
    // the result: work that is only wanted if convergence is confirmed can ride on the same wait (the augmented
    // Lagrangian's multiplier update, whose kernel looks at the status word itself).
    void (*after_retest)(void*) = nullptr;
    void* after_retest_ctx = nullptr;
    bool last_read_was_retest = false;   // the scalar block was last read behind such a call
    // lbfgsb_solve looks at the status after this many steps the first time (0: after poll_every, as always later).
    // A warm-started solve that may be over at once (the augmented Lagrangian's later inner solves) sets 1: every step
    // enqueued behind the one that converged is four launches that return at once.
    int first_batch = 0;
    int steps_since_refresh;
    long long steps_since_set_x;
    bool x_set;
    // timing
    bool timing;
    std::vector<hipEvent_t> ev0, ev1;
    int timed;
};

namespace {

// objective is a quadratic along every direction: closed-form line search, gradient carried by recurrence
bool is_quadratic(int kind) { return kind != LBFGSB_OBJ_LOGISTIC_L2 && kind != LBFGSB_OBJ_OT_ENTROPY; }

int check_objective(int64_t n, int m, const lbfgsb_objective* o) {
    if (!o) return fail(LBFGSB_E_INVALID_ARG, "objective is NULL");
    if (n <= 0) return fail(LBFGSB_E_INVALID_ARG, "n must be positive (got %lld)", (long long)n);
    if (m <= 0 || m > LBFGSB_MAX_M) return fail(LBFGSB_E_INVALID_ARG, "m must be in 1..%d (got %d)", LBFGSB_MAX_M, m);
    if (o->kind < LBFGSB_OBJ_LSQ || o->kind > LBFGSB_OBJ_OT_ENTROPY)
        return fail(LBFGSB_E_INVALID_ARG, "unknown objective kind %d", o->kind);
    if (o->kind == LBFGSB_OBJ_QP && o->rows != o->cols)
        return fail(LBFGSB_E_INVALID_ARG, "the quadratic form needs a square matrix (got %lld x %lld)", (long long)o->rows,
                    (long long)o->cols);
    if (o->n_extra < 0 || o->n_extra > kMaxExtra) return fail(LBFGSB_E_INVALID_ARG, "n_extra must be in 0..%d", kMaxExtra);
    if (o->n_extra > 0 && (o->kind == LBFGSB_OBJ_LOGISTIC_L2 || is_transport(o->kind)))
        return fail(LBFGSB_E_INVALID_ARG, "extra rows go with the least-squares and quadratic-form kinds");
    if (is_transport(o->kind) && !(o->lambda > 0.0))
        return fail(LBFGSB_E_INVALID_ARG, "the transport kinds need lambda > 0");
    if (o->dtype != LBFGSB_F64 && o->dtype != LBFGSB_F32) return fail(LBFGSB_E_INVALID_ARG, "unknown dtype %d", o->dtype);
    if (o->rows <= 0 || o->cols <= 0) return fail(LBFGSB_E_INVALID_ARG, "rows and cols must be positive");
    if (o->rows > (1ll << 31) - 1 || o->cols > (1ll << 31) - 1) return fail(LBFGSB_E_INVALID_ARG, "rows/cols exceed 2^31-1");
    if (o->ld < o->cols) return fail(LBFGSB_E_INVALID_ARG, "ld (%lld) < cols (%lld)", (long long)o->ld, (long long)o->cols);
    if (is_transport(o->kind) && o->rows > ((1ll << 40) / o->cols))
        return fail(LBFGSB_E_INVALID_ARG, "rows*cols exceeds 2^40 variables");
    const int64_t expect = is_transport(o->kind) ? o->rows * o->cols
                         : o->kind == LBFGSB_OBJ_LSQ_L1SPLIT ? 2 * o->cols : o->cols;
    if (n != expect) return fail(LBFGSB_E_INVALID_ARG, "n = %lld does not match the objective (%lld variables)", (long long)n, (long long)expect);
    return LBFGSB_OK;
}

int check_options(const lbfgsb_options* o) {
    if (!(o->eps >= 0.0) || !(o->armijo_c1 > 0.0 && o->armijo_c1 < 1.0) || !(o->backtrack > 0.0 && o->backtrack < 1.0) ||
        o->max_backtracks < 0 || !(o->tol >= 0.0) || o->max_iter < 0 || o->refresh_every < 0 || o->poll_every < 1 ||
        o->a_pass < LBFGSB_APASS_AUTO || o->a_pass > LBFGSB_APASS_RESIDENT)
        return fail(LBFGSB_E_INVALID_ARG, "bad option value");
    return LBFGSB_OK;
}

Geometry make_geometry(const Dims& dm, const void* A) {
    Geometry ge{};
    const int per16 = dm.dtype == LBFGSB_F32 ? 4 : 2;
    const bool aligned = ((uintptr_t)A % 16 == 0) && (dm.cols % per16 == 0) && (dm.ld % per16 == 0);
    ge.vec = aligned ? per16 : 1;
    int64_t gb = (dm.rows + kWaves * 4 - 1) / (kWaves * 4);
    ge.gemv_blocks = (int)(gb > 2048 ? 2048 : gb);
    const int64_t cols_per_tile = (int64_t)kBlock * ge.vec;
    ge.gemvt_col_tiles = (int)((dm.cols + cols_per_tile - 1) / cols_per_tile);
    int64_t rb = 2048 / ge.gemvt_col_tiles;
    const int64_t rb_max = (dm.rows + 31) / 32;
    if (rb > rb_max) rb = rb_max;
    if (rb > 512) rb = 512;
    if (rb < 1) rb = 1;
    ge.gemvt_rows_per_block = (dm.rows + rb - 1) / rb;
    ge.gemvt_row_blocks = (int)((dm.rows + ge.gemvt_rows_per_block - 1) / ge.gemvt_rows_per_block);
    ge.fused_ok = !is_transport(dm.kind) && fused_shape_ok(dm, A, &ge.fused_variant, &ge.fused_blocks) ? 1 : 0;
    ge.gram_blocks = gram_blocks_for(dm.n, dm.m);
    int64_t db = (dm.n + kBlock - 1) / kBlock;
    ge.dir_blocks = (int)(db > kDirBlocksMax ? kDirBlocksMax : db);
    int64_t ub = (dm.cols + 15) / 16;   // 16 columns per workgroup in the column-sum kernels
    ge.upd_blocks = ge.fin_blocks = (int)(ub > 2048 ? 2048 : ub);
    int64_t lb_ = (dm.rows + kBlock - 1) / kBlock;
    ge.ls_blocks = (int)(lb_ > 128 ? 128 : lb_);   // (the line search ends in a single-address arrival: few workgroups)
    ge.lrows_blocks = (int)(lb_ > 512 ? 512 : lb_);   // the margins' update has no such ending: 512 measured faster than 128
    {
        // workgroups for the columns plus workgroups for the margins (four rows per thread), at most 512 in all
        int64_t rb4 = (dm.rows + 4 * kBlock - 1) / (4 * kBlock);
        int64_t tot = rb4 + ge.upd_blocks;
        ge.updl_blocks = (int)(tot > 512 ? 512 : tot);
    }
    if (is_transport(dm.kind)) {
        int rpw = 1;
        while (rpw < kOtRpwMax && (dm.rows + rpw - 1) / rpw > 512) rpw *= 2;
        ge.ot_rpw = rpw;
        ge.ot_row_blocks = (int)((dm.rows + rpw - 1) / rpw);
        int64_t cb = (dm.cols + kCX - 1) / kCX;
        ge.ot_col_blocks = (int)(cb > 2048 ? 2048 : cb);
        ge.ot_el_blocks = (int)(dm.rows > 512 ? 512 : dm.rows);
        int64_t eb = (dm.n + kBlock - 1) / kBlock;
        ge.ls_blocks = (int)(eb > 512 ? 512 : eb);
    }
    return ge;
}

struct Layout {
    size_t scal, scal_next, x, g, l, u, d, p1, p2, mask, S, Y, row, t, psi, wpart, losspart, grampart, redpart, lspart, wextra, xres, hist, total;
};

Layout make_layout(const Dims& dm, const Geometry& ge) {
    Layout L{};
    size_t off = 0;
    // (wextra / xres are appended at the end so that the offsets of everything else do not depend on n_extra)
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    const size_t nb = (size_t)dm.n * 8, rb = (size_t)row_entries(dm.kind, dm.rows, dm.cols) * 8;
    L.scal = take(sizeof(Scal));
    L.scal_next = take(sizeof(Scal));
    L.x = take(nb); L.g = take(nb); L.l = take(nb); L.u = take(nb); L.d = take(nb); L.p1 = take(nb); L.p2 = take(nb);
    L.mask = take((size_t)dm.n);
    L.S = take(nb * dm.m); L.Y = take(nb * dm.m);
    L.row = take(rb); L.t = take(rb); L.psi = take(rb);
    int wparts = ge.gemvt_row_blocks;
    if (ge.fused_ok && ge.fused_blocks > wparts) wparts = ge.fused_blocks;
    if (is_transport(dm.kind)) wparts = ge.ot_row_blocks;
    L.wpart = take((size_t)wparts * dm.cols * 8);
    int lparts = ge.gemv_blocks;
    if (ge.fused_ok && ge.fused_blocks > lparts) lparts = ge.fused_blocks;
    if (ge.ls_blocks > lparts) lparts = ge.ls_blocks;
    if (ge.lrows_blocks > lparts) lparts = ge.lrows_blocks;
    if (is_transport(dm.kind) && ge.ot_row_blocks + ge.ot_col_blocks > lparts) lparts = ge.ot_row_blocks + ge.ot_col_blocks;
    L.losspart = take((size_t)lparts * 8);
    L.grampart = take(gram_partial_bytes(dm.n, dm.m));
    size_t red = (size_t)ge.dir_blocks * (8 + 2 * kFoldMax);
    if ((size_t)ge.upd_blocks * 2 > red) red = (size_t)ge.upd_blocks * 2;
    if ((size_t)ge.updl_blocks * 2 > red) red = (size_t)ge.updl_blocks * 2;
    if (is_transport(dm.kind) && (size_t)ge.ot_el_blocks > red) red = (size_t)ge.ot_el_blocks;
    L.redpart = take(red * 8);
    L.lspart = take((size_t)ge.ls_blocks * 64 * 8);   // up to 64 step lengths per sweep (entropy line search: 51)
    L.wextra = take(dm.n_extra > 0 ? (size_t)dm.n * 8 : 8);
    L.xres = take((size_t)(dm.n_extra + 1) * 8);
    L.hist = take((size_t)LBFGSB_HISTORY_CAPACITY * sizeof(lbfgsb_iter_record));
    L.total = off;
    return L;
}

Dims make_dims(int64_t n, int m, const lbfgsb_objective* o) {
    Dims dm{};
    dm.n = n; dm.rows = o->rows; dm.cols = o->cols; dm.ld = o->ld; dm.m = m; dm.kind = o->kind; dm.dtype = o->dtype;
    dm.lambda = o->lambda; dm.mu = o->mu;
    dm.n_extra = (int)o->n_extra;
    return dm;
}

void enqueue_step(lbfgsb_solver* s);

// Reads the scalar block after applying any update the last step left pending.  If the short logistic launch sequence
// has parked the solver (first trial step rejected: kStatusBail), the iteration is finished here with the launches
// that sequence leaves out, the steps that found the solver parked are enqueued again, and the block is read anew.
hipError_t read_scal(lbfgsb_solver* s) {
    for (;;) {
        // (the resident solver applies its updates itself; only its evaluations by the multi-kernel path leave one pending)
        if (!s->use_resident || s->commit_needed) launch_commit(s->dm, s->bf, s->stream);
        s->commit_needed = false;
        hipError_t e = hipMemcpyAsync(s->h_scal, s->bf.scal, sizeof(Scal), hipMemcpyDeviceToHost, s->stream);
        if (e != hipSuccess) return e;
        e = hipStreamSynchronize(s->stream);
        if (e != hipSuccess) return e;
        s->short_steps_unseen = 0;
        if (s->h_scal->status != kStatusBail) return hipSuccess;
        const int redo = s->h_scal->bail_skipped;
        launch_clear_bail(s->bf, s->stream);
        // the rest of the interrupted iteration: more step lengths, new margins and row weights, the transposed
        // pass for the accepted step, the update
        launch_ls_logistic(s->dm, s->op, s->ge, s->bf, s->obj.b, 1, 2, s->stream);
        launch_rows_logistic(s->dm, s->ge, s->bf, s->obj.b, s->stream);
        launch_gemvt_from(s->dm, s->ge, s->bf, s->obj.A, s->bf.psi, 2, s->stream, nullptr, nullptr);
        launch_update_logistic(s->dm, s->op, s->ge, s->bf, s->ge.lrows_blocks, 0, s->stream);
        s->logi_full_left = 8 + redo;   // a problem that backtracks once tends to do so again: full sequence for a while
        for (int k = 0; k < redo; ++k) enqueue_step(s);
    }
}

// Uploads a fresh scalar block (host template in h_scal) and waits for it.
hipError_t write_scal(lbfgsb_solver* s) {
    hipError_t e = hipMemcpyAsync(s->bf.scal, s->h_scal, sizeof(Scal), hipMemcpyHostToDevice, s->stream);
    if (e != hipSuccess) return e;
    return hipStreamSynchronize(s->stream);
}

void fill_info(const Scal& sc, lbfgsb_info* info) {
    info->status = sc.status; info->iters = sc.iters; info->fevals = sc.fevals; info->f = sc.f;
    info->pg2 = sc.pg2; info->pginf = sc.pginf; info->n_fixed = sc.n_fixed; info->branch = sc.branch;
    info->backtracks = sc.backtracks; info->pairs_used = sc.pairs_used; info->memory_resets = sc.memory_resets;
    info->alpha = sc.alpha; info->alpha_ub = sc.alpha_ub; info->gp = sc.gp;
}

// Events for the next launch of a kernel that reads A (null when timing is off or the store is full).
struct TimedSlot {
    hipEvent_t e0 = nullptr, e1 = nullptr;
    explicit TimedSlot(lbfgsb_solver* s, bool wanted = true) {
        if (wanted && s->timing && s->timed < kMaxTimed) {
            e0 = s->ev0[s->timed];
            e1 = s->ev1[s->timed];
            s->timed++;
        }
    }
};

APassArgs base_args(const lbfgsb_solver* s) {
    APassArgs a{};
    a.A = s->obj.A; a.b = s->obj.b;
    a.w = (s->dm.kind == LBFGSB_OBJ_LSQ || s->dm.kind == LBFGSB_OBJ_LSQ_L1SPLIT) ? s->obj.row_weight : nullptr;
    a.vs = s->dm.kind == LBFGSB_OBJ_QP ? s->obj.sign : nullptr;
    a.p1 = s->bf.p1; a.p2 = s->bf.p2;
    a.split = s->dm.kind == LBFGSB_OBJ_LSQ_L1SPLIT;
    return a;
}

OtArgs ot_args(const lbfgsb_solver* s) {
    return OtArgs{s->obj.A, s->obj.b, s->obj.row_weight};
}

// f, g (and the residual / margins) from scratch at the current x.
void enqueue_eval(lbfgsb_solver* s, int check_status) {
    launch_commit(s->dm, s->bf, s->stream);   // a pending f must not overwrite the one computed here
    if (is_transport(s->dm.kind)) {
        const OtArgs oa = ot_args(s);
        launch_ot_sums(s->dm, s->ge, s->bf, oa, 1, check_status, s->stream);
        launch_ot_eval_finish(s->dm, s->ge, s->bf, oa, s->stream);
        return;
    }
    APassArgs a = base_args(s);
    a.va = s->bf.x;
    a.vb = a.split ? s->bf.x + s->dm.cols : nullptr;
    a.select_p = 0;
    const bool qp = s->dm.kind == LBFGSB_OBJ_QP;
    a.mode = qp ? kRowQpEval : (is_quadratic(s->dm.kind) ? kRowLsqEval : kRowLogiEval);
    a.check_status = check_status;
    if (qp) {
        // symmetric matrix: the gradient needs the row products only
        TimedSlot ts(s);
        if (s->use_fused) launch_fused(s->dm, s->ge, s->bf, a, s->stream, ts.e0, ts.e1);
        else launch_gemv(s->dm, s->ge, s->bf, a, s->stream, ts.e0, ts.e1);
    } else if (s->use_fused) {
        TimedSlot ts(s);
        launch_fused(s->dm, s->ge, s->bf, a, s->stream, ts.e0, ts.e1);
    } else {
        { TimedSlot ts(s); launch_gemv(s->dm, s->ge, s->bf, a, s->stream, ts.e0, ts.e1); }
        { TimedSlot ts(s); launch_gemvt_from(s->dm, s->ge, s->bf, s->obj.A, s->bf.psi, check_status, s->stream, ts.e0, ts.e1); }
    }
    if (s->dm.n_extra > 0)
        launch_extra_rows(s->dm, s->bf, s->obj.extra_rows, s->obj.extra_target, s->obj.extra_weight, 1, s->stream);
    launch_eval_finish(s->dm, s->ge, s->bf, s->obj.b, s->obj.sign, s->stream);
}

// One iteration of Algorithm 1 as a fixed sequence of launches; nothing here waits for the device.
void enqueue_step(lbfgsb_solver* s) {
    if (s->use_resident) {
        // (the periodic recomputation and the pending-update bookkeeping happen inside the kernel)
        launch_resident(s->dm, s->op, s->bf, s->obj.A, s->obj.b, 1, s->options.refresh_every, s->stream);
        return;
    }
    const bool quad = is_quadratic(s->dm.kind);
    if (quad && s->options.refresh_every > 0 && s->steps_since_refresh >= s->options.refresh_every) {
        enqueue_eval(s, 1);
        s->steps_since_refresh = 0;
    }
    if (is_transport(s->dm.kind)) {
        // no matrix product: the iteration streams the pair memory twice (Gram matrix, direction) and the
        // iterate-sized vectors a few times.  The Gram kernel is the longest and the one that is timed.
        // (timed only once the pair memory is full, so that every timed launch moves the same bytes)
        {
            TimedSlot ts(s, s->steps_since_set_x >= s->dm.m);
            launch_gram(s->dm, s->op, s->ge, s->bf, 0, 1, s->stream, ts.e0, ts.e1);
        }
        // (the direction kernel ends without its closing step: the row-sum kernel, the first to need Algorithm 2's
        // choice, makes it from the per-workgroup sums)
        launch_dir(s->dm, s->op, s->ge, s->bf, 0, 0, s->stream, nullptr, nullptr, 1);
        const OtArgs oa = ot_args(s);
        launch_ot_sums(s->dm, s->ge, s->bf, oa, 0, 1, s->stream, s->ge.dir_blocks, s->op.eps);
        if (quad) launch_ot_update_gauss(s->dm, s->op, s->ge, s->bf, oa, s->stream);
        else launch_ot_step_entropy(s->dm, s->op, s->ge, s->bf, oa, s->stream);
        s->steps_since_refresh++;
        s->steps_since_set_x++;
        return;
    }
    // one or two extra rows ride along with the direction kernel; more get the kernel of their own
    const bool fold = quad && dir_folds_extra_rows(s->dm);
    const double* fold_rows = fold ? s->obj.extra_rows : nullptr;
    // The single-read pass can make Algorithm 2's choice itself from the direction kernel's partial sums, which then
    // needs no closing step (not with extra rows that have a kernel of their own, which reads the choice from the
    // scalar block; rows folded into the direction kernel get their coefficients in the update kernel)
    const bool defer = s->use_fused && (s->dm.n_extra == 0 || fold);
    // ... and then the Gram kernel needs no closing step either, where its grid is small enough for the direction
    // kernel's workgroups to add its partial sums themselves: they finish its work on private copies of the scalar
    // block, and the pass moves workgroup 0's copy into place (Buffers::scal_next)
    const bool open_gram = defer && gram_can_skip_close(s->dm, s->ge);
    launch_gram(s->dm, s->op, s->ge, s->bf, 0, 1, s->stream, nullptr, nullptr, open_gram ? 1 : 0);
    launch_dir(s->dm, s->op, s->ge, s->bf, 0, 0, s->stream, fold_rows, s->obj.extra_weight, defer ? 1 : 0,
               open_gram ? s->ge.gram_blocks : 0);
    APassArgs a = base_args(s);
    a.select_p = 1;
    a.check_status = 1;
    if (defer) {
        a.dir_part = s->bf.redpart; a.dir_blocks = s->ge.dir_blocks; a.eps = s->op.eps;
        if (open_gram) a.scal_next = s->bf.scal_next;
    }
    const int fold_blocks = defer && fold ? s->ge.dir_blocks : 0;   // the update kernel forms the folded rows' coefficients
    if (quad && s->dm.n_extra > 0 && !fold)
        launch_extra_rows(s->dm, s->bf, s->obj.extra_rows, s->obj.extra_target, s->obj.extra_weight, 0, s->stream);
    if (s->dm.kind == LBFGSB_OBJ_QP) {
        a.mode = kRowQpDir;
        {
            TimedSlot ts(s);
            if (s->use_fused) launch_fused(s->dm, s->ge, s->bf, a, s->stream, ts.e0, ts.e1);
            else launch_gemv(s->dm, s->ge, s->bf, a, s->stream, ts.e0, ts.e1);
        }
        launch_update_quadratic(s->dm, s->op, s->ge, s->bf, s->obj.sign, s->stream, fold_rows, s->obj.extra_weight, fold_blocks);
    } else if (quad) {
        a.mode = kRowDir;
        if (s->use_fused) {
            TimedSlot ts(s);
            launch_fused(s->dm, s->ge, s->bf, a, s->stream, ts.e0, ts.e1);
        } else {
            { TimedSlot ts(s); launch_gemv(s->dm, s->ge, s->bf, a, s->stream, ts.e0, ts.e1); }
            { TimedSlot ts(s); launch_gemvt_from(s->dm, s->ge, s->bf, s->obj.A, s->bf.psi, 1, s->stream, ts.e0, ts.e1); }
        }
        launch_update_quadratic(s->dm, s->op, s->ge, s->bf, nullptr, s->stream, fold_rows, s->obj.extra_weight, fold_blocks);
    } else if (s->use_fused) {
        // One read of X yields t = X p AND X^T psi for the first trial step min(1, alpha_ub).  The line
        // search over the margins then decides; only if it does not accept that first step does a second
        // (transposed) pass over X run, otherwise that launch returns at once.  The transposed pass is not
        // among the timed launches: it reads A only in the iterations that backtrack.
        a.mode = kRowLogiSpec;
        const bool full = s->logi_full_left > 0 || !s->short_ok;
        a.ls_first = full ? 0 : 1;
        { TimedSlot ts(s); launch_fused(s->dm, s->ge, s->bf, a, s->stream, ts.e0, ts.e1); }
        if (full) {
            if (s->logi_full_left > 0) s->logi_full_left--;
            launch_ls_logistic(s->dm, s->op, s->ge, s->bf, s->obj.b, 1, 3, s->stream);
            launch_rows_logistic(s->dm, s->ge, s->bf, s->obj.b, s->stream);
            launch_gemvt_from(s->dm, s->ge, s->bf, s->obj.A, s->bf.psi, 2, s->stream, nullptr, nullptr);
            launch_update_logistic(s->dm, s->op, s->ge, s->bf, s->ge.lrows_blocks, 0, s->stream);
        } else {
            // Short sequence: the pass itself sums the loss differences of the first trial step over each workgroup's
            // rows, and the update kernel takes the Armijo decision from those partials; the update of an accepted
            // first step also moves the margins.  The search kernels, the recomputation of the row weights and the
            // second transposed pass -- launches that almost never do work -- are left out; should the first step be
            // rejected, the solver parks itself and read_scal() supplies them.
            launch_update_logistic(s->dm, s->op, s->ge, s->bf, s->ge.fused_blocks, 1, s->stream);
            s->short_steps_unseen++;
        }
    } else {
        a.mode = kRowLogiDir;
        { TimedSlot ts(s); launch_gemv(s->dm, s->ge, s->bf, a, s->stream, ts.e0, ts.e1); }
        launch_ls_logistic(s->dm, s->op, s->ge, s->bf, s->obj.b, 0, 3, s->stream);
        launch_rows_logistic(s->dm, s->ge, s->bf, s->obj.b, s->stream);
        { TimedSlot ts(s); launch_gemvt_from(s->dm, s->ge, s->bf, s->obj.A, s->bf.psi, 1, s->stream, ts.e0, ts.e1); }
        launch_update_logistic(s->dm, s->op, s->ge, s->bf, s->ge.lrows_blocks, 0, s->stream);
    }
    s->steps_since_refresh++;
}

void fresh_scal(lbfgsb_solver* s) {
    std::memset(s->h_scal, 0, sizeof(Scal));
    s->h_scal->status = LBFGSB_RUNNING;
    s->h_scal->alpha_ub = 1.0;
    s->h_scal->hist = s->bf.hist;
}

// trusted: x0 is the solver's own iterate (feasible by construction): only f is checked for finiteness and
// nothing iterate-sized crosses to the host
int set_x_impl(lbfgsb_solver* s, const double* x0, bool trusted) {
    const int64_t n = s->dm.n;
    std::vector<double> hx;
    if (!trusted) {
        std::vector<double> hl((size_t)n), hu((size_t)n);
        hx.resize((size_t)n);
        HIP_TRY(hipMemcpyAsync(hx.data(), x0, (size_t)n * 8, hipMemcpyDeviceToHost, s->stream));
        HIP_TRY(hipMemcpyAsync(hl.data(), s->bf.l, (size_t)n * 8, hipMemcpyDeviceToHost, s->stream));
        HIP_TRY(hipMemcpyAsync(hu.data(), s->bf.u, (size_t)n * 8, hipMemcpyDeviceToHost, s->stream));
        HIP_TRY(hipStreamSynchronize(s->stream));
        for (int64_t i = 0; i < n; ++i) {
            const double v = hx[(size_t)i];
            if (!(v >= hl[(size_t)i]) || !(v <= hu[(size_t)i]))
                return fail(LBFGSB_E_INFEASIBLE_X0, "x0[%lld] = %g is outside [%g, %g]", (long long)i, v, hl[(size_t)i],
                            hu[(size_t)i]);
        }
    }
    if (x0 != s->bf.x) HIP_TRY(hipMemcpyAsync(s->bf.x, x0, (size_t)n * 8, hipMemcpyDeviceToDevice, s->stream));
    fresh_scal(s);
    // (no wait: the pinned block is next touched by the read below, which the stream orders after this upload)
    HIP_TRY(hipMemcpyAsync(s->bf.scal, s->h_scal, sizeof(Scal), hipMemcpyHostToDevice, s->stream));
    enqueue_eval(s, 0);
    s->steps_since_refresh = 0;
    s->steps_since_set_x = 0;
    s->logi_full_left = 0;
    s->short_steps_unseen = 0;
    if (!trusted) HIP_TRY(hipMemcpyAsync(hx.data(), s->bf.g, (size_t)n * 8, hipMemcpyDeviceToHost, s->stream));
    HIP_TRY(read_scal(s));
    HIP_TRY(hipGetLastError());
    bool finite = std::isfinite(s->h_scal->f);
    for (int64_t i = 0; finite && !trusted && i < n; ++i) finite = std::isfinite(hx[(size_t)i]);
    if (!finite) { s->x_set = false; return fail(LBFGSB_E_NONFINITE, "f or grad f is not finite at x0"); }
    s->x_set = true;
    return LBFGSB_OK;
}


// Argument checks shared by the entry points that set a solver up; *o receives the options (defaults when opt is NULL).
int check_create_args(int64_t n, int m, const double* l, const double* u, const lbfgsb_objective* obj,
                      const lbfgsb_options* opt, const void* workspace, lbfgsb_options* o) {
    int rc = check_objective(n, m, obj);
    if (rc) return rc;
    const bool ot = is_transport(obj->kind);
    if (!l || !u || !obj->A || !workspace) return fail(LBFGSB_E_INVALID_ARG, "NULL device pointer");
    if (ot ? (obj->row_weight && !obj->b) : !obj->b) return fail(LBFGSB_E_INVALID_ARG, "NULL device pointer (b)");
    if (obj->n_extra > 0 && (!obj->extra_rows || !obj->extra_target))
        return fail(LBFGSB_E_INVALID_ARG, "NULL extra_rows / extra_target");
    if (opt) *o = *opt; else lbfgsb_default_options(o);
    rc = check_options(o);
    if (rc) return rc;
    if ((uintptr_t)workspace % 256) return fail(LBFGSB_E_INVALID_ARG, "workspace must be 256-byte aligned");
    const int esz = obj->dtype == LBFGSB_F32 ? 4 : 8;
    if ((uintptr_t)obj->A % esz || (uintptr_t)obj->b % 8 || (uintptr_t)obj->row_weight % 8 || (uintptr_t)l % 8 ||
        (uintptr_t)u % 8)
        return fail(LBFGSB_E_INVALID_ARG, "misaligned device pointer");
    return LBFGSB_OK;
}

// Fills the host object for a checked problem: launch geometry, kernel preparation, and the device arrays carved
// out of `workspace`.  Allocates nothing and touches no device memory; *total receives the bytes of workspace in use.
int setup_solver(lbfgsb_solver* s, int64_t n, int m, const lbfgsb_objective* obj, const lbfgsb_options& o,
                 void* workspace, size_t workspace_bytes, hipStream_t stream, size_t* total) {
    s->dm = make_dims(n, m, obj);
    s->options = o;
    s->op = Opts{o.eps, o.armijo_c1, o.backtrack, o.tol, o.max_backtracks, o.tol_relative, o.max_iter, 0, 0.0, 0.0};
    s->obj = *obj;
    s->ge = make_geometry(s->dm, obj->A);
    s->stream = stream;
    s->h_scal = nullptr;
    s->owns_h_scal = false;
    s->steps_since_refresh = 0;
    s->steps_since_set_x = 0;
    s->logi_full_left = 0;
    s->short_steps_unseen = 0;
    s->commit_needed = true;
    s->x_set = false;
    s->timing = false;
    s->timed = 0;
    const Layout L = make_layout(s->dm, s->ge);
    *total = L.total;
    if (workspace_bytes < L.total)
        return fail(LBFGSB_E_INVALID_ARG, "workspace too small: %zu < %zu bytes", workspace_bytes, L.total);
    if (o.a_pass == LBFGSB_APASS_FUSED && !s->ge.fused_ok)
        return fail(LBFGSB_E_UNSUPPORTED, "the fused A pass does not support this shape");
    {
        const hipError_t ge_ = gram_prepare(n, m);
        if (ge_ != hipSuccess) return fail(LBFGSB_E_HIP, "preparing the Gram kernel: %s", hipGetErrorString(ge_));
    }
    const bool resident_ok = resident_shape_ok(s->dm, obj->row_weight != nullptr);
    if (o.a_pass == LBFGSB_APASS_RESIDENT && !resident_ok)
        return fail(LBFGSB_E_UNSUPPORTED, "the resident solver does not take this problem (kind, shape or size)");
    s->use_resident = resident_ok && (o.a_pass == LBFGSB_APASS_AUTO || o.a_pass == LBFGSB_APASS_RESIDENT);
    if (s->use_resident) {
        const hipError_t re = resident_prepare(s->dm);
        if (re != hipSuccess) return fail(LBFGSB_E_HIP, "preparing the resident solver: %s", hipGetErrorString(re));
    }
    s->use_fused = s->ge.fused_ok && o.a_pass != LBFGSB_APASS_TWO_PASS;
    if (s->use_fused) {
        const hipError_t fe = fused_prepare(s->dm, s->ge);
        if (fe != hipSuccess) return fail(LBFGSB_E_HIP, "preparing the fused A pass: %s", hipGetErrorString(fe));
    }
    s->short_ok = s->use_fused && s->dm.kind == LBFGSB_OBJ_LOGISTIC_L2 && fused_ls_first_ok(s->dm, s->ge);
    s->ge.w_parts = s->use_fused ? s->ge.fused_blocks : s->ge.gemvt_row_blocks;
    s->ge.loss_parts = s->use_fused ? s->ge.fused_blocks : s->ge.gemv_blocks;

    char* w = (char*)workspace;
    Buffers& b = s->bf;
    b.scal = (Scal*)(w + L.scal);
    b.scal_next = (Scal*)(w + L.scal_next);
    b.x = (double*)(w + L.x); b.g = (double*)(w + L.g); b.l = (double*)(w + L.l); b.u = (double*)(w + L.u);
    b.d = (double*)(w + L.d); b.p1 = (double*)(w + L.p1); b.p2 = (double*)(w + L.p2);
    b.mask = (uint8_t*)(w + L.mask);
    b.S = (double*)(w + L.S); b.Y = (double*)(w + L.Y);
    b.row = (double*)(w + L.row); b.t = (double*)(w + L.t); b.psi = (double*)(w + L.psi);
    b.wpart = (double*)(w + L.wpart); b.losspart = (double*)(w + L.losspart);
    b.grampart = (double*)(w + L.grampart); b.redpart = (double*)(w + L.redpart); b.lspart = (double*)(w + L.lspart);
    b.wextra = (double*)(w + L.wextra); b.xres = (double*)(w + L.xres);
    b.hist = (lbfgsb_iter_record*)(w + L.hist);
    return LBFGSB_OK;
}

// The workspace starts from all-zero memory (fill kernel: no memset node ever enters a captured graph); the bounds
// are copied in.  Waits for both.
int init_workspace(lbfgsb_solver* s, const double* l, const double* u, void* workspace, size_t total) {
    launch_fill_zero(workspace, total, s->stream);
    hipError_t e = hipMemcpyAsync(s->bf.l, l, (size_t)s->dm.n * 8, hipMemcpyDeviceToDevice, s->stream);
    if (e == hipSuccess) e = hipMemcpyAsync(s->bf.u, u, (size_t)s->dm.n * 8, hipMemcpyDeviceToDevice, s->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(s->stream);
    if (e == hipSuccess) e = hipGetLastError();
    if (e != hipSuccess) return fail(LBFGSB_E_HIP, "initialising the workspace: %s", hipGetErrorString(e));
    return LBFGSB_OK;
}

constexpr int kPollMax = 64;   // steps between two looks at the device status, at most

// The stopping logic of lbfgsb_solve, for a solver whose arguments have been checked.
int solve_impl(lbfgsb_solver* s, lbfgsb_info* info) {
    const bool quad = is_quadratic(s->dm.kind);
    const long long cap = 2ll * s->options.max_iter + 64;   // accepted iterations + memory-reset retries
    if (s->use_resident) {
        // one launch runs until the device-side status changes (it re-evaluates the gradient from x before it
        // reports convergence) or the cap is reached
        const int steps_cap = (int)(cap > 0x3fffffff ? 0x3fffffff : cap);
        if (s->owns_h_scal) {
            // (pinned host copy: the kernel writes the scalar block there itself, with every pending update applied)
            launch_resident(s->dm, s->op, s->bf, s->obj.A, s->obj.b, steps_cap, s->options.refresh_every, s->stream, s->h_scal);
            s->commit_needed = false;
            HIP_TRY(hipStreamSynchronize(s->stream));
        } else {
            launch_resident(s->dm, s->op, s->bf, s->obj.A, s->obj.b, steps_cap, s->options.refresh_every, s->stream);
            HIP_TRY(read_scal(s));
        }
        HIP_TRY(hipGetLastError());
        if (info) fill_info(*s->h_scal, info);
        return LBFGSB_OK;
    }
    long long steps = 0;
    s->last_read_was_retest = false;
    // A poll leaves the device idle for about 30 us (commit, copy of the scalar block, the host's wake-up and the next
    // launches), a step enqueued after the solver has stopped costs about 6.  Long runs are therefore polled less
    // often: the interval doubles whenever eight intervals' worth of steps have gone by, up to 64.
    int batch = s->first_batch > 0 ? s->first_batch : s->options.poll_every;
    bool first = s->first_batch > 0;
    for (;;) {
        for (int k = 0; k < batch; ++k) enqueue_step(s);
        steps += batch;
        if (first) { batch = s->options.poll_every; first = false; }
        else if (batch < kPollMax && steps >= 8ll * batch) batch = 2 * batch > kPollMax ? kPollMax : 2 * batch;
        HIP_TRY(read_scal(s));
        s->last_read_was_retest = false;
        int st = s->h_scal->status;
        if (st == LBFGSB_CONVERGED && quad && s->steps_since_refresh > 0 && s->h_scal->iters > 0) {
            // the stopping quantity was computed from a gradient carried by recurrence: recompute
            // residual and gradient from x and test again before declaring convergence
            launch_set_status(s->bf, LBFGSB_RUNNING, s->stream);
            enqueue_eval(s, 0);
            s->steps_since_refresh = 0;
            launch_gram(s->dm, s->op, s->ge, s->bf, 0, 1, s->stream);
            if (s->after_retest) s->after_retest(s->after_retest_ctx);
            HIP_TRY(read_scal(s));
            s->last_read_was_retest = s->after_retest != nullptr;
            st = s->h_scal->status;
        }
        if (st != LBFGSB_RUNNING) break;
        if (steps >= cap) break;
    }
    HIP_TRY(hipGetLastError());
    if (info) fill_info(*s->h_scal, info);
    return LBFGSB_OK;
}


// ---- lbfgsb_solve_static: per-device state, nothing of it allocated at run time ----------------------------

constexpr int kMaxDevices = 64;
constexpr int kHostChunk = 2048;   // doubles per host-side validation chunk (stack arrays)

struct StaticSlot {
    void* ptr = nullptr;       // device address of this device's copy of `scratch`
    lbfgsb_solver solver;      // host object, reused by every call on the device
    Scal h_scal;               // host copy of the scalar block (pageable: allocating pinned memory is an allocation)
};
StaticSlot g_static[kMaxDevices];

// The calling thread's current device's slot, with the address of that device's scratch array resolved.
int static_slot(StaticSlot** out) {
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(LBFGSB_E_INVALID_ARG, "device index %d is not supported", dev);
    StaticSlot* sl = &g_static[dev];
    if (!sl->ptr) {
        void* p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p || (uintptr_t)p % 256) return fail(LBFGSB_E_HIP, "the scratch array has no usable device address");
        sl->ptr = p;
    }
    *out = sl;
    return LBFGSB_OK;
}

// Bounds and start point checked on the host in chunks that live on the stack: l <= u, l <= x0 <= u, no NaN,
// l > 0 for the entropy kind; also finds out whether all variables share one pair of bounds.
int check_box_chunked(lbfgsb_solver* s, const double* l, const double* u, const double* x0) {
    double hl[kHostChunk], hu[kHostChunk], hx[kHostChunk];
    const int64_t n = s->dm.n;
    bool same = true;
    double lo0 = 0.0, hi0 = 0.0;
    for (int64_t i0 = 0; i0 < n; i0 += kHostChunk) {
        const int64_t cnt = n - i0 < kHostChunk ? n - i0 : kHostChunk;
        HIP_TRY(hipMemcpyAsync(hl, l + i0, (size_t)cnt * 8, hipMemcpyDeviceToHost, s->stream));
        HIP_TRY(hipMemcpyAsync(hu, u + i0, (size_t)cnt * 8, hipMemcpyDeviceToHost, s->stream));
        HIP_TRY(hipMemcpyAsync(hx, x0 + i0, (size_t)cnt * 8, hipMemcpyDeviceToHost, s->stream));
        HIP_TRY(hipStreamSynchronize(s->stream));
        if (i0 == 0) { lo0 = hl[0]; hi0 = hu[0]; }
        for (int64_t k = 0; k < cnt; ++k) {
            if (!(hl[k] <= hu[k]))
                return fail(LBFGSB_E_BOUNDS, "bounds cross or are NaN at index %lld (l = %g, u = %g)", (long long)(i0 + k),
                            hl[k], hu[k]);
            if (s->dm.kind == LBFGSB_OBJ_OT_ENTROPY && !(hl[k] > 0.0))
                return fail(LBFGSB_E_BOUNDS, "the entropy regulariser needs l > 0 (l[%lld] = %g)", (long long)(i0 + k), hl[k]);
            if (!(hx[k] >= hl[k]) || !(hx[k] <= hu[k]))
                return fail(LBFGSB_E_INFEASIBLE_X0, "x0[%lld] = %g is outside [%g, %g]", (long long)(i0 + k), hx[k], hl[k],
                            hu[k]);
            same = same && hl[k] == lo0 && hu[k] == hi0;
        }
    }
    s->op.uniform_bounds = same ? 1 : 0;
    s->op.lo = lo0;
    s->op.hi = hi0;
    return LBFGSB_OK;
}

int check_finite_chunked(lbfgsb_solver* s, const double* v) {
    double hv[kHostChunk];
    for (int64_t i0 = 0; i0 < s->dm.n; i0 += kHostChunk) {
        const int64_t cnt = s->dm.n - i0 < kHostChunk ? s->dm.n - i0 : kHostChunk;
        HIP_TRY(hipMemcpyAsync(hv, v + i0, (size_t)cnt * 8, hipMemcpyDeviceToHost, s->stream));
        HIP_TRY(hipStreamSynchronize(s->stream));
        for (int64_t k = 0; k < cnt; ++k)
            if (!std::isfinite(hv[k])) return fail(LBFGSB_E_NONFINITE, "f or grad f is not finite at x0");
    }
    return LBFGSB_OK;
}

}  // namespace

extern "C" {

const char* lbfgsb_last_error(void) { return g_err.c_str(); }

void lbfgsb_default_options(lbfgsb_options* o) {
    if (!o) return;
    o->eps = 1e-10; o->armijo_c1 = 1e-4; o->backtrack = 0.5; o->max_backtracks = 60; o->tol = 1e-8;
    o->tol_relative = 0; o->max_iter = 1000; o->refresh_every = 32; o->poll_every = 8; o->a_pass = LBFGSB_APASS_AUTO;
}

size_t lbfgsb_workspace_bytes(int64_t n, int m, const lbfgsb_objective* obj, const lbfgsb_options* opt) {
    (void)opt;
    if (check_objective(n, m, obj) != LBFGSB_OK) return 0;
    const Dims dm = make_dims(n, m, obj);
    const Geometry ge = make_geometry(dm, obj->A);
    return make_layout(dm, ge).total;
}

int lbfgsb_create(lbfgsb_solver** out, int64_t n, int m, const double* l, const double* u, const lbfgsb_objective* obj,
                  const lbfgsb_options* opt, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!out) return fail(LBFGSB_E_INVALID_ARG, "out is NULL");
    *out = nullptr;
    lbfgsb_options o;
    int rc = check_create_args(n, m, l, u, obj, opt, workspace, &o);
    if (rc) return rc;
    lbfgsb_solver* s = new (std::nothrow) lbfgsb_solver();
    if (!s) return fail(LBFGSB_E_INVALID_ARG, "out of host memory");
    size_t total = 0;
    rc = setup_solver(s, n, m, obj, o, workspace, workspace_bytes, (hipStream_t)hip_stream, &total);
    if (rc) { delete s; return rc; }

    auto bail = [&](int code) { lbfgsb_destroy(s); return code; };
    {
        hipError_t e = hipHostMalloc((void**)&s->h_scal, sizeof(Scal), hipHostMallocDefault);
        if (e != hipSuccess) { s->h_scal = nullptr; return bail(fail(LBFGSB_E_HIP, "hipHostMalloc: %s", hipGetErrorString(e))); }
        s->owns_h_scal = true;
    }
    // validate the bounds on the host
    std::vector<double> hl((size_t)n), hu((size_t)n);
    hipError_t e = hipMemcpyAsync(hl.data(), l, (size_t)n * 8, hipMemcpyDeviceToHost, s->stream);
    if (e == hipSuccess) e = hipMemcpyAsync(hu.data(), u, (size_t)n * 8, hipMemcpyDeviceToHost, s->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(s->stream);
    if (e != hipSuccess) return bail(fail(LBFGSB_E_HIP, "reading the bounds: %s", hipGetErrorString(e)));
    for (int64_t i = 0; i < n; ++i)
        if (!(hl[(size_t)i] <= hu[(size_t)i]))
            return bail(fail(LBFGSB_E_BOUNDS, "bounds cross or are NaN at index %lld (l = %g, u = %g)", (long long)i,
                             hl[(size_t)i], hu[(size_t)i]));
    {
        bool same = true;
        for (int64_t i = 1; same && i < n; ++i) same = hl[(size_t)i] == hl[0] && hu[(size_t)i] == hu[0];
        s->op.uniform_bounds = same ? 1 : 0;
        s->op.lo = hl[0];
        s->op.hi = hu[0];
    }
    if (obj->kind == LBFGSB_OBJ_OT_ENTROPY)
        for (int64_t i = 0; i < n; ++i)
            if (!(hl[(size_t)i] > 0.0))
                return bail(fail(LBFGSB_E_BOUNDS, "the entropy regulariser needs l > 0 (l[%lld] = %g)", (long long)i,
                                 hl[(size_t)i]));
    rc = init_workspace(s, l, u, workspace, total);
    if (rc) return bail(rc);
    *out = s;
    return LBFGSB_OK;
}

void lbfgsb_destroy(lbfgsb_solver* s) {
    if (!s) return;
    for (hipEvent_t ev : s->ev0) (void)hipEventDestroy(ev);
    for (hipEvent_t ev : s->ev1) (void)hipEventDestroy(ev);
    if (s->h_scal && s->owns_h_scal) (void)hipHostFree(s->h_scal);
    delete s;
}

int lbfgsb_set_x(lbfgsb_solver* s, const double* x0) {
    if (!s || !x0) return fail(LBFGSB_E_INVALID_ARG, "NULL argument");
    return set_x_impl(s, x0, false);
}

int lbfgsb_step(lbfgsb_solver* s, lbfgsb_info* info) {
    if (!s) return fail(LBFGSB_E_INVALID_ARG, "solver is NULL");
    if (!s->x_set) return fail(LBFGSB_E_INVALID_ARG, "lbfgsb_set_x has not been called");
    enqueue_step(s);
    if (info) {
        HIP_TRY(read_scal(s));
        HIP_TRY(hipGetLastError());
        fill_info(*s->h_scal, info);
    }
    return LBFGSB_OK;
}

int lbfgsb_solve(lbfgsb_solver* s, lbfgsb_info* info) {
    if (!s) return fail(LBFGSB_E_INVALID_ARG, "solver is NULL");
    if (!s->x_set) return fail(LBFGSB_E_INVALID_ARG, "lbfgsb_set_x has not been called");
    return solve_impl(s, info);
}

int lbfgsb_solve_static(int64_t n, int m, const double* l, const double* u, const lbfgsb_objective* obj,
                        const lbfgsb_options* opt, double* x, lbfgsb_info* info, void* hip_stream) {
    if (!x) return fail(LBFGSB_E_INVALID_ARG, "x is NULL");
    if ((uintptr_t)x % 8) return fail(LBFGSB_E_INVALID_ARG, "misaligned device pointer");
    StaticSlot* sl = nullptr;
    int rc = static_slot(&sl);
    if (rc) return rc;
    lbfgsb_options o;
    rc = check_create_args(n, m, l, u, obj, opt, sl->ptr, &o);
    if (rc) return rc;
    const size_t need = lbfgsb_workspace_bytes(n, m, obj, &o);
    if (need == 0 || need > (size_t)LBFGSB_STATIC_SCRATCH_BYTES)
        return fail(LBFGSB_E_INVALID_ARG,
                    "this problem needs %zu bytes of workspace, lbfgsb_solve_static holds %zu: use lbfgsb_create with a "
                    "workspace of your own", need, (size_t)LBFGSB_STATIC_SCRATCH_BYTES);
    lbfgsb_solver* s = &sl->solver;
    if (s->timing || !s->ev0.empty()) return fail(LBFGSB_E_INVALID_ARG, "the static solver object is in an unexpected state");
    size_t total = 0;
    rc = setup_solver(s, n, m, obj, o, sl->ptr, (size_t)LBFGSB_STATIC_SCRATCH_BYTES, (hipStream_t)hip_stream, &total);
    if (rc) return rc;
    s->h_scal = &sl->h_scal;
    rc = check_box_chunked(s, l, u, x);
    if (rc) return rc;
    // the array keeps the previous call's contents: everything this problem uses starts from zero again
    rc = init_workspace(s, l, u, sl->ptr, total);
    if (rc) return rc;
    rc = set_x_impl(s, x, true);
    if (rc) return rc;
    rc = check_finite_chunked(s, s->bf.g);
    if (rc) { s->x_set = false; return rc; }
    rc = solve_impl(s, info);
    if (rc) return rc;
    HIP_TRY(hipMemcpyAsync(x, s->bf.x, (size_t)n * 8, hipMemcpyDeviceToDevice, s->stream));
    HIP_TRY(hipStreamSynchronize(s->stream));
    s->x_set = false;
    return LBFGSB_OK;
}

int lbfgsb_get_history(lbfgsb_solver* s, lbfgsb_iter_record* records, int capacity, int* count) {
    if (!s || !records || !count || capacity < 0) return fail(LBFGSB_E_INVALID_ARG, "NULL argument or negative capacity");
    *count = 0;
    HIP_TRY(read_scal(s));
    const long long written = s->h_scal->hist_count;
    long long have = written < LBFGSB_HISTORY_CAPACITY ? written : LBFGSB_HISTORY_CAPACITY;
    if (have > capacity) have = capacity;
    // the `have` most recent records, oldest first: ring positions (written - have) .. (written - 1)
    for (long long k = 0; k < have; ++k) {
        const long long pos = (written - have + k) % LBFGSB_HISTORY_CAPACITY;
        HIP_TRY(hipMemcpyAsync(records + k, s->bf.hist + pos, sizeof(lbfgsb_iter_record), hipMemcpyDeviceToHost, s->stream));
    }
    HIP_TRY(hipStreamSynchronize(s->stream));
    *count = (int)have;
    return LBFGSB_OK;
}

int lbfgsb_get_info(lbfgsb_solver* s, lbfgsb_info* info) {
    if (!s || !info) return fail(LBFGSB_E_INVALID_ARG, "NULL argument");
    HIP_TRY(read_scal(s));
    fill_info(*s->h_scal, info);
    return LBFGSB_OK;
}

int lbfgsb_get_x(lbfgsb_solver* s, double* x_out) {
    if (!s || !x_out) return fail(LBFGSB_E_INVALID_ARG, "NULL argument");
    if (s->short_steps_unseen > 0) HIP_TRY(read_scal(s));   // a parked solver is brought up to date first (this waits)
    HIP_TRY(hipMemcpyAsync(x_out, s->bf.x, (size_t)s->dm.n * 8, hipMemcpyDeviceToDevice, s->stream));
    return LBFGSB_OK;
}

int lbfgsb_get_g(lbfgsb_solver* s, double* g_out) {
    if (!s || !g_out) return fail(LBFGSB_E_INVALID_ARG, "NULL argument");
    if (s->short_steps_unseen > 0) HIP_TRY(read_scal(s));
    HIP_TRY(hipMemcpyAsync(g_out, s->bf.g, (size_t)s->dm.n * 8, hipMemcpyDeviceToDevice, s->stream));
    return LBFGSB_OK;
}

int lbfgsb_enable_apass_timing(lbfgsb_solver* s, int enable) {
    if (!s) return fail(LBFGSB_E_INVALID_ARG, "solver is NULL");
    if (enable && s->ev0.empty()) {
        s->ev0.resize(kMaxTimed);
        s->ev1.resize(kMaxTimed);
        for (int i = 0; i < kMaxTimed; ++i) {
            HIP_TRY(hipEventCreate(&s->ev0[i]));
            HIP_TRY(hipEventCreate(&s->ev1[i]));
        }
    }
    s->timing = enable != 0;
    if (enable == 2) s->timed = 0;
    return LBFGSB_OK;
}

int lbfgsb_apass_timing(lbfgsb_solver* s, int64_t* count, double* total_ms, double* bytes_per_pass) {
    if (!s || !count || !total_ms || !bytes_per_pass) return fail(LBFGSB_E_INVALID_ARG, "NULL argument");
    HIP_TRY(hipStreamSynchronize(s->stream));
    // launches enqueued after the solver had stopped return at once without touching A: they are recognised
    // by their duration (below half of a typical long launch: the 90th percentile, so that a single launch
    // stretched by a profiler or a clock ramp does not set the scale) and left out
    std::vector<float> dur((size_t)s->timed);
    for (int i = 0; i < s->timed; ++i) HIP_TRY(hipEventElapsedTime(&dur[(size_t)i], s->ev0[i], s->ev1[i]));
    float longest = 0.f;
    if (!dur.empty()) {
        std::vector<float> sorted(dur);
        std::sort(sorted.begin(), sorted.end());
        longest = sorted[(size_t)((sorted.size() - 1) * 9 / 10)];
    }
    double tot = 0.0;
    int64_t n = 0;
    for (int i = 0; i < s->timed; ++i)
        if (dur[(size_t)i] >= 0.5f * longest) { tot += dur[(size_t)i]; ++n; }
    *count = n;
    *total_ms = tot;
    *bytes_per_pass = (double)s->dm.rows * (double)s->dm.cols * (s->dm.dtype == LBFGSB_F32 ? 4.0 : 8.0);
    // transport kinds: the timed kernel is the Gram kernel, timed in iterations m, m+1, ... after lbfgsb_set_x, when
    // all m pairs are stored.  It reads x, g, the newest y (and l, u unless every variable has the same bounds) in
    // full and writes the one-byte free mask; the 2m pair vectors are read at the free variables only (count taken
    // from the last status the host has seen)
    if (is_transport(s->dm.kind)) {
        const double n_free = (double)(s->dm.n - s->h_scal->n_fixed);
        *bytes_per_pass = (double)s->dm.n * (s->op.uniform_bounds ? 25.0 : 41.0) + n_free * 2.0 * s->dm.m * 8.0;
    }
    return LBFGSB_OK;
}


const char* lbfgsb_apass_name(const lbfgsb_solver* s) {
    if (s && s->use_resident) return "resident";
    return s && s->use_fused ? "fused" : "two_pass";
}

// ---- primitive-level hooks ------------------------------------------------------------------------------

int lbfgsb_dbg_fg(lbfgsb_solver* s, const double* x, double* f_host, double* g, double* rowvec) {
    if (!s || !x || !f_host || !g) return fail(LBFGSB_E_INVALID_ARG, "NULL argument");
    s->x_set = false;
    HIP_TRY(hipMemcpyAsync(s->bf.x, x, (size_t)s->dm.n * 8, hipMemcpyDeviceToDevice, s->stream));
    fresh_scal(s);
    HIP_TRY(write_scal(s));
    enqueue_eval(s, 0);
    HIP_TRY(hipMemcpyAsync(g, s->bf.g, (size_t)s->dm.n * 8, hipMemcpyDeviceToDevice, s->stream));
    if (rowvec)
        HIP_TRY(hipMemcpyAsync(rowvec, s->bf.row, (size_t)row_entries(s->dm.kind, s->dm.rows, s->dm.cols) * 8,
                               hipMemcpyDeviceToDevice, s->stream));
    HIP_TRY(read_scal(s));
    HIP_TRY(hipGetLastError());
    *f_host = s->h_scal->f;
    return LBFGSB_OK;
}

int lbfgsb_dbg_free_mask(lbfgsb_solver* s, const double* x, const double* g, uint8_t* mask) {
    if (!s || !x || !g || !mask) return fail(LBFGSB_E_INVALID_ARG, "NULL argument");
    s->x_set = false;
    HIP_TRY(hipMemcpyAsync(s->bf.x, x, (size_t)s->dm.n * 8, hipMemcpyDeviceToDevice, s->stream));
    HIP_TRY(hipMemcpyAsync(s->bf.g, g, (size_t)s->dm.n * 8, hipMemcpyDeviceToDevice, s->stream));
    fresh_scal(s);
    HIP_TRY(write_scal(s));
    launch_gram(s->dm, s->op, s->ge, s->bf, 0, 0, s->stream);
    HIP_TRY(hipMemcpyAsync(mask, s->bf.mask, (size_t)s->dm.n, hipMemcpyDeviceToDevice, s->stream));
    HIP_TRY(hipStreamSynchronize(s->stream));
    HIP_TRY(hipGetLastError());
    return LBFGSB_OK;
}

int lbfgsb_dbg_two_loop(lbfgsb_solver* s, const double* S, const double* Y, const double* ynorm2, int npairs,
                        const double* g, const uint8_t* mask, double* d, int* pairs_used) {
    if (!s || !g || !mask || !d) return fail(LBFGSB_E_INVALID_ARG, "NULL argument");
    if (npairs < 0 || npairs > s->dm.m) return fail(LBFGSB_E_INVALID_ARG, "npairs must be in 0..m");
    if (npairs > 0 && (!S || !Y || !ynorm2)) return fail(LBFGSB_E_INVALID_ARG, "NULL pair arrays");
    s->x_set = false;
    const size_t nb = (size_t)s->dm.n * 8;
    fresh_scal(s);
    if (npairs > 0) {
        HIP_TRY(hipMemcpyAsync(s->bf.S, S, nb * npairs, hipMemcpyDeviceToDevice, s->stream));
        HIP_TRY(hipMemcpyAsync(s->bf.Y, Y, nb * npairs, hipMemcpyDeviceToDevice, s->stream));
        HIP_TRY(hipMemcpyAsync(s->h_scal->ynorm2, ynorm2, (size_t)npairs * 8, hipMemcpyDeviceToHost, s->stream));
        HIP_TRY(hipStreamSynchronize(s->stream));
    }
    s->h_scal->count = npairs;
    s->h_scal->head = npairs % s->dm.m;
    HIP_TRY(write_scal(s));
    HIP_TRY(hipMemcpyAsync(s->bf.g, g, nb, hipMemcpyDeviceToDevice, s->stream));
    HIP_TRY(hipMemcpyAsync(s->bf.mask, mask, (size_t)s->dm.n, hipMemcpyDeviceToDevice, s->stream));
    launch_gram(s->dm, s->op, s->ge, s->bf, 1, 0, s->stream);
    launch_dir(s->dm, s->op, s->ge, s->bf, 0, 1, s->stream);
    HIP_TRY(hipMemcpyAsync(d, s->bf.d, nb, hipMemcpyDeviceToDevice, s->stream));
    HIP_TRY(read_scal(s));
    HIP_TRY(hipGetLastError());
    if (pairs_used) *pairs_used = s->h_scal->pairs_used;
    return LBFGSB_OK;
}

int lbfgsb_dbg_project_direction(lbfgsb_solver* s, const double* x, const double* g, const double* d, double* p,
                                 int* branch, double* alpha_ub) {
    if (!s || !x || !g || !d || !p) return fail(LBFGSB_E_INVALID_ARG, "NULL argument");
    s->x_set = false;
    const size_t nb = (size_t)s->dm.n * 8;
    HIP_TRY(hipMemcpyAsync(s->bf.x, x, nb, hipMemcpyDeviceToDevice, s->stream));
    HIP_TRY(hipMemcpyAsync(s->bf.g, g, nb, hipMemcpyDeviceToDevice, s->stream));
    HIP_TRY(hipMemcpyAsync(s->bf.d, d, nb, hipMemcpyDeviceToDevice, s->stream));
    fresh_scal(s);
    HIP_TRY(write_scal(s));
    launch_dir(s->dm, s->op, s->ge, s->bf, 1, 1, s->stream);
    HIP_TRY(read_scal(s));
    HIP_TRY(hipGetLastError());
    const int br = s->h_scal->branch;
    HIP_TRY(hipMemcpyAsync(p, br == 1 ? s->bf.p1 : s->bf.p2, nb, hipMemcpyDeviceToDevice, s->stream));
    HIP_TRY(hipStreamSynchronize(s->stream));
    if (branch) *branch = br;
    if (alpha_ub) *alpha_ub = s->h_scal->alpha_ub;
    return LBFGSB_OK;
}


// ---- augmented Lagrangian algorithm (Algorithm 4 of the appendix, Eq. (augLag)) ------------------------------
//
// Linear equality constraints h(x) = C x - d = 0 on the least-squares objective.  The rows of C are
// appended to A, and   rho/2 ||C x - d + lambda/rho||^2   is then a block of least-squares rows with weight
// rho and target d - lambda/rho: every outer iteration rewrites those targets and weights and runs the box
// solver on  L(., lambda, rho) = 0.5 sum_r w_r (a_r . x - beta_r)^2,  so the single-read pass, the closed-form
// line search and everything else of the path serve the constrained problem unchanged.

}  // extern "C"

struct lbfgsb_auglag {
    lbfgsb_solver* inner;
    lbfgsb_auglag_options ao;
    int64_t n_eq, n;
    // the constraint rows' targets d (caller's), and the targets / weights the algorithm rewrites (workspace):
    // entries of the stacked matrix's row vectors, or the inner objective's extra rows
    const double* d_c;
    double *beta_c, *omega_c;
    const double* res_c;     // where the inner solver leaves a_r . x - beta_r of the constraint rows after an evaluation
    double *lambda, *red;    // multipliers; red[0] = violation, red[1] = penalty term
    double* h_red;           // pinned host copy of red
    double rho;
    hipStream_t stream;
    // stacked variant only: the constraint rows inside the caller's matrix, and n_eq doubles of scratch (the
    // change of weight*residual per constraint row), for re-evaluating f and g after the targets changed
    const void* c_rows = nullptr;
    double* coef = nullptr;
};

namespace {

__global__ void k_al_init(int64_t rows, const double* __restrict__ bd, double* __restrict__ beta,
                          double* __restrict__ omega) {
    for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < rows; r += (int64_t)gridDim.x * blockDim.x) {
        beta[r] = bd[r];
        omega[r] = 1.0;
    }
}

// targets d - lambda/rho and weights rho of the constraint rows for the next inner solve
__global__ void k_al_prepare(int64_t n_eq, double rho, const double* __restrict__ d, const double* __restrict__ lambda,
                             double* __restrict__ beta, double* __restrict__ omega) {
    for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < n_eq; r += (int64_t)gridDim.x * blockDim.x) {
        beta[r] = d[r] - lambda[r] / rho;
        omega[r] = rho;
    }
}

// Stacked variant, between two inner solves: only the targets beta and the weights omega of the constraint rows
// change, so f and g at the unchanged x follow from the fresh residuals without another pass over the whole matrix:
// with c_r . x = res_r + beta_r,  res_r' = c_r . x - beta_r',  f' = f + 0.5 sum (omega' res'^2 - omega res^2),
// g' = g + C^T (omega' res' - omega res).  First kernel (one workgroup): new targets, weights and residuals, the
// coefficients omega' res' - omega res, and f; second kernel: the n_eq x n product into g.
__global__ __launch_bounds__(kBlock) void k_al_shift_rows(int64_t n_eq, double rho, const double* __restrict__ d,
                                                          const double* __restrict__ lambda, double* __restrict__ beta,
                                                          double* __restrict__ omega, double* __restrict__ res,
                                                          double* __restrict__ coef, Scal* __restrict__ scal) {
    __shared__ double lds[kWaves];
    double df[1] = {0.0};
    for (int64_t r = threadIdx.x; r < n_eq; r += kBlock) {
        const double res_old = res[r], w_old = omega[r];
        const double cx = res_old + beta[r];
        const double b_new = d[r] - lambda[r] / rho;
        const double res_new = cx - b_new;
        coef[r] = rho * res_new - w_old * res_old;
        df[0] += 0.5 * (rho * res_new * res_new - w_old * res_old * res_old);
        beta[r] = b_new;
        omega[r] = rho;
        res[r] = res_new;
    }
    block_sum<1, kWaves>(df, lds);
    if (threadIdx.x == 0) scal->f += df[0];
}

template <typename T>
__global__ void k_al_shift_g(int64_t n_eq, int64_t cols, int64_t ld, const T* __restrict__ Crows,
                             const double* __restrict__ coef, double* __restrict__ g) {
    for (int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < cols; j += (int64_t)gridDim.x * blockDim.x) {
        double acc = 0.0;
        for (int64_t r = 0; r < n_eq; ++r) acc = fma(coef[r], (double)Crows[r * ld + j], acc);
        g[j] += acc;
    }
}

// One workgroup.  res holds a_r . x - beta_r of the constraint rows, freshly evaluated at x:
// h_r = res_r - lambda_r/rho; with update != 0 the multipliers become lambda + rho h.  red[0] = ||h||_inf,
// red[1] = rho/2 sum (h + lambda/rho)^2 (the penalty term at the OLD multipliers).
// gate (or NULL): do nothing unless that scalar block says CONVERGED.
__global__ __launch_bounds__(kBlock) void k_al_update(int64_t n_eq, double rho, int update,
                                                      const double* __restrict__ res, double* __restrict__ lambda,
                                                      double* __restrict__ red, const Scal* __restrict__ gate) {
    __shared__ double lds[kWaves * 2];
    if (gate && gate->status != LBFGSB_CONVERGED) return;
    double viol = 0.0, pen = 0.0;
    for (int64_t r = threadIdx.x; r < n_eq; r += kBlock) {
        const double a = res[r];
        const double h = a - lambda[r] / rho;
        viol = fmax(viol, fabs(h));
        pen = fma(a, a, pen);
        if (update) lambda[r] += rho * h;
    }
    double pv[1] = {pen};
    block_sum<1, kWaves>(pv, lds);
    viol = wave_max(viol);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = viol;
    __syncthreads();
    if (threadIdx.x == 0) {
        double v = lds[0];
        for (int w = 1; w < kWaves; ++w) v = fmax(v, lds[w]);
        red[0] = v;
        red[1] = 0.5 * rho * pv[0];
    }
}

size_t al_extra_bytes(int64_t rows, int64_t n_eq) {
    return align_up((size_t)rows * 8) * 2 + 2 * align_up((size_t)(n_eq > 0 ? n_eq : 1) * 8) + align_up(64);
}

int check_al(int64_t n, const lbfgsb_objective* o, int64_t n_eq) {
    if (!o) return fail(LBFGSB_E_INVALID_ARG, "objective is NULL");
    if (o->kind != LBFGSB_OBJ_LSQ) return fail(LBFGSB_E_INVALID_ARG, "lbfgsb_auglag_create takes the least-squares objective with the constraint rows stacked under A");
    if (n_eq < 0 || n_eq >= o->rows) return fail(LBFGSB_E_INVALID_ARG, "n_eq must be in 0..rows-1 (rows counts the constraint rows)");
    if (o->row_weight) return fail(LBFGSB_E_INVALID_ARG, "row_weight must be NULL: the weights are the algorithm's");
    if (o->n_extra) return fail(LBFGSB_E_INVALID_ARG, "n_extra must be 0");
    (void)n;
    return LBFGSB_OK;
}

int check_al_rows(const lbfgsb_objective* o, int64_t n_eq, const double* C, const double* d) {
    if (!o) return fail(LBFGSB_E_INVALID_ARG, "objective is NULL");
    if (o->kind == LBFGSB_OBJ_LOGISTIC_L2) return fail(LBFGSB_E_INVALID_ARG, "the augmented Lagrangian entry points take the quadratic objective kinds");
    if (n_eq < 0 || n_eq > kMaxExtra) return fail(LBFGSB_E_INVALID_ARG, "n_eq must be in 0..%d for constraint rows passed separately", kMaxExtra);
    if (o->n_extra) return fail(LBFGSB_E_INVALID_ARG, "n_extra must be 0: the extra rows are the algorithm's");
    if (n_eq > 0 && (!C || !d)) return fail(LBFGSB_E_INVALID_ARG, "NULL constraint rows / targets");
    return LBFGSB_OK;
}

size_t al_rows_extra_bytes(int64_t n_eq) {
    return 3 * align_up((size_t)(n_eq > 0 ? n_eq : 1) * 8) + align_up(64);
}

// residual (all rows) and gradient recomputed from x unless they already are
// (called right behind lbfgsb_solve, whose last act was to read the scalar block: the host copy is current)
hipError_t al_fresh_eval(lbfgsb_solver* s) {
    if (s->steps_since_refresh > 0) {
        const int status = s->h_scal->status;
        launch_set_status(s->bf, LBFGSB_RUNNING, s->stream);   // the evaluation's last kernel only runs in this state
        enqueue_eval(s, 0);
        launch_set_status(s->bf, status, s->stream);
        s->steps_since_refresh = 0;
    }
    return hipGetLastError();
}

}  // namespace

extern "C" {

void lbfgsb_auglag_default_options(lbfgsb_auglag_options* o) {
    if (!o) return;
    o->rho0 = 1.0; o->ctol = 1e-8; o->max_outer = 100;
}

size_t lbfgsb_auglag_workspace_bytes(int64_t n, int m, const lbfgsb_objective* obj, int64_t n_eq,
                                     const lbfgsb_options* opt) {
    if (check_al(n, obj, n_eq) != LBFGSB_OK) return 0;
    const size_t inner = lbfgsb_workspace_bytes(n, m, obj, opt);
    return inner ? inner + al_extra_bytes(obj->rows, n_eq) : 0;
}

int lbfgsb_auglag_create(lbfgsb_auglag** out, int64_t n, int m, const double* l, const double* u,
                         const lbfgsb_objective* obj, int64_t n_eq, const lbfgsb_options* opt,
                         const lbfgsb_auglag_options* aopt, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!out) return fail(LBFGSB_E_INVALID_ARG, "out is NULL");
    *out = nullptr;
    int rc = check_al(n, obj, n_eq);
    if (rc) return rc;
    lbfgsb_auglag_options ao;
    if (aopt) ao = *aopt; else lbfgsb_auglag_default_options(&ao);
    if (!(ao.rho0 > 0.0) || !(ao.ctol >= 0.0) || ao.max_outer < 1) return fail(LBFGSB_E_INVALID_ARG, "bad option value");
    if (!workspace || !obj->b) return fail(LBFGSB_E_INVALID_ARG, "NULL device pointer");
    const size_t inner_bytes = lbfgsb_workspace_bytes(n, m, obj, opt);
    if (inner_bytes == 0) return LBFGSB_E_INVALID_ARG;
    const size_t extra = al_extra_bytes(obj->rows, n_eq);
    if (workspace_bytes < inner_bytes + extra)
        return fail(LBFGSB_E_INVALID_ARG, "workspace too small: %zu < %zu bytes", workspace_bytes, inner_bytes + extra);
    if ((uintptr_t)workspace % 256) return fail(LBFGSB_E_INVALID_ARG, "workspace must be 256-byte aligned");

    lbfgsb_auglag* al = new (std::nothrow) lbfgsb_auglag();
    if (!al) return fail(LBFGSB_E_INVALID_ARG, "out of host memory");
    const int64_t rows_data = obj->rows - n_eq;
    al->ao = ao; al->n_eq = n_eq; al->n = n; al->d_c = obj->b + rows_data;
    al->stream = (hipStream_t)hip_stream; al->rho = ao.rho0; al->inner = nullptr; al->h_red = nullptr;
    char* w = (char*)workspace + align_up(inner_bytes);
    double* beta = (double*)w; w += align_up((size_t)obj->rows * 8);
    double* omega = (double*)w; w += align_up((size_t)obj->rows * 8);
    al->beta_c = beta + rows_data; al->omega_c = omega + rows_data;
    al->lambda = (double*)w; w += align_up((size_t)(n_eq > 0 ? n_eq : 1) * 8);
    al->coef = (double*)w; w += align_up((size_t)(n_eq > 0 ? n_eq : 1) * 8);
    al->red = (double*)w;
    al->c_rows = (const char*)obj->A + (size_t)rows_data * (size_t)obj->ld * (obj->dtype == LBFGSB_F64 ? 8 : 4);
    lbfgsb_objective inner_obj = *obj;
    inner_obj.b = beta;
    inner_obj.row_weight = omega;
    rc = lbfgsb_create(&al->inner, n, m, l, u, &inner_obj, opt, workspace, inner_bytes, hip_stream);
    if (rc) { delete al; return rc; }
    al->res_c = al->inner->bf.row + rows_data;
    hipError_t e = hipHostMalloc((void**)&al->h_red, 64, hipHostMallocDefault);
    if (e != hipSuccess) { al->h_red = nullptr; lbfgsb_auglag_destroy(al); return fail(LBFGSB_E_HIP, "hipHostMalloc: %s", hipGetErrorString(e)); }
    int blocks = (int)((obj->rows + 255) / 256);
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(k_al_init, dim3(blocks), dim3(256), 0, al->stream, obj->rows, obj->b, beta, omega);
    launch_fill_zero(al->lambda, align_up((size_t)(n_eq > 0 ? n_eq : 1) * 8), al->stream);
    e = hipStreamSynchronize(al->stream);
    if (e == hipSuccess) e = hipGetLastError();
    if (e != hipSuccess) { lbfgsb_auglag_destroy(al); return fail(LBFGSB_E_HIP, "initialising: %s", hipGetErrorString(e)); }
    *out = al;
    return LBFGSB_OK;
}

size_t lbfgsb_auglag_rows_workspace_bytes(int64_t n, int m, const lbfgsb_objective* obj, int64_t n_eq,
                                          const lbfgsb_options* opt) {
    if (check_al_rows(obj, n_eq, (const double*)8, (const double*)8) != LBFGSB_OK) return 0;
    lbfgsb_objective o = *obj;
    o.n_extra = n_eq;
    const size_t inner = lbfgsb_workspace_bytes(n, m, &o, opt);
    return inner ? align_up(inner) + al_rows_extra_bytes(n_eq) : 0;
}

int lbfgsb_auglag_create_rows(lbfgsb_auglag** out, int64_t n, int m, const double* l, const double* u,
                              const lbfgsb_objective* obj, int64_t n_eq, const double* C, const double* d,
                              const lbfgsb_options* opt, const lbfgsb_auglag_options* aopt, void* workspace,
                              size_t workspace_bytes, void* hip_stream) {
    if (!out) return fail(LBFGSB_E_INVALID_ARG, "out is NULL");
    *out = nullptr;
    int rc = check_al_rows(obj, n_eq, C, d);
    if (rc) return rc;
    lbfgsb_auglag_options ao;
    if (aopt) ao = *aopt; else lbfgsb_auglag_default_options(&ao);
    if (!(ao.rho0 > 0.0) || !(ao.ctol >= 0.0) || ao.max_outer < 1) return fail(LBFGSB_E_INVALID_ARG, "bad option value");
    if (!workspace) return fail(LBFGSB_E_INVALID_ARG, "NULL device pointer");
    lbfgsb_objective inner_obj = *obj;
    inner_obj.n_extra = n_eq;
    inner_obj.extra_rows = C;
    inner_obj.extra_target = (const double*)8;   // placeholders for the size computation; set below
    const size_t inner_bytes = lbfgsb_workspace_bytes(n, m, &inner_obj, opt);
    if (inner_bytes == 0) return LBFGSB_E_INVALID_ARG;
    const size_t extra = al_rows_extra_bytes(n_eq);
    if (workspace_bytes < align_up(inner_bytes) + extra)
        return fail(LBFGSB_E_INVALID_ARG, "workspace too small: %zu < %zu bytes", workspace_bytes, align_up(inner_bytes) + extra);
    if ((uintptr_t)workspace % 256) return fail(LBFGSB_E_INVALID_ARG, "workspace must be 256-byte aligned");

    lbfgsb_auglag* al = new (std::nothrow) lbfgsb_auglag();
    if (!al) return fail(LBFGSB_E_INVALID_ARG, "out of host memory");
    const size_t slot = align_up((size_t)(n_eq > 0 ? n_eq : 1) * 8);
    al->ao = ao; al->n_eq = n_eq; al->n = n; al->d_c = d;
    al->stream = (hipStream_t)hip_stream; al->rho = ao.rho0; al->inner = nullptr; al->h_red = nullptr;
    char* w = (char*)workspace + align_up(inner_bytes);
    al->beta_c = (double*)w; w += slot;
    al->omega_c = (double*)w; w += slot;
    al->lambda = (double*)w; w += slot;
    al->red = (double*)w;
    inner_obj.extra_target = al->beta_c;
    inner_obj.extra_weight = al->omega_c;
    rc = lbfgsb_create(&al->inner, n, m, l, u, &inner_obj, opt, workspace, inner_bytes, hip_stream);
    if (rc) { delete al; return rc; }
    al->res_c = al->inner->bf.xres;
    hipError_t e = hipHostMalloc((void**)&al->h_red, 64, hipHostMallocDefault);
    if (e != hipSuccess) { al->h_red = nullptr; lbfgsb_auglag_destroy(al); return fail(LBFGSB_E_HIP, "hipHostMalloc: %s", hipGetErrorString(e)); }
    launch_fill_zero(al->beta_c, 3 * slot, al->stream);
    e = hipStreamSynchronize(al->stream);
    if (e == hipSuccess) e = hipGetLastError();
    if (e != hipSuccess) { lbfgsb_auglag_destroy(al); return fail(LBFGSB_E_HIP, "initialising: %s", hipGetErrorString(e)); }
    *out = al;
    return LBFGSB_OK;
}

size_t lbfgsb_auglag_marginals_workspace_bytes(int m, const lbfgsb_objective* obj, const lbfgsb_options* opt) {
    if (!obj || !is_transport(obj->kind)) { fail(LBFGSB_E_INVALID_ARG, "the marginal constraints go with the transport kinds"); return 0; }
    lbfgsb_objective o = *obj;
    o.n_extra = 0;
    const size_t inner = lbfgsb_workspace_bytes(o.rows * o.cols, m, &o, opt);
    return inner ? align_up(inner) + al_rows_extra_bytes(o.rows + o.cols) : 0;
}

int lbfgsb_auglag_create_marginals(lbfgsb_auglag** out, int m, const double* l, const double* u,
                                   const lbfgsb_objective* obj, const double* marginals, const lbfgsb_options* opt,
                                   const lbfgsb_auglag_options* aopt, void* workspace, size_t workspace_bytes,
                                   void* hip_stream) {
    if (!out) return fail(LBFGSB_E_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (!obj || !is_transport(obj->kind)) return fail(LBFGSB_E_INVALID_ARG, "the marginal constraints go with the transport kinds");
    if (!marginals || !workspace) return fail(LBFGSB_E_INVALID_ARG, "NULL device pointer");
    lbfgsb_auglag_options ao;
    if (aopt) ao = *aopt; else lbfgsb_auglag_default_options(&ao);
    if (!(ao.rho0 > 0.0) || !(ao.ctol >= 0.0) || ao.max_outer < 1) return fail(LBFGSB_E_INVALID_ARG, "bad option value");
    lbfgsb_objective inner_obj = *obj;
    inner_obj.n_extra = 0;
    inner_obj.b = nullptr;
    inner_obj.row_weight = nullptr;
    const int64_t n = obj->rows * obj->cols, n_eq = obj->rows + obj->cols;
    const size_t inner_bytes = lbfgsb_workspace_bytes(n, m, &inner_obj, opt);
    if (inner_bytes == 0) return LBFGSB_E_INVALID_ARG;
    const size_t extra = al_rows_extra_bytes(n_eq);
    if (workspace_bytes < align_up(inner_bytes) + extra)
        return fail(LBFGSB_E_INVALID_ARG, "workspace too small: %zu < %zu bytes", workspace_bytes, align_up(inner_bytes) + extra);
    if ((uintptr_t)workspace % 256) return fail(LBFGSB_E_INVALID_ARG, "workspace must be 256-byte aligned");

    lbfgsb_auglag* al = new (std::nothrow) lbfgsb_auglag();
    if (!al) return fail(LBFGSB_E_INVALID_ARG, "out of host memory");
    const size_t slot = align_up((size_t)n_eq * 8);
    al->ao = ao; al->n_eq = n_eq; al->n = n; al->d_c = marginals;
    al->stream = (hipStream_t)hip_stream; al->rho = ao.rho0; al->inner = nullptr; al->h_red = nullptr;
    char* w = (char*)workspace + align_up(inner_bytes);
    al->beta_c = (double*)w; w += slot;
    al->omega_c = (double*)w; w += slot;
    al->lambda = (double*)w; w += slot;
    al->red = (double*)w;
    inner_obj.b = al->beta_c;
    inner_obj.row_weight = al->omega_c;
    int rc = lbfgsb_create(&al->inner, n, m, l, u, &inner_obj, opt, workspace, inner_bytes, hip_stream);
    if (rc) { delete al; return rc; }
    al->res_c = al->inner->bf.row;
    hipError_t e = hipHostMalloc((void**)&al->h_red, 64, hipHostMallocDefault);
    if (e != hipSuccess) { al->h_red = nullptr; lbfgsb_auglag_destroy(al); return fail(LBFGSB_E_HIP, "hipHostMalloc: %s", hipGetErrorString(e)); }
    launch_fill_zero(al->beta_c, 3 * slot, al->stream);
    e = hipStreamSynchronize(al->stream);
    if (e == hipSuccess) e = hipGetLastError();
    if (e != hipSuccess) { lbfgsb_auglag_destroy(al); return fail(LBFGSB_E_HIP, "initialising: %s", hipGetErrorString(e)); }
    *out = al;
    return LBFGSB_OK;
}

void lbfgsb_auglag_destroy(lbfgsb_auglag* al) {
    if (!al) return;
    lbfgsb_destroy(al->inner);
    if (al->h_red) (void)hipHostFree(al->h_red);
    delete al;
}

int lbfgsb_auglag_solve(lbfgsb_auglag* al, const double* x0, lbfgsb_auglag_info* info) {
    if (!al || !x0) return fail(LBFGSB_E_INVALID_ARG, "NULL argument");
    lbfgsb_solver* s = al->inner;
    lbfgsb_auglag_info out{};
    out.status = LBFGSB_MAX_ITER;
    const int pb = (int)((al->n_eq + 255) / 256) > 0 ? (int)((al->n_eq + 255) / 256) : 1;
    // lambda^0 = 0, rho = rho0; the violation at x^0 is what the first iteration is compared with
    launch_fill_zero(al->lambda, align_up((size_t)(al->n_eq > 0 ? al->n_eq : 1) * 8), al->stream);
    al->rho = al->ao.rho0;
    hipLaunchKernelGGL(k_al_prepare, dim3(pb), dim3(256), 0, al->stream, al->n_eq, al->rho, al->d_c, al->lambda,
                       al->beta_c, al->omega_c);
    int rc = lbfgsb_set_x(s, x0);
    if (rc) return rc;
    // constraint violation and penalty term at the current x (and the multiplier update); wait: whether to wait
    // here or let a following read of the scalar block do it
    auto measure = [&](int update, bool wait) -> hipError_t {
        hipLaunchKernelGGL(k_al_update, dim3(1), dim3(kBlock), 0, al->stream, al->n_eq, al->rho, update, al->res_c,
                           al->lambda, al->red, (const Scal*)nullptr);
        hipError_t e = hipMemcpyAsync(al->h_red, al->red, 16, hipMemcpyDeviceToHost, al->stream);
        if (e != hipSuccess || !wait) return e;
        return hipStreamSynchronize(al->stream);
    };
    // The multiplier update of an inner solve whose convergence is being confirmed rides on that confirmation's wait:
    // residuals are fresh behind the re-evaluation, and the kernel does nothing unless the status says CONVERGED.
    s->after_retest = [](void* ctx) {
        lbfgsb_auglag* a = (lbfgsb_auglag*)ctx;
        hipLaunchKernelGGL(k_al_update, dim3(1), dim3(kBlock), 0, a->stream, a->n_eq, a->rho, 1, a->res_c, a->lambda,
                           a->red, (const Scal*)a->inner->bf.scal);
        (void)hipMemcpyAsync(a->h_red, a->red, 16, hipMemcpyDeviceToHost, a->stream);
    };
    s->after_retest_ctx = al;
    struct HookReset { lbfgsb_solver* s; ~HookReset() { s->after_retest = nullptr; s->after_retest_ctx = nullptr; } } hook_reset{s};
    HIP_TRY(measure(0, true));
    double viol_prev = al->h_red[0];
    out.violation = viol_prev;
    long long prev_inner = 0;
    for (int it = 0; it < al->ao.max_outer; ++it) {
        if (it > 0 && al->c_rows) {
            // new targets/weights of the stacked constraint rows: the pair memory is cleared, and f and g at the
            // unchanged x are shifted by the constraint rows' share (residuals and gradient are fresh at this point)
            const double f_old = s->h_scal->f;
            fresh_scal(s);
            s->h_scal->f = f_old;
            HIP_TRY(hipMemcpyAsync(s->bf.scal, s->h_scal, sizeof(Scal), hipMemcpyHostToDevice, s->stream));
            hipLaunchKernelGGL(k_al_shift_rows, dim3(1), dim3(kBlock), 0, al->stream, al->n_eq, al->rho, al->d_c,
                               (const double*)al->lambda, al->beta_c, al->omega_c, (double*)al->res_c, al->coef, s->bf.scal);
            int gb = (int)((s->dm.cols + 255) / 256);
            if (gb > 1024) gb = 1024;
            if (s->dm.dtype == LBFGSB_F64)
                hipLaunchKernelGGL(k_al_shift_g<double>, dim3(gb), dim3(256), 0, al->stream, al->n_eq, s->dm.cols, s->dm.ld,
                                   (const double*)al->c_rows, (const double*)al->coef, s->bf.g);
            else
                hipLaunchKernelGGL(k_al_shift_g<float>, dim3(gb), dim3(256), 0, al->stream, al->n_eq, s->dm.cols, s->dm.ld,
                                   (const float*)al->c_rows, (const double*)al->coef, s->bf.g);
            s->steps_since_refresh = 0;
            s->steps_since_set_x = 0;
        } else if (it > 0) {
            // new targets/weights: the objective changed, so f and g are re-evaluated at x and the pair memory is cleared
            hipLaunchKernelGGL(k_al_prepare, dim3(pb), dim3(256), 0, al->stream, al->n_eq, al->rho, al->d_c, al->lambda,
                               al->beta_c, al->omega_c);
            rc = set_x_impl(s, s->bf.x, true);
            if (rc) return rc;
        }
        lbfgsb_info ii;
        // (an inner solve that follows one which needed at most two iterations is likely to be over at once)
        s->first_batch = (it > 0 && prev_inner <= 2) ? 1 : 0;
        rc = lbfgsb_solve(s, &ii);
        s->first_batch = 0;
        if (rc) return rc;
        prev_inner = ii.iters;
        out.outer = it + 1;
        out.inner_iters += ii.iters;
        out.pg2 = ii.pg2;
        if (ii.status == LBFGSB_LINESEARCH_FAILED) { out.status = ii.status; break; }
        if (!(ii.status == LBFGSB_CONVERGED && s->last_read_was_retest)) {
            HIP_TRY(al_fresh_eval(s));
            HIP_TRY(measure(1, false));           // lambda += rho h(x); violation; penalty term
            HIP_TRY(read_scal(s));                // (one wait for both)
        }                                         // (else: done behind the solve's last wait)
        out.L = s->h_scal->f;
        out.violation = al->h_red[0];
        out.f = out.L - al->h_red[1];
        if (out.violation <= al->ao.ctol && ii.status == LBFGSB_CONVERGED) { out.status = LBFGSB_CONVERGED; break; }
        if (out.violation > 0.5 * viol_prev) al->rho *= 2.0;
        viol_prev = out.violation;
    }
    out.rho = al->rho;
    if (info) *info = out;
    return LBFGSB_OK;
}

int lbfgsb_auglag_get_x(lbfgsb_auglag* al, double* x_out) {
    if (!al) return fail(LBFGSB_E_INVALID_ARG, "NULL argument");
    return lbfgsb_get_x(al->inner, x_out);
}

int lbfgsb_auglag_get_lambda(lbfgsb_auglag* al, double* lambda_out) {
    if (!al || !lambda_out) return fail(LBFGSB_E_INVALID_ARG, "NULL argument");
    if (al->n_eq > 0)
        HIP_TRY(hipMemcpyAsync(lambda_out, al->lambda, (size_t)al->n_eq * 8, hipMemcpyDeviceToDevice, al->stream));
    return LBFGSB_OK;
}

lbfgsb_solver* lbfgsb_auglag_inner(lbfgsb_auglag* al) { return al ? al->inner : nullptr; }

}  // extern "C"
