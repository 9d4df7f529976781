// Shared declarations of the HIP implementation: device-resident solver state, reduction
// helpers, and the launchers each translation unit exports to the C-ABI layer.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "../../include/lbfgsb.h"

namespace lb {

constexpr int kMaxM = LBFGSB_MAX_M;
constexpr int kMaxV = 64;          // 2*m + 1 <= 64 vectors enter the batched two-loop
constexpr int kBlock = 256;        // threads per workgroup of every vector kernel (4 waves of 64)
constexpr int kWaves = kBlock / 64;
constexpr int kFoldMax = 2;       // extra dense rows the direction kernel handles itself (more: a kernel of their own)
constexpr int kLsBatch = 8;        // step lengths the logistic line search evaluates per sweep over the rows

// Which per-kernel arrival counter (Scal::counters) a kernel uses to find its last workgroup.
enum { kCntGram = 0, kCntDir, kCntUpdate, kCntEvalFinish, kCntLs, kCntCount };
// Grids of the kernels whose last workgroup finishes the job (arrive_is_last) stay at two workgroups per compute
// unit: every workgroup ends with an atomic on one address, and those serialise (4096 workgroups measured 90 us
// slower per launch than 512 on the same data).
constexpr int kDirBlocksMax = 512;    // workgroups of the direction kernel, at most
constexpr int kGramGroups = 16;    // large-n Gram kernel: groups of workgroups whose partials are summed first
constexpr int kOtRpwMax = 16;      // rows of P one workgroup of the marginal-sum kernel owns, at most

// All scalars of the iteration live here, in device memory, so that no data-dependent decision
// needs the host.  Only the last workgroup of a kernel to finish ever writes it; every other
// workgroup has read what it needs before it signals arrival.
struct Scal {
    int status;             // LBFGSB_RUNNING ...
    int head;               // ring slot the next pair is written to
    int count;              // stored pairs (<= m)
    int branch;             // Algorithm 2 branch of the current direction (1 or 2)
    int tol_resolved;       // tol_abs has been fixed (first free-set evaluation after set_x)
    int backtracks;
    int pairs_used;
    int memory_resets;
    int ls_ok;              // the last line search found an acceptable step
    // update left pending by the quadratic update kernel (no workgroup of that kernel reads these);
    // applied by the last workgroup of the next Gram kernel, or by k_commit
    int pend_valid, pend_ok, pend_bt;
    int spec_ok;            // logistic: the accepted step is the first trial step, whose X^T psi the single-read pass already holds
    double pend_alpha, pend_f;
    long long iters;
    long long fevals;
    long long n_fixed;
    double f;
    double gp;              // <g, p> for the selected p
    double alpha_ub;        // step bound for the selected p
    double alpha;           // accepted step
    double pg2, pginf, tol_abs;
    double xp, pp;          // <x, p>, <p, p> for the selected p (separable terms of the line search)
    double ynorm2[kMaxM + 1];   // ||y||^2 over the full vector, per ring slot
    double delta[kMaxV];        // coefficients of q = sum_j delta_j b_j in the batched two-loop
    unsigned counters[kCntCount];
    unsigned gram_cnt[kGramGroups + 1];   // two-level arrival of the large-n Gram kernel: one per group, then the top
    // Only in the copy the direction kernel hands to the pass (Buffers::scal_next): this copy holds a state the scalar
    // block itself does not have yet
    int fresh;
    int since_refresh;      // resident solver: iterations since residual and gradient were last computed from x
    // logistic objective, short launch sequence (see kStatusBail)
    int bail_skipped;       // whole steps that found the status kStatusBail and did nothing
    // per-iteration records (ring in the workspace; null: none kept)
    lbfgsb_iter_record* hist;
    long long hist_count;   // records written since lbfgsb_set_x
};

// Internal status of the short logistic launch sequence.  That sequence has no launches for the rare continuation of
// the line search (more step lengths, a second transposed pass): when the first trial step is rejected, the search
// kernel parks the solver in this state, every later kernel returns at once (as for any status other than RUNNING),
// and the host finishes the iteration with the missing launches when it next looks at the scalar block.  Never
// reported to the caller.
constexpr int kStatusBail = 64;

struct Dims {
    int64_t n, rows, cols, ld;
    int m, kind, dtype;
    double lambda, mu;
    int n_extra;            // extra dense rows on top of a quadratic kind (0 = none)
};

constexpr int kMaxExtra = 64;

__host__ __device__ inline bool is_transport(int kind) {
    return kind == LBFGSB_OBJ_OT_GAUSS || kind == LBFGSB_OBJ_OT_ENTROPY;
}
// entries of the row vectors (Buffers::row, t, psi): rows of A, or the rows + cols marginals of the transport kinds
__host__ __device__ inline int64_t row_entries(int kind, int64_t rows, int64_t cols) {
    return is_transport(kind) ? rows + cols : rows;
}

struct Opts {
    double eps, c1, backtrack, tol;
    int max_backtracks, tol_relative, max_iter;
    // every variable has the same bounds (found when the bounds are validated): the long-vector kernels then take
    // them from here instead of streaming l and u
    int uniform_bounds;
    double lo, hi;
};

// ---- reductions ---------------------------------------------------------------------------------

// Reductions over the 64 lanes of a wave: lane permutations of the data-parallel-primitive unit inside a row of 16
// lanes (an operand modifier of a move: a few cycles, where a shuffle goes through the LDS crossbar and costs ~130
// cycles per dependent step), then the four row totals through scalar registers.  Every lane gets the result; the
// order of the operations is fixed: lane pairs, quads, halves of a row, rows 0..3.  ALL 64 lanes must be active
// where these are called (a permutation reads zero from an inactive lane).
template <int CTRL>
__device__ __forceinline__ double dpp_move(double v) {
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, 0xf, 0xf, true);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, 0xf, 0xf, true);
    return __hiloint2double(hi, lo);
}
constexpr int kDppXor1 = 0xB1;          // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;          // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;   // lane i <-> 7 - i within each half row
constexpr int kDppMirror = 0x140;       // lane i <-> 15 - i within each row
__device__ __forceinline__ double lane_bcast(double v, int l) {   // l: compile-time lane index
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), l);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), l);
    return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double wave_sum(double v) {
    v += dpp_move<kDppXor1>(v);
    v += dpp_move<kDppXor2>(v);
    v += dpp_move<kDppHalfMirror>(v);
    v += dpp_move<kDppMirror>(v);
    return ((lane_bcast(v, 0) + lane_bcast(v, 16)) + lane_bcast(v, 32)) + lane_bcast(v, 48);
}
__device__ __forceinline__ double wave_min(double v) {
    v = fmin(v, dpp_move<kDppXor1>(v));
    v = fmin(v, dpp_move<kDppXor2>(v));
    v = fmin(v, dpp_move<kDppHalfMirror>(v));
    v = fmin(v, dpp_move<kDppMirror>(v));
    return fmin(fmin(lane_bcast(v, 0), lane_bcast(v, 16)), fmin(lane_bcast(v, 32), lane_bcast(v, 48)));
}
__device__ __forceinline__ double wave_max(double v) { return -wave_min(-v); }

// Sum of K values over a workgroup of NW waves; every thread gets the totals.  The order of the
// additions is fixed (butterfly inside a wave, waves in index order), so results are bit-reproducible.
template <int K, int NW>
__device__ __forceinline__ void block_sum(double (&v)[K], double* lds /* NW*K doubles */) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int k = 0; k < K; ++k) v[k] = wave_sum(v[k]);
    __syncthreads();   // protect lds against readers of a previous use
    if (lane == 0) {
#pragma unroll
        for (int k = 0; k < K; ++k) lds[wave * K + k] = v[k];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < K; ++k) {
        double t = 0.0;
#pragma unroll
        for (int w = 0; w < NW; ++w) t += lds[w * K + k];
        v[k] = t;
    }
}

// Signals that this workgroup's partial results are in memory and tells whether it is the last
// one of the grid to do so.  Every wave first waits for its own stores to be acknowledged; after the
// barrier thread 0 alone issues the device-scope release fence (which writes the L2 back) and the
// relaxed device-scope atomic, and in the last workgroup the acquire fence; the barrier that follows
// extends that to the other waves.  Fencing in every wave instead costs ~60 ns per workgroup of
// serialised time on MI355X.  The last workgroup resets the counter for the next launch.  Must be
// called by all threads of the workgroup.
__device__ __forceinline__ bool arrive_is_last(unsigned* counter, int* lds_flag, unsigned expected = 0u) {
    __builtin_amdgcn_s_waitcnt(0);   // vmcnt(0) expcnt(0) lgkmcnt(0): this wave's stores have reached L2
    __syncthreads();
    if (threadIdx.x == 0) {
        __threadfence();
        const unsigned total = expected ? expected : gridDim.x * gridDim.y;   // expected: arrivals at this counter
        const unsigned old = atomicAdd(counter, 1u);
        const int last = old == total - 1u;
        if (last) {
            __threadfence();
            *counter = 0u;
        }
        *lds_flag = last;
    }
    __syncthreads();
    return *lds_flag != 0;
}

// Ring bookkeeping.  Logical vector j of [s^0..s^{c-1}, y^0..y^{c-1}, g], pair 0 being the oldest;
// `head` is the slot the next pair goes to.
__device__ __forceinline__ const double* ring_vec(int j, int c, int head, int m, int64_t n, const double* S,
                                                  const double* Y, const double* g) {
    if (j < c) return S + (int64_t)((head - c + j + 2 * m) % m) * n;
    if (j < 2 * c) return Y + (int64_t)((head - c + (j - c) + 2 * m) % m) * n;
    return g;
}

// head/count as they will be once a pending update has been applied.  ls_dead: the pending update is
// a failed line search with no pair left to drop (the solver is about to stop).
__device__ __forceinline__ void effective_ring(const Scal* s, int m, int& head, int& count, bool& ls_dead) {
    head = s->head;
    count = s->count;
    ls_dead = false;
    if (s->pend_valid) {
        if (s->pend_ok) {
            head = (head + 1) % m;
            count = count < m ? count + 1 : m;
        } else if (count > 0) {
            count = 0;
        } else {
            ls_dead = true;
        }
    }
}

// One record per accepted iteration, written by the thread that has just completed the iteration's bookkeeping:
// the scalar block then holds the stopping quantities of the iterate the iteration started from (the next free-set
// pass has not run yet), the direction's branch and bound, and the accepted step.
__device__ __forceinline__ void fill_record(const Scal* s, lbfgsb_iter_record* r) {
    r->iter = s->iters; r->f = s->f; r->pg2 = s->pg2; r->pginf = s->pginf; r->n_fixed = s->n_fixed;
    r->alpha = s->alpha; r->alpha_ub = s->alpha_ub; r->gp = s->gp;
    r->branch = s->branch; r->backtracks = s->backtracks; r->pairs_used = s->pairs_used; r->memory_resets = s->memory_resets;
}
__device__ __forceinline__ void record_iteration(Scal* s) {
    if (!s->hist) return;
    fill_record(s, s->hist + (s->hist_count % LBFGSB_HISTORY_CAPACITY));
    s->hist_count += 1;
}

// Applies the pending update: accepted step (pair stored at slot `head`), or an exhausted line search
// (clear the pair memory and retry once from the steepest-descent direction, else stop).
// record: also write the per-iteration record (false where several workgroups apply the same update to private copies)
__device__ __forceinline__ void apply_pending(Scal* s, int m, bool record = true) {
    if (!s->pend_valid) return;
    s->pend_valid = 0;
    s->ls_ok = s->pend_ok;
    s->backtracks = s->pend_bt;
    s->fevals += s->pend_bt + (s->pend_ok ? 1 : 0);
    if (s->pend_ok) {
        s->alpha = s->pend_alpha;
        s->f = s->pend_f;
        s->head = (s->head + 1) % m;
        s->count = s->count < m ? s->count + 1 : m;
        s->iters += 1;
        if (record) record_iteration(s);
        else if (s->hist) s->hist_count += 1;
    } else if (s->count > 0) {
        s->count = 0;
        s->memory_resets += 1;
    } else {
        s->status = LBFGSB_LINESEARCH_FAILED;
    }
}

__device__ __forceinline__ double clampd(double v, double lo, double hi) {
    return v < lo ? lo : (v > hi ? hi : v);
}

__device__ __forceinline__ double softplus_d(double t) { return fmax(t, 0.0) + log1p(exp(-fabs(t))); }
__device__ __forceinline__ double sigmoid_d(double t) {
    if (t >= 0.0) return 1.0 / (1.0 + exp(-t));
    const double e = exp(t);
    return e / (1.0 + e);
}

// softplus(q + dq) - softplus(q) without differencing two rounded values; sq = sigmoid(q).
__device__ __forceinline__ double softplus_diff(double q, double sq, double dq) {
    if (fabs(dq) >= 30.0) return softplus_d(q + dq) - softplus_d(q);
    // log(1 + sigmoid(q) (e^dq - 1)).  Where the product comes close to -1 (a saturated margin that the step undoes)
    // log1p of it would itself take the logarithm of a difference of nearly equal numbers; there the same number is
    // log(sigmoid(-q) + sigmoid(q) e^dq), a sum of two positive terms.
    const double u = sq * expm1(dq);
    if (u > -0.5) return log1p(u);
    return log(sigmoid_d(-q) + sq * exp(dq));
}

// ---- Algorithm 2's choice between the two candidate directions, from the direction kernel's partial sums ----------
//
// Per workgroup of the direction kernel one record of kDirRed doubles: p1.g, p1.p1, x.p1, p2.g, p2.p2, x.p2, the
// smallest step bound of p2, one unused; then e_r.p1, e_r.p2 per folded extra row.
constexpr int kDirRed = 8 + 2 * kFoldMax;

struct DirChoice {
    int branch;              // 1: p = P(x + d) - x, step bound 1;  2: p = d with outward components zeroed
    double gp, alpha_ub, pp, xp;
};

// The choice, computed by ONE FULL WAVE from the records of `nblocks` workgroups: lane l adds records l, l + 64, ...
// in that order, then the fixed-order wave reductions.  Every wave that calls this on the same records gets the same
// bits, whatever its workgroup's size, so a kernel that needs the choice can make it itself instead of waiting for a
// last workgroup of the direction kernel to publish it (that closing step -- fences, an atomic on one address, a
// dependent round of loads -- is about half of that kernel's duration).
__device__ __forceinline__ DirChoice dir_choice_from_partials(const double* __restrict__ redpart, int nblocks, double eps) {
    const int lane = threadIdx.x & 63;
    double t6[6] = {0, 0, 0, 0, 0, 0};
    double tmin = INFINITY;
    for (int b0 = 0; b0 < nblocks; b0 += 2 * 64) {          // two records per lane and trip, their loads issued together
        double v[2][7];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int b = b0 + 64 * j + lane;
            const bool in = b < nblocks;
            const double* r = redpart + (int64_t)(in ? b : 0) * kDirRed;
#pragma unroll
            for (int k = 0; k < 7; ++k) v[j][k] = r[k];
            if (!in) {
#pragma unroll
                for (int k = 0; k < 6; ++k) v[j][k] = 0.0;
                v[j][6] = INFINITY;
            }
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
#pragma unroll
            for (int k = 0; k < 6; ++k) t6[k] += v[j][k];
            tmin = fmin(tmin, v[j][6]);
        }
    }
#pragma unroll
    for (int k = 0; k < 6; ++k) t6[k] = wave_sum(t6[k]);
    tmin = wave_min(tmin);
    DirChoice c;
    c.branch = (t6[0] <= -eps * t6[1] && t6[1] >= eps) ? 1 : 2;
    if (c.branch == 1) { c.gp = t6[0]; c.alpha_ub = 1.0; c.pp = t6[1]; c.xp = t6[2]; }
    else { c.gp = t6[3]; c.alpha_ub = tmin; c.pp = t6[4]; c.xp = t6[5]; }
    return c;
}

// Sums, over the same records, of the folded extra rows' products with both candidates (one full wave; lane l adds
// records l, l + 64, ...): tx[2r] with the first candidate, tx[2r+1] with the second.
__device__ __forceinline__ void dir_fold_from_partials(const double* __restrict__ redpart, int nblocks,
                                                       double (&tx)[2 * kFoldMax]) {
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int k = 0; k < 2 * kFoldMax; ++k) tx[k] = 0.0;
    for (int b0 = 0; b0 < nblocks; b0 += 2 * 64) {
        double v[2][2 * kFoldMax];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int b = b0 + 64 * j + lane;
            const bool in = b < nblocks;
            const double* r = redpart + (int64_t)(in ? b : 0) * kDirRed + 8;
#pragma unroll
            for (int k = 0; k < 2 * kFoldMax; ++k) v[j][k] = r[k];
            if (!in) {
#pragma unroll
                for (int k = 0; k < 2 * kFoldMax; ++k) v[j][k] = 0.0;
            }
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
#pragma unroll
            for (int k = 0; k < 2 * kFoldMax; ++k) tx[k] += v[j][k];
        }
    }
#pragma unroll
    for (int k = 0; k < 2 * kFoldMax; ++k) tx[k] = wave_sum(tx[k]);
}

// The same choice made by a whole workgroup of kBlock threads: thread t adds records t, t + kBlock, ... (their loads
// issued together), then the fixed-order sums over the workgroup; every thread gets the result.  lds: kWaves * 7 doubles.
__device__ __forceinline__ DirChoice dir_choice_block(const double* __restrict__ redpart, int nblocks, double eps,
                                                      double* lds) {
    const int tid = threadIdx.x;
    double t6[6] = {0, 0, 0, 0, 0, 0};
    double tmin = INFINITY;
    for (int b0 = 0; b0 < nblocks; b0 += 2 * kBlock) {
        double v[2][7];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int b = b0 + kBlock * j + tid;
            const bool in = b < nblocks;
            const double* r = redpart + (int64_t)(in ? b : 0) * kDirRed;
#pragma unroll
            for (int k = 0; k < 7; ++k) v[j][k] = r[k];
            if (!in) {
#pragma unroll
                for (int k = 0; k < 6; ++k) v[j][k] = 0.0;
                v[j][6] = INFINITY;
            }
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
#pragma unroll
            for (int k = 0; k < 6; ++k) t6[k] += v[j][k];
            tmin = fmin(tmin, v[j][6]);
        }
    }
    block_sum<6, kWaves>(t6, lds);
    tmin = wave_min(tmin);
    __syncthreads();
    if ((tid & 63) == 0) lds[tid >> 6] = tmin;
    __syncthreads();
    tmin = lds[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) tmin = fmin(tmin, lds[w]);
    DirChoice c;
    c.branch = (t6[0] <= -eps * t6[1] && t6[1] >= eps) ? 1 : 2;
    if (c.branch == 1) { c.gp = t6[0]; c.alpha_ub = 1.0; c.pp = t6[1]; c.xp = t6[2]; }
    else { c.gp = t6[3]; c.alpha_ub = tmin; c.pp = t6[4]; c.xp = t6[5]; }
    return c;
}

// ---- helpers shared by the column-wise consumers of the A pass ---------------------------------------------

constexpr int kCX = 16;             // columns per workgroup
constexpr int kGY = kBlock / kCX;   // partial-row groups per workgroup

// Sum over the A pass's partial columns for column c0 + (tid % kCX); valid in threads with tid < kCX.
__device__ __forceinline__ double column_sum(const double* __restrict__ wpart, int parts, int64_t cols, int64_t c,
                                             double* lds /* kBlock doubles */) {
    const int cx = threadIdx.x % kCX, gy = threadIdx.x / kCX;
    double s = 0.0;
    if (c < cols) {
        for (int k0 = gy; k0 < parts; k0 += kGY * 8) {
            double v[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int kk = k0 + kGY * k;
                v[k] = kk < parts ? wpart[(int64_t)kk * cols + c] : 0.0;
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) s += v[k];
        }
    }
    __syncthreads();
    lds[gy * kCX + cx] = s;
    __syncthreads();
    double tot = 0.0;
    if (gy == 0) {
#pragma unroll
        for (int k = 0; k < kGY; ++k) tot += lds[k * kCX + cx];
    }
    return tot;
}

// Sum of `count` doubles, identical in every workgroup that calls it (same order everywhere).
__device__ __forceinline__ double sum_all(const double* __restrict__ v, int count, double* lds) {
    double s[1] = {0.0};
    for (int k0 = threadIdx.x; k0 < count; k0 += kBlock * 8) {
        double t[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) t[k] = k0 + kBlock * k < count ? v[k0 + kBlock * k] : 0.0;
#pragma unroll
        for (int k = 0; k < 8; ++k) s[0] += t[k];
    }
    block_sum<1, kWaves>(s, lds);
    return s[0];
}

// ---- launch geometry decided once at creation -------------------------------------------------------

struct Geometry {
    // two-pass A kernels
    int gemv_blocks;        // workgroups of the row-dot kernel (each writes one loss partial)
    int gemvt_col_tiles;    // column tiles of the transposed kernel
    int gemvt_row_blocks;   // row blocks of the transposed kernel = partial vectors per column
    int64_t gemvt_rows_per_block;
    int vec;                // elements per 16-byte load (1 if alignment forbids vector loads)
    // fused A kernel
    int fused_ok;           // shape fits the fused kernel
    int fused_variant;      // index into the instantiation table
    int fused_blocks;       // workgroups = partial vectors per column and loss partials
    // vector kernels
    int gram_blocks, dir_blocks, upd_blocks, fin_blocks, ls_blocks, lrows_blocks;
    int updl_blocks;        // logistic update of the short sequence (it also moves the margins: rows / 1024 workgroups, at most 512)
    // transport kinds: workgroups of the marginal-sum kernel (each owns ot_rpw consecutive rows of P), of the
    // column-sum kernel, and of the entrywise kernels
    int ot_row_blocks, ot_rpw, ot_col_blocks, ot_el_blocks;
    // partial counts consumers have to sum
    int w_parts;            // partial vectors per column written by the A pass in use
    int loss_parts;         // loss partials written by the A pass in use
};

// Device arrays carved out of the caller's workspace.
struct Buffers {
    Scal* scal;
    // Second scalar block for the sequence in which the Gram kernel has no closing step: every workgroup of the
    // direction kernel works the closing step out on a private copy, workgroup 0 leaves its copy here (nothing in that
    // kernel reads it), and workgroup 0 of the pass, whose other workgroups read only the status word of this copy,
    // moves it into `scal`.
    Scal* scal_next;
    double *x, *g, *l, *u, *d, *p1, *p2;
    uint8_t* mask;
    double *S, *Y;          // m x n rings
    double *row;            // residual A v - b (least squares) or margins (logistic), rows entries
    double *t;              // A p, rows entries
    double *psi;            // per-row weights of the transposed product, rows entries
    double *wpart;          // w_parts x cols partial columns of A^T psi
    double *losspart;       // loss partials of the A pass
    double *grampart;       // gram_blocks x gram_entries
    double *redpart;        // partials of the direction / update / finish kernels
    double *lspart;         // ls_blocks x (step lengths per sweep, at most 64)
    double *wextra;         // n: contribution of the extra rows to the columns of the gradient (or of its change)
    double *xres;           // n_extra residuals e_r.x - target_r of the last evaluation, then [n_extra] the loss term
    lbfgsb_iter_record* hist;   // LBFGSB_HISTORY_CAPACITY per-iteration records
};

// ---- launchers (defined in apass.hip / vec.hip) -------------------------------------------------------

enum RowMode {
    kRowLsqEval = 0,   // u = a_r.v; res = u - b_r -> row; psi = w_r res; loss += 0.5 w_r res^2
    kRowDir = 1,       // u = a_r.v -> t; psi = w_r u;              loss += w_r u^2
    kRowLogiEval = 2,  // u = a_r.v -> row (margin); psi = -y sigma(-y u)/rows; loss += softplus(-y u)/rows
    kRowLogiDir = 3,   // u = a_r.v -> t only (no transposed product follows)
    kRowLogiSpec = 4,  // fused kernel only: u = a_r.v -> t; psi of the first trial step min(1, alpha_ub)
    kRowQpEval = 5,    // two-pass row kernel only: u = a_r.v -> row; loss += 0.5 v_r u   (A symmetric, v = s.x)
    kRowQpDir = 6      // two-pass row kernel only: u = a_r.v -> t;   loss += v_r u       (v = s.p)
};

struct APassArgs {
    const void* A;
    const double* b;
    const double* w;        // per-row weights of the least-squares kinds (null = all ones)
    const double* vs;       // QP: v is multiplied entrywise by this sign vector (null = ones)
    const double* va;       // v = va[c] - (vb ? vb[c] : 0)
    const double* vb;
    const double* p1;       // when select_p != 0: va/vb are taken from p1 or p2 according to Scal::branch
    const double* p2;
    int select_p;
    int split;              // L1SPLIT: vb = va + cols
    int mode;               // RowMode
    int check_status;       // skip all work unless Scal::status == RUNNING
    // kRowLogiSpec only: every workgroup also sums, over its own rows, the loss differences of the first trial step
    // (softplus(-y (z + alpha0 t)) - softplus(-y z)) into its loss partial, so that the update kernel can take the
    // Armijo decision on that step without a sweep over the margins in a kernel of its own
    int ls_first;
    // select_p with dir_blocks > 0: the direction kernel has left its partial sums in dir_part without choosing; every
    // workgroup of the pass makes Algorithm 2's choice itself (dir_choice_from_partials) and workgroup 0 records it in
    // the scalar block.  dir_blocks == 0: the choice is read from the scalar block.
    const double* dir_part;
    int dir_blocks;
    double eps;
    // non-null: the status word is read from this copy of the scalar block, and workgroup 0 first moves the copy into the
    // scalar block itself if the direction kernel marked it fresh (see Buffers::scal_next)
    Scal* scal_next;
};

// ev0/ev1 (both or neither): HIP events attached to the dispatch itself, so that their difference is
// the kernel's own duration
void launch_gemv(const Dims& dm, const Geometry& ge, const Buffers& bf, const APassArgs& a, hipStream_t st,
                 hipEvent_t ev0 = nullptr, hipEvent_t ev1 = nullptr);
// w partials = A^T psi_src (psi_src: Buffers::psi after an evaluation, Buffers::t after a direction pass)
void launch_gemvt_from(const Dims& dm, const Geometry& ge, const Buffers& bf, const void* A, const double* psi_src,
                       int check_status, hipStream_t st, hipEvent_t ev0 = nullptr, hipEvent_t ev1 = nullptr);
bool fused_shape_ok(const Dims& dm, const void* A, int* variant, int* blocks);
bool fused_ls_first_ok(const Dims& dm, const Geometry& ge);   // APassArgs::ls_first may be set (its LDS fits)
hipError_t fused_prepare(const Dims& dm, const Geometry& ge);   // once per solver, before the first launch_fused
void launch_fused(const Dims& dm, const Geometry& ge, const Buffers& bf, const APassArgs& a, hipStream_t st,
                  hipEvent_t ev0 = nullptr, hipEvent_t ev1 = nullptr);

void launch_fill_zero(void* p, size_t bytes, hipStream_t st);
void launch_set_status(const Buffers& bf, int status, hipStream_t st);
void launch_eval_finish(const Dims& dm, const Geometry& ge, const Buffers& bf, const double* lin, const double* sign,
                        hipStream_t st);   // lin, sign: QP only (linear term b, sign vector)
// no_close (wide kernel with a one-level grid only, see gram_can_skip_close): the kernel ends when its workgroups'
// partial sums are written; the direction kernel does the rest (launch_dir with gram_blocks > 0)
void launch_gram(const Dims& dm, const Opts& op, const Geometry& ge, const Buffers& bf, int dbg_inputs,
                 int evaluate_stop, hipStream_t st, hipEvent_t ev0 = nullptr, hipEvent_t ev1 = nullptr, int no_close = 0);
bool gram_can_skip_close(const Dims& dm, const Geometry& ge);
void launch_commit(const Dims& dm, const Buffers& bf, hipStream_t st);
// store_d: also keep d itself (the primitive-level hooks read it; an iteration only needs the two candidates)
bool dir_folds_extra_rows(const Dims& dm);
// fold_rows / fold_weight: the objective's extra rows and their weights when they are to ride along (else NULL)
// defer_choice: the kernel stops after its partial sums (no last workgroup, nothing written to the scalar block): the
// consumer of the direction makes Algorithm 2's choice from them (APassArgs::dir_part); not with folded rows
// gram_blocks > 0 (short vectors only): the Gram kernel left its workgroups' partial sums without a closing step; every
// workgroup of the direction kernel adds them, applies the pending update and runs the recursion on a private copy of
// the scalar block, and workgroup 0 leaves its copy in Buffers::scal_next
void launch_dir(const Dims& dm, const Opts& op, const Geometry& ge, const Buffers& bf, int d_given, int store_d,
                hipStream_t st, const double* fold_rows = nullptr, const double* fold_weight = nullptr,
                int defer_choice = 0, int gram_blocks = 0);
// fold_weight, dir_blocks > 0: the direction kernel ended without its closing step; the update kernel forms the folded
// rows' coefficients itself from that kernel's per-workgroup sums (Buffers::redpart)
void launch_update_quadratic(const Dims& dm, const Opts& op, const Geometry& ge, const Buffers& bf, const double* sign,
                             hipStream_t st, const double* fold_rows = nullptr, const double* fold_weight = nullptr,
                             int dir_blocks = 0);
// extra rows: e_r.z for z = x (eval != 0: residuals against the targets) or the selected direction (eval == 0)
void launch_extra_rows(const Dims& dm, const Buffers& bf, const double* rows, const double* target, const double* weight,
                       int eval, hipStream_t st);
// spec != 0: the A pass already holds X^T psi of the first trial step (recorded in Scal::spec_ok if that step is accepted)
// stages: 2 = the continuation only (eight more step lengths per sweep, then one at a time: what the host supplies
// after the short sequence has rejected the first trial step), 3 = the first trial step in a sweep of its own, then
// the continuation
void launch_ls_logistic(const Dims& dm, const Opts& op, const Geometry& ge, const Buffers& bf, const double* labels,
                        int spec, int stages, hipStream_t st);
void launch_rows_logistic(const Dims& dm, const Geometry& ge, const Buffers& bf, const double* labels, hipStream_t st);
// short != 0: the short sequence's update.  The pass over X has left the loss differences of the first trial step in
// its loss partials; every workgroup adds them up and takes the Armijo decision itself.  Accepted: margins z += alpha t
// here, f from that difference.  Rejected: the solver is parked in kStatusBail and nothing is updated.
void launch_update_logistic(const Dims& dm, const Opts& op, const Geometry& ge, const Buffers& bf, int loss_parts,
                            int short_seq, hipStream_t st);
void launch_clear_bail(const Buffers& bf, hipStream_t st);   // status kStatusBail -> RUNNING, bail_skipped -> 0

// transport kinds (transport.hip).  M: cost matrix; beta/omega: targets and weights of the rows + cols marginal
// terms (omega null = no such terms).  eval: z = x, residuals against beta -> Buffers::row; else z = the selected
// direction, K z -> Buffers::t.  Loss partials: ot_row_blocks + ot_col_blocks entries.
struct OtArgs {
    const void* M;
    const double* beta;
    const double* omega;
};
// dir_blocks > 0 (direction sums only): the direction kernel has left its partial sums in Buffers::redpart without
// choosing between Algorithm 2's candidates; the row-sum kernel makes the choice and records it in the scalar block
void launch_ot_sums(const Dims& dm, const Geometry& ge, const Buffers& bf, const OtArgs& a, int eval, int check_status,
                    hipStream_t st, int dir_blocks = 0, double eps = 0.0);
void launch_ot_eval_finish(const Dims& dm, const Geometry& ge, const Buffers& bf, const OtArgs& a, hipStream_t st);
void launch_ot_update_gauss(const Dims& dm, const Opts& op, const Geometry& ge, const Buffers& bf, const OtArgs& a,
                            hipStream_t st);
void launch_ot_step_entropy(const Dims& dm, const Opts& op, const Geometry& ge, const Buffers& bf, const OtArgs& a,
                            hipStream_t st);

// single-workgroup resident solver for small least-squares problems (resident.hip)
bool resident_shape_ok(const Dims& dm, bool has_row_weight);
hipError_t resident_prepare(const Dims& dm);   // once per solver, before the first launch_resident
// host_scal: pinned host memory that receives the scalar block as well when the launch ends (null: device copy only)
void launch_resident(const Dims& dm, const Opts& op, const Buffers& bf, const void* A, const double* b, int max_steps,
                     int refresh_every, hipStream_t st, Scal* host_scal = nullptr);

int gram_blocks_for(int64_t n, int m);
size_t gram_partial_bytes(int64_t n, int m);   // Buffers::grampart
hipError_t gram_prepare(int64_t n, int m);     // once per solver, before the first launch_gram

}  // namespace lb
