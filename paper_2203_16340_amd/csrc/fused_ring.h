// Fused single-read A pass for the quadratic objectives, software-pipelined.
//
// For f(x) = 0.5*||A v(x) - b||^2 (+ linear terms) one iteration needs t = A v_p and w = A^T t
// (direction pass), and an evaluation needs r = A v - b and A^T r.  Both have the shape
//     u_r = a_r . v,   psi_r = rowop(u_r),   w += a_r * psi_r      for every row r,
// so a workgroup that owns WHOLE rows can keep a row on chip between its dot product and its
// contribution to w, and A is read from HBM exactly once per pass instead of twice.
//
// What limits such a kernel on MI355X is not arithmetic but the bytes it keeps in flight: a row
// cannot be released before its dot product has been reduced over the workgroup, so unless later
// rows are already being loaded the memory system idles during every reduction.  On-chip storage
// per compute unit is 512 KiB of vector registers and 160 KiB of LDS, and the per-column state
// (v and the fp64 accumulators of w) already takes 16 bytes per column.  Layout chosen here:
//   * v lives in LDS (read once per row by every thread: ~1/5 of the LDS bandwidth),
//   * the accumulators of w live in registers (thread `tid` owns the 16-byte chunks
//     (k*NT + tid), k = 0..KC-1, of every row: a wave reads 1 KiB contiguous per load),
//   * the rest of the register file is a RING of NB slots, each holding this thread's chunks
//     of one row fraction (a row is U slots of KCU chunks, KC = U*KCU).  A slot is refilled
//     with the row fraction NB slots ahead as soon as its contribution to w has been taken,
//     so loads stay in flight across the reduction and the barrier.
// Rows are dealt to workgroups in contiguous ranges and processed R at a time (one barrier per R
// rows).  Each workgroup writes its partial w (summed later in workgroup order, so results are
// bit-reproducible) and one loss partial.
//
// Bytes: rows*cols*sizeof(T) read once, plus G*cols*8 written (G workgroups) and rows*8 for t or r.
#pragma once

#include "common.h"
#include "apass_rowop.h"

namespace lb {
namespace ring {

// 16 bytes of a row as the compiler's native vector types (the non-temporal load builtin takes these)
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef double f64x2 __attribute__((ext_vector_type(2)));
template <typename T> struct Raw;
template <> struct Raw<float> { using type = f32x4; };
template <> struct Raw<double> { using type = f64x2; };

__device__ __forceinline__ void widen(const f32x4& r, double (&o)[4]) { o[0] = r.x; o[1] = r.y; o[2] = r.z; o[3] = r.w; }
__device__ __forceinline__ void widen(const f64x2& r, double (&o)[2]) { o[0] = r.x; o[1] = r.y; }
__device__ __forceinline__ f32x4 zero_raw(const float*) { return f32x4{0.f, 0.f, 0.f, 0.f}; }
__device__ __forceinline__ f64x2 zero_raw(const double*) { return f64x2{0.0, 0.0}; }

// Makes the compiler forget what it knows about a loaded fp32 chunk, so that it converts it to fp64 a
// second time instead of holding both copies in registers.
__device__ __forceinline__ void forget(f32x4& r) { asm volatile("" : "+v"(r)); }
__device__ __forceinline__ void forget(f64x2&) {}

constexpr int gcd_i(int a, int b) { return b == 0 ? a : gcd_i(b, a % b); }

// The objective's per-row operation on u = a_r . v, as pure arithmetic (b and z are the row's entries of
// the target/label vector and of the stored margins, read ahead of time):
//   psi  : the row's weight in the transposed product,
//   loss : the row's contribution to the loss partial,
//   keep : the value stored for the row (into t for the direction modes, into row for the evaluations).
// LOGI selects the family at compile time: 0 = quadratic objectives, 1 = logistic (evaluation and
// direction pass), 2 = logistic direction pass only, whose chain is short enough to leave registers for
// a deeper ring (the transcendental code of the logistic modes would
// otherwise cost the quadratic kernels registers they need for the ring).
template <int LOGI>
__device__ __forceinline__ void row_eval(int mode, double u, double b, double z, double alpha0, double invn,
                                         double& psi, double& loss, double& keep) {
    if constexpr (LOGI == 0) {
        // z carries the row's weight here (1 when the objective has none); in the quadratic-form modes the
        // row's own entry of v (the row index is also a column index of the symmetric matrix)
        if (mode == kRowQpEval || mode == kRowQpDir) {
            psi = 0.0; keep = u;
            loss = (mode == kRowQpEval ? 0.5 : 1.0) * z * u;
        } else if (mode == kRowDir) {       // t = A p for the closed-form line search; w = A^T (weights * t)
            psi = z * u; loss = psi * u; keep = u;
        } else {                            // kRowLsqEval: r = A v - b; w = A^T (weights * r)
            const double res = u - b;
            psi = z * res; loss = 0.5 * psi * res; keep = res;
        }
    } else {
        // one exponential serves sigma and softplus of the same argument
        if (LOGI == 1 && mode == kRowLogiEval) {   // margins z = X w; psi = -y sigma(-y z)/N
            const double q = -b * u;
            const double e = exp(-fabs(q));
            psi = -b * ((q >= 0.0 ? 1.0 : e) / (1.0 + e)) * invn;
            loss = (fmax(q, 0.0) + log1p(e)) * invn;
            keep = u;
        } else {                            // kRowLogiSpec: t = X p, and the weights of the FIRST trial step alpha0
            // psi = -y sigma(-y (z + alpha0 t))/N: what the transposed product needs if alpha0 is accepted.
            // Whether it is accepted is decided after this pass, from the margins (k_ls_logistic), so the
            // chain every stage waits for is one exponential and one division.
            const double q = -b * fma(alpha0, u, z);
            const double e = exp(-fabs(q));
            psi = -b * ((q >= 0.0 ? 1.0 : e) / (1.0 + e)) * invn;
            loss = 0.0;
            keep = u;
        }
    }
}

// After the barrier of a stage: lane r (< R) of EVERY wave sums the partial dot products of row r of the
// stage and evaluates its row operation -- the transcendental functions of the logistic modes run once
// per stage, not once per row -- wave 0 stores the row's entry of t / row, and the weights psi are
// handed to all lanes through scalar registers.  red: [R][NW] partial dot products of this stage;
// bcur/zcur: the rows' entries of b and of the stored margins; row0: global index of the stage's first row.
template <int R, int NW, int LOGI>
__device__ __forceinline__ void stage_row_op(const double* red, int lane, int wave, int mode, const double (&bcur)[R],
                                             const double (&zcur)[R], int64_t row0, int64_t r_end, double alpha0,
                                             double invn, double* __restrict__ row, double* __restrict__ t,
                                             double& loss, double (&psi)[R], double* lsq = nullptr, int64_t r_begin = 0) {
    const int rl = lane < R ? lane : 0;
    double u = 0.0;
#pragma unroll
    for (int q = 0; q < NW; ++q) u += red[rl * NW + q];
    // lane r takes entry r: a chain of selects on values made opaque first (left transparent, the compiler
    // turns the chain into an array in scratch memory indexed by the lane, i.e. into vector memory traffic
    // in the middle of the stage)
    double bl = 0.0, zl = 0.0;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        double bv = bcur[r], zv = zcur[r];
        asm volatile("" : "+v"(bv), "+v"(zv));
        if (lane == r) { bl = bv; zl = zv; }
    }
    const int64_t grow = row0 + rl;
    const bool valid = lane < R && grow < r_end;
    double psil, lossl, keep;
    row_eval<LOGI>(mode, u, bl, zl, alpha0, invn, psil, lossl, keep);
    if (!valid) { psil = 0.0; lossl = 0.0; }
    loss += lossl;
    if (valid && wave == 0) {
        if (mode == kRowDir || mode == kRowLogiSpec || mode == kRowQpDir) t[grow] = keep; else row[grow] = keep;
        if constexpr (LOGI == 2) {
            // what the first trial step's loss difference of this row needs (summed after the row loop): q = -y z and
            // dq = -y alpha0 t, kept in LDS at the row's local index
            if (lsq) {
                lsq[2 * (grow - r_begin)] = -bl * zl;
                lsq[2 * (grow - r_begin) + 1] = -bl * alpha0 * u;
            }
        }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) psi[r] = lane_bcast(psil, r);
}

// v[c] = (va[c] - vb[c]) * sc[c] (difference and scaling optional) for c < lcols into LDS: E entries per thread
// and round, every load of a round issued before the first value is used (a round is one trip to memory).
// `after_last_issue` runs once, in every thread, when the loads of the last round have been issued and before they are
// waited for: loads return in the order they were issued, so whatever it requests arrives behind v, not in front of it.
template <int NT, int E, bool HAS_VB, bool HAS_VS, class Hook>
__device__ __forceinline__ void stage_v_looped(const double* __restrict__ va, const double* __restrict__ vb,
                                        const double* __restrict__ sc, double* vs, int lcols, int tid,
                                        Hook&& after_last_issue) {
    const int rounds = (lcols + NT * E - 1) / (NT * E);      // the same in every thread
    if (rounds == 0) after_last_issue();
    for (int r = 0; r < rounds; ++r) {
        const int c0 = tid + r * NT * E;
        double v8[E], b8[E], s8[E];
#pragma unroll
        for (int k = 0; k < E; ++k) {
            const int c = c0 + k * NT;
            const int cc = c < lcols ? c : lcols - 1;
            v8[k] = va[cc];
            if (HAS_VB) b8[k] = vb[cc];
            if (HAS_VS) s8[k] = sc[cc];
        }
        if (r == rounds - 1) {
            __builtin_amdgcn_sched_barrier(0);
            after_last_issue();
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int k = 0; k < E; ++k) {
            const int c = c0 + k * NT;
            double v = v8[k];
            if (HAS_VB) v -= b8[k];
            if (HAS_VS) v *= s8[k];
            if (c < lcols) vs[c] = v;
        }
    }
}

// The same with the last round outside the loop.
template <int NT, int E, bool HAS_VB, bool HAS_VS, class Hook>
__device__ __forceinline__ void stage_v_peeled(const double* __restrict__ va, const double* __restrict__ vb,
                                        const double* __restrict__ sc, double* vs, int lcols, int tid,
                                        Hook&& after_last_issue) {
    const int rounds = (lcols + NT * E - 1) / (NT * E);      // the same in every thread, at least one (lcols >= 1)
    // The last round stands outside the loop, in straight-line code: inside it, under a test of the round number, the
    // wait the compiler puts in front of the use of v covers half of the hook's loads as well (it has to assume the
    // path on which the hook did not run).
    for (int r = 0; r + 1 < rounds; ++r) {
        const int c0 = tid + r * NT * E;
        double v8[E], b8[E], s8[E];
#pragma unroll
        for (int k = 0; k < E; ++k) {
            const int c = c0 + k * NT;                       // (not the last round: every entry exists)
            v8[k] = va[c];
            if (HAS_VB) b8[k] = vb[c];
            if (HAS_VS) s8[k] = sc[c];
        }
#pragma unroll
        for (int k = 0; k < E; ++k) {
            double v = v8[k];
            if (HAS_VB) v -= b8[k];
            if (HAS_VS) v *= s8[k];
            vs[c0 + k * NT] = v;
        }
    }
    {
        const int c0 = tid + (rounds - 1) * NT * E;
        double v8[E], b8[E], s8[E];
#pragma unroll
        for (int k = 0; k < E; ++k) {
            const int c = c0 + k * NT;
            const int cc = c < lcols ? c : lcols - 1;
            v8[k] = va[cc];
            if (HAS_VB) b8[k] = vb[cc];
            if (HAS_VS) s8[k] = sc[cc];
        }
        __builtin_amdgcn_sched_barrier(0);
        after_last_issue();
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int k = 0; k < E; ++k) {
            const int c = c0 + k * NT;
            double v = v8[k];
            if (HAS_VB) v -= b8[k];
            if (HAS_VS) v *= s8[k];
            if (c < lcols) vs[c] = v;
        }
    }
}

// Which of the two: the peeled form where several workgroups share a compute unit (the narrow variants: C4's pass is
// 4 us shorter with it), the loop where one workgroup of 512 threads has it to itself (there the peeled form measured
// 0.7 us slower at C3 and no different at C2 and C5).
template <int NT, int E, bool HAS_VB, bool HAS_VS, class Hook>
__device__ __forceinline__ void stage_v(const double* __restrict__ va, const double* __restrict__ vb,
                                        const double* __restrict__ sc, double* vs, int lcols, int tid,
                                        Hook&& after_last_issue) {
    if constexpr (NT < 512) stage_v_peeled<NT, E, HAS_VB, HAS_VS>(va, vb, sc, vs, lcols, tid, after_last_issue);
    else stage_v_looped<NT, E, HAS_VB, HAS_VS>(va, vb, sc, vs, lcols, tid, after_last_issue);
}

// dynamic LDS a launch needs: v for the columns held there (all of them unless the variant keeps the v of
// its last KR chunks per thread in registers), one all-zero chunk, then the reduction scratch
constexpr int kPad = 4;
template <typename T, int NT, int KC, int KR>
inline int64_t lds_cols(int64_t cols) {
    const int64_t cap = (int64_t)(KC - KR) * NT * (16 / (int)sizeof(T));
    return KR > 0 && cols > cap ? cap : cols;
}
template <typename T, int NT, int KC, int KR, int R>
inline size_t lds_bytes(int64_t cols) {
    return ((size_t)lds_cols<T, NT, KC, KR>(cols) + kPad) * 8 + (size_t)2 * R * (NT / 64) * 8;
}

// TRANS = false: the transposed accumulation is left out (quadratic form with a symmetric matrix: the row
// products are all an iteration needs), and the registers it would take go to a deeper ring.
template <typename T, int NT, int KCU, int U, int R, int NB, int WPE, int LOGI, int KR = 0, bool TRANS = true>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(WPE, WPE)))
void k_fused_ring(const T* __restrict__ A, int64_t ld, int64_t rows, int64_t cols, int64_t rows_per_wg, APassArgs a,
                  Scal* __restrict__ scal, double* __restrict__ row, double* __restrict__ t,
                  double* __restrict__ wpart, double* __restrict__ losspart) {
    using RawT = typename Raw<T>::type;
    constexpr int VEC = 16 / sizeof(T);
    constexpr int KC = KCU * U;
    constexpr int NW = NT / 64;
    constexpr int SPS = R * U;                               // slots one stage (R rows) consumes
    constexpr int STAGES = NB / gcd_i(NB, SPS);              // stages after which the ring is back at slot 0
    static_assert(NB >= SPS, "the ring must hold at least one stage");
    static_assert(R <= 16, "one lane per row of a stage evaluates the row operation");
    extern __shared__ __align__(16) double lds[];
    // Rows too wide for v to fit in LDS: the v of each thread's last KR chunks stays in registers instead
    static_assert(KR == 0 || U == 1, "register-resident v is only combined with whole-row slots");
    constexpr int KL = KC - KR;                              // chunks whose v is read from LDS
    const int lcols = KR > 0 && cols > (int64_t)KL * NT * VEC ? KL * NT * VEC : (int)cols;
    double* vs = lds;                                        // v, `lcols` entries, then kPad zeros
    double* red = lds + lcols + kPad;                        // [2][R][NW]
    // logistic direction pass that also sums the first trial step's loss differences: (q, dq) per row of this workgroup
    double* lsq = (LOGI == 2 && a.ls_first) ? red + 2 * R * NW : nullptr;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // chunk k of this thread starts at column (k*NT + tid)*VEC.  A chunk at or past `cols` does not
    // exist: its loads are redirected to the last chunk of the row (valid memory) and its v to the
    // zero pad, so it adds nothing to a dot product, and its w is never stored.  No load is predicated.
    const int c0 = tid * VEC;
    constexpr int kStride = NT * VEC;
    const int icols = (int)cols;
    double w[TRANS ? KC : 1][VEC];
#pragma unroll
    for (int k = 0; k < (TRANS ? KC : 1); ++k)
#pragma unroll
        for (int j = 0; j < VEC; ++j) w[k][j] = 0.0;

    const int64_t r_begin = (int64_t)blockIdx.x * rows_per_wg;
    const int64_t r_end = r_begin + rows_per_wg < rows ? r_begin + rows_per_wg : rows;
    const int nstage = r_end > r_begin ? (int)((r_end - r_begin + R - 1) / R) : 0;   // (the grid is sized so that no range is empty)

    RawT raw[NB][KCU];
    // fills a ring slot with row fraction j of local row lr (past the last row: that row again, whose
    // psi is zero; the few repeated loads hit in L2)
    auto fetch = [&](RawT (&dst)[KCU], int64_t lr, int j) {
        const int64_t gr = r_begin + lr < r_end ? r_begin + lr : r_end - 1;
        const char* rp = reinterpret_cast<const char*>(A + gr * ld);   // uniform: lives in scalar registers
        // 32-bit byte offsets, recomputed at every use (two integer operations) rather than kept in
        // registers; scalar base + 32-bit vector offset is the addressing form wanted here
        unsigned cb = (unsigned)c0;
        asm volatile("" : "+v"(cb));
#pragma unroll
        for (int k = 0; k < KCU; ++k) {
            unsigned c = cb + (unsigned)((j * KCU + k) * kStride);
            c = c < (unsigned)(icols - VEC) ? c : (unsigned)(icols - VEC);
            dst[k] = __builtin_nontemporal_load(reinterpret_cast<const RawT*>(rp + c * (unsigned)sizeof(T)));
        }
    };
    // The ring is primed as early as it can be without getting in the way: loads return in the order they were issued,
    // so rows requested before the status word, the direction kernel's records and v would have to arrive in full
    // (a whole ring: hundreds of kilobytes per workgroup) before any of those small reads did.  The rows are therefore
    // requested right behind the last of v's loads and arrive while v is written to LDS.
    auto prime = [&]() {
#pragma unroll
        for (int s = 0; s < NB; ++s) fetch(raw[s], (s / SPS) * R + (s % SPS) / U, (s % SPS) % U);
    };
    // Algorithm 2's choice between the candidate directions: from the scalar block, or made here from the direction
    // kernel's partial sums (every wave of every workgroup gets the same bits; workgroup 0 records them).  The status
    // word is requested first and looked at afterwards, so that its trip to memory and the records' are one.
    // With a.scal_next the status word comes from the copy of the scalar block the direction kernel's workgroup 0 left
    // there, and the first wave of workgroup 0 moves that copy into the scalar block itself (no other workgroup of this
    // kernel reads the scalar block then), with the choice just made written into it on the way.
    const Scal* st_src = a.scal_next ? a.scal_next : scal;
    const int status = a.check_status ? st_src->status : LBFGSB_RUNNING;
    constexpr int kScalWords = (int)(sizeof(Scal) / 4), kScalPerLane = (kScalWords + 63) / 64;
    const bool mover = a.scal_next && blockIdx.x == 0 && tid < 64;
    int moved[kScalPerLane];
    int fresh = 0;
    if (mover) {
        fresh = a.scal_next->fresh;
#pragma unroll
        for (int j = 0; j < kScalPerLane; ++j) {
            const int idx = tid + 64 * j;
            moved[j] = idx < kScalWords ? reinterpret_cast<const int*>(a.scal_next)[idx] : 0;
        }
    }
    int branch = 0;
    double alpha_ub = 1.0;
    DirChoice ch{};
    const bool own_choice = a.select_p && a.dir_blocks > 0;
    if (own_choice) ch = dir_choice_from_partials(a.dir_part, a.dir_blocks, a.eps);
    if (mover && fresh) {
        const bool with_choice = own_choice && status == LBFGSB_RUNNING;
#pragma unroll
        for (int j = 0; j < kScalPerLane; ++j) {
            const int idx = tid + 64 * j;
            int v = moved[j];
            auto put_double = [&](size_t off, double val) {
                if (idx == (int)(off / 4)) v = __double2loint(val);
                if (idx == (int)(off / 4) + 1) v = __double2hiint(val);
            };
            if (with_choice) {
                if (idx == (int)(offsetof(Scal, branch) / 4)) v = ch.branch;
                put_double(offsetof(Scal, gp), ch.gp);
                put_double(offsetof(Scal, alpha_ub), ch.alpha_ub);
                put_double(offsetof(Scal, pp), ch.pp);
                put_double(offsetof(Scal, xp), ch.xp);
            }
            if (idx == (int)(offsetof(Scal, fresh) / 4)) v = 0;
            if (idx < kScalWords) reinterpret_cast<int*>(scal)[idx] = v;
        }
        if (tid == 0) a.scal_next->fresh = 0;
    }
    if (status != LBFGSB_RUNNING) return;
    if (own_choice) {
        branch = ch.branch;
        alpha_ub = ch.alpha_ub;
        if (blockIdx.x == 0 && tid == 0 && !(a.scal_next && fresh)) {
            scal->branch = ch.branch; scal->gp = ch.gp; scal->alpha_ub = ch.alpha_ub; scal->pp = ch.pp; scal->xp = ch.xp;
        }
    } else if (LOGI != 0 && a.mode == kRowLogiSpec) {
        alpha_ub = scal->alpha_ub;
    }
    const double *va, *vb;
    resolve_v(a, scal, cols, va, vb, branch);

    // v into LDS, eight entries per thread and round with all their loads issued before the first is used (one
    // entry at a time this loop was a chain of dependent trips to memory: 3.5 us at 5000 columns).  The optional
    // difference and scaling are decided outside the loop, whose body then has no branch for a load to wait at.
    constexpr int VE = 8;                                    // entries per thread and round (12 and 16 measured no faster; 16 spills in the widest variants)
    double vreg[KR > 0 ? KR : 1][VEC];
#pragma unroll
    for (int k = 0; k < KR; ++k) {
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
            const int64_t c = (int64_t)((KL + k) * NT + tid) * VEC + j;
            vreg[k][j] = c < cols ? (vb ? va[c] - vb[c] : va[c]) * (a.vs ? a.vs[c] : 1.0) : 0.0;
        }
    }
    if (vb) {
        if (a.vs) stage_v<NT, VE, true, true>(va, vb, a.vs, vs, lcols, tid, prime); else stage_v<NT, VE, true, false>(va, vb, a.vs, vs, lcols, tid, prime);
    } else {
        if (a.vs) stage_v<NT, VE, false, true>(va, vb, a.vs, vs, lcols, tid, prime); else stage_v<NT, VE, false, false>(va, vb, a.vs, vs, lcols, tid, prime);
    }
    if (tid < kPad) vs[lcols + tid] = 0.0;

    // The row's entries of b (targets or labels) and of the row weights (quadratic kinds) or, for the
    // speculative logistic pass, of the stored margins are read one stage ahead through the scalar unit (the row index is uniform and neither
    // vector is written by this kernel in the modes that read it): scalar loads are not ordered with
    // the vector loads of the ring, so waiting for one does not drain the rows in flight.
    typedef const double __attribute__((address_space(4))) * ConstD;
    const int mode = a.mode;
    const bool need_b = mode != kRowDir && mode != kRowQpEval && mode != kRowQpDir, need_z = LOGI != 0 && mode == kRowLogiSpec;
    auto read_rows = [&](double (&db)[R], double (&dz)[R], int64_t lr) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int64_t gr = r_begin + lr + r < r_end ? r_begin + lr + r : r_end - 1;
            db[r] = need_b ? *(ConstD)(uintptr_t)(a.b + gr) : 0.0;
            if constexpr (LOGI != 0) {
                dz[r] = need_z ? *(ConstD)(uintptr_t)(row + gr) : 0.0;
            } else if (mode == kRowQpEval || mode == kRowQpDir) {
                // (v is not written by this kernel: the scalar reads are safe)
                double vr = *(ConstD)(uintptr_t)(va + gr);
                if (vb) vr -= *(ConstD)(uintptr_t)(vb + gr);
                if (a.vs) vr *= *(ConstD)(uintptr_t)(a.vs + gr);
                dz[r] = vr;
            } else {
                dz[r] = a.w ? *(ConstD)(uintptr_t)(a.w + gr) : 1.0;
            }
        }
    };
    const double alpha0 = need_z ? fmin(1.0, alpha_ub) : 0.0;   // first trial step of the line search
    const double invn = 1.0 / (double)rows;
    double bcur[R], zcur[R];
    read_rows(bcur, zcur, 0);
    __syncthreads();                                         // v is in LDS

    double loss = 0.0;
    int par = 0;
    int prio_now = -1;
    constexpr int kSegStages = 6;                            // stages per priority segment
    const int nseg = (nstage + kSegStages - 1) / kSegStages;
    for (int st0 = 0; st0 < nstage; st0 += STAGES) {
        // Where two workgroups share a compute unit, the one dispatched first wins every arbitration between waves of
        // equal priority: it runs at almost the speed it would have alone, the other at two thirds of that, and when
        // the first has finished the second is left with a compute unit it cannot fill on its own.  So a workgroup
        // steps its waves' priority down as it gets on with its rows -- 3, 2, 1, 0 over four segments of a few stages,
        // then again, counted from the END so that the last four segments are one descent: whichever workgroup is
        // ahead is in a lower segment of the descent and yields to the other.
        const int prio = (nseg - 1 - st0 / kSegStages) & 3;
        if (prio != prio_now) {
            prio_now = prio;
            switch (prio) {
                case 3: __builtin_amdgcn_s_setprio(3); break;
                case 2: __builtin_amdgcn_s_setprio(2); break;
                case 1: __builtin_amdgcn_s_setprio(1); break;
                default: __builtin_amdgcn_s_setprio(0); break;
            }
        }
#pragma unroll
        for (int ss = 0; ss < STAGES; ++ss) {
            const int64_t lr0 = (int64_t)(st0 + ss) * R;     // first local row of the stage
            double acc[R];
#pragma unroll
            for (int r = 0; r < R; ++r) acc[r] = 0.0;
            // v does not change between rows, but holding it in registers is exactly what this kernel
            // avoids: an offset the compiler cannot see through keeps the LDS reads inside the loop
            int cb = c0;
            asm volatile("" : "+v"(cb));
#pragma unroll
            for (int q = 0; q < SPS; ++q) {
                const int slot = (ss * SPS + q) % NB;
                const int r = q / U, j = q % U;
#pragma unroll
                for (int k = 0; k < KCU; ++k) {
                    const int kk = j * KCU + k;
                    double e[VEC];
                    widen(raw[slot][k], e);
                    if (kk >= KL) {                          // (compile-time) v of this chunk is in registers
#pragma unroll
                        for (int i = 0; i < VEC; ++i) acc[r] = fma(e[i], vreg[kk - KL][i], acc[r]);
                        continue;
                    }
                    int c = cb + kk * kStride;
                    c = c < lcols ? c : lcols;               // zero pad for a chunk that does not exist
#pragma unroll
                    for (int i = 0; i < VEC; i += 2) {       // 16-byte LDS reads
                        const double2 vv = *reinterpret_cast<const double2*>(vs + c + i);
                        acc[r] = fma(e[i], vv.x, acc[r]);
                        acc[r] = fma(e[i + 1], vv.y, acc[r]);
                    }
                }
            }
#pragma unroll
            for (int r = 0; r < R; ++r) acc[r] = wave_sum(acc[r]);
            if (lane == 0) {
#pragma unroll
                for (int r = 0; r < R; ++r) red[(par * R + r) * NW + wave] = acc[r];
            }
            __syncthreads();
            double bnext[R], znext[R];
            read_rows(bnext, znext, lr0 + R);
            double psi[R];
            stage_row_op<R, NW, LOGI>(red + par * R * NW, lane, wave, mode, bcur, zcur, r_begin + lr0, r_end, alpha0,
                                      invn, row, t, loss, psi, lsq, r_begin);
#pragma unroll
            for (int r = 0; r < R; ++r) {
                bcur[r] = bnext[r];
                zcur[r] = znext[r];
            }
#pragma unroll
            for (int q = 0; q < SPS; ++q) {
                const int slot = (ss * SPS + q) % NB;
                const int r = q / U, j = q % U;
#pragma unroll
                for (int k = 0; k < KCU; ++k) {
                    if constexpr (!TRANS) break;
                    const int kk = j * KCU + k;
                    forget(raw[slot][k]);                    // fp32 data is widened again here rather than kept widened across the barrier
                    double e[VEC];
                    widen(raw[slot][k], e);
#pragma unroll
                    for (int i = 0; i < VEC; ++i) w[TRANS ? kk : 0][i] = fma(e[i], psi[r], w[TRANS ? kk : 0][i]);
                }
                // the slot is free: refill it with the row fraction NB slots ahead.  The scheduling
                // barriers keep the loads from being hoisted above the last use of the old contents
                // (which would need a second set of registers for the slot)
                const int g = ss * SPS + q + NB;             // slot sequence number relative to stage st0
                __builtin_amdgcn_sched_barrier(0);
                fetch(raw[slot], (int64_t)(st0 + g / SPS) * R + (g % SPS) / U, (g % SPS) % U);
                __builtin_amdgcn_sched_barrier(0);
            }
            par ^= 1;
        }
    }
    if constexpr (TRANS) {
        double* out = wpart + (int64_t)blockIdx.x * cols + c0;
#pragma unroll
        for (int k = 0; k < KC; ++k) {
            if (c0 + k * kStride < icols) {
#pragma unroll
                for (int j = 0; j < VEC; ++j) out[k * kStride + j] = w[k][j];
            }
        }
    }
    if constexpr (LOGI == 2) {
        // First trial step of the line search: this workgroup's share of sum_r softplus(-y (z + alpha0 t)) - softplus(-y z)
        // over its own rows, from the (q, dq) the row loop left in LDS.  Done here, after the row loop, where nothing
        // waits for it and no trip to memory is needed, so that the Armijo decision on that step takes no sweep over
        // the margins in a kernel of its own.  (The partial columns are already on their way: their stores were
        // issued above and drain meanwhile.)
        if (lsq) {
            __syncthreads();
            const int nloc = (int)(r_end - r_begin);
            double s2[2] = {0.0, 0.0};
            for (int i0 = tid; i0 < nloc; i0 += 2 * NT) {
                double q[2], dq[2];
#pragma unroll
                for (int k = 0; k < 2; ++k) {
                    const int i = i0 + k * NT;
                    q[k] = i < nloc ? lsq[2 * i] : 0.0;      // q = dq = 0: the row contributes log1p(0.5 * expm1(0)) = 0
                    dq[k] = i < nloc ? lsq[2 * i + 1] : 0.0;
                }
#pragma unroll
                for (int k = 0; k < 2; ++k) s2[k] += softplus_diff(q[k], sigmoid_d(q[k]), dq[k]);
            }
            loss = wave_sum(s2[0] + s2[1]);
            if (lane == 0) red[wave] = loss;
        }
    }
    if constexpr (LOGI == 2) {
        if (lsq) {
            __syncthreads();
            if (tid == 0) {
                double tot = 0.0;
#pragma unroll
                for (int q = 0; q < NW; ++q) tot += red[q];
                losspart[blockIdx.x] = tot;
            }
            return;
        }
    }
    loss = wave_sum(loss);                                   // lanes 0..R-1 of a wave hold the row losses
    if (tid == 0) losspart[blockIdx.x] = loss;

}

}  // namespace ring
}  // namespace lb
