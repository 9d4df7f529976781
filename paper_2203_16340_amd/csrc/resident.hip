// Small least-squares problems: the whole of Algorithm 1 in ONE workgroup that stays on its compute unit for as many
// iterations as the caller asks for.  The multi-kernel path spends four dependent launches of 5-9 us each on an
// iteration of a 200 x 100 problem, i.e. it is bound by launch latency; here an iteration is a handful of
// workgroup barriers.
//
//   * the matrix lives in REGISTERS for the whole launch: the 512 threads form 32 groups of 16 lanes (a row of the
//     lane-permutation unit); group q owns rows q, q + 32, q + 64, ..., lane j of a group owns columns j, j + 16, ...
//     of those rows, up to 64 elements per lane, loaded once at the start (fp32 storage is widened there).  One
//     "pass over A" per iteration is then arithmetic only: t_r = a_r . p by four lane permutations inside the group,
//     which leaves t_r in exactly the lanes that need it for w = A^T t, accumulated from the same registers; the 32
//     groups' partial columns meet in LDS and are added in group order;
//   * x, g, l, u, the pair memory and the Gram matrix live in LDS; the scalar block is an LDS copy of the device one;
//   * every phase is the arithmetic of the corresponding kernel of the multi-kernel path (Eq. (ws), masked Gram matrix,
//     Algorithm 3 on coefficients -- the same device function --, Algorithm 2 with both candidate directions, the
//     closed-form Armijo search of the quadratic objectives, update and pair storage), with its own fixed summation
//     orders; iterate, gradient, pair memory, free mask and the scalar block go to device memory when the launch
//     ends, so the other entry points find the state they expect (the per-iteration records are written as they arise:
//     keeping them in LDS until the end measured slower).
// The gradient is carried by recurrence as on the multi-kernel path; it is recomputed from x every refresh_every
// iterations and before convergence is declared.
#include "common.h"
#include "recursion.h"

namespace lb {

namespace {

constexpr int kResThreads = 512;                // 8 waves, two per SIMD: 256 registers per lane, half of them hold the matrix
constexpr int kResWaves = kResThreads / 64;
constexpr int kResGroups = kResThreads / 16;    // 16-lane groups, each owning whole rows of the matrix
constexpr size_t kResLdsLimit = 150 * 1024;

struct ResArgs {
    Dims dm;
    Opts op;
    const void* A;
    const double* b;
    Scal* scal;
    double *x, *g, *S, *Y;
    const double *l, *u;
    uint8_t* mask;
    int max_steps;         // iterations this launch may take
    int refresh_every;
    int f32;               // storage type of the matrix (it is widened when it is loaded into the registers)
    Scal* host_scal;       // pinned host memory that also receives the scalar block when the launch ends (or null)
};

// LDS layout in doubles
struct ResLayout {
    int x, g, l, u, p1, p2, msk, w, S, Y, G, wred, red, alpha, total;
};
// every n-vector has npad = n rounded up to 16 entries, the padding kept at zero, so that loops over elements in
// steps of 16 need no bounds checks
__host__ __device__ inline int res_npad(int n) { return (n + 15) & ~15; }
__host__ __device__ inline ResLayout res_layout(int n, int m, int cpad) {
    ResLayout L;
    const int np = res_npad(n);
    int off = 0;
    auto take = [&](int k) { int o = off; off += (k + 1) & ~1; return o; };
    L.x = take(np); L.g = take(np); L.l = take(np); L.u = take(np); L.p1 = take(np); L.p2 = take(np); L.msk = take(np); L.w = take(np);
    L.S = take(m * np); L.Y = take(m * np);
    L.G = take((2 * m + 2) * (2 * m + 2));
    L.wred = take(kResGroups * cpad);
    L.red = take(96);               // per-phase exchange areas of the waves' partial results
    L.alpha = take(kMaxM + 1);
    L.total = off;
    return L;
}

// CPL: columns per lane (of each row its group owns); RG: rows per group (instantiated for a few sizes so that the
// matrix of a problem smaller than the largest one leaves registers for everything else).
//
// What bounds an iteration here is the latency of dependent steps (an LDS access or a shuffle is ~130 cycles when
// the next instruction waits for it), so: thread i owns element i of every n-vector (n <= 512 = threads) and keeps
// x_i, g_i, l_i, u_i in registers; sums over a wave use the lane permutations of wave_sum; LDS loads that feed a
// chain are issued in groups before they are used; reductions over the workgroup that can share a barrier do.
template <int CPL, int RG>
__global__ __launch_bounds__(kResThreads) void k_resident(ResArgs a) {
    extern __shared__ __align__(16) double lds[];
    __shared__ Scal sc;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int grp = tid >> 4, gj = tid & 15;    // this lane's group and its place in it
    const int n = (int)a.dm.cols, rows = (int)a.dm.rows, m = a.dm.m;
    const int np = res_npad(n);
    const int64_t ld = a.dm.ld;
    const ResLayout L = res_layout(n, m, CPL * 16);
    double *gs = lds + L.g, *p1s = lds + L.p1, *p2s = lds + L.p2, *xs = lds + L.x;
    double *msk = lds + L.msk, *Ss = lds + L.S, *Ys = lds + L.Y, *G = lds + L.G, *wred = lds + L.wred;
    double *red = lds + L.red, *alpha_s = lds + L.alpha;
    double *redA = red, *redD = red + 16, *redP = red + 16 + 56, *redU = red + 16 + 56 + 8;   // one region per phase
    const Opts op = a.op;
    const bool act = tid < n;                   // this thread owns element `tid`
    const int nw = (n + 63) >> 6;               // waves that own elements; the others only help with Gram and pass
    const bool wact = wave < nw;

    // ---- the matrix into registers (requested before the scalar block is looked at: it depends on nothing)
    double at[RG][CPL];
#pragma unroll
    for (int q = 0; q < RG; ++q) {
        const int r = grp + kResGroups * q;
#pragma unroll
        for (int k = 0; k < CPL; ++k) {
            const int col = gj + 16 * k;
            const int64_t o = (int64_t)r * ld + col;
            const bool in = r < rows && col < n;
            if (a.f32) at[q][k] = in ? (double)reinterpret_cast<const float*>(a.A)[o] : 0.0;
            else at[q][k] = in ? reinterpret_cast<const double*>(a.A)[o] : 0.0;
        }
    }

    // ---- the scalar block; nothing to do when the solver has stopped
    for (int k = tid; k < (int)(sizeof(Scal) / 4); k += kResThreads)
        reinterpret_cast<int*>(&sc)[k] = reinterpret_cast<const int*>(a.scal)[k];
    for (int k = tid; k < L.G; k += kResThreads) lds[k] = 0.0;   // the vectors, their padding included
    __syncthreads();
    if (sc.status != LBFGSB_RUNNING) {
        if (a.host_scal) {
            for (int k = tid; k < (int)(sizeof(Scal) / 4); k += kResThreads)
                reinterpret_cast<int*>(a.host_scal)[k] = reinterpret_cast<const int*>(&sc)[k];
        }
        return;
    }
    if (tid == 0 && sc.pend_valid) apply_pending(&sc, m);   // (left by a step of the multi-kernel path; normally none)

    // ---- the vectors into LDS and registers
    double xi = 0.0, gi = 0.0, li = 0.0, ui = 0.0, mi = 0.0;
    if (act) { xi = a.x[tid]; gi = a.g[tid]; li = a.l[tid]; ui = a.u[tid]; mi = a.mask[tid] ? 1.0 : 0.0; xs[tid] = xi; gs[tid] = gi; }
    for (int i = tid; i < m * n; i += kResThreads) {
        const int sl = i / n, e = i - sl * n;
        Ss[sl * np + e] = a.S[i];
        Ys[sl * np + e] = a.Y[i];
    }
    __syncthreads();
    // loop state every thread carries in registers (the same values in all of them)
    int c = sc.count, head = sc.head, since = sc.since_refresh;


    // Every trip of the loop makes ONE product pass: either an evaluation from scratch (r = A x - b, f = 0.5 ||r||^2,
    // g = A^T r: the periodic recomputation, and the one before convergence is declared), or the pass of an iteration.
    int steps = 0;
    bool want_eval = false;
    for (;;) {
        if (!want_eval && steps >= a.max_steps) break;
        if (!want_eval && a.refresh_every > 0 && since >= a.refresh_every) want_eval = true;

        const int V = 2 * c + 1, Vp = V + 1;
        const int base_slot = c > 0 ? (head - c + 2 * m) % m : 0;
        auto vec = [&](int j) __attribute__((always_inline)) -> const double* {
            if (j >= 2 * c) return gs;
            const bool is_y = j >= c;
            int sl = base_slot + (is_y ? j - c : j);
            if (sl >= m) sl -= m;
            return (is_y ? Ys : Ss) + sl * np;
        };
        double s6[6] = {0, 0, 0, 0, 0, 0};
        double gp = 0.0, alpha_ub = 1.0, pa = 0.0, pb = 0.0;
        int branch = 1;
        const double* ps = xs;

        if (!want_eval) {
            // ---- Eq. (ws): free set; the epsilon-free KKT residual and the number of fixed variables
            if (wact) {
                const bool fr = !(((xi <= li + op.eps) && (gi >= 0.0)) || ((xi >= ui - op.eps) && (gi <= 0.0)));
                mi = (act && fr) ? 1.0 : 0.0;
                if (act) msk[tid] = mi;
                const double nf = wave_sum((act && !fr) ? 1.0 : 0.0);
                const double pg = wave_max(act ? fabs(xi - clampd(xi - gi, li, ui)) : 0.0);
                if (lane == 0) { redA[wave] = nf; redA[kResWaves + wave] = pg; }
            }
            __syncthreads();                        // msk and the waves' partial statistics are in LDS

            // ---- masked Gram matrix of [s^0 .. s^{c-1}, y^0 .. y^{c-1}, g]: four lanes per entry, each taking every
            // fourth element; the loads of four elements are issued before their products
            {
                const int E = V * (V + 1) / 2;
                const int eg = tid >> 2, sub = tid & 3;
                for (int e0 = 0; e0 < E; e0 += kResThreads / 4) {
                    const int e = e0 + eg;
                    int ra = 0, rb = 0;
                    double s = 0.0;
                    if (e < E) {
                        int q = e;
                        while (q >= V - ra) { q -= V - ra; ++ra; }
                        rb = ra + q;
                        const double *va = vec(ra) + sub, *vb = vec(rb) + sub, *vm = msk + sub;
                        for (int i0 = 0; i0 < np; i0 += 16) {
                            double mv[4], av[4], bv[4];
#pragma unroll
                            for (int k = 0; k < 4; ++k) { mv[k] = vm[i0 + 4 * k]; av[k] = va[i0 + 4 * k]; bv[k] = vb[i0 + 4 * k]; }
#pragma unroll
                            for (int k = 0; k < 4; ++k) s = fma(mv[k] * av[k], bv[k], s);
                        }
                    }
                    s += dpp_move<kDppXor1>(s);
                    s += dpp_move<kDppXor2>(s);
                    if (e < E && sub == 0) { G[ra * Vp + rb] = s; G[rb * Vp + ra] = s; }
                }
            }
            __syncthreads();
            // ---- Algorithm 3 on coefficients (wave 0), the stopping test with it
            if (tid < 64) {
                double nfix = 0.0, pginf = 0.0;
                for (int w = 0; w < nw; ++w) { nfix += redA[w]; pginf = fmax(pginf, redA[kResWaves + w]); }
                const double ynew = c > 0 ? sc.ynorm2[(head - 1 + m) % m] : 0.0;
                const double yn_old = prefetch_ynorm2(&sc, c, head, m);
                recursion_on_coefficients(G, Vp, c, head, m, op, &sc, G[(2 * c) * Vp + 2 * c], pginf, nfix, ynew, yn_old,
                                          alpha_s, 0, 1);
            }
            __syncthreads();
            const int st = sc.status;
            const bool recheck = st == LBFGSB_CONVERGED && since > 0 && sc.iters > 0;
            if (recheck) {
                // the stopping quantity came from a gradient carried by recurrence: recompute it from x, test again
                __syncthreads();                    // every thread has read the status
                if (tid == 0) sc.status = LBFGSB_RUNNING;
                want_eval = true;
                continue;
            }
            if (st != LBFGSB_RUNNING) break;
            ++steps;

            // ---- d = -B delta on the free set; both candidate directions of Algorithm 2 and their sums
            if (wact) {
                double de = 0.0;
                if (mi != 0.0) {
                    double q = 0.0;
                    for (int j0 = 0; j0 < V; j0 += 8) {
                        double dv[8], vv[8];
#pragma unroll
                        for (int k = 0; k < 8; ++k) {
                            const bool in = j0 + k < V;
                            dv[k] = in ? sc.delta[j0 + k] : 0.0;
                            vv[k] = in ? vec(j0 + k)[tid] : 0.0;
                        }
#pragma unroll
                        for (int k = 0; k < 8; ++k) q = fma(dv[k], vv[k], q);
                    }
                    de = -q;
                }
                double ub = INFINITY;
                if (act) {
                    pa = clampd(xi + de, li, ui) - xi;
                    pb = de;
                    if (de < 0.0 && xi <= li + op.eps) pb = 0.0;
                    if (de > 0.0 && xi >= ui - op.eps) pb = 0.0;
                    p1s[tid] = pa;
                    p2s[tid] = pb;
                    if (pb > 0.0) ub = (ui - xi) / pb;
                    else if (pb < 0.0) ub = (li - xi) / pb;
                }
                double w6[6] = {pa * gi, pa * pa, xi * pa, pb * gi, pb * pb, xi * pb};
#pragma unroll
                for (int k = 0; k < 6; ++k) w6[k] = wave_sum(w6[k]);
                ub = wave_min(ub);
                if (lane == 0) {
#pragma unroll
                    for (int k = 0; k < 6; ++k) redD[wave * 7 + k] = w6[k];
                    redD[wave * 7 + 6] = ub;
                }
            }
            __syncthreads();                        // (also publishes p1s / p2s)
            {
                double ubt = INFINITY;
                for (int w = 0; w < nw; ++w) {
#pragma unroll
                    for (int k = 0; k < 6; ++k) s6[k] += redD[w * 7 + k];
                    ubt = fmin(ubt, redD[w * 7 + 6]);
                }
                branch = (s6[0] <= -op.eps * s6[1] && s6[1] >= op.eps) ? 1 : 2;
                gp = branch == 1 ? s6[0] : s6[3];
                alpha_ub = branch == 1 ? 1.0 : ubt;
                ps = branch == 1 ? p1s : p2s;
            }
        }

        // ---- the pass: u_r = a_r . v for this group's rows, psi_r = u_r - (evaluation ? b_r : 0), w = A^T psi, sum psi^2
        double tt = 0.0, wi = 0.0;
        {
            double pv[CPL], wl[CPL];
#pragma unroll
            for (int k = 0; k < CPL; ++k) {
                const int col = gj + 16 * k;
                pv[k] = col < n ? ps[col] : 0.0;
                wl[k] = 0.0;
            }
            double ttg = 0.0;
#pragma unroll
            for (int q = 0; q < RG; ++q) {
                double s = 0.0;
#pragma unroll
                for (int k = 0; k < CPL; ++k) s = fma(at[q][k], pv[k], s);
                // the sum over the 16 lanes of the group; every lane of the group gets it
                s += dpp_move<kDppXor1>(s);
                s += dpp_move<kDppXor2>(s);
                s += dpp_move<kDppHalfMirror>(s);
                s += dpp_move<kDppMirror>(s);
                const int r = grp + kResGroups * q;
                double psi = r < rows ? s : 0.0;
                if (want_eval && r < rows) psi -= a.b[r];      // (the targets are read in the rare evaluations only)
                ttg = fma(psi, psi, ttg);
#pragma unroll
                for (int k = 0; k < CPL; ++k) wl[k] = fma(at[q][k], psi, wl[k]);
            }
#pragma unroll
            for (int k = 0; k < CPL; ++k) wred[grp * (CPL * 16) + gj + 16 * k] = wl[k];
            // the four groups of a wave in group order, then the waves in wave order
            const double ttw = ((lane_bcast(ttg, 0) + lane_bcast(ttg, 16)) + lane_bcast(ttg, 32)) + lane_bcast(ttg, 48);
            if (lane == 0) redP[wave] = ttw;
            __syncthreads();
            if (act) {
                // four chains of eight groups each, so that the additions do not wait for one another
                double w4[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
                for (int q = 0; q < kResGroups / 4; ++q) {
#pragma unroll
                    for (int h = 0; h < 4; ++h) w4[h] += wred[(h * (kResGroups / 4) + q) * (CPL * 16) + tid];
                }
                wi = (w4[0] + w4[1]) + (w4[2] + w4[3]);
            }
#pragma unroll
            for (int w = 0; w < kResWaves; ++w) tt += redP[w];
        }
        if (want_eval) {
            gi = wi;
            if (act) gs[tid] = gi;
            if (tid == 0) { sc.f = 0.5 * tt; sc.fevals += 1; sc.since_refresh = 0; }
            since = 0;
            want_eval = false;
            continue;                               // (the next trip's first barrier orders these writes before their readers)
        }

        // ---- closed-form Armijo search (every thread takes the same decisions)
        double alpha = fmin(1.0, alpha_ub);
        int ok = 0, bt = 0;
        for (int k = 0; k <= op.max_backtracks; ++k) {
            const double lhs = gp + 0.5 * alpha * tt;            // (f(x + alpha p) - f(x)) / alpha
            if (isfinite(alpha * lhs) && lhs <= op.c1 * gp) { ok = 1; bt = k; break; }
            alpha *= op.backtrack;
        }
        if (!ok) bt = op.max_backtracks + 1;

        // ---- update: x+, g+ = g + alpha w, the new pair into the ring (LDS and device memory)
        const int slot = head;
        if (wact) {
            double ysq = 0.0;
            if (ok && act) {
                const double y = alpha * wi;
                const double pi = branch == 1 ? pa : pb;
                const double xn = clampd(fma(alpha, pi, xi), li, ui);
                const double sn = xn - xi;
                xi = xn;
                gi += y;
                Ss[slot * np + tid] = sn;
                Ys[slot * np + tid] = y;
                xs[tid] = xi;
                gs[tid] = gi;
                ysq = y * y;
            }
            ysq = wave_sum(ysq);
            if (lane == 0) redU[wave] = ysq;
        }
        __syncthreads();
        if (tid == 0) {
            double yn = 0.0;
            for (int w = 0; w < nw; ++w) yn += redU[w];
            sc.branch = branch; sc.gp = gp; sc.alpha_ub = alpha_ub;
            sc.pp = branch == 1 ? s6[1] : s6[4];
            sc.xp = branch == 1 ? s6[2] : s6[5];
            sc.ls_ok = ok;
            sc.backtracks = bt;
            sc.fevals += bt + (ok ? 1 : 0);
            if (ok) {
                sc.f = sc.f + alpha * (gp + 0.5 * alpha * tt);
                sc.alpha = alpha;
                sc.ynorm2[slot] = yn;
                sc.head = (slot + 1) % m;
                sc.count = c < m ? c + 1 : m;
                sc.iters += 1;
                sc.since_refresh = since + 1;
                record_iteration(&sc);
            } else if (c > 0) {
                sc.count = 0;
                sc.memory_resets += 1;
            } else {
                sc.status = LBFGSB_LINESEARCH_FAILED;
            }
        }
        // the same bookkeeping in every thread's registers; the next trip's first barrier orders thread 0's writes to
        // the scalar block before the recursion reads them
        if (ok) { head = (slot + 1) % m; c = c < m ? c + 1 : m; since += 1; }
        else if (c > 0) c = 0;
    }

    // ---- state the other entry points read: iterate, gradient, pair memory, free mask and the scalar block.  Written
    // once, here: a store to device memory inside the loop is waited for at the next barrier (the barrier orders
    // memory for the workgroup), which costs every iteration a trip to memory for values nobody reads before the
    // launch has ended.
    __syncthreads();
    if (act) { a.x[tid] = xi; a.g[tid] = gi; a.mask[tid] = mi != 0.0 ? 1 : 0; }
    for (int i = tid; i < m * n; i += kResThreads) {
        const int sl = i / n, e = i - sl * n;
        a.S[i] = Ss[sl * np + e];
        a.Y[i] = Ys[sl * np + e];
    }
    for (int k = tid; k < (int)(sizeof(Scal) / 4); k += kResThreads)
        reinterpret_cast<int*>(a.scal)[k] = reinterpret_cast<const int*>(&sc)[k];
    // the host's copy directly (pinned memory is visible to the device): the caller then only waits for the launch,
    // where a copy command behind it costs several microseconds more
    if (a.host_scal) {
        for (int k = tid; k < (int)(sizeof(Scal) / 4); k += kResThreads)
            reinterpret_cast<int*>(a.host_scal)[k] = reinterpret_cast<const int*>(&sc)[k];
    }
}

// The instantiations, smallest register footprint first: (columns per lane, rows per group) holds a matrix of up
// to 32 * RG rows and 16 * CPL columns.  (7, 7) is the one the 200 x 100 benchmark configuration runs on: its 49
// matrix elements per lane leave the rest of the iteration its registers, which (8, 8) does not.
typedef void (*ResKernel)(ResArgs);
struct ResVariant { int cpl, rg; ResKernel kernel; };
const ResVariant kResVariants[] = {
    {8, 4, &k_resident<8, 4>}, {4, 8, &k_resident<4, 8>}, {7, 7, &k_resident<7, 7>},
    {8, 8, &k_resident<8, 8>}, {16, 4, &k_resident<16, 4>},
};
const ResVariant* resident_variant(const Dims& dm) {
    for (const ResVariant& v : kResVariants)
        if (dm.cols <= 16 * v.cpl && dm.rows <= (int64_t)kResGroups * v.rg) return &v;
    return nullptr;
}

}  // namespace

// The resident solver takes plain least squares (no row weights, no extra rows) whose matrix fits the registers of
// one workgroup (up to 256 rows of at most 128 columns, or 128 rows of at most 256) and whose vectors fit its LDS.
bool resident_shape_ok(const Dims& dm, bool has_row_weight) {
    if (dm.kind != LBFGSB_OBJ_LSQ || has_row_weight || dm.n_extra > 0 || dm.n != dm.cols) return false;
    const ResVariant* v = resident_variant(dm);
    return v && (size_t)res_layout((int)dm.n, dm.m, v->cpl * 16).total * 8 <= kResLdsLimit;
}

hipError_t resident_prepare(const Dims& dm) {
    const ResVariant* v = resident_variant(dm);
    const size_t bytes = (size_t)res_layout((int)dm.n, dm.m, v->cpl * 16).total * 8;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(v->kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

void launch_resident(const Dims& dm, const Opts& op, const Buffers& bf, const void* A, const double* b, int max_steps,
                     int refresh_every, hipStream_t st, Scal* host_scal) {
    const ResVariant* v = resident_variant(dm);
    const size_t bytes = (size_t)res_layout((int)dm.n, dm.m, v->cpl * 16).total * 8;
    ResArgs a{dm, op, A, b, bf.scal, bf.x, bf.g, bf.S, bf.Y, bf.l, bf.u, bf.mask, max_steps, refresh_every,
              dm.dtype == LBFGSB_F32 ? 1 : 0, host_scal};
    hipLaunchKernelGGL(v->kernel, dim3(1), dim3(kResThreads), bytes, st, a);
}

}  // namespace lb
