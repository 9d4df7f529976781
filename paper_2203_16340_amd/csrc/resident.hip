// Small least-squares problems: the whole of Algorithm 1 in ONE workgroup that stays on its compute unit for as many
// iterations as the caller asks for.  The multi-kernel path spends four dependent launches of 5-9 us each on an
// iteration of a 200 x 100 problem, i.e. it is bound by launch latency; here an iteration is a handful of
// workgroup barriers.
//
//   * the matrix lives in REGISTERS for the whole launch: wave w of the 8 owns rows w, w + 8, w + 16, ..., lane l of a
//     wave owns columns 2l, 2l + 1 of every 128-column chunk, so a lane holds up to 32 (row, chunk) tiles of two
//     elements, loaded once at the start (fp32 storage is widened there).  One "pass over A" per iteration is then
//     arithmetic and cross-lane sums only: t_r = a_r . p by a butterfly over the wave, and w = A^T t accumulated from
//     the same registers, per wave, summed over the waves in wave order;
//   * x, g, l, u, the pair memory and the Gram matrix live in LDS; the scalar block is an LDS copy of the device one;
//   * every phase is the arithmetic of the corresponding kernel of the multi-kernel path (Eq. (ws), masked Gram matrix,
//     Algorithm 3 on coefficients -- the same device function --, Algorithm 2 with both candidate directions, the
//     closed-form Armijo search of the quadratic objectives, update and pair storage), with its own fixed summation
//     orders; iterate, gradient and new pair are also written through to device memory every iteration, the scalar
//     block and the free mask when the launch ends, so the other entry points find the state they expect.
// The gradient is carried by recurrence as on the multi-kernel path; it is recomputed from x every refresh_every
// iterations and before convergence is declared.
#include "common.h"
#include "recursion.h"

namespace lb {

namespace {

constexpr int kResThreads = 512;                // 8 waves, two per SIMD: 256 registers per lane, half of them hold the matrix
constexpr int kResWaves = kResThreads / 64;
constexpr int kResTiles = 32;                   // (row, chunk) tiles of two elements a lane holds, at most
constexpr int kResBatch = 8;                    // rows whose cross-lane sums are in flight together
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
};

// LDS layout in doubles
struct ResLayout {
    int x, g, l, u, p1, p2, msk, w, S, Y, G, wred, red, alpha, total;
};
__host__ __device__ inline ResLayout res_layout(int n, int m, int cpad) {
    ResLayout L;
    int off = 0;
    auto take = [&](int k) { int o = off; off += (k + 1) & ~1; return o; };
    L.x = take(n); L.g = take(n); L.l = take(n); L.u = take(n); L.p1 = take(n); L.p2 = take(n); L.msk = take(n); L.w = take(n);
    L.S = take(m * n); L.Y = take(m * n);
    L.G = take((2 * m + 2) * (2 * m + 2));
    L.wred = take(kResWaves * cpad);
    L.red = take(96);               // per-phase exchange areas of the waves' partial results
    L.alpha = take(kMaxM + 1);
    L.total = off;
    return L;
}

// CH: 128-column chunks of a row; NT: tiles a lane holds (instantiated for a few sizes so that the matrix of a
// problem smaller than the largest one leaves registers for everything else).
//
// What bounds an iteration here is the latency of dependent steps (an LDS access or a shuffle is ~130 cycles when
// the next instruction waits for it), so: thread i owns element i of every n-vector (n <= 512 = threads) and keeps
// x_i, g_i, l_i, u_i in registers; sums over a wave use the lane permutations of wave_sum_dpp; LDS loads that feed a
// chain are issued in groups before they are used; reductions over the workgroup that can share a barrier do.
template <int CH, int NT>
__global__ __launch_bounds__(kResThreads) void k_resident(ResArgs a) {
    extern __shared__ __align__(16) double lds[];
    __shared__ Scal sc;
    constexpr int RW = NT / CH;                 // rows a wave can own
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = (int)a.dm.cols, rows = (int)a.dm.rows, m = a.dm.m;
    const int64_t ld = a.dm.ld;
    const ResLayout L = res_layout(n, m, CH * 128);
    double *gs = lds + L.g, *p1s = lds + L.p1, *p2s = lds + L.p2, *xs = lds + L.x;
    double *msk = lds + L.msk, *Ss = lds + L.S, *Ys = lds + L.Y, *G = lds + L.G, *wred = lds + L.wred;
    double *red = lds + L.red, *alpha_s = lds + L.alpha;
    double *redA = red, *redD = red + 16, *redP = red + 16 + 56, *redU = red + 16 + 56 + 8;   // one region per phase
    const Opts op = a.op;
    const bool act = tid < n;                   // this thread owns element `tid`

    // ---- the scalar block; nothing to do when the solver has stopped
    for (int k = tid; k < (int)(sizeof(Scal) / 4); k += kResThreads)
        reinterpret_cast<int*>(&sc)[k] = reinterpret_cast<const int*>(a.scal)[k];
    __syncthreads();
    if (sc.status != LBFGSB_RUNNING) return;
    if (tid == 0 && sc.pend_valid) apply_pending(&sc, m);   // (left by a step of the multi-kernel path; normally none)

    // ---- the matrix into registers, the vectors into LDS and registers
    double at[NT][2];
#pragma unroll
    for (int k = 0; k < NT; ++k) {
        const int r = wave + kResWaves * (k / CH), c0 = (k % CH) * 128 + 2 * lane;
        const int64_t o = (int64_t)r * ld + c0;
        const bool in0 = r < rows && c0 < n, in1 = r < rows && c0 + 1 < n;
        if (a.f32) {
            const float* A = reinterpret_cast<const float*>(a.A);
            at[k][0] = in0 ? (double)A[o] : 0.0;
            at[k][1] = in1 ? (double)A[o + 1] : 0.0;
        } else {
            const double* A = reinterpret_cast<const double*>(a.A);
            at[k][0] = in0 ? A[o] : 0.0;
            at[k][1] = in1 ? A[o + 1] : 0.0;
        }
    }
    double xi = 0.0, gi = 0.0, li = 0.0, ui = 0.0, mi = 0.0;
    if (act) { xi = a.x[tid]; gi = a.g[tid]; li = a.l[tid]; ui = a.u[tid]; mi = a.mask[tid] ? 1.0 : 0.0; xs[tid] = xi; gs[tid] = gi; }
    for (int i = tid; i < m * n; i += kResThreads) { Ss[i] = a.S[i]; Ys[i] = a.Y[i]; }
    __syncthreads();

#ifdef LBFGSB_RESIDENT_PROFILE
    unsigned long long pt[8] = {0, 0, 0, 0, 0, 0, 0, 0}, pt0 = 0;
#define RES_MARK(k) do { if (tid == 0) { const unsigned long long now_ = wall_clock64(); pt[k] += now_ - pt0; pt0 = now_; } } while (0)
    if (tid == 0) pt0 = wall_clock64();
#else
#define RES_MARK(k) do { } while (0)
#endif

    // Every trip of the loop makes ONE product pass: either an evaluation from scratch (r = A x - b, f = 0.5 ||r||^2,
    // g = A^T r: the periodic recomputation, and the one before convergence is declared), or the pass of an iteration.
    int steps = 0;
    bool want_eval = false;
    for (;;) {
        if (!want_eval && steps >= a.max_steps) break;
        if (!want_eval && a.refresh_every > 0 && sc.since_refresh >= a.refresh_every) want_eval = true;

        const int c = sc.count, head = sc.head;
        const int V = 2 * c + 1, Vp = V + 1;
        const int base_slot = c > 0 ? (head - c + 2 * m) % m : 0;
        auto vec = [&](int j) __attribute__((always_inline)) -> const double* {
            if (j >= 2 * c) return gs;
            const bool is_y = j >= c;
            int sl = base_slot + (is_y ? j - c : j);
            if (sl >= m) sl -= m;
            return (is_y ? Ys : Ss) + sl * n;
        };
        double s6[6] = {0, 0, 0, 0, 0, 0};
        double gp = 0.0, alpha_ub = 1.0, pa = 0.0, pb = 0.0;
        int branch = 1;
        const double* ps = xs;

        if (!want_eval) {
            // ---- Eq. (ws): free set; the epsilon-free KKT residual and the number of fixed variables
            {
                const bool fr = !(((xi <= li + op.eps) && (gi >= 0.0)) || ((xi >= ui - op.eps) && (gi <= 0.0)));
                mi = (act && fr) ? 1.0 : 0.0;
                if (act) msk[tid] = mi;
                const double nf = wave_sum_dpp((act && !fr) ? 1.0 : 0.0);
                const double pg = wave_max_dpp(act ? fabs(xi - clampd(xi - gi, li, ui)) : 0.0);
                if (lane == 0) { redA[wave] = nf; redA[kResWaves + wave] = pg; }
            }
            __syncthreads();                        // msk and the waves' partial statistics are in LDS
            RES_MARK(0);

            // ---- masked Gram matrix of [s^0 .. s^{c-1}, y^0 .. y^{c-1}, g]: four lanes per entry, each taking every
            // fourth element; the loads of four elements are issued before their products
            {
                const int E = V * (V + 1) / 2;
                const int grp = tid >> 2, sub = tid & 3;
                for (int e0 = 0; e0 < E; e0 += kResThreads / 4) {
                    const int e = e0 + grp;
                    int ra = 0, rb = 0;
                    double s = 0.0;
                    if (e < E) {
                        int q = e;
                        while (q >= V - ra) { q -= V - ra; ++ra; }
                        rb = ra + q;
                        const double *va = vec(ra), *vb = vec(rb);
                        for (int i0 = sub; i0 < n; i0 += 16) {
                            double mv[4], av[4], bv[4];
#pragma unroll
                            for (int k = 0; k < 4; ++k) {
                                const int i = i0 + 4 * k;
                                const bool in = i < n;
                                mv[k] = in ? msk[i] : 0.0;
                                av[k] = in ? va[i] : 0.0;
                                bv[k] = in ? vb[i] : 0.0;
                            }
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
            RES_MARK(1);
            // ---- Algorithm 3 on coefficients (wave 0), the stopping test with it
            if (tid < 64) {
                double nfix = 0.0, pginf = 0.0;
#pragma unroll
                for (int w = 0; w < kResWaves; ++w) { nfix += redA[w]; pginf = fmax(pginf, redA[kResWaves + w]); }
                const double ynew = c > 0 ? sc.ynorm2[(head - 1 + m) % m] : 0.0;
                const double yn_old = prefetch_ynorm2(&sc, c, head, m);
                recursion_on_coefficients(G, Vp, c, head, m, op, &sc, G[(2 * c) * Vp + 2 * c], pginf, nfix, ynew, yn_old,
                                          alpha_s, 0, 1);
            }
            __syncthreads();
            RES_MARK(2);
            const int st = sc.status;
            const bool recheck = st == LBFGSB_CONVERGED && sc.since_refresh > 0 && sc.iters > 0;
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
            {
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
                for (int k = 0; k < 6; ++k) w6[k] = wave_sum_dpp(w6[k]);
                ub = wave_min_dpp(ub);
                if (lane == 0) {
#pragma unroll
                    for (int k = 0; k < 6; ++k) redD[wave * 7 + k] = w6[k];
                    redD[wave * 7 + 6] = ub;
                }
                __syncthreads();                    // (also publishes p1s / p2s)
                double ubt = INFINITY;
#pragma unroll
                for (int w = 0; w < kResWaves; ++w) {
#pragma unroll
                    for (int k = 0; k < 6; ++k) s6[k] += redD[w * 7 + k];
                    ubt = fmin(ubt, redD[w * 7 + 6]);
                }
                branch = (s6[0] <= -op.eps * s6[1] && s6[1] >= op.eps) ? 1 : 2;
                gp = branch == 1 ? s6[0] : s6[3];
                alpha_ub = branch == 1 ? 1.0 : ubt;
                ps = branch == 1 ? p1s : p2s;
            }
            RES_MARK(3);
        }

        // ---- the pass: u_r = a_r . v for this wave's rows, psi_r = u_r - (evaluation ? b_r : 0), w = A^T psi, sum psi^2
        double tt = 0.0, wi = 0.0;
        {
            double pv[CH][2];
#pragma unroll
            for (int ch = 0; ch < CH; ++ch) {
                const int c0 = ch * 128 + 2 * lane;
                pv[ch][0] = c0 < n ? ps[c0] : 0.0;
                pv[ch][1] = c0 + 1 < n ? ps[c0 + 1] : 0.0;
            }
            double wl[CH][2];
#pragma unroll
            for (int ch = 0; ch < CH; ++ch) wl[ch][0] = wl[ch][1] = 0.0;
            double ttw = 0.0;
#pragma unroll
            for (int q = 0; q < RW; ++q) {
                double s = 0.0;
#pragma unroll
                for (int ch = 0; ch < CH; ++ch) {
                    s = fma(at[q * CH + ch][0], pv[ch][0], s);
                    s = fma(at[q * CH + ch][1], pv[ch][1], s);
                }
                s = wave_sum_dpp(s);
                const int r = wave + kResWaves * q;
                double psi = r < rows ? s : 0.0;
                if (want_eval && r < rows) psi -= a.b[r];      // (the targets are read in the rare evaluations only)
                ttw = fma(psi, psi, ttw);
#pragma unroll
                for (int ch = 0; ch < CH; ++ch) {
                    wl[ch][0] = fma(at[q * CH + ch][0], psi, wl[ch][0]);
                    wl[ch][1] = fma(at[q * CH + ch][1], psi, wl[ch][1]);
                }
            }
#pragma unroll
            for (int ch = 0; ch < CH; ++ch) {
                wred[wave * (CH * 128) + ch * 128 + 2 * lane] = wl[ch][0];
                wred[wave * (CH * 128) + ch * 128 + 2 * lane + 1] = wl[ch][1];
            }
            if (lane == 0) redP[wave] = ttw;
            __syncthreads();
#pragma unroll
            for (int w = 0; w < kResWaves; ++w) {
                wi += act ? wred[w * (CH * 128) + tid] : 0.0;
                tt += redP[w];
            }
        }
        RES_MARK(4);
        if (want_eval) {
            gi = wi;
            if (act) { gs[tid] = gi; a.g[tid] = gi; }
            if (tid == 0) { sc.f = 0.5 * tt; sc.fevals += 1; sc.since_refresh = 0; }
            __syncthreads();
            want_eval = false;
            continue;
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
        double ysq = 0.0;
        if (ok && act) {
            const double y = alpha * wi;
            const double pi = branch == 1 ? pa : pb;
            const double xn = clampd(fma(alpha, pi, xi), li, ui);
            const double sn = xn - xi;
            xi = xn;
            gi += y;
            Ss[slot * n + tid] = sn;
            Ys[slot * n + tid] = y;
            xs[tid] = xi;
            gs[tid] = gi;
            a.S[(int64_t)slot * n + tid] = sn;
            a.Y[(int64_t)slot * n + tid] = y;
            a.x[tid] = xi;
            a.g[tid] = gi;
            ysq = y * y;
        }
        ysq = wave_sum_dpp(ysq);
        if (lane == 0) redU[wave] = ysq;
        __syncthreads();
        if (tid == 0) {
            double yn = 0.0;
#pragma unroll
            for (int w = 0; w < kResWaves; ++w) yn += redU[w];
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
                sc.since_refresh += 1;
            } else if (c > 0) {
                sc.count = 0;
                sc.memory_resets += 1;
            } else {
                sc.status = LBFGSB_LINESEARCH_FAILED;
            }
        }
        __syncthreads();
        RES_MARK(5);
    }
#ifdef LBFGSB_RESIDENT_PROFILE
    if (tid == 0 && steps > 8)
        printf("resident: %d steps; per step (10 ns ticks): mask %llu gram %llu recursion %llu direction %llu pass %llu update %llu\n",
               steps, pt[0] / steps, pt[1] / steps, pt[2] / steps, pt[3] / steps, pt[4] / steps, pt[5] / steps);
#endif

    // ---- state the other entry points read: the scalar block and the free mask
    __syncthreads();
    if (act) a.mask[tid] = mi != 0.0 ? 1 : 0;
    for (int k = tid; k < (int)(sizeof(Scal) / 4); k += kResThreads)
        reinterpret_cast<int*>(a.scal)[k] = reinterpret_cast<const int*>(&sc)[k];
}

int resident_chunks(const Dims& dm) { return dm.cols <= 128 ? 1 : 4; }

// tiles per lane of the instantiation that holds this problem (0: none does)
int resident_tiles(const Dims& dm) {
    const int ch = resident_chunks(dm);
    const int64_t need = (dm.rows + kResWaves - 1) / kResWaves * ch;
    if (ch == 1) return need <= 8 ? 8 : (need <= 16 ? 16 : (need <= 26 ? 26 : (need <= 32 ? 32 : 0)));
    return need <= 16 ? 16 : (need <= 32 ? 32 : 0);
}

typedef void (*ResKernel)(ResArgs);
ResKernel resident_kernel(const Dims& dm) {
    const int nt = resident_tiles(dm);
    if (resident_chunks(dm) == 1) {
        switch (nt) {
            case 8: return &k_resident<1, 8>;
            case 16: return &k_resident<1, 16>;
            case 26: return &k_resident<1, 26>;
            default: return &k_resident<1, 32>;
        }
    }
    return nt == 16 ? &k_resident<4, 16> : &k_resident<4, 32>;
}

}  // namespace

// The resident solver takes plain least squares (no row weights, no extra rows) whose matrix fits the register tiles
// of one workgroup and whose vectors fit its LDS.
bool resident_shape_ok(const Dims& dm, bool has_row_weight) {
    if (dm.kind != LBFGSB_OBJ_LSQ || has_row_weight || dm.n_extra > 0) return false;
    if (dm.cols > 512 || dm.n != dm.cols) return false;
    if (resident_tiles(dm) == 0) return false;
    return (size_t)res_layout((int)dm.n, dm.m, resident_chunks(dm) * 128).total * 8 <= kResLdsLimit;
}

hipError_t resident_prepare(const Dims& dm) {
    const size_t bytes = (size_t)res_layout((int)dm.n, dm.m, resident_chunks(dm) * 128).total * 8;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(resident_kernel(dm)), hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)bytes);
}

void launch_resident(const Dims& dm, const Opts& op, const Buffers& bf, const void* A, const double* b, int max_steps,
                     int refresh_every, hipStream_t st) {
    const size_t bytes = (size_t)res_layout((int)dm.n, dm.m, resident_chunks(dm) * 128).total * 8;
    ResArgs a{dm, op, A, b, bf.scal, bf.x, bf.g, bf.S, bf.Y, bf.l, bf.u, bf.mask, max_steps, refresh_every,
              dm.dtype == LBFGSB_F32 ? 1 : 0};
    hipLaunchKernelGGL(resident_kernel(dm), dim3(1), dim3(kResThreads), bytes, st, a);
}

}  // namespace lb
