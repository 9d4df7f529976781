// Regularised optimal-transport objective of the paper's section "Joint Probability Distribution":
//     f(P) = <M,P> + lambda sum_ij phi(P_ij) + 0.5 sum_k omega_k ((K P)_k - beta_k)^2,
// P a rows x cols matrix stored row by row (the solver's variable vector), phi(p) = p^2/2 (Gaussian
// regulariser) or p log p (entropy), K P = [P 1; P^T 1] the rows + cols marginals.  The last term is how the
// augmented Lagrangian of Eq. (augLag) enters for the constraints P 1 = u, P^T 1 = v: omega = rho and
// beta = [u; v] - multipliers/rho, rewritten by Algorithm 4 between inner solves.
//
// There is no matrix-vector product here: every kernel streams n = rows*cols-entry vectors once.
//   k_ot_sums + k_ot_cols   K z for z = x (evaluation) or the selected direction p, the loss partials
//   k_ot_eval_finish        gradient M + lambda phi'(P) + K^T (omega . residual), objective value
//   k_ot_update_gauss       closed-form Armijo search (the objective is quadratic along p) and the update
//   k_ot_ls_entropy / k_ot_update_entropy   the same for the entropy, whose line search
//                           needs one pass over (x, p) per batch of trial steps
#include "common.h"

namespace lb {

namespace {

__device__ __forceinline__ double m_at(const void* M, int dtype, int64_t idx) {
    return dtype == LBFGSB_F32 ? (double)((const float*)M)[idx] : ((const double*)M)[idx];
}

// lambda * phi(p) and lambda * phi'(p)
__device__ __forceinline__ double reg_value(int kind, double lambda, double p) {
    if (kind == LBFGSB_OBJ_OT_GAUSS) return 0.5 * lambda * p * p;
    return p > 0.0 ? lambda * p * log(p) : 0.0;
}
__device__ __forceinline__ double reg_slope(int kind, double lambda, double p) {
    if (kind == LBFGSB_OBJ_OT_GAUSS) return lambda * p;
    return lambda * (log(p) + 1.0);
}

// K z, first half: the sums of the RPW rows this workgroup owns, and its partial column sums.
template <int RPW>
__global__ __launch_bounds__(kBlock) void k_ot_sums(Dims dm, OtArgs a, int eval, int check_status,
                                                    const double* __restrict__ x, const double* __restrict__ p1,
                                                    const double* __restrict__ p2, Scal* __restrict__ scal,
                                                    double* __restrict__ out, double* __restrict__ wpart,
                                                    double* __restrict__ losspart, const double* __restrict__ dir_part,
                                                    int dir_blocks, double eps) {
    __shared__ double red[kWaves * (RPW + 1 > 7 ? RPW + 1 : 7)];
    const int tid = threadIdx.x;
    const int status = check_status ? scal->status : LBFGSB_RUNNING;
    const double* z = x;
    if (!eval && dir_blocks > 0) {
        // Algorithm 2's choice from the direction kernel's per-workgroup sums (requested together with the status
        // word); workgroup 0 records it for the kernels that follow
        const DirChoice ch = dir_choice_block(dir_part, dir_blocks, eps, red);
        if (status != LBFGSB_RUNNING) return;
        if (blockIdx.x == 0 && tid == 0) {
            scal->branch = ch.branch; scal->gp = ch.gp; scal->alpha_ub = ch.alpha_ub; scal->pp = ch.pp; scal->xp = ch.xp;
        }
        z = ch.branch == 1 ? p1 : p2;
    } else {
        if (status != LBFGSB_RUNNING) return;
        if (!eval) z = scal->branch == 1 ? p1 : p2;
    }
    const int64_t r0 = (int64_t)blockIdx.x * RPW;
    const int nr = dm.rows - r0 < RPW ? (int)(dm.rows - r0) : RPW;
    double acc[RPW + 1];   // row sums, then the objective terms of these entries
#pragma unroll
    for (int r = 0; r <= RPW; ++r) acc[r] = 0.0;
    // several column tiles per round, all their loads issued before the first is used: the loop over the tiles is
    // otherwise a chain of dependent trips to memory, and this kernel is nothing else
    constexpr int JT = RPW <= 4 ? 4 : 2;
    for (int64_t j0 = 0; j0 < dm.cols; j0 += JT * kBlock) {
        double zv[JT][RPW];
#pragma unroll
        for (int t = 0; t < JT; ++t) {
            const int64_t j = j0 + t * kBlock + tid;
#pragma unroll
            for (int r = 0; r < RPW; ++r) zv[t][r] = (j < dm.cols && r < nr) ? z[(r0 + r) * dm.cols + j] : 0.0;
        }
#pragma unroll
        for (int t = 0; t < JT; ++t) {
            const int64_t j = j0 + t * kBlock + tid;
            const bool in = j < dm.cols;
            double cs = 0.0;
#pragma unroll
            for (int r = 0; r < RPW; ++r) { cs += zv[t][r]; acc[r] += zv[t][r]; }
            if (eval) {
#pragma unroll
                for (int r = 0; r < RPW; ++r) {
                    if (in && r < nr) {
                        acc[RPW] = fma(m_at(a.M, dm.dtype, (r0 + r) * dm.ld + j), zv[t][r], acc[RPW]);
                        acc[RPW] += reg_value(dm.kind, dm.lambda, zv[t][r]);
                    }
                }
            }
            if (in) wpart[(int64_t)blockIdx.x * dm.cols + j] = cs;
        }
    }
    block_sum<RPW + 1, kWaves>(acc, red);
    if (tid == 0) {
        double loss = eval ? acc[RPW] : 0.0;
#pragma unroll
        for (int r = 0; r < RPW; ++r) {
            if (r < nr) {
                // beta is only there together with omega (no marginal terms: the plain sums are left in `out`)
                const double res = (eval && a.omega) ? acc[r] - a.beta[r0 + r] : acc[r];
                out[r0 + r] = res;
                if (a.omega) loss += (eval ? 0.5 : 1.0) * a.omega[r0 + r] * res * res;
            }
        }
        losspart[blockIdx.x] = loss;
    }
}

// K z, second half: the column sums from the workgroups' partials.
__global__ __launch_bounds__(kBlock) void k_ot_cols(Dims dm, OtArgs a, int eval, int check_status, int parts,
                                                    const double* __restrict__ wpart, const Scal* __restrict__ scal,
                                                    double* __restrict__ out, double* __restrict__ losspart) {
    __shared__ double lds[kBlock];
    __shared__ double red[kWaves];
    if (check_status && scal->status != LBFGSB_RUNNING) return;
    const int tid = threadIdx.x;
    double loss[1] = {0.0};
    for (int64_t c0 = (int64_t)blockIdx.x * kCX; c0 < dm.cols; c0 += (int64_t)gridDim.x * kCX) {
        const int64_t c = c0 + tid % kCX;
        const double s = column_sum(wpart, parts, dm.cols, c, lds);
        if (tid < kCX && c < dm.cols) {
            const double res = (eval && a.omega) ? s - a.beta[dm.rows + c] : s;
            out[dm.rows + c] = res;
            if (a.omega) loss[0] += (eval ? 0.5 : 1.0) * a.omega[dm.rows + c] * res * res;
        }
    }
    block_sum<1, kWaves>(loss, red);
    if (tid == 0) losspart[blockIdx.x] = loss[0];
}

// g = M + lambda phi'(x) + K^T (omega . residual); the last workgroup adds up f.
__global__ __launch_bounds__(kBlock) void k_ot_eval_finish(Dims dm, OtArgs a, int loss_parts,
                                                           const double* __restrict__ x, const double* __restrict__ res,
                                                           const double* __restrict__ losspart, double* __restrict__ g,
                                                           Scal* __restrict__ scal) {
    __shared__ double red[kWaves];
    __shared__ int flag;
    if (scal->status != LBFGSB_RUNNING) return;
    const int tid = threadIdx.x;
    for (int64_t i = blockIdx.x; i < dm.rows; i += gridDim.x) {
        const double ri = a.omega ? a.omega[i] * res[i] : 0.0;
        for (int64_t j = tid; j < dm.cols; j += kBlock) {
            const int64_t e = i * dm.cols + j;
            const double cj = a.omega ? a.omega[dm.rows + j] * res[dm.rows + j] : 0.0;
            g[e] = m_at(a.M, dm.dtype, i * dm.ld + j) + reg_slope(dm.kind, dm.lambda, x[e]) + (ri + cj);
        }
    }
    if (!arrive_is_last(&scal->counters[kCntEvalFinish], &flag)) return;
    const double f = sum_all(losspart, loss_parts, red);
    if (tid == 0) {
        scal->f = f;
        scal->fevals += 1;
    }
}

constexpr int kOtTiles = 4;   // column tiles of a row whose loads the Gaussian update kernel keeps in flight together

// Gaussian regulariser: along p the objective is the quadratic  a <g,p> + a^2/2 (lambda <p,p> + sum omega (K p)^2),
// so the Armijo search is the closed form of the least-squares kinds; the change of the gradient is
// y = a (lambda p + K^T (omega . K p)).
__global__ __launch_bounds__(kBlock) void k_ot_update_gauss(Dims dm, Opts op, OtArgs a, int loss_parts,
                                                            const double* __restrict__ losspart,
                                                            const double* __restrict__ t, const double* __restrict__ p1,
                                                            const double* __restrict__ p2, const double* __restrict__ l,
                                                            const double* __restrict__ u, double* __restrict__ x,
                                                            double* __restrict__ g, double* __restrict__ S,
                                                            double* __restrict__ Y, Scal* __restrict__ scal) {
    __shared__ double red[kWaves];
    __shared__ double ls_alpha;
    __shared__ int ls_ok, ls_bt;
    if (scal->status != LBFGSB_RUNNING) return;
    const int tid = threadIdx.x;
    const double gp = scal->gp, alpha_ub = scal->alpha_ub, f_old = scal->f;
    const int slot = scal->head;
    const double* p = scal->branch == 1 ? p1 : p2;
    const double tt = sum_all(losspart, loss_parts, red) + dm.lambda * scal->pp;
    if (tid == 0) {
        double al = fmin(1.0, alpha_ub);
        int ok = 0, bt = 0;
        for (int k = 0; k <= op.max_backtracks; ++k) {
            const double lhs = gp + 0.5 * al * tt;          // (f(x + a p) - f(x)) / a
            if (isfinite(al * lhs) && lhs <= op.c1 * gp) { ok = 1; bt = k; break; }
            al *= op.backtrack;
        }
        ls_alpha = al; ls_ok = ok; ls_bt = ok ? bt : op.max_backtracks + 1;
    }
    __syncthreads();
    const double alpha = ls_alpha;
    const int ok = ls_ok;
    if (ok) {
        double* Sn = S + (int64_t)slot * dm.n;
        double* Yn = Y + (int64_t)slot * dm.n;
        // kOtTiles column tiles of a row per round, all their loads issued before the first is used (one tile at a
        // time the row is a chain of dependent trips to memory)
        for (int64_t i = blockIdx.x; i < dm.rows; i += gridDim.x) {
            const double ri = a.omega ? a.omega[i] * t[i] : 0.0;
            for (int64_t j0 = 0; j0 < dm.cols; j0 += kOtTiles * kBlock) {
                double pv[kOtTiles], xv[kOtTiles], gv[kOtTiles], cv[kOtTiles], lv[kOtTiles], uv[kOtTiles];
#pragma unroll
                for (int k = 0; k < kOtTiles; ++k) {
                    const int64_t j = j0 + k * kBlock + tid;
                    const bool in = j < dm.cols;
                    const int64_t e = i * dm.cols + (in ? j : 0);
                    pv[k] = p[e]; xv[k] = x[e]; gv[k] = g[e];
                    cv[k] = (a.omega && in) ? a.omega[dm.rows + j] * t[dm.rows + j] : 0.0;
                    lv[k] = op.uniform_bounds ? op.lo : l[e];
                    uv[k] = op.uniform_bounds ? op.hi : u[e];
                }
#pragma unroll
                for (int k = 0; k < kOtTiles; ++k) {
                    const int64_t j = j0 + k * kBlock + tid;
                    if (j < dm.cols) {
                        const int64_t e = i * dm.cols + j;
                        const double y = alpha * fma(dm.lambda, pv[k], ri + cv[k]);
                        const double xn = clampd(fma(alpha, pv[k], xv[k]), lv[k], uv[k]);
                        Sn[e] = xn - xv[k];
                        Yn[e] = y;
                        x[e] = xn;
                        g[e] = gv[k] + y;
                    }
                }
            }
        }
    }
    // as in the least-squares update: no workgroup of this kernel reads the pend_* fields
    if (blockIdx.x == 0 && tid == 0) {
        scal->pend_ok = ok;
        scal->pend_bt = ls_bt;
        scal->pend_alpha = alpha;
        scal->pend_f = f_old + alpha * (gp + 0.5 * alpha * tt);
        scal->pend_valid = 1;
    }
}

// Entropy: f(x + a p) - f(x) = a <g,p> + a^2/2 sum omega (K p)^2 + lambda sum_ij D(x_ij + a p_ij ; x_ij) with the
// Bregman divergence of p log p,  D(xt; x) = xt log(xt/x) - (xt - x) = x h(r),  r = (xt - x)/x,
// h(r) = (1 + r) log(1 + r) - r  (series for small r, where the closed form cancels).
__device__ __forceinline__ double entropy_h(double r) {
    if (r <= -1.0) return 1.0;                       // xt = 0: 0 log 0 = 0
    if (fabs(r) < 1e-2) {
        const double r2 = r * r;
        return r2 * (0.5 + r * (-1.0 / 6.0 + r * (1.0 / 12.0 + r * (-1.0 / 20.0 + r * (1.0 / 30.0 + r * (-1.0 / 42.0))))));
    }
    return (1.0 + r) * log1p(r) - r;
}

// NTRY step lengths a0 backtrack^first, ... per sweep over (x, p).  The first launch tries two; two further
// launches, which return at once when an earlier one found the step (such a launch still costs ~4.5 us: the scalar
// block was just written, so its status word comes from memory), try the next kLsBatch and then kLsTail (a long run
// of rejected steps happens at a start on the lower bound, where p/x is huge).  Together they cover the default
// limit of 60 backtracks; only beyond those does the last workgroup of the last launch go on alone, one length at
// a time.
constexpr int kLsTail = 51;   // 2 + kLsBatch + kLsTail = 61 step lengths

// Armijo test of NTRY step lengths a_first, a_first * backtrack, ... (indices first, first + 1, ...) given their sums
// tot[k] = sum_e x_e h(a_k p_e / x_e): the first acceptable one, or found = -1.
template <int NTRY>
__device__ __forceinline__ void entropy_decide(const double (&tot)[NTRY], int first, double a_first, double gp, double tt,
                                               double lambda, const Opts& op, int& found, double& a_acc, double& a_last) {
    found = -1;
    a_acc = 0.0;
    double av = a_first;
#pragma unroll
    for (int k = 0; k < NTRY; ++k) {
        const double df = av * (gp + 0.5 * av * tt) + lambda * tot[k];
        if (found < 0 && first + k <= op.max_backtracks && isfinite(df) && df <= op.c1 * av * gp) { found = first + k; a_acc = av; }
        if (k + 1 < NTRY) av *= op.backtrack;
    }
    a_last = av;
}

// NPREV > 0: the launch before this one (NPREV step lengths from index first - NPREV on) ended without deciding;
// every workgroup of this launch adds that launch's partial sums (prev) and takes its decision, and only if none of
// those step lengths was acceptable goes on with its own.  NPREV == 0 with defer != 0: this launch leaves its decision
// to the next one (no closing arrival).
template <int NTRY, int NPREV>
__global__ __launch_bounds__(kBlock) void k_ot_ls_entropy(Dims dm, Opts op, int loss_parts, int first, int last_resort,
                                                          int defer, const double* __restrict__ losspart,
                                                          const double* __restrict__ x, const double* __restrict__ p1,
                                                          const double* __restrict__ p2, Scal* __restrict__ scal,
                                                          const double* __restrict__ prev, double* __restrict__ lspart) {
    __shared__ double red[kWaves * (NTRY > NPREV ? NTRY : NPREV)];
    __shared__ int flag;
    if (scal->status != LBFGSB_RUNNING) return;
    if (NPREV == 0 && first > 0 && scal->ls_ok) return;   // an earlier launch of this iteration found the step
    const int tid = threadIdx.x;
    const double* p = scal->branch == 1 ? p1 : p2;
    const double a0 = fmin(1.0, scal->alpha_ub);     // step lengths by repeated multiplication, the same everywhere
    if constexpr (NPREV > 0) {
        const double gp = scal->gp;
        double tp[NPREV];
#pragma unroll
        for (int k = 0; k < NPREV; ++k) tp[k] = 0.0;
        for (int b = tid; b < (int)gridDim.x; b += kBlock) {
#pragma unroll
            for (int k = 0; k < NPREV; ++k) tp[k] += prev[(int64_t)b * NPREV + k];
        }
        const double tt = sum_all(losspart, loss_parts, red);
        block_sum<NPREV, kWaves>(tp, red);
        double a_prev = a0;
        for (int k = 0; k < first - NPREV; ++k) a_prev *= op.backtrack;
        int found;
        double a_acc, a_last;
        entropy_decide<NPREV>(tp, first - NPREV, a_prev, gp, tt, dm.lambda, op, found, a_acc, a_last);
        if (found >= 0) {
            if (blockIdx.x == 0 && tid == 0) {
                scal->ls_ok = 1;
                scal->backtracks = found;
                scal->fevals += found + 1;
                scal->alpha = a_acc;
            }
            return;
        }
        __syncthreads();   // (red is used again below)
    }
    double s[NTRY];
    double a_first = a0;
    for (int k = 0; k < first; ++k) a_first *= op.backtrack;
#pragma unroll
    for (int k = 0; k < NTRY; ++k) s[k] = 0.0;
    for (int64_t e = (int64_t)blockIdx.x * kBlock + tid; e < dm.n; e += (int64_t)gridDim.x * kBlock) {
        const double xe = x[e], ratio = p[e] / xe;
        double a = a_first;
#pragma unroll
        for (int k = 0; k < NTRY; ++k) {
            s[k] = fma(xe, entropy_h(a * ratio), s[k]);
            a *= op.backtrack;
        }
    }
    block_sum<NTRY, kWaves>(s, red);
    if (tid == 0) {
#pragma unroll
        for (int k = 0; k < NTRY; ++k) lspart[(int64_t)blockIdx.x * NTRY + k] = s[k];
    }
    if (NPREV == 0 && defer) return;
    if (!arrive_is_last(&scal->counters[kCntLs], &flag)) return;
    const double gp = scal->gp;
    const double tt = sum_all(losspart, loss_parts, red);
    double tot[NTRY];
#pragma unroll
    for (int k = 0; k < NTRY; ++k) tot[k] = 0.0;
    for (int b = tid; b < (int)gridDim.x; b += kBlock) {
#pragma unroll
        for (int k = 0; k < NTRY; ++k) tot[k] += lspart[(int64_t)b * NTRY + k];
    }
    block_sum<NTRY, kWaves>(tot, red);
    int found;
    double a_acc, av;
    entropy_decide<NTRY>(tot, first, a_first, gp, tt, dm.lambda, op, found, a_acc, av);
    // rare: continue one step length at a time (every thread holds the same totals: uniform control flow)
    for (int k = first + NTRY; last_resort && found < 0 && k <= op.max_backtracks; ++k) {
        av *= op.backtrack;
        double sv[1] = {0.0};
        for (int64_t e = tid; e < dm.n; e += kBlock) {
            const double xe = x[e];
            sv[0] = fma(xe, entropy_h(av * p[e] / xe), sv[0]);
        }
        block_sum<1, kWaves>(sv, red);
        const double df = av * (gp + 0.5 * av * tt) + dm.lambda * sv[0];
        if (isfinite(df) && df <= op.c1 * av * gp) { found = k; a_acc = av; }
    }
    if (tid == 0) {
        scal->ls_ok = found >= 0;
        if (found >= 0 || last_resort) {
            scal->backtracks = found >= 0 ? found : op.max_backtracks + 1;
            scal->fevals += found >= 0 ? found + 1 : op.max_backtracks + 1;
        }
        if (found >= 0) scal->alpha = a_acc;
    }
}

// x+ = P(x + a p); g+ = M + lambda (log x+ + 1) + K^T (omega . (res + a K p)); pair; f+ from scratch at x+.
__global__ __launch_bounds__(kBlock) void k_ot_update_entropy(Dims dm, Opts op, OtArgs a, double* res,
                                                              const double* __restrict__ t, const double* __restrict__ p1,
                                                              const double* __restrict__ p2, const double* __restrict__ l,
                                                              const double* __restrict__ u, double* __restrict__ x,
                                                              double* __restrict__ g, double* __restrict__ S,
                                                              double* __restrict__ Y, Scal* __restrict__ scal,
                                                              double* __restrict__ redpart) {
    __shared__ double red[kWaves];
    __shared__ int flag;
    if (scal->status != LBFGSB_RUNNING) return;
    const int tid = threadIdx.x;
    const int ok = scal->ls_ok;
    const double alpha = scal->alpha;
    const int slot = scal->head;
    const double* p = scal->branch == 1 ? p1 : p2;
    double fs[1] = {0.0};
    if (ok) {
        double* Sn = S + (int64_t)slot * dm.n;
        double* Yn = Y + (int64_t)slot * dm.n;
        for (int64_t i = blockIdx.x; i < dm.rows; i += gridDim.x) {
            const double ri = a.omega ? a.omega[i] * fma(alpha, t[i], res[i]) : 0.0;
            for (int64_t j = tid; j < dm.cols; j += kBlock) {
                const int64_t e = i * dm.cols + j;
                const double cj = a.omega ? a.omega[dm.rows + j] * fma(alpha, t[dm.rows + j], res[dm.rows + j]) : 0.0;
                const double mij = m_at(a.M, dm.dtype, i * dm.ld + j);
                const double xi = x[e];
                const double xn = op.uniform_bounds ? clampd(fma(alpha, p[e], xi), op.lo, op.hi)
                                                    : clampd(fma(alpha, p[e], xi), l[e], u[e]);
                const double lg = log(xn);
                const double gn = mij + dm.lambda * (lg + 1.0) + (ri + cj);
                Sn[e] = xn - xi;
                Yn[e] = gn - g[e];
                x[e] = xn;
                g[e] = gn;
                fs[0] = fma(mij, xn, fs[0]);
                if (xn > 0.0) fs[0] = fma(dm.lambda * xn, lg, fs[0]);
            }
        }
    }
    block_sum<1, kWaves>(fs, red);
    if (tid == 0) redpart[blockIdx.x] = fs[0];
    if (!arrive_is_last(&scal->counters[kCntUpdate], &flag)) return;
    double tot[1] = {0.0};
    for (int b = tid; b < (int)gridDim.x; b += kBlock) tot[0] += redpart[b];
    if (ok) {
        // the residuals of the marginal terms move to the new point here, res += a K p: every other workgroup has
        // finished reading them (it has arrived)
        for (int64_t k = tid; k < dm.rows + dm.cols; k += kBlock) {
            const double rn = fma(alpha, t[k], res[k]);
            res[k] = rn;
            if (a.omega) tot[0] = fma(0.5 * a.omega[k] * rn, rn, tot[0]);
        }
    }
    block_sum<1, kWaves>(tot, red);
    if (tid == 0) {
        if (ok) {
            scal->f = tot[0];
            scal->head = (slot + 1) % dm.m;
            scal->count = scal->count < dm.m ? scal->count + 1 : dm.m;
            scal->iters += 1;
            record_iteration(scal);
        } else if (scal->count > 0) {
            scal->count = 0;
            scal->memory_resets += 1;
        } else {
            scal->status = LBFGSB_LINESEARCH_FAILED;
        }
    }
}

template <int RPW>
void launch_sums_t(const Dims& dm, const Geometry& ge, const Buffers& bf, const OtArgs& a, int eval, int check_status,
                   hipStream_t st, int dir_blocks, double eps) {
    hipLaunchKernelGGL(k_ot_sums<RPW>, dim3(ge.ot_row_blocks), dim3(kBlock), 0, st, dm, a, eval, check_status,
                       (const double*)bf.x, (const double*)bf.p1, (const double*)bf.p2, bf.scal, eval ? bf.row : bf.t,
                       bf.wpart, bf.losspart, (const double*)bf.redpart, eval ? 0 : dir_blocks, eps);
}

}  // namespace

void launch_ot_sums(const Dims& dm, const Geometry& ge, const Buffers& bf, const OtArgs& a, int eval, int check_status,
                    hipStream_t st, int dir_blocks, double eps) {
    switch (ge.ot_rpw) {
        case 1: launch_sums_t<1>(dm, ge, bf, a, eval, check_status, st, dir_blocks, eps); break;
        case 2: launch_sums_t<2>(dm, ge, bf, a, eval, check_status, st, dir_blocks, eps); break;
        case 4: launch_sums_t<4>(dm, ge, bf, a, eval, check_status, st, dir_blocks, eps); break;
        case 8: launch_sums_t<8>(dm, ge, bf, a, eval, check_status, st, dir_blocks, eps); break;
        default: launch_sums_t<kOtRpwMax>(dm, ge, bf, a, eval, check_status, st, dir_blocks, eps); break;
    }
    hipLaunchKernelGGL(k_ot_cols, dim3(ge.ot_col_blocks), dim3(kBlock), 0, st, dm, a, eval, check_status, ge.ot_row_blocks,
                       (const double*)bf.wpart, (const Scal*)bf.scal, eval ? bf.row : bf.t, bf.losspart + ge.ot_row_blocks);
}

void launch_ot_eval_finish(const Dims& dm, const Geometry& ge, const Buffers& bf, const OtArgs& a, hipStream_t st) {
    hipLaunchKernelGGL(k_ot_eval_finish, dim3(ge.ot_el_blocks), dim3(kBlock), 0, st, dm, a,
                       ge.ot_row_blocks + ge.ot_col_blocks, (const double*)bf.x, (const double*)bf.row,
                       (const double*)bf.losspart, bf.g, bf.scal);
}

void launch_ot_update_gauss(const Dims& dm, const Opts& op, const Geometry& ge, const Buffers& bf, const OtArgs& a,
                            hipStream_t st) {
    // (no closing arrival in this kernel: one workgroup per row)
    hipLaunchKernelGGL(k_ot_update_gauss, dim3((unsigned)(dm.rows > 2048 ? 2048 : dm.rows)), dim3(kBlock), 0, st, dm, op, a,
                       ge.ot_row_blocks + ge.ot_col_blocks, (const double*)bf.losspart, (const double*)bf.t,
                       (const double*)bf.p1, (const double*)bf.p2, (const double*)bf.l, (const double*)bf.u, bf.x, bf.g,
                       bf.S, bf.Y, bf.scal);
}

void launch_ot_step_entropy(const Dims& dm, const Opts& op, const Geometry& ge, const Buffers& bf, const OtArgs& a,
                            hipStream_t st) {
    // three launches, each with a region of lspart of its own: the first (two step lengths) only leaves its partial
    // sums, the second takes the first's decision before anything else
    double* part0 = bf.lspart;
    double* part1 = part0 + (size_t)ge.ls_blocks * 2;
    double* part2 = part1 + (size_t)ge.ls_blocks * kLsBatch;
    static_assert(2 + kLsBatch + kLsTail <= 64, "lspart holds 64 step lengths per workgroup");
    hipLaunchKernelGGL((k_ot_ls_entropy<2, 0>), dim3(ge.ls_blocks), dim3(kBlock), 0, st, dm, op,
                       ge.ot_row_blocks + ge.ot_col_blocks, 0, 0, 1, (const double*)bf.losspart, (const double*)bf.x,
                       (const double*)bf.p1, (const double*)bf.p2, bf.scal, (const double*)nullptr, part0);
    hipLaunchKernelGGL((k_ot_ls_entropy<kLsBatch, 2>), dim3(ge.ls_blocks), dim3(kBlock), 0, st, dm, op,
                       ge.ot_row_blocks + ge.ot_col_blocks, 2, 0, 0, (const double*)bf.losspart, (const double*)bf.x,
                       (const double*)bf.p1, (const double*)bf.p2, bf.scal, (const double*)part0, part1);
    hipLaunchKernelGGL((k_ot_ls_entropy<kLsTail, 0>), dim3(ge.ls_blocks), dim3(kBlock), 0, st, dm, op,
                       ge.ot_row_blocks + ge.ot_col_blocks, 2 + kLsBatch, 1, 0, (const double*)bf.losspart,
                       (const double*)bf.x, (const double*)bf.p1, (const double*)bf.p2, bf.scal, (const double*)nullptr,
                       part2);
    hipLaunchKernelGGL(k_ot_update_entropy, dim3(ge.ot_el_blocks), dim3(kBlock), 0, st, dm, op, a, bf.row,
                       (const double*)bf.t, (const double*)bf.p1, (const double*)bf.p2, (const double*)bf.l,
                       (const double*)bf.u, bf.x, bf.g, bf.S, bf.Y, bf.scal, bf.redpart);
}

}  // namespace lb
