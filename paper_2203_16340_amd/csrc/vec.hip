// The O(m*n) part of an iteration of Algorithm 1: free set (Eq. (ws)), the modified two-loop
// recursion (Algorithm 3) in batched form, projectDirection (Algorithm 2), the line search and the
// update of iterate, gradient and pair memory.  Every data-dependent decision is taken on the
// device by the last workgroup of the kernel that produces the numbers it depends on.
//
// Batched form of Algorithm 3.  Let b_0..b_{V-1} = s^0[S]..s^{c-1}[S], y^0[S]..y^{c-1}[S], g[S]
// (c stored pairs, oldest first, S the current free set) and G = B^T B.  Every vector q the
// recursion forms is B*delta for a coefficient vector delta (initially e_{V-1}); the dot products it
// needs are rows of G times delta:  rho^i = G[s_i][y_i], <s^i,q> = (G delta)[s_i], <y^i,q> =
// (G delta)[y_i].  So one pass over the V vectors gives G (k_gram), one wave runs the recursion on
// V coefficients, and one more pass forms d = -B*delta (k_dir).  G has to be rebuilt every
// iteration because S changes.
#include "common.h"

namespace lb {

constexpr int kGramE = 64;   // elements staged per chunk

__host__ __device__ inline int gram_tiles(int V) {
    const int T = (V + 1) / 2;
    return T * (T + 1) / 2;
}
int gram_entries(int m) { return 4 + 4 * gram_tiles(2 * m + 1); }
int gram_blocks_for(int64_t n) {
    // a few chunks per workgroup: the kernel is latency-bound, and every partial written here is
    // read again by the last workgroup
    int64_t b = (n + 4 * kGramE - 1) / (4 * kGramE);
    return (int)(b < 1 ? 1 : (b > 128 ? 128 : b));
}

__device__ __forceinline__ const double* ring_vec(int j, int c, int head, int m, int64_t n, const double* S,
                                                  const double* Y, const double* g) {
    // logical vector j of [s^0..s^{c-1}, y^0..y^{c-1}, g], pair 0 being the oldest
    if (j < c) return S + (int64_t)((head - c + j + 2 * m) % m) * n;
    if (j < 2 * c) return Y + (int64_t)((head - c + (j - c) + 2 * m) % m) * n;
    return g;
}

__global__ void k_fill_zero(uint64_t* p, size_t words) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < words; i += (size_t)gridDim.x * blockDim.x)
        p[i] = 0ull;
}
void launch_fill_zero(void* p, size_t bytes, hipStream_t st) {
    const size_t words = bytes / 8;
    int blocks = (int)((words + 255) / 256);
    if (blocks > 4096) blocks = 4096;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(k_fill_zero, dim3(blocks), dim3(256), 0, st, (uint64_t*)p, words);
}

__global__ void k_set_status(Scal* scal, int status) {
    if (threadIdx.x == 0 && blockIdx.x == 0) scal->status = status;
}
void launch_set_status(const Buffers& bf, int status, hipStream_t st) {
    hipLaunchKernelGGL(k_set_status, dim3(1), dim3(64), 0, st, bf.scal, status);
}

// ---- free set + masked Gram matrix + two-loop coefficients ------------------------------------------

__global__ __launch_bounds__(kBlock) void k_gram(int64_t n, int m, Opts op, const double* __restrict__ x,
                                                 const double* __restrict__ g, const double* __restrict__ l,
                                                 const double* __restrict__ u, const double* __restrict__ S,
                                                 const double* __restrict__ Y, uint8_t* __restrict__ mask,
                                                 Scal* __restrict__ scal, double* __restrict__ grampart, int NE,
                                                 int use_given_mask, int evaluate_stop) {
    __shared__ __align__(16) double tileb[kGramE * kMaxV];   // staged chunk [element][vector]; later G
    __shared__ const double* vecp[kMaxV];
    __shared__ double red[kWaves * 2];
    __shared__ double alpha_s[kMaxM + 1];
    __shared__ int flag;

    if (scal->status != LBFGSB_RUNNING) return;
    const int tid = threadIdx.x;
    const int c = scal->count, head = scal->head;
    const int V = 2 * c + 1;
    const int Vp = (V + 1) & ~1;
    const int T = Vp / 2;
    const int ntiles = T * (T + 1) / 2;
    if (tid < V) vecp[tid] = ring_vec(tid, c, head, m, n, S, Y, g);

    // tiles this thread accumulates
    constexpr int kTPT = 3;   // ceil(528 / 256)
    int ti[kTPT], tj[kTPT];
    double acc[kTPT][4];
#pragma unroll
    for (int k = 0; k < kTPT; ++k) {
        int q = tid + k * kBlock, a = 0;
        if (q < ntiles) {
            while (q >= T - a) { q -= T - a; ++a; }
            ti[k] = a; tj[k] = a + q;
        } else {
            ti[k] = -1; tj[k] = 0;
        }
        acc[k][0] = acc[k][1] = acc[k][2] = acc[k][3] = 0.0;
    }
    double pg2 = 0.0, pginf = 0.0, nfixed = 0.0;
    __syncthreads();

    const int lane = tid & 63, wave = tid >> 6;
    for (int64_t e0 = (int64_t)blockIdx.x * kGramE; e0 < n; e0 += (int64_t)gridDim.x * kGramE) {
        // every wave derives the free flag of element e0 + lane (wave 0 also records it); wave w then
        // stages vectors w, w + 4, w + 8, ... of that element, all loads issued before any is used
        const int64_t e = e0 + lane;
        double mf = 0.0;
        double stage[kMaxV / kWaves];
        if (e < n) {
#pragma unroll
            for (int k = 0; k < kMaxV / kWaves; ++k) {
                const int j = wave + kWaves * k;
                stage[k] = j < V ? vecp[j][e] : 0.0;
            }
            const double xe = x[e], ge = g[e], le = l[e], ue = u[e];
            int fr;
            if (use_given_mask) {
                fr = mask[e] != 0;
            } else {
                const bool at_lower = (xe <= le + op.eps) && (ge >= 0.0);
                const bool at_upper = (xe >= ue - op.eps) && (ge <= 0.0);
                fr = !(at_lower || at_upper);
            }
            mf = fr ? 1.0 : 0.0;
            if (wave == 0) {
                if (!use_given_mask) mask[e] = (uint8_t)fr;
                if (fr) pg2 = fma(ge, ge, pg2); else nfixed += 1.0;
                pginf = fmax(pginf, fabs(xe - clampd(xe - ge, le, ue)));
            }
        } else {
#pragma unroll
            for (int k = 0; k < kMaxV / kWaves; ++k) stage[k] = 0.0;
        }
#pragma unroll
        for (int k = 0; k < kMaxV / kWaves; ++k) {
            const int j = wave + kWaves * k;
            if (j < Vp) tileb[lane * Vp + j] = stage[k] * mf;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < kTPT; ++k) {
            if (ti[k] >= 0) {
                const double* pa = tileb + 2 * ti[k];
                const double* pb = tileb + 2 * tj[k];
#pragma unroll 4
                for (int el = 0; el < kGramE; ++el) {
                    const double2 a = *reinterpret_cast<const double2*>(pa + el * Vp);
                    const double2 b = *reinterpret_cast<const double2*>(pb + el * Vp);
                    acc[k][0] = fma(a.x, b.x, acc[k][0]);
                    acc[k][1] = fma(a.x, b.y, acc[k][1]);
                    acc[k][2] = fma(a.y, b.x, acc[k][2]);
                    acc[k][3] = fma(a.y, b.y, acc[k][3]);
                }
            }
        }
        __syncthreads();
    }

    double* part = grampart + (int64_t)blockIdx.x * NE;
#pragma unroll
    for (int k = 0; k < kTPT; ++k) {
        if (ti[k] >= 0) {
            const int q = tid + k * kBlock;
#pragma unroll
            for (int s = 0; s < 4; ++s) part[4 + 4 * q + s] = acc[k][s];
        }
    }
    {
        double sv[2] = {pg2, nfixed};
        block_sum<2, kWaves>(sv, red);
        double mx = wave_max(pginf);
        __syncthreads();
        if ((tid & 63) == 0) red[tid >> 6] = mx;
        __syncthreads();
        if (tid == 0) {
            mx = red[0];
            for (int w = 1; w < kWaves; ++w) mx = fmax(mx, red[w]);
            part[0] = sv[0]; part[1] = mx; part[2] = sv[1];
        }
    }
    if (!arrive_is_last(&scal->counters[kCntGram], &flag)) return;

    // ---- last workgroup: total G, then the recursion on coefficients ----
    const int nb = gridDim.x;
    double* G = tileb;   // Vp x Vp, row-major
    // 64 entries at a time; wave w sums the partials of workgroups w, w + 4, ... (8 loads in flight),
    // the four wave results are added in wave order
    __shared__ double wsum[kWaves][64];
    for (int q0 = 0; q0 < 4 * ntiles; q0 += 64) {
        const int q4 = q0 + lane;
        double s = 0.0;
        if (q4 < 4 * ntiles) {
            const double* src = grampart + 4 + q4;
            for (int b0 = wave; b0 < nb; b0 += kWaves * 8) {
                double v[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const int b = b0 + kWaves * k;
                    v[k] = b < nb ? src[(int64_t)b * NE] : 0.0;
                }
#pragma unroll
                for (int k = 0; k < 8; ++k) s += v[k];
            }
        }
        wsum[wave][lane] = s;
        __syncthreads();
        if (wave == 0 && q4 < 4 * ntiles) {
            const double tot = ((wsum[0][lane] + wsum[1][lane]) + wsum[2][lane]) + wsum[3][lane];
            int q = q4 >> 2, a = 0;
            while (q >= T - a) { q -= T - a; ++a; }
            const int row = 2 * a + ((q4 >> 1) & 1), col = 2 * (a + q) + (q4 & 1);
            G[row * Vp + col] = tot;
            G[col * Vp + row] = tot;
        }
        __syncthreads();
    }
    {
        // per-workgroup statistics (at most 128 workgroups): one thread each, fixed-order reductions
        const bool have = tid < nb;
        double sv[2] = {have ? grampart[(int64_t)tid * NE] : 0.0, have ? grampart[(int64_t)tid * NE + 2] : 0.0};
        double mx = have ? grampart[(int64_t)tid * NE + 1] : 0.0;
        __shared__ double stat[kWaves * 2];
        __shared__ double stat_mx[kWaves];
        block_sum<2, kWaves>(sv, stat);
        mx = wave_max(mx);
        if (lane == 0) stat_mx[wave] = mx;
        __syncthreads();
        if (tid == 0) {
            red[0] = sv[0];
            red[1] = fmax(fmax(stat_mx[0], stat_mx[1]), fmax(stat_mx[2], stat_mx[3]));
            red[2] = sv[1];
        }
    }
    __syncthreads();
    if (tid < 64) {
        // lane j holds delta_j
        double delta = (lane == 2 * c) ? 1.0 : 0.0;
        int used = 0;
        unsigned long long passmask = 0ull;
        for (int i = c - 1; i >= 0; --i) {
            const double rho = G[i * Vp + (c + i)];
            const double yn = scal->ynorm2[(head - c + i + 2 * m) % m];
            if (rho > op.eps * yn) {
                passmask |= 1ull << i;
                ++used;
                const double sq = wave_sum(lane < V ? G[i * Vp + lane] * delta : 0.0);
                const double al = sq / rho;
                if (lane == 0) alpha_s[i] = al;
                if (lane == c + i) delta -= al;
            }
        }
        if (c > 0 && ((passmask >> (c - 1)) & 1ull)) {
            const double rho = G[(c - 1) * Vp + (2 * c - 1)];
            const double yn = scal->ynorm2[(head - 1 + 2 * m) % m];
            delta *= rho / yn;
        }
        for (int i = 0; i < c; ++i) {
            if ((passmask >> i) & 1ull) {
                const double rho = G[i * Vp + (c + i)];
                const double yq = wave_sum(lane < V ? G[(c + i) * Vp + lane] * delta : 0.0);
                const double beta = yq / rho;
                const double al = alpha_s[i];
                if (lane == i) delta += al - beta;
            }
        }
        scal->delta[lane] = lane < V ? delta : 0.0;
        if (lane == 0) {
            scal->pairs_used = used;
            if (evaluate_stop) {
                const double pgn = sqrt(red[0]);
                scal->pg2 = pgn;
                scal->pginf = red[1];
                scal->n_fixed = (long long)red[2];
                if (!scal->tol_resolved) {
                    scal->tol_abs = op.tol_relative ? op.tol * fmax(1.0, pgn) : op.tol;
                    scal->tol_resolved = 1;
                }
                if (pgn <= scal->tol_abs) scal->status = LBFGSB_CONVERGED;
                else if (scal->iters >= op.max_iter) scal->status = LBFGSB_MAX_ITER;
            }
        }
    }
}

void launch_gram(const Dims& dm, const Opts& op, const Geometry& ge, const Buffers& bf, int use_given_mask,
                 int evaluate_stop, hipStream_t st) {
    hipLaunchKernelGGL(k_gram, dim3(ge.gram_blocks), dim3(kBlock), 0, st, dm.n, dm.m, op, bf.x, bf.g, bf.l, bf.u, bf.S,
                       bf.Y, bf.mask, bf.scal, bf.grampart, gram_entries(dm.m), use_given_mask, evaluate_stop);
}

// ---- d = -B delta on the free set, then Algorithm 2 ------------------------------------------------------

constexpr int kDirRed = 8;   // p1.g, p1.p1, x.p1, p2.g, p2.p2, x.p2, min step bound of p2, unused

__global__ __launch_bounds__(kBlock) void k_dir(int64_t n, int m, Opts op, const double* __restrict__ x,
                                                const double* __restrict__ g, const double* __restrict__ l,
                                                const double* __restrict__ u, const uint8_t* __restrict__ mask,
                                                const double* __restrict__ S, const double* __restrict__ Y,
                                                Scal* __restrict__ scal, double* __restrict__ d,
                                                double* __restrict__ p1, double* __restrict__ p2,
                                                double* __restrict__ redpart, int d_given) {
    __shared__ double delta_s[kMaxV + 8];
    __shared__ const double* vecp[kMaxV + 8];
    __shared__ double red[kWaves * 7];
    __shared__ int flag;
    if (scal->status != LBFGSB_RUNNING) return;
    const int tid = threadIdx.x;
    const int c = scal->count, head = scal->head;
    const int V = 2 * c + 1;
    if (tid < kMaxV + 8) {
        vecp[tid] = tid < V ? ring_vec(tid, c, head, m, n, S, Y, g) : g;
        delta_s[tid] = tid < V ? scal->delta[tid] : 0.0;
    }
    __syncthreads();
    double s[6] = {0, 0, 0, 0, 0, 0};
    double ub = INFINITY;
    for (int64_t e = (int64_t)blockIdx.x * kBlock + tid; e < n; e += (int64_t)gridDim.x * kBlock) {
        double de;
        if (d_given) {
            de = d[e];
        } else {
            de = 0.0;
            if (mask[e]) {
                double q = 0.0;
                for (int j0 = 0; j0 < V; j0 += 8) {
                    double v[8];
#pragma unroll
                    for (int k = 0; k < 8; ++k) v[k] = j0 + k < V ? vecp[j0 + k][e] : 0.0;
#pragma unroll
                    for (int k = 0; k < 8; ++k) q = fma(delta_s[j0 + k], v[k], q);
                }
                de = -q;
            }
            d[e] = de;
        }
        const double xe = x[e], ge = g[e], le = l[e], ue = u[e];
        const double a = clampd(xe + de, le, ue) - xe;
        double b = de;
        if (de < 0.0 && xe <= le + op.eps) b = 0.0;
        if (de > 0.0 && xe >= ue - op.eps) b = 0.0;
        p1[e] = a;
        p2[e] = b;
        s[0] = fma(a, ge, s[0]); s[1] = fma(a, a, s[1]); s[2] = fma(xe, a, s[2]);
        s[3] = fma(b, ge, s[3]); s[4] = fma(b, b, s[4]); s[5] = fma(xe, b, s[5]);
        if (b > 0.0) ub = fmin(ub, (ue - xe) / b);
        else if (b < 0.0) ub = fmin(ub, (le - xe) / b);
    }
    block_sum<6, kWaves>(s, red);
    double mn = wave_min(ub);
    __syncthreads();
    if ((tid & 63) == 0) red[tid >> 6] = mn;
    __syncthreads();
    if (tid == 0) {
        mn = red[0];
        for (int w = 1; w < kWaves; ++w) mn = fmin(mn, red[w]);
        double* part = redpart + (int64_t)blockIdx.x * kDirRed;
        for (int k = 0; k < 6; ++k) part[k] = s[k];
        part[6] = mn;
    }
    if (!arrive_is_last(&scal->counters[kCntDir], &flag)) return;
    {
        // at most kBlock workgroups wrote partials: one thread each, then the fixed-order reductions
        double t6[6];
        double tmin = INFINITY;
        const bool have = tid < (int)gridDim.x;
#pragma unroll
        for (int k = 0; k < 6; ++k) t6[k] = have ? redpart[(int64_t)tid * kDirRed + k] : 0.0;
        if (have) tmin = redpart[(int64_t)tid * kDirRed + 6];
        block_sum<6, kWaves>(t6, red);
        tmin = wave_min(tmin);
        __syncthreads();
        if ((tid & 63) == 0) red[tid >> 6] = tmin;
        __syncthreads();
        if (tid == 0) {
            tmin = red[0];
            for (int w = 1; w < kWaves; ++w) tmin = fmin(tmin, red[w]);
        }
        __syncthreads();
        if (tid == 0) {
            for (int k = 0; k < 6; ++k) red[k] = t6[k];
            red[6] = tmin;
        }
    }
    __syncthreads();
    if (tid == 0) {
        const double p1g = red[0], p1p1 = red[1];
        if (p1g <= -op.eps * p1p1 && p1p1 >= op.eps) {
            scal->branch = 1; scal->gp = p1g; scal->alpha_ub = 1.0; scal->pp = p1p1; scal->xp = red[2];
        } else {
            scal->branch = 2; scal->gp = red[3]; scal->alpha_ub = red[6]; scal->pp = red[4]; scal->xp = red[5];
        }
    }
}

void launch_dir(const Dims& dm, const Opts& op, const Geometry& ge, const Buffers& bf, int d_given, hipStream_t st) {
    hipLaunchKernelGGL(k_dir, dim3(ge.dir_blocks), dim3(kBlock), 0, st, dm.n, dm.m, op, bf.x, bf.g, bf.l, bf.u, bf.mask,
                       bf.S, bf.Y, bf.scal, bf.d, bf.p1, bf.p2, bf.redpart, d_given);
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

// ---- after an evaluation pass: g and f ------------------------------------------------------------------

__global__ __launch_bounds__(kBlock) void k_eval_finish(Dims dm, int w_parts, int loss_parts,
                                                        const double* __restrict__ wpart,
                                                        const double* __restrict__ losspart,
                                                        const double* __restrict__ x, double* __restrict__ g,
                                                        Scal* __restrict__ scal, double* __restrict__ redpart) {
    __shared__ double lds[kBlock];
    __shared__ double red[kWaves];
    __shared__ int flag;
    if (scal->status != LBFGSB_RUNNING) return;
    const int tid = threadIdx.x;
    double reg = 0.0;
    for (int64_t c0 = (int64_t)blockIdx.x * kCX; c0 < dm.cols; c0 += (int64_t)gridDim.x * kCX) {
        const int64_t c = c0 + tid % kCX;
        const double w = column_sum(wpart, w_parts, dm.cols, c, lds);
        if (tid < kCX && c < dm.cols) {
            if (dm.kind == LBFGSB_OBJ_LSQ) {
                g[c] = w;
            } else if (dm.kind == LBFGSB_OBJ_LSQ_L1SPLIT) {
                g[c] = w + dm.lambda;
                g[c + dm.cols] = -w + dm.lambda;
                reg += x[c] + x[c + dm.cols];
            } else {
                const double xc = x[c];
                g[c] = fma(dm.mu, xc, w);
                reg = fma(xc, xc, reg);
            }
        }
    }
    double rv[1] = {reg};
    block_sum<1, kWaves>(rv, red);
    if (tid == 0) redpart[blockIdx.x] = rv[0];
    if (!arrive_is_last(&scal->counters[kCntEvalFinish], &flag)) return;
    const double loss = sum_all(losspart, loss_parts, red);
    const double regt = sum_all(redpart, gridDim.x, red);
    if (tid == 0) {
        double f = loss;
        if (dm.kind == LBFGSB_OBJ_LSQ_L1SPLIT) f += dm.lambda * regt;
        else if (dm.kind == LBFGSB_OBJ_LOGISTIC_L2) f += 0.5 * dm.mu * regt;
        scal->f = f;
        scal->fevals += 1;
    }
}

void launch_eval_finish(const Dims& dm, const Geometry& ge, const Buffers& bf, hipStream_t st) {
    hipLaunchKernelGGL(k_eval_finish, dim3(ge.fin_blocks), dim3(kBlock), 0, st, dm, ge.w_parts, ge.loss_parts, bf.wpart,
                       bf.losspart, bf.x, bf.g, bf.scal, bf.redpart);
}

// ---- quadratic objectives: closed-form Armijo search, then the update ---------------------------------------
//
// With t = A v_p and w = A^T t from the direction pass:  f(x + a p) - f(x) = a <g,p> + a^2/2 ||t||^2,
// residual r + a t, gradient g + a w~ (w~ = w, or [w; -w] for the split form), y = a w~.
// The Armijo inequality  a gp + a^2/2 tt <= c1 a gp  is tested after division by a > 0.
__global__ __launch_bounds__(kBlock) void k_update_quadratic(Dims dm, Opts op, int w_parts, int loss_parts,
                                                             const double* __restrict__ wpart,
                                                             const double* __restrict__ losspart,
                                                             const double* __restrict__ p1,
                                                             const double* __restrict__ p2,
                                                             const double* __restrict__ l, const double* __restrict__ u,
                                                             const double* __restrict__ t, double* __restrict__ x,
                                                             double* __restrict__ g, double* __restrict__ row,
                                                             double* __restrict__ S, double* __restrict__ Y,
                                                             Scal* __restrict__ scal, double* __restrict__ redpart) {
    __shared__ double lds[kBlock];
    __shared__ double red[kWaves];
    __shared__ double ls_alpha;
    __shared__ int ls_ok, ls_bt, flag;
    if (scal->status != LBFGSB_RUNNING) return;
    const int tid = threadIdx.x;
    const double tt = sum_all(losspart, loss_parts, red);
    const double gp = scal->gp;
    if (tid == 0) {
        double a = fmin(1.0, scal->alpha_ub);
        int ok = 0, bt = 0;
        for (int k = 0; k <= op.max_backtracks; ++k) {
            const double lhs = gp + 0.5 * a * tt;          // (f(x + a p) - f(x)) / a
            const double df = a * lhs;
            if (isfinite(df) && lhs <= op.c1 * gp) { ok = 1; bt = k; break; }
            a *= op.backtrack;
        }
        ls_alpha = a; ls_ok = ok; ls_bt = ok ? bt : op.max_backtracks + 1;
    }
    __syncthreads();
    const double alpha = ls_alpha;
    const int ok = ls_ok;
    const int slot = scal->head;
    const double* p = scal->branch == 1 ? p1 : p2;
    double yy = 0.0;
    if (ok) {
        double* Sn = S + (int64_t)slot * dm.n;
        double* Yn = Y + (int64_t)slot * dm.n;
        for (int64_t c0 = (int64_t)blockIdx.x * kCX; c0 < dm.cols; c0 += (int64_t)gridDim.x * kCX) {
            const int64_t c = c0 + tid % kCX;
            const double w = column_sum(wpart, w_parts, dm.cols, c, lds);
            if (tid < kCX && c < dm.cols) {
                const int nvar = dm.kind == LBFGSB_OBJ_LSQ_L1SPLIT ? 2 : 1;
                for (int h = 0; h < nvar; ++h) {
                    const int64_t i = c + h * dm.cols;
                    const double y = alpha * (h ? -w : w);
                    const double xi = x[i];
                    const double xn = clampd(fma(alpha, p[i], xi), l[i], u[i]);
                    Sn[i] = xn - xi;
                    Yn[i] = y;
                    x[i] = xn;
                    g[i] += y;
                    yy = fma(y, y, yy);
                }
            }
        }
        for (int64_t r = (int64_t)blockIdx.x * kBlock + tid; r < dm.rows; r += (int64_t)gridDim.x * kBlock)
            row[r] = fma(alpha, t[r], row[r]);
    }
    double yv[1] = {yy};
    block_sum<1, kWaves>(yv, red);
    if (tid == 0) redpart[blockIdx.x] = yv[0];
    if (!arrive_is_last(&scal->counters[kCntUpdate], &flag)) return;
    const double yyt = sum_all(redpart, gridDim.x, red);
    if (tid == 0) {
        scal->ls_ok = ok;
        scal->backtracks = ls_bt;
        scal->fevals += ls_bt + (ok ? 1 : 0);
        if (ok) {
            scal->alpha = alpha;
            scal->f += alpha * (gp + 0.5 * alpha * tt);
            scal->ynorm2[slot] = yyt;
            scal->head = (slot + 1) % dm.m;
            scal->count = scal->count < dm.m ? scal->count + 1 : dm.m;
            scal->iters += 1;
        } else if (scal->count > 0) {
            scal->count = 0;                 // clear the pair memory; the next step retries from -g[S]
            scal->memory_resets += 1;
        } else {
            scal->status = LBFGSB_LINESEARCH_FAILED;
        }
    }
}

void launch_update_quadratic(const Dims& dm, const Opts& op, const Geometry& ge, const Buffers& bf, hipStream_t st) {
    hipLaunchKernelGGL(k_update_quadratic, dim3(ge.upd_blocks), dim3(kBlock), 0, st, dm, op, ge.w_parts, ge.loss_parts,
                       bf.wpart, bf.losspart, bf.p1, bf.p2, bf.l, bf.u, bf.t, bf.x, bf.g, bf.row, bf.S, bf.Y, bf.scal,
                       bf.redpart);
}

// ---- logistic objective: line search on the margins --------------------------------------------------------
//
// With z = X w (kept in `row`) and t = X p:  f(x + a p) - f(x) = (1/N) sum_r [softplus(-y_r (z_r + a t_r))
// - softplus(-y_r z_r)] + mu (a <x,p> + a^2/2 <p,p>).  The bracket is evaluated in the cancellation-free
// form log1p(sigmoid(q) expm1(dq)), q = -y z, dq = -y a t.  kLsBatch step lengths are evaluated in one
// sweep over the rows; if none is acceptable the last workgroup goes on alone, one length at a time.
__device__ __forceinline__ double softplus_diff(double q, double sq, double dq) {
    return fabs(dq) < 30.0 ? log1p(sq * expm1(dq)) : softplus_d(q + dq) - softplus_d(q);
}

__global__ __launch_bounds__(kBlock) void k_ls_logistic(Dims dm, Opts op, const double* __restrict__ yl,
                                                        const double* __restrict__ z, const double* __restrict__ t,
                                                        Scal* __restrict__ scal, double* __restrict__ lspart) {
    __shared__ double red[kWaves * kLsBatch];
    __shared__ int flag;
    __shared__ double sh_alpha;
    __shared__ int sh_done;
    if (scal->status != LBFGSB_RUNNING) return;
    const int tid = threadIdx.x;
    const double a0 = fmin(1.0, scal->alpha_ub);
    double al[kLsBatch], s[kLsBatch];
    {
        double a = a0;
#pragma unroll
        for (int j = 0; j < kLsBatch; ++j) { al[j] = a; s[j] = 0.0; a *= op.backtrack; }
    }
    for (int64_t r = (int64_t)blockIdx.x * kBlock + tid; r < dm.rows; r += (int64_t)gridDim.x * kBlock) {
        const double y = yl[r], q = -y * z[r], sq = sigmoid_d(q), ty = -y * t[r];
#pragma unroll
        for (int j = 0; j < kLsBatch; ++j) s[j] += softplus_diff(q, sq, al[j] * ty);
    }
    block_sum<kLsBatch, kWaves>(s, red);
    if (tid == 0) {
#pragma unroll
        for (int j = 0; j < kLsBatch; ++j) lspart[(int64_t)blockIdx.x * kLsBatch + j] = s[j];
    }
    if (!arrive_is_last(&scal->counters[kCntLs], &flag)) return;
    const double gp = scal->gp, xp = scal->xp, pp = scal->pp;
    const double invn = 1.0 / (double)dm.rows;
    // totals of the batch
    double tot[kLsBatch];
#pragma unroll
    for (int j = 0; j < kLsBatch; ++j) tot[j] = 0.0;
    for (int b = tid; b < (int)gridDim.x; b += kBlock) {
#pragma unroll
        for (int j = 0; j < kLsBatch; ++j) tot[j] += lspart[(int64_t)b * kLsBatch + j];
    }
    block_sum<kLsBatch, kWaves>(tot, red);
    int found = -1;
    double a_acc = 0.0;
    for (int j = 0; j < kLsBatch && j <= op.max_backtracks; ++j) {
        const double df = tot[j] * invn + dm.mu * al[j] * (xp + 0.5 * al[j] * pp);
        if (isfinite(df) && df <= op.c1 * al[j] * gp) { found = j; a_acc = al[j]; break; }
    }
    // rare: continue one step length at a time (uniform control flow: every thread holds the same totals)
    double a = al[kLsBatch - 1];
    for (int k = kLsBatch; found < 0 && k <= op.max_backtracks; ++k) {
        a *= op.backtrack;
        double sv[1] = {0.0};
        for (int64_t r = tid; r < dm.rows; r += kBlock) {
            const double y = yl[r], q = -y * z[r];
            sv[0] += softplus_diff(q, sigmoid_d(q), -y * a * t[r]);
        }
        block_sum<1, kWaves>(sv, red);
        const double df = sv[0] * invn + dm.mu * a * (xp + 0.5 * a * pp);
        if (isfinite(df) && df <= op.c1 * a * gp) { found = k; a_acc = a; }
    }
    if (tid == 0) {
        scal->ls_ok = found >= 0;
        scal->backtracks = found >= 0 ? found : op.max_backtracks + 1;
        scal->fevals += found >= 0 ? found + 1 : op.max_backtracks + 1;
        if (found >= 0) scal->alpha = a_acc;
    }
    (void)sh_alpha; (void)sh_done;
}

void launch_ls_logistic(const Dims& dm, const Opts& op, const Geometry& ge, const Buffers& bf, const double* labels,
                        hipStream_t st) {
    hipLaunchKernelGGL(k_ls_logistic, dim3(ge.ls_blocks), dim3(kBlock), 0, st, dm, op, labels, bf.row, bf.t, bf.scal,
                       bf.lspart);
}

// z += alpha t; psi = -y sigma(-y z)/N; loss partials of the new point (from the new margins).
__global__ __launch_bounds__(kBlock) void k_rows_logistic(Dims dm, const double* __restrict__ yl,
                                                          const double* __restrict__ t, double* __restrict__ z,
                                                          double* __restrict__ psi, const Scal* __restrict__ scal,
                                                          double* __restrict__ losspart) {
    __shared__ double red[kWaves];
    if (scal->status != LBFGSB_RUNNING || !scal->ls_ok) return;
    const double alpha = scal->alpha;
    const double invn = 1.0 / (double)dm.rows;
    double s[1] = {0.0};
    for (int64_t r = (int64_t)blockIdx.x * kBlock + threadIdx.x; r < dm.rows; r += (int64_t)gridDim.x * kBlock) {
        const double y = yl[r];
        const double zn = fma(alpha, t[r], z[r]);
        const double q = -y * zn;
        z[r] = zn;
        psi[r] = -y * sigmoid_d(q) * invn;
        s[0] += softplus_d(q) * invn;
    }
    block_sum<1, kWaves>(s, red);
    if (threadIdx.x == 0) losspart[blockIdx.x] = s[0];
}

void launch_rows_logistic(const Dims& dm, const Geometry& ge, const Buffers& bf, const double* labels, hipStream_t st) {
    hipLaunchKernelGGL(k_rows_logistic, dim3(ge.ls_blocks), dim3(kBlock), 0, st, dm, labels, bf.t, bf.row, bf.psi, bf.scal,
                       bf.losspart);
}

// x+ = P(x + alpha p), g+ = X^T psi + mu x+, pair (x+ - x, g+ - g), f+ from the new margins.
__global__ __launch_bounds__(kBlock) void k_update_logistic(Dims dm, int w_parts, int loss_parts,
                                                            const double* __restrict__ wpart,
                                                            const double* __restrict__ losspart,
                                                            const double* __restrict__ p1, const double* __restrict__ p2,
                                                            const double* __restrict__ l, const double* __restrict__ u,
                                                            double* __restrict__ x, double* __restrict__ g,
                                                            double* __restrict__ S, double* __restrict__ Y,
                                                            Scal* __restrict__ scal, double* __restrict__ redpart) {
    __shared__ double lds[kBlock];
    __shared__ double red[kWaves * 2];
    __shared__ int flag;
    if (scal->status != LBFGSB_RUNNING) return;
    const int tid = threadIdx.x;
    const int ok = scal->ls_ok;
    const double alpha = scal->alpha;
    const int slot = scal->head;
    const double* p = scal->branch == 1 ? p1 : p2;
    double sums[2] = {0.0, 0.0};   // ||y||^2, ||x+||^2
    if (ok) {
        double* Sn = S + (int64_t)slot * dm.n;
        double* Yn = Y + (int64_t)slot * dm.n;
        for (int64_t c0 = (int64_t)blockIdx.x * kCX; c0 < dm.cols; c0 += (int64_t)gridDim.x * kCX) {
            const int64_t c = c0 + tid % kCX;
            const double w = column_sum(wpart, w_parts, dm.cols, c, lds);
            if (tid < kCX && c < dm.cols) {
                const double xi = x[c];
                const double xn = clampd(fma(alpha, p[c], xi), l[c], u[c]);
                const double gn = fma(dm.mu, xn, w);
                const double y = gn - g[c];
                Sn[c] = xn - xi;
                Yn[c] = y;
                x[c] = xn;
                g[c] = gn;
                sums[0] = fma(y, y, sums[0]);
                sums[1] = fma(xn, xn, sums[1]);
            }
        }
    }
    block_sum<2, kWaves>(sums, red);
    if (tid == 0) { redpart[2 * blockIdx.x] = sums[0]; redpart[2 * blockIdx.x + 1] = sums[1]; }
    if (!arrive_is_last(&scal->counters[kCntUpdate], &flag)) return;
    double tot[2] = {0.0, 0.0};
    for (int b = tid; b < (int)gridDim.x; b += kBlock) { tot[0] += redpart[2 * b]; tot[1] += redpart[2 * b + 1]; }
    block_sum<2, kWaves>(tot, red);
    const double loss = ok ? sum_all(losspart, loss_parts, red) : 0.0;
    if (tid == 0) {
        if (ok) {
            scal->f = loss + 0.5 * dm.mu * tot[1];
            scal->ynorm2[slot] = tot[0];
            scal->head = (slot + 1) % dm.m;
            scal->count = scal->count < dm.m ? scal->count + 1 : dm.m;
            scal->iters += 1;
        } else if (scal->count > 0) {
            scal->count = 0;
            scal->memory_resets += 1;
        } else {
            scal->status = LBFGSB_LINESEARCH_FAILED;
        }
    }
}

void launch_update_logistic(const Dims& dm, const Geometry& ge, const Buffers& bf, int loss_parts, hipStream_t st) {
    hipLaunchKernelGGL(k_update_logistic, dim3(ge.upd_blocks), dim3(kBlock), 0, st, dm, ge.w_parts, loss_parts, bf.wpart,
                       bf.losspart, bf.p1, bf.p2, bf.l, bf.u, bf.x, bf.g, bf.S, bf.Y, bf.scal, bf.redpart);
}

}  // namespace lb
