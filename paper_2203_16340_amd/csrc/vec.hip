// The O(m*n) part of an iteration of Algorithm 1: free set (Eq. (ws)), the modified two-loop
// recursion (Algorithm 3) in batched form, projectDirection (Algorithm 2), the line search and the
// update of iterate, gradient and pair memory.  Every data-dependent decision is taken on the
// device by the last workgroup of the kernel that produces the numbers it depends on.
// (The free set, the Gram matrix and the recursion of Algorithm 3 are in gram.hip.)
#include "common.h"
#include "wide_close.h"

namespace lb {

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

__global__ void k_clear_bail(Scal* scal) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        if (scal->status == kStatusBail) scal->status = LBFGSB_RUNNING;
        scal->bail_skipped = 0;
    }
}
void launch_clear_bail(const Buffers& bf, hipStream_t st) {
    hipLaunchKernelGGL(k_clear_bail, dim3(1), dim3(64), 0, st, bf.scal);
}

// ---- d = -B delta on the free set, then Algorithm 2 ------------------------------------------------------

// Extra dense rows of the objective (at most kFoldMax of them) folded into the direction kernel: their products
// with both candidate directions ride along with the other sums, the last workgroup turns the selected one into the
// coefficient weight_r (e_r . p) of the row's contribution to the gradient change and into the curvature term
// sum weight_r (e_r . p)^2, and the update kernel adds coef_r e_r on the fly.  (A kernel of its own for this, one
// workgroup between the direction kernel and the pass over A, cost 9 us plus a launch gap per iteration.)
struct FoldArgs {
    int n_fold;              // 0: nothing folded
    const double* E;         // n_fold x n, row-major
    const double* weight;    // n_fold entries or NULL (= ones)
    double* coef;            // out: n_fold coefficients
    double* total;           // out: sum weight_r (e_r . p)^2
};

// Partial sums of the direction kernels -> Algorithm 2's choice between the two candidate directions (last workgroup).
__device__ __forceinline__ void dir_finish(double (&s)[6], double ub, double eps, Scal* __restrict__ scal,
                                           double* __restrict__ redpart, double* red, int* flag_p,
                                           double (&sx)[2 * kFoldMax], const FoldArgs& fold, int defer_choice = 0) {
    const int tid = threadIdx.x;
    block_sum<6, kWaves>(s, red);
    if (fold.n_fold > 0) block_sum<2 * kFoldMax, kWaves>(sx, red);
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
        for (int k = 0; k < 2 * kFoldMax; ++k) part[8 + k] = sx[k];
    }
    if (defer_choice) return;   // the consumer of the direction chooses between the candidates from the records
    if (!arrive_is_last(&scal->counters[kCntDir], flag_p)) return;
    double tx[2 * kFoldMax];
    {
        // the workgroups' partials, strided over the threads in a fixed order, then the fixed-order reductions
        double t6[6] = {0, 0, 0, 0, 0, 0};
        double tmin = INFINITY;
#pragma unroll
        for (int k = 0; k < 2 * kFoldMax; ++k) tx[k] = 0.0;
        for (int b = tid; b < (int)gridDim.x; b += kBlock) {
#pragma unroll
            for (int k = 0; k < 6; ++k) t6[k] += redpart[(int64_t)b * kDirRed + k];
            tmin = fmin(tmin, redpart[(int64_t)b * kDirRed + 6]);
            if (fold.n_fold > 0) {
#pragma unroll
                for (int k = 0; k < 2 * kFoldMax; ++k) tx[k] += redpart[(int64_t)b * kDirRed + 8 + k];
            }
        }
        block_sum<6, kWaves>(t6, red);
        if (fold.n_fold > 0) block_sum<2 * kFoldMax, kWaves>(tx, red);
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
        const int branch = (p1g <= -eps * p1p1 && p1p1 >= eps) ? 1 : 2;
        if (branch == 1) {
            scal->branch = 1; scal->gp = p1g; scal->alpha_ub = 1.0; scal->pp = p1p1; scal->xp = red[2];
        } else {
            scal->branch = 2; scal->gp = red[3]; scal->alpha_ub = red[6]; scal->pp = red[4]; scal->xp = red[5];
        }
        if (fold.n_fold > 0) {
            double total = 0.0;
#pragma unroll
            for (int r = 0; r < kFoldMax; ++r) {
                if (r < fold.n_fold) {
                    const double te = branch == 1 ? tx[2 * r] : tx[2 * r + 1];
                    const double wr = fold.weight ? fold.weight[r] : 1.0;
                    fold.coef[r] = wr * te;
                    total += wr * te * te;
                }
            }
            *fold.total = total;
        }
    }
}

// CLOSE: the wide Gram kernel before this one ended without its closing step (gram_blocks workgroups' partial sums in
// grampart).  Every workgroup here then does that step on a private copy of the scalar block: adds the partial sums in
// workgroup order, applies the pending update, runs Algorithm 3 on coefficients and the stopping test -- the same
// functions in the same order as the Gram kernel's last workgroup, so the same bits -- and takes the coefficients from
// its copy.  Workgroup 0 leaves its copy in scal_next for the pass (nothing in this kernel reads that); the scalar
// block itself is only read here.  What this saves is the Gram kernel's arrival (a fence, an atomic, a dependent round
// of loads) and this kernel's own dependent reads of the status word and the coefficients.
template <bool CLOSE>
__global__ __launch_bounds__(kBlock) void k_dir(int64_t n, int m, Opts op, const double* __restrict__ x,
                                                const double* __restrict__ g, const double* __restrict__ l,
                                                const double* __restrict__ u, const uint8_t* __restrict__ mask,
                                                const double* __restrict__ S, const double* __restrict__ Y,
                                                Scal* __restrict__ scal, double* __restrict__ d,
                                                double* __restrict__ p1, double* __restrict__ p2,
                                                double* __restrict__ redpart, int d_given, int store_d, FoldArgs fold,
                                                int defer_choice, const double* __restrict__ grampart, int gram_blocks,
                                                Scal* __restrict__ scal_next) {
    __shared__ double delta_s[kMaxV + 8];
    __shared__ const double* vecp[kMaxV + 8];
    __shared__ double red[kWaves * 7];
    __shared__ int flag;
    const int tid = threadIdx.x;
    // What depends on nothing the scalar block says is requested together with it: the coefficients (masked by the
    // number of vectors afterwards) and the first element's x, g, l, u and mask -- otherwise three dependent trips.
    const int64_t e_first = (int64_t)blockIdx.x * kBlock + tid;
    const int64_t e_safe = e_first < n ? e_first : n - 1;
    double xn = x[e_safe], gn = g[e_safe], ln = l[e_safe], un = u[e_safe];
    uint8_t mkn = mask[e_safe];
    int c, head;
    constexpr int kDirPre = CLOSE ? 2 * kWideM + 1 : 1;      // (the wide Gram kernel takes at most kWideM pairs)
    double vpre[kDirPre];
#pragma unroll
    for (int j = 0; j < kDirPre; ++j) vpre[j] = 0.0;
    if constexpr (CLOSE) {
        __shared__ Scal sc;
        __shared__ double Gs[(2 * kWideM + 2) * (2 * kWideM + 2)];
        __shared__ double tot[kWideNE];
        __shared__ double alpha_s[kMaxM + 1];
        constexpr int kScalWords = (int)(sizeof(Scal) / 4);
        for (int k = tid; k < kScalWords; k += kBlock)
            reinterpret_cast<int*>(&sc)[k] = reinterpret_cast<const int*>(scal)[k];
        gram_sum_partials_flat(grampart, kWideNE, gram_blocks, tot);
        __syncthreads();
        if (sc.status != LBFGSB_RUNNING) {
            // (the pass reads its status word from scal_next: it must not find an older one there)
            if (blockIdx.x == 0 && tid == 0) { scal_next->status = sc.status; scal_next->fresh = 0; }
            return;
        }
        head = sc.head; c = sc.count;
        if (sc.pend_valid) {                                       // same rule as effective_ring()
            if (sc.pend_ok) { head = (head + 1) % m; c = c < m ? c + 1 : m; }
            else c = 0;
        }
        const int base_slot = c > 0 ? (head - c + 2 * m) % m : 0;
        const double yn_old = prefetch_ynorm2(&sc, c, head, m);
        // the first element's vectors are requested now (which ring slots hold them is known), so that their trip to
        // memory runs under the closing step instead of behind it
        if (tid < kMaxV + 8) vecp[tid] = tid < 2 * c + 1 ? ring_vec(tid, c, head, m, n, S, Y, g) : g;
        __syncthreads();
        if (!d_given && mkn && e_first < n) {
#pragma unroll
            for (int j = 0; j < kDirPre; ++j) vpre[j] = j < 2 * c + 1 ? vecp[j][e_first] : 0.0;
        }
        __syncthreads();                                           // every thread has read the ring before it changes
        wide_finish(tot, Gs, alpha_s, &sc, m, c, head, base_slot, op, yn_old, 0, 1, blockIdx.x == 0);
        __syncthreads();                                           // the first wave's results are in the copy
        if (blockIdx.x == 0) {
            for (int k = tid; k < kScalWords; k += kBlock) {
                int v = reinterpret_cast<const int*>(&sc)[k];
                if (k == (int)(offsetof(Scal, fresh) / 4)) v = 1;
                reinterpret_cast<int*>(scal_next)[k] = v;
            }
        }
        if (sc.status != LBFGSB_RUNNING) return;
        c = sc.count; head = sc.head;                              // (as computed above: the update has been applied)
        const int V = 2 * c + 1;
        if (tid < kMaxV + 8) delta_s[tid] = tid < V ? sc.delta[tid] : 0.0;
    } else {
        const int status = scal->status;
        const double delta_raw = tid < kMaxV ? scal->delta[tid] : 0.0;
        if (status != LBFGSB_RUNNING) return;
        c = scal->count; head = scal->head;
        const int V = 2 * c + 1;
        if (tid < kMaxV + 8) {
            vecp[tid] = tid < V ? ring_vec(tid, c, head, m, n, S, Y, g) : g;
            delta_s[tid] = tid < V ? delta_raw : 0.0;
        }
    }
    const int V = 2 * c + 1;
    __syncthreads();
    double s[6] = {0, 0, 0, 0, 0, 0};
    double sx[2 * kFoldMax];
#pragma unroll
    for (int k = 0; k < 2 * kFoldMax; ++k) sx[k] = 0.0;
    double ub = INFINITY;
    for (int64_t e = e_first; e < n; e += (int64_t)gridDim.x * kBlock) {
        const double xe = xn, ge = gn, le = ln, ue = un;
        const uint8_t mk = mkn;
        {
            // the next element's, one trip ahead
            const int64_t e2 = e + (int64_t)gridDim.x * kBlock;
            const int64_t e2s = e2 < n ? e2 : n - 1;
            xn = x[e2s]; gn = g[e2s]; ln = l[e2s]; un = u[e2s]; mkn = mask[e2s];
        }
        double de;
        if (d_given) {
            de = d[e];
        } else {
            de = 0.0;
            if (mk) {
                double q = 0.0;
                if (CLOSE && e == e_first) {
                    // (same order of additions as below; entries past the last vector are zero times zero)
#pragma unroll
                    for (int j = 0; j < kDirPre; ++j) q = fma(delta_s[j], vpre[j], q);
                } else {
                    for (int j0 = 0; j0 < V; j0 += 8) {
                        double v[8];
#pragma unroll
                        for (int k = 0; k < 8; ++k) v[k] = j0 + k < V ? vecp[j0 + k][e] : 0.0;
#pragma unroll
                        for (int k = 0; k < 8; ++k) q = fma(delta_s[j0 + k], v[k], q);
                    }
                }
                de = -q;
            }
            if (store_d) d[e] = de;
        }
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
#pragma unroll
        for (int r = 0; r < kFoldMax; ++r) {
            if (r < fold.n_fold) {
                const double ev = fold.E[(int64_t)r * n + e];
                sx[2 * r] = fma(ev, a, sx[2 * r]);
                sx[2 * r + 1] = fma(ev, b, sx[2 * r + 1]);
            }
        }
    }
    dir_finish(s, ub, op.eps, scal, redpart, red, &flag, sx, fold, defer_choice);
}

// The same for long vectors (n even, from 2^17 entries on): two elements per lane through 16-byte accesses; lanes
// whose elements are fixed skip the pair memory.
typedef double dir_f64x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ void dir_element(double xe, double ge, double le, double ue, double de, double eps, double& a,
                                            double& b, double (&s)[6], double& ub) {
    a = clampd(xe + de, le, ue) - xe;
    b = de;
    if (de < 0.0 && xe <= le + eps) b = 0.0;
    if (de > 0.0 && xe >= ue - eps) b = 0.0;
    s[0] = fma(a, ge, s[0]); s[1] = fma(a, a, s[1]); s[2] = fma(xe, a, s[2]);
    s[3] = fma(b, ge, s[3]); s[4] = fma(b, b, s[4]); s[5] = fma(xe, b, s[5]);
    if (b > 0.0) ub = fmin(ub, (ue - xe) / b);
    else if (b < 0.0) ub = fmin(ub, (le - xe) / b);
}

__global__ __launch_bounds__(kBlock) void k_dir_pairs(int64_t n, int m, Opts op, const double* __restrict__ x,
                                                      const double* __restrict__ g, const double* __restrict__ l,
                                                      const double* __restrict__ u, const uint8_t* __restrict__ mask,
                                                      const double* __restrict__ S, const double* __restrict__ Y,
                                                      Scal* __restrict__ scal, double* __restrict__ d,
                                                      double* __restrict__ p1, double* __restrict__ p2,
                                                      double* __restrict__ redpart, int d_given, int store_d,
                                                      int defer_choice) {
    __shared__ double delta_s[kMaxV + 24];
    __shared__ double red[kWaves * 7];
    __shared__ int flag;
    if (scal->status != LBFGSB_RUNNING) return;
    const int tid = threadIdx.x;
    const int c = scal->count, head = scal->head;
    const int V = 2 * c + 1;
    if (tid < kMaxV + 24) delta_s[tid] = tid < V ? scal->delta[tid] : 0.0;
    __syncthreads();
    double s[6] = {0, 0, 0, 0, 0, 0};
    double ub = INFINITY;
    const int64_t nchunks = (n + 2 * kBlock - 1) / (2 * kBlock);
    // the mask decides which lanes read the pair memory at all, so it (with x, g, l, u) is fetched one chunk ahead
    auto pair_index = [&](int64_t ch, bool& in) -> int64_t {
        const int64_t e = ch * (2 * kBlock) + 2 * tid;
        in = ch < nchunks && e < n;                              // n is even: both elements or neither
        return in ? e : n - 2;
    };
    bool in_next;
    int64_t ec_next = pair_index(blockIdx.x, in_next);
    const bool ub_same = op.uniform_bounds != 0;                 // same bounds everywhere: l and u are not streamed
    dir_f64x2 xn = *reinterpret_cast<const dir_f64x2*>(x + ec_next), gn = *reinterpret_cast<const dir_f64x2*>(g + ec_next);
    dir_f64x2 ln = dir_f64x2{op.lo, op.lo}, un = dir_f64x2{op.hi, op.hi};
    if (!ub_same) { ln = *reinterpret_cast<const dir_f64x2*>(l + ec_next); un = *reinterpret_cast<const dir_f64x2*>(u + ec_next); }
    unsigned short mkn = *reinterpret_cast<const unsigned short*>(mask + ec_next);
    for (int64_t ch = blockIdx.x; ch < nchunks; ch += gridDim.x) {
        const bool in = in_next;
        const int64_t ec = ec_next, e = ec_next;
        const dir_f64x2 xe = xn, ge = gn, le = ln, ue = un;
        const unsigned short mk = in ? mkn : (unsigned short)0;
        ec_next = pair_index(ch + gridDim.x, in_next);
        xn = *reinterpret_cast<const dir_f64x2*>(x + ec_next); gn = *reinterpret_cast<const dir_f64x2*>(g + ec_next);
        if (!ub_same) { ln = *reinterpret_cast<const dir_f64x2*>(l + ec_next); un = *reinterpret_cast<const dir_f64x2*>(u + ec_next); }
        mkn = *reinterpret_cast<const unsigned short*>(mask + ec_next);
        dir_f64x2 de;
        if (d_given) {
            de = *reinterpret_cast<const dir_f64x2*>(d + ec);
        } else {
            double q0 = 0.0, q1 = 0.0;
            if (mk != 0) {                                       // lanes whose two elements are both fixed read nothing
                // 24 vectors per round: with m <= 11 every load of an element is in flight at once
                for (int j0 = 0; j0 < V; j0 += 24) {
                    dir_f64x2 v[24];
#pragma unroll
                    for (int k = 0; k < 24; ++k) {
                        v[k] = dir_f64x2{0.0, 0.0};
                        if (j0 + k < V) v[k] = *reinterpret_cast<const dir_f64x2*>(ring_vec(j0 + k, c, head, m, n, S, Y, g) + ec);
                    }
#pragma unroll
                    for (int k = 0; k < 24; ++k) {
                        q0 = fma(delta_s[j0 + k], v[k].x, q0);
                        q1 = fma(delta_s[j0 + k], v[k].y, q1);
                    }
                }
            }
            de.x = (mk & 0xffu) ? -q0 : 0.0;
            de.y = (mk >> 8) ? -q1 : 0.0;
            if (in && store_d) *reinterpret_cast<dir_f64x2*>(d + e) = de;
        }
        if (in) {
            double a0, b0, a1, b1;
            dir_element(xe.x, ge.x, le.x, ue.x, de.x, op.eps, a0, b0, s, ub);
            dir_element(xe.y, ge.y, le.y, ue.y, de.y, op.eps, a1, b1, s, ub);
            *reinterpret_cast<dir_f64x2*>(p1 + e) = dir_f64x2{a0, a1};
            *reinterpret_cast<dir_f64x2*>(p2 + e) = dir_f64x2{b0, b1};
        }
    }
    double sx[2 * kFoldMax];
#pragma unroll
    for (int k = 0; k < 2 * kFoldMax; ++k) sx[k] = 0.0;
    dir_finish(s, ub, op.eps, scal, redpart, red, &flag, sx, FoldArgs{0, nullptr, nullptr, nullptr, nullptr}, defer_choice);
}

// extra rows can ride along with the direction kernel for short vectors only
bool dir_folds_extra_rows(const Dims& dm) {
    return dm.n_extra > 0 && dm.n_extra <= kFoldMax && !(dm.n >= (1 << 17) && dm.n % 2 == 0);
}

void launch_dir(const Dims& dm, const Opts& op, const Geometry& ge, const Buffers& bf, int d_given, int store_d,
                hipStream_t st, const double* fold_rows, const double* fold_weight, int defer_choice, int gram_blocks) {
    FoldArgs fold{0, nullptr, nullptr, nullptr, nullptr};
    if (fold_rows && dir_folds_extra_rows(dm)) fold = FoldArgs{dm.n_extra, fold_rows, fold_weight, bf.wextra, bf.xres + dm.n_extra};
    if (dm.n >= (1 << 17) && dm.n % 2 == 0) {
        hipLaunchKernelGGL(k_dir_pairs, dim3(ge.dir_blocks), dim3(kBlock), 0, st, dm.n, dm.m, op, bf.x, bf.g, bf.l, bf.u,
                           bf.mask, bf.S, bf.Y, bf.scal, bf.d, bf.p1, bf.p2, bf.redpart, d_given, store_d, defer_choice);
        return;
    }
    if (gram_blocks > 0) {
        hipLaunchKernelGGL(k_dir<true>, dim3(ge.dir_blocks), dim3(kBlock), 0, st, dm.n, dm.m, op, bf.x, bf.g, bf.l, bf.u,
                           bf.mask, bf.S, bf.Y, bf.scal, bf.d, bf.p1, bf.p2, bf.redpart, d_given, store_d, fold, defer_choice,
                           (const double*)bf.grampart, gram_blocks, bf.scal_next);
        return;
    }
    hipLaunchKernelGGL(k_dir<false>, dim3(ge.dir_blocks), dim3(kBlock), 0, st, dm.n, dm.m, op, bf.x, bf.g, bf.l, bf.u,
                       bf.mask, bf.S, bf.Y, bf.scal, bf.d, bf.p1, bf.p2, bf.redpart, d_given, store_d, fold, defer_choice,
                       (const double*)nullptr, 0, (Scal*)nullptr);
}

// ---- after an evaluation pass: g and f ------------------------------------------------------------------

__global__ __launch_bounds__(kBlock) void k_eval_finish(Dims dm, int w_parts, int loss_parts,
                                                        const double* __restrict__ wpart,
                                                        const double* __restrict__ losspart,
                                                        const double* __restrict__ x, double* __restrict__ g,
                                                        Scal* __restrict__ scal, double* __restrict__ redpart,
                                                        const double* __restrict__ lin, const double* __restrict__ sign,
                                                        const double* __restrict__ wextra,
                                                        const double* __restrict__ xres) {
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
            // wextra: the extra rows' contribution E^T (weight * residual), one entry per variable
            if (dm.kind == LBFGSB_OBJ_LSQ) {
                g[c] = w + (wextra ? wextra[c] : 0.0);
            } else if (dm.kind == LBFGSB_OBJ_LSQ_L1SPLIT) {
                g[c] = w + dm.lambda + (wextra ? wextra[c] : 0.0);
                g[c + dm.cols] = -w + dm.lambda + (wextra ? wextra[c + dm.cols] : 0.0);
                reg += x[c] + x[c + dm.cols];
            } else if (dm.kind == LBFGSB_OBJ_QP) {
                // w = (A (s.x))_c (a single "partial": the row kernel's output); g = s w + b, f = loss + b.x
                g[c] = (sign ? sign[c] : 1.0) * w + lin[c] + (wextra ? wextra[c] : 0.0);
                reg = fma(lin[c], x[c], reg);
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
        else if (dm.kind == LBFGSB_OBJ_QP) f += regt;
        if (xres) f += xres[dm.n_extra];   // 0.5 sum weight * residual^2 of the extra rows
        scal->f = f;
        scal->fevals += 1;
    }
}

void launch_eval_finish(const Dims& dm, const Geometry& ge, const Buffers& bf, const double* lin, const double* sign,
                        hipStream_t st) {
    const bool qp = dm.kind == LBFGSB_OBJ_QP;
    hipLaunchKernelGGL(k_eval_finish, dim3(ge.fin_blocks), dim3(kBlock), 0, st, dm, qp ? 1 : ge.w_parts, ge.loss_parts,
                       qp ? (const double*)bf.row : (const double*)bf.wpart, bf.losspart, bf.x, bf.g, bf.scal, bf.redpart,
                       lin, sign, dm.n_extra > 0 ? (const double*)bf.wextra : nullptr,
                       dm.n_extra > 0 ? (const double*)bf.xres : nullptr);
}

// ---- quadratic objectives: closed-form Armijo search, then the update ---------------------------------------
//
// With t = A v_p and w = A^T t from the direction pass:  f(x + a p) - f(x) = a <g,p> + a^2/2 ||t||^2,
// gradient g + a w~ (w~ = w, or [w; -w] for the split form), y = a w~.  The residual is not carried
// along: nothing in the iteration reads it, and an evaluation from x recomputes it.
// The Armijo inequality  a gp + a^2/2 tt <= c1 a gp  is tested after division by a > 0.
__global__ __launch_bounds__(kBlock) void k_update_quadratic(Dims dm, Opts op, int w_parts, int loss_parts,
                                                             const double* __restrict__ wpart,
                                                             const double* __restrict__ losspart,
                                                             const double* __restrict__ p1,
                                                             const double* __restrict__ p2,
                                                             const double* __restrict__ l, const double* __restrict__ u,
                                                             double* __restrict__ x, double* __restrict__ g,
                                                             double* __restrict__ S, double* __restrict__ Y,
                                                             Scal* __restrict__ scal, const double* __restrict__ sign,
                                                             const double* __restrict__ wextra,
                                                             const double* __restrict__ xres, int n_fold,
                                                             const double* __restrict__ fold_rows,
                                                             const double* __restrict__ fold_weight,
                                                             const double* __restrict__ dir_part, int dir_blocks) {
    __shared__ double lds[kBlock];
    __shared__ double red[kWaves];
    __shared__ double ls_alpha;
    __shared__ int ls_ok, ls_bt;
    __shared__ double fold_s[kFoldMax + 1];   // folded rows: coefficients weight_r (e_r . p), then sum weight_r (e_r . p)^2
    if (scal->status != LBFGSB_RUNNING) return;
    const int tid = threadIdx.x;
    const double gp = scal->gp, alpha_ub = scal->alpha_ub, f_old = scal->f;
    const int slot = scal->head;
    const int branch = scal->branch;
    const double* p = branch == 1 ? p1 : p2;
    const bool own_fold = n_fold > 0 && dir_blocks > 0;
    if (own_fold) {
        // the direction kernel left only its per-workgroup sums: the first wave adds the folded rows' products with
        // the chosen candidate (every workgroup the same bits)
        if (tid < 64) {
            double tx[2 * kFoldMax];
            dir_fold_from_partials(dir_part, dir_blocks, tx);
            if (tid == 0) {
                double total = 0.0;
#pragma unroll
                for (int r = 0; r < kFoldMax; ++r) {
                    double cr = 0.0;
                    if (r < n_fold) {
                        const double te = branch == 1 ? tx[2 * r] : tx[2 * r + 1];
                        const double wr = fold_weight ? fold_weight[r] : 1.0;
                        cr = wr * te;
                        total += wr * te * te;
                    }
                    fold_s[r] = cr;
                }
                fold_s[kFoldMax] = total;
            }
        }
        __syncthreads();
    }
    // curvature along p: ||t||^2 (weighted) from the A pass, plus the extra rows' sum weight (e_r.p)^2
    const double tt = sum_all(losspart, loss_parts, red) + (own_fold ? fold_s[kFoldMax] : (xres ? xres[dm.n_extra] : 0.0));
    if (tid == 0) {
        double a = fmin(1.0, alpha_ub);
        int ok = 0, bt = 0;
        for (int k = 0; k <= op.max_backtracks; ++k) {
            const double lhs = gp + 0.5 * a * tt;          // (f(x + a p) - f(x)) / a
            if (isfinite(a * lhs) && lhs <= op.c1 * gp) { ok = 1; bt = k; break; }
            a *= op.backtrack;
        }
        ls_alpha = a; ls_ok = ok; ls_bt = ok ? bt : op.max_backtracks + 1;
    }
    __syncthreads();
    const double alpha = ls_alpha;
    const int ok = ls_ok;
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
                    double wi = h ? -w : w;
                    if (sign) wi *= sign[i];               // QP: the change of the gradient is s.(A (s.p))
                    if (n_fold > 0) {                       // folded extra rows: wextra[0 .. n_fold) holds their coefficients
                        for (int r = 0; r < n_fold; ++r) wi = fma(own_fold ? fold_s[r] : wextra[r], fold_rows[(int64_t)r * dm.n + i], wi);
                    } else if (wextra) {
                        wi += wextra[i];
                    }
                    const double y = alpha * wi;
                    const double xi = x[i];
                    const double xn = clampd(fma(alpha, p[i], xi), l[i], u[i]);
                    Sn[i] = xn - xi;
                    Yn[i] = y;
                    x[i] = xn;
                    g[i] += y;
                }
            }
        }
    }
    // No workgroup of this kernel reads the pend_* fields, so one thread may write them while others
    // are still running; the next Gram kernel (or k_commit) turns them into head/count/iters/f.
    if (blockIdx.x == 0 && tid == 0) {
        scal->pend_ok = ok;
        scal->pend_bt = ls_bt;
        scal->pend_alpha = alpha;
        scal->pend_f = f_old + alpha * (gp + 0.5 * alpha * tt);
        scal->pend_valid = 1;
    }
}

void launch_update_quadratic(const Dims& dm, const Opts& op, const Geometry& ge, const Buffers& bf, const double* sign,
                             hipStream_t st, const double* fold_rows, const double* fold_weight, int dir_blocks) {
    const int n_fold = fold_rows && dir_folds_extra_rows(dm) ? dm.n_extra : 0;
    const bool qp = dm.kind == LBFGSB_OBJ_QP;   // its "partial columns" are the single vector t = A (s.p)
    hipLaunchKernelGGL(k_update_quadratic, dim3(ge.upd_blocks), dim3(kBlock), 0, st, dm, op, qp ? 1 : ge.w_parts,
                       ge.loss_parts, qp ? (const double*)bf.t : (const double*)bf.wpart, bf.losspart, bf.p1, bf.p2, bf.l,
                       bf.u, bf.x, bf.g, bf.S, bf.Y, bf.scal, qp ? sign : nullptr,
                       dm.n_extra > 0 ? (const double*)bf.wextra : nullptr,
                       dm.n_extra > 0 ? (const double*)bf.xres : nullptr, n_fold, fold_rows, fold_weight,
                       (const double*)bf.redpart, n_fold > 0 ? dir_blocks : 0);
}

// ---- extra dense rows ------------------------------------------------------------------------------------
//
// One workgroup.  z = x (eval) or the direction Algorithm 2 selected.  te_r = e_r . z; coefficient
// c_r = weight_r (te_r - target_r) (eval) or weight_r te_r (direction);
//   wextra[i] = sum_r c_r E[r][i],   xres[r] = te_r - target_r (eval only),
//   xres[n_extra] = 0.5 sum weight_r (te_r - target_r)^2 (eval)  or  sum weight_r te_r^2 (direction).
__global__ __launch_bounds__(kBlock) void k_extra_rows(Dims dm, const double* __restrict__ E,
                                                       const double* __restrict__ target,
                                                       const double* __restrict__ weight, int eval,
                                                       const double* __restrict__ x, const double* __restrict__ p1,
                                                       const double* __restrict__ p2, const Scal* __restrict__ scal,
                                                       double* __restrict__ wextra, double* __restrict__ xres) {
    __shared__ double red[kWaves];
    __shared__ double coef[kMaxExtra];
    if (!eval && scal->status != LBFGSB_RUNNING) return;
    const int tid = threadIdx.x;
    const double* z = eval ? x : (scal->branch == 1 ? p1 : p2);
    double total = 0.0;
    for (int r = 0; r < dm.n_extra; ++r) {
        double s[1] = {0.0};
        const double* er = E + (int64_t)r * dm.n;
        for (int64_t i0 = tid; i0 < dm.n; i0 += kBlock * 8) {   // 16 loads in flight per thread: the kernel is latency-bound
            double ev[8], zv[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int64_t i = i0 + (int64_t)k * kBlock;
                ev[k] = i < dm.n ? er[i] : 0.0;
                zv[k] = i < dm.n ? z[i] : 0.0;
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) s[0] = fma(ev[k], zv[k], s[0]);
        }
        block_sum<1, kWaves>(s, red);
        const double wr = weight ? weight[r] : 1.0;
        const double res = eval ? s[0] - target[r] : s[0];
        total += (eval ? 0.5 : 1.0) * wr * res * res;
        if (tid == 0) {
            coef[r] = wr * res;
            if (eval) xres[r] = res;
        }
    }
    __syncthreads();
    for (int64_t i0 = tid; i0 < dm.n; i0 += kBlock * 8) {
        double acc[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) acc[k] = 0.0;
        for (int r = 0; r < dm.n_extra; ++r) {
            double ev[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int64_t i = i0 + (int64_t)k * kBlock;
                ev[k] = i < dm.n ? E[(int64_t)r * dm.n + i] : 0.0;
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) acc[k] = fma(coef[r], ev[k], acc[k]);
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int64_t i = i0 + (int64_t)k * kBlock;
            if (i < dm.n) wextra[i] = acc[k];
        }
    }
    if (tid == 0) xres[dm.n_extra] = total;
}

void launch_extra_rows(const Dims& dm, const Buffers& bf, const double* rows, const double* target, const double* weight,
                       int eval, hipStream_t st) {
    hipLaunchKernelGGL(k_extra_rows, dim3(1), dim3(kBlock), 0, st, dm, rows, target, weight, eval, bf.x, bf.p1, bf.p2,
                       (const Scal*)bf.scal, bf.wextra, bf.xres);
}

// ---- logistic objective: line search on the margins --------------------------------------------------------
//
// With z = X w (kept in `row`) and t = X p:  f(x + a p) - f(x) = (1/N) sum_r [softplus(-y_r (z_r + a t_r))
// - softplus(-y_r z_r)] + mu (a <x,p> + a^2/2 <p,p>).  The bracket is evaluated in the cancellation-free
// form log(1 + sigmoid(q) expm1(dq)), q = -y z, dq = -y a t (softplus_diff).  Step lengths are evaluated NTRY at a time per sweep
// over the rows: the first launch tries the first one alone (it is accepted in almost every quasi-Newton
// iteration; the short launch sequence has the pass over X form that sum itself and the update kernel decide,
// see k_update_logistic), a second launch, which returns at once when the first found the step, tries the next kLsBatch, and
// if none of them is acceptable its last workgroup goes on alone, one length at a time.
template <int NTRY>
__global__ __launch_bounds__(kBlock) void k_ls_logistic(Dims dm, Opts op, int first, int last_resort, int spec,
                                                        const double* __restrict__ yl, const double* __restrict__ z,
                                                        const double* __restrict__ t, Scal* __restrict__ scal,
                                                        double* __restrict__ lspart) {
    __shared__ double red[kWaves * NTRY];
    __shared__ int flag;
    if (scal->status != LBFGSB_RUNNING) return;
    if (first > 0 && scal->ls_ok) return;            // an earlier launch of this iteration found the step
    const int tid = threadIdx.x;
    double al[NTRY], s[NTRY];
    {
        double a = fmin(1.0, scal->alpha_ub);
        for (int k = 0; k < first; ++k) a *= op.backtrack;
#pragma unroll
        for (int j = 0; j < NTRY; ++j) { al[j] = a; s[j] = 0.0; a *= op.backtrack; }
    }
    // four rows per trip: the transcendental chains of different rows are independent, and the few waves of this
    // kernel are latency-bound, so interleaving them is what shortens it
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    for (int64_t r0 = (int64_t)blockIdx.x * kBlock + tid; r0 < dm.rows; r0 += 4 * stride) {
        double q[4], sq[4], ty[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int64_t r = r0 + k * stride;
            const bool in = r < dm.rows;
            const double y = in ? yl[r] : 0.0;          // y = 0: q = ty = 0, the row contributes log1p(0.5 * expm1(0)) = 0
            q[k] = -y * (in ? z[r] : 0.0);
            ty[k] = -y * (in ? t[r] : 0.0);
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) sq[k] = sigmoid_d(q[k]);
#pragma unroll
        for (int j = 0; j < NTRY; ++j) {
#pragma unroll
            for (int k = 0; k < 4; ++k) s[j] += softplus_diff(q[k], sq[k], al[j] * ty[k]);
        }
    }
    block_sum<NTRY, kWaves>(s, red);
    if (tid == 0) {
#pragma unroll
        for (int j = 0; j < NTRY; ++j) lspart[(int64_t)blockIdx.x * NTRY + j] = s[j];
    }
    if (!arrive_is_last(&scal->counters[kCntLs], &flag)) return;
    const double gp = scal->gp, xp = scal->xp, pp = scal->pp;
    const double invn = 1.0 / (double)dm.rows;
    // totals of the batch
    double tot[NTRY];
#pragma unroll
    for (int j = 0; j < NTRY; ++j) tot[j] = 0.0;
    for (int b = tid; b < (int)gridDim.x; b += kBlock) {
#pragma unroll
        for (int j = 0; j < NTRY; ++j) tot[j] += lspart[(int64_t)b * NTRY + j];
    }
    block_sum<NTRY, kWaves>(tot, red);
    int found = -1;
    double a_acc = 0.0;
#pragma unroll
    for (int j = 0; j < NTRY; ++j) {
        const double df = tot[j] * invn + dm.mu * al[j] * (xp + 0.5 * al[j] * pp);
        if (found < 0 && first + j <= op.max_backtracks && isfinite(df) && df <= op.c1 * al[j] * gp) { found = first + j; a_acc = al[j]; }
    }
    // rare: continue one step length at a time (uniform control flow: every thread holds the same totals)
    double a = al[NTRY - 1];
    for (int k = first + NTRY; last_resort && found < 0 && k <= op.max_backtracks; ++k) {
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
        if (first == 0) scal->spec_ok = spec && found == 0;
        if (found >= 0 || last_resort) {
            scal->backtracks = found >= 0 ? found : op.max_backtracks + 1;
            scal->fevals += found >= 0 ? found + 1 : op.max_backtracks + 1;
        }
        if (found >= 0) scal->alpha = a_acc;
    }
}

void launch_ls_logistic(const Dims& dm, const Opts& op, const Geometry& ge, const Buffers& bf, const double* labels,
                        int spec, int stages, hipStream_t st) {
    if (stages & 1)
        hipLaunchKernelGGL(k_ls_logistic<1>, dim3(ge.ls_blocks), dim3(kBlock), 0, st, dm, op, 0, 0, spec, labels, (const double*)bf.row, (const double*)bf.t, bf.scal, bf.lspart);
    if (stages & 2)
        hipLaunchKernelGGL(k_ls_logistic<kLsBatch>, dim3(ge.ls_blocks), dim3(kBlock), 0, st, dm, op, 1, 1, spec, labels,
                           (const double*)bf.row, (const double*)bf.t, bf.scal, bf.lspart);
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
    hipLaunchKernelGGL(k_rows_logistic, dim3(ge.lrows_blocks), dim3(kBlock), 0, st, dm, labels, bf.t, bf.row, bf.psi, bf.scal,
                       bf.losspart);
}

// x+ = P(x + alpha p), g+ = X^T psi + mu x+, pair (x+ - x, g+ - g), f+ from the new margins.
// short_seq: the pass over X has left, in its loss partials, the sums over its workgroups' rows of
// softplus(-y (z + a0 t)) - softplus(-y z) for the first trial step a0 = min(1, alpha_ub).  Every workgroup adds
// them in the same order and takes the same Armijo decision; an accepted step is applied here (the margins move
// too), a rejected one parks the solver (kStatusBail) with nothing changed and no arrival counted.
__global__ __launch_bounds__(kBlock) void k_update_logistic(Dims dm, double c1, int w_parts_two_pass, int w_parts_spec,
                                                            int loss_parts, int short_seq, const double* __restrict__ t,
                                                            double* __restrict__ z, const double* __restrict__ wpart,
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
    int ok = scal->ls_ok;
    double alpha = scal->alpha;
    const int slot = scal->head;
    const double* p = scal->branch == 1 ? p1 : p2;
    int w_parts = scal->spec_ok ? w_parts_spec : w_parts_two_pass;   // which kernel wrote the partial columns
    double df = 0.0, f_old = 0.0;
    if (short_seq) {
        const double gp = scal->gp, xp = scal->xp, pp = scal->pp;
        f_old = scal->f;
        alpha = fmin(1.0, scal->alpha_ub);
        df = sum_all(losspart, loss_parts, red) / (double)dm.rows + dm.mu * alpha * (xp + 0.5 * alpha * pp);
        ok = isfinite(df) && df <= c1 * alpha * gp;
        w_parts = w_parts_spec;
        if (!ok) {
            // (a workgroup that starts after this store finds the solver parked and returns at once: same outcome)
            if (blockIdx.x == 0 && tid == 0) {
                scal->ls_ok = 0;
                scal->spec_ok = 0;
                scal->status = kStatusBail;
            }
            return;
        }
    }
    double sums[2] = {0.0, 0.0};   // ||y||^2, ||x+||^2
    // short sequence: the first `col_blocks` workgroups take the columns, the others the margins (side by side, not
    // one after the other: a workgroup's trips to memory are dependent and nothing else runs on its compute unit);
    // a grid of one workgroup does both
    int col_first = 0, col_stride = (int)gridDim.x;
    if (ok && short_seq) {
        // the margins of the new point (the full sequence has a kernel for this, which also recomputes the row weights:
        // here the single-read pass already holds X^T psi of this step)
        const int want = (int)((dm.cols + kCX - 1) / kCX);
        const int col_blocks = want < (int)gridDim.x / 2 ? want : (int)gridDim.x / 2;
        int rb = (int)blockIdx.x, nrb = (int)gridDim.x;
        if (col_blocks > 0) {
            col_stride = col_blocks;
            if ((int)blockIdx.x >= col_blocks) col_first = -1;   // this workgroup takes no columns
            rb = (int)blockIdx.x - col_blocks;                   // (negative: no rows)
            nrb = (int)gridDim.x - col_blocks;
        }
        if (rb >= 0) {
            // (four rows per trip with their loads issued together)
            const int64_t stride = (int64_t)nrb * kBlock;
            for (int64_t r0 = (int64_t)rb * kBlock + tid; r0 < dm.rows; r0 += 4 * stride) {
                double tv[4], zv[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int64_t r = r0 + k * stride;
                    tv[k] = r < dm.rows ? t[r] : 0.0;
                    zv[k] = r < dm.rows ? z[r] : 0.0;
                }
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int64_t r = r0 + k * stride;
                    if (r < dm.rows) z[r] = fma(alpha, tv[k], zv[k]);
                }
            }
        }
    }
    if (ok && col_first >= 0) {
        double* Sn = S + (int64_t)slot * dm.n;
        double* Yn = Y + (int64_t)slot * dm.n;
        for (int64_t c0 = (int64_t)blockIdx.x * kCX; c0 < dm.cols; c0 += (int64_t)col_stride * kCX) {
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
    if (short_seq) {
        // Nothing is left to add up: f moves by the line search's difference, and the new pair's ||y||^2 comes from
        // the next free-set pass (as for the quadratic kinds).  No workgroup of this kernel reads the pend_* fields,
        // so one thread may write them while others are still running; the next Gram kernel (or k_commit) turns
        // them into head/count/iters/f.  Without an arrival at one address the grid need not stay small.
        if (blockIdx.x == 0 && tid == 0) {
            scal->spec_ok = 1;
            scal->pend_ok = 1;
            scal->pend_bt = 0;
            scal->pend_alpha = alpha;
            scal->pend_f = f_old + df;
            scal->pend_valid = 1;
        }
        return;
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
            // f from the new margins and the new iterate
            scal->f = loss + 0.5 * dm.mu * tot[1];
            scal->ynorm2[slot] = tot[0];
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

void launch_update_logistic(const Dims& dm, const Opts& op, const Geometry& ge, const Buffers& bf, int loss_parts,
                            int short_seq, hipStream_t st) {
    hipLaunchKernelGGL(k_update_logistic, dim3(short_seq ? ge.updl_blocks : ge.upd_blocks), dim3(kBlock), 0, st, dm, op.c1, ge.gemvt_row_blocks,
                       ge.fused_blocks, loss_parts, short_seq, (const double*)bf.t, bf.row, bf.wpart,
                       bf.losspart, bf.p1, bf.p2, bf.l, bf.u, bf.x, bf.g, bf.S, bf.Y, bf.scal, bf.redpart);
}

}  // namespace lb
