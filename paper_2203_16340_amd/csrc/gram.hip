// Free set (Eq. (ws)), masked Gram matrix of the stored pairs and the gradient, and the modified
// two-loop recursion (Algorithm 3) carried out on coefficients.
//
// Batched form of Algorithm 3.  Let b_0..b_{V-1} = s^0[S]..s^{c-1}[S], y^0[S]..y^{c-1}[S], g[S]
// (c stored pairs, oldest first, S the current free set) and G = B^T B.  Every vector the recursion
// forms is B*delta for some coefficient vector delta, and every dot product it needs is an entry of
// G*delta.  Written out, with rho_i = G[s_i][y_i], pass_i = rho_i > eps*||y^i||^2 (full norm):
//   first loop  (i = c-1 .. 0):  alpha_i = (G[s_i][g] - sum_{k>i} alpha_k G[s_i][y_k]) / rho_i
//   scaling:                     gamma = rho_{c-1}/||y^{c-1}||^2 if pass_{c-1}, else 1
//   second loop (i = 0 .. c-1):  beta_i = (gamma (G[y_i][g] - sum_k alpha_k G[y_i][y_k])
//                                          + sum_{k<i} (alpha_k - beta_k) G[y_i][s_k]) / rho_i
//   result:  q = gamma g - gamma sum_k alpha_k y_k + sum_k (alpha_k - beta_k) s_k,  d = -q on S
// (pairs that fail the gate have alpha = beta = 0).  Both loops are triangular solves; lane i of one
// wave owns row i, so a step is one broadcast and one multiply-add, with no cross-lane reduction.
// G must be rebuilt every iteration because S changes; it costs one pass over the 2c+1 vectors.
#include <cstddef>

#include "common.h"

#ifdef LB_PROFILE_GRAM
#define LB_TICK(i) do { if (threadIdx.x == 0) ticks[i] = wall_clock64(); } while (0)
#else
#define LB_TICK(i) do {} while (0)
#endif

namespace lb {

namespace {
constexpr int kStageMax = 32;   // vectors one thread stages per chunk
constexpr int kHdr = 8;         // per-workgroup partial: [0] sum g[S]^2, [1] max KKT residual, [2] #fixed, [3] ||y_new||^2
constexpr int kTPT = 3;         // tiles per thread when there are more 2x2 tiles than threads (<= 528)

__host__ __device__ inline int gram_tiles(int V) {
    const int T = (V + 1) / 2;
    return T * (T + 1) / 2;
}
}  // namespace

int gram_entries(int m) { return kHdr + 4 * gram_tiles(2 * m + 1); }

// elements staged per chunk: as many as a 60 KiB tile [chunk][2m+2] allows
int gram_chunk(int m) {
    const int vp = 2 * m + 2;
    return vp <= 30 ? 256 : (vp <= 60 ? 128 : 64);
}
size_t gram_lds_bytes(int m) {
    size_t d = (size_t)gram_chunk(m) * (2 * m + 2);
    if (d < 1024) d = 1024;
    return d * 8;
}
// Few workgroups keep the last one's sum over the partials short, which is what matters while the vectors are
// short; from 2^17 entries on, reading the vectors dominates and the whole chip is put to it.
int gram_blocks_for(int64_t n, int m) {
    const int e = gram_chunk(m);
    int64_t b = (n + e - 1) / e;
    const int64_t cap = n >= (1 << 17) ? 512 : 128;
    return (int)(b < 1 ? 1 : (b > cap ? cap : b));
}

// value of v in lane l (l uniform across the wave): a scalar-register read, not a trip through LDS
__device__ __forceinline__ double lane_value(double v, int l) {
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), l);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), l);
    return __hiloint2double(hi, lo);
}

__device__ __forceinline__ void tile_of(int q, int T, int& ti, int& tj) {
    int a = 0;
    while (q >= T - a) { q -= T - a; ++a; }
    ti = a; tj = a + q;
}

__global__ __launch_bounds__(kBlock) void k_gram(int64_t n, int m, int E, Opts op, const double* __restrict__ x,
                                                 const double* __restrict__ g, const double* __restrict__ l,
                                                 const double* __restrict__ u, const double* __restrict__ S,
                                                 const double* __restrict__ Y, uint8_t* __restrict__ mask,
                                                 Scal* __restrict__ scal, double* __restrict__ grampart, int NE,
                                                 int dbg_inputs, int evaluate_stop) {
    extern __shared__ __align__(16) double dyn[];   // staged chunk [element][vector]; later scratch and G
    __shared__ double red[kWaves * 4];
    __shared__ double alpha_s[kMaxM + 1];
    __shared__ int flag;

#ifdef LB_PROFILE_GRAM
    __shared__ unsigned long long ticks[16];
#endif
    LB_TICK(0);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // one load per wave fetches the integer header of the scalar block (status, ring position, pending
    // update); readlanes hand the fields to every lane
    static_assert(offsetof(Scal, pend_ok) < 64, "header fields must sit in the first 16 ints");
    const int hdr = lane < 16 ? reinterpret_cast<const int*>(scal)[lane] : 0;
    if (__shfl(hdr, offsetof(Scal, status) / 4) != LBFGSB_RUNNING) return;
    int head = __shfl(hdr, offsetof(Scal, head) / 4), c = __shfl(hdr, offsetof(Scal, count) / 4);
    if (__shfl(hdr, offsetof(Scal, pend_valid) / 4)) {          // same rule as effective_ring()
        if (__shfl(hdr, offsetof(Scal, pend_ok) / 4)) { head = (head + 1) % m; c = c < m ? c + 1 : m; }
        else c = 0;
    }
    const int V = 2 * c + 1;
    const int Vp = V + 1;
    const int T = Vp / 2;
    const int TT = T * (T + 1) / 2;
    const int jnew = 2 * c - 1;   // newest y (none when c == 0)
    const int base_slot = c > 0 ? (head - c + 2 * m) % m : 0;   // ring slot of the oldest pair
    auto vec_ptr = [&](int j) -> const double* {
        if (j >= 2 * c) return g;
        const bool is_y = j >= c;
        int sl = base_slot + (is_y ? j - c : j);
        if (sl >= m) sl -= m;
        return (is_y ? Y : S) + (int64_t)sl * n;
    };

    // which 2x2 tiles of G this thread accumulates, and over which elements of a chunk
    const bool split = TT <= kBlock;                  // several threads share a tile, each takes a slice of the elements
    const int groups = split ? kBlock / TT : 1;
    const int h = split ? tid / TT : 0;
    int ti[kTPT], tj[kTPT];
    double acc[kTPT][4];
#pragma unroll
    for (int k = 0; k < kTPT; ++k) {
        const int q = split ? (k == 0 && h < groups ? tid % TT : -1) : (tid + k * kBlock < TT ? tid + k * kBlock : -1);
        if (q >= 0) tile_of(q, T, ti[k], tj[k]); else { ti[k] = -1; tj[k] = 0; }
        acc[k][0] = acc[k][1] = acc[k][2] = acc[k][3] = 0.0;
    }
    double pg2 = 0.0, pginf = 0.0, nfixed = 0.0, ynew = 0.0;
    const int ngrp = kBlock / E;
    const int el = tid % E, grp = tid / E;
    __syncthreads();
    LB_TICK(1);

    for (int64_t e0 = (int64_t)blockIdx.x * E; e0 < n; e0 += (int64_t)gridDim.x * E) {
        // thread (el, grp) stages vectors grp, grp + ngrp, ... of element e0 + el: every load is issued
        // before any is used
        const int64_t e = e0 + el;
        double st[kStageMax];
        double mf = 0.0;
        if (e < n) {
            // unconditional loads (an index past the last vector re-reads g[e]) so that nothing
            // separates them and all are in flight together; the surplus ones are zeroed afterwards
#pragma unroll
            for (int k = 0; k < kStageMax; ++k) {
                const int j = grp + ngrp * k;
                st[k] = vec_ptr(j < V ? j : V - 1)[e];
            }
            const double xe = x[e], ge = g[e], le = l[e], ue = u[e];
            int fr;
            if (dbg_inputs) {
                fr = mask[e] != 0;
            } else {
                const bool at_lower = (xe <= le + op.eps) && (ge >= 0.0);
                const bool at_upper = (xe >= ue - op.eps) && (ge <= 0.0);
                fr = !(at_lower || at_upper);
            }
            mf = fr ? 1.0 : 0.0;
#pragma unroll
            for (int k = 0; k < kStageMax; ++k)
                if (grp + ngrp * k >= V) st[k] = 0.0;
            if (grp == 0) {
                if (!dbg_inputs) mask[e] = (uint8_t)fr;
                if (fr) pg2 = fma(ge, ge, pg2); else nfixed += 1.0;
                pginf = fmax(pginf, fabs(xe - clampd(xe - ge, le, ue)));
            }
#pragma unroll
            for (int k = 0; k < kStageMax; ++k)
                if (grp + ngrp * k == jnew) ynew = fma(st[k], st[k], ynew);
        } else {
#pragma unroll
            for (int k = 0; k < kStageMax; ++k) st[k] = 0.0;
        }
        __syncthreads();   // the previous chunk has been consumed
#pragma unroll
        for (int k = 0; k < kStageMax; ++k) {
            const int j = grp + ngrp * k;
            if (j < Vp) dyn[el * Vp + j] = st[k] * mf;
        }
        __syncthreads();
        LB_TICK(8);
#pragma unroll
        for (int k = 0; k < kTPT; ++k) {
            if (ti[k] >= 0) {
                const double* pa = dyn + 2 * ti[k];
                const double* pb = dyn + 2 * tj[k];
#pragma unroll 4
                for (int i = h; i < E; i += groups) {
                    const double2 a = *reinterpret_cast<const double2*>(pa + i * Vp);
                    const double2 b = *reinterpret_cast<const double2*>(pb + i * Vp);
                    acc[k][0] = fma(a.x, b.x, acc[k][0]);
                    acc[k][1] = fma(a.x, b.y, acc[k][1]);
                    acc[k][2] = fma(a.y, b.x, acc[k][2]);
                    acc[k][3] = fma(a.y, b.y, acc[k][3]);
                }
            }
        }
    }

    LB_TICK(2);
    double* part = grampart + (int64_t)blockIdx.x * NE;
    if (split && groups > 1) {
        // add the element slices of each tile in slice order
        __syncthreads();
        if (ti[0] >= 0) {
#pragma unroll
            for (int s = 0; s < 4; ++s) dyn[(h * TT + tid % TT) * 4 + s] = acc[0][s];
        }
        __syncthreads();
        if (h == 0) {
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                double t = 0.0;
                for (int hh = 0; hh < groups; ++hh) t += dyn[(hh * TT + tid) * 4 + s];
                part[kHdr + 4 * tid + s] = t;
            }
        }
    } else {
#pragma unroll
        for (int k = 0; k < kTPT; ++k) {
            if (ti[k] >= 0) {
                const int q = split ? tid : tid + k * kBlock;
#pragma unroll
                for (int s = 0; s < 4; ++s) part[kHdr + 4 * q + s] = acc[k][s];
            }
        }
    }
    {
        double sv[3] = {pg2, nfixed, ynew};
        block_sum<3, kWaves>(sv, red);
        double mx = wave_max(pginf);
        __syncthreads();
        if (lane == 0) red[wave] = mx;
        __syncthreads();
        if (tid == 0) {
            mx = fmax(fmax(red[0], red[1]), fmax(red[2], red[3]));
            part[0] = sv[0]; part[1] = mx; part[2] = sv[1]; part[3] = sv[2];
        }
    }
    LB_TICK(3);
    if (!arrive_is_last(&scal->counters[kCntGram], &flag)) return;
    LB_TICK(4);

    // ---- last workgroup: total G, then the recursion on coefficients ----
    const int nb = gridDim.x;
    double* G = dyn;   // Vp x Vp, row-major
    __shared__ double wsum[kWaves];
    // statistics header of every workgroup (strided over the threads): issued first, used after the G sums
    double sv[3] = {0.0, 0.0, 0.0};
    double mx = 0.0;
    for (int b = tid; b < nb; b += kBlock) {
        const double* hp = grampart + (int64_t)b * NE;
        sv[0] += hp[0]; sv[1] += hp[2]; sv[2] += hp[3];
        mx = fmax(mx, hp[1]);
    }
    // one thread per entry adds the partials in workgroup order, 24 loads in flight (larger batches
    // measured no faster: one compute unit's load bandwidth is the limit once there are ~100 partials)
    for (int q4 = tid; q4 < 4 * TT; q4 += kBlock) {
        const double* src = grampart + kHdr + q4;
        double s = 0.0;
        for (int b0 = 0; b0 < nb; b0 += 24) {
            double v[24];
#pragma unroll
            for (int k = 0; k < 24; ++k) v[k] = b0 + k < nb ? src[(int64_t)(b0 + k) * NE] : 0.0;
#pragma unroll
            for (int k = 0; k < 24; ++k) s += v[k];
        }
        int a, bq;
        tile_of(q4 >> 2, T, a, bq);
        const int row = 2 * a + ((q4 >> 1) & 1), col = 2 * bq + (q4 & 1);
        G[row * Vp + col] = s;
        G[col * Vp + row] = s;
    }
    LB_TICK(5);
    {
        // per-workgroup statistics: fixed-order reductions
        block_sum<3, kWaves>(sv, red);
        mx = wave_max(mx);
        __syncthreads();
        if (lane == 0) wsum[wave] = mx;
        __syncthreads();
        if (tid == 0) {
            red[0] = sv[0];
            red[1] = fmax(fmax(wsum[0], wsum[1]), fmax(wsum[2], wsum[3]));
            red[2] = sv[1];
            red[3] = sv[2];
            // apply the update the previous kernel left pending, then record the newest pair's norm
            apply_pending(scal, m);
            if (c > 0 && !dbg_inputs) scal->ynorm2[(head - 1 + m) % m] = sv[2];
        }
    }
    __syncthreads();
    LB_TICK(6);
    if (tid < 64) {
        const int i = lane;   // lane i owns pair i (oldest = 0)
        double rho = 1.0, yn = 1.0, inv = 0.0;
        bool pass = false;
        if (i < c) {
            rho = G[i * Vp + (c + i)];
            // the newest pair's norm was just summed (tid 0 also stored it for later iterations)
            yn = (i == c - 1 && !dbg_inputs) ? red[3] : scal->ynorm2[(head - c + i + 2 * m) % m];
            pass = rho > op.eps * yn;
            inv = 1.0 / rho;
        }
        const unsigned long long pm = __ballot(pass);
        // first loop: alpha_k, newest to oldest.  Steps of pairs that fail the gate run with alpha_k = 0;
        // a lane's row is dead once its own alpha has been taken, so updating it further is harmless.
        double part_s = i < c ? G[i * Vp + 2 * c] : 0.0;   // <s_i, g>
        double alpha_i = 0.0;
#pragma unroll 4
        for (int k = c - 1; k >= 0; --k) {
            const double gsy = i < c ? G[i * Vp + (c + k)] : 0.0;   // <s_i, y_k>
            double ak = lane_value(part_s * inv, k);
            if (!((pm >> k) & 1ull)) ak = 0.0;
            if (i == k) alpha_i = ak;
            part_s = fma(-ak, gsy, part_s);
        }
        if (i < c) alpha_s[i] = alpha_i;
        double gamma = 1.0;
        if (c > 0 && ((pm >> (c - 1)) & 1ull)) gamma = lane_value(rho / yn, c - 1);
        // <y_i, gamma (g - sum_k alpha_k y_k)>
        double by = 0.0;
        {
            double tsum = i < c ? G[(c + i) * Vp + 2 * c] : 0.0;
#pragma unroll 4
            for (int k = 0; k < c; ++k) {
                const double gyy = i < c ? G[(c + i) * Vp + (c + k)] : 0.0;
                tsum = fma(-alpha_s[k], gyy, tsum);
            }
            by = gamma * tsum;
        }
        // second loop: alpha_k - beta_k, oldest to newest
        double coef_s = 0.0;
#pragma unroll 4
        for (int k = 0; k < c; ++k) {
            const double gys = i < c ? G[(c + i) * Vp + k] : 0.0;   // <y_i, s_k>
            double ck = lane_value(alpha_i - by * inv, k);
            if (!((pm >> k) & 1ull)) ck = 0.0;
            if (i == k) coef_s = ck;
            if (i > k) by = fma(ck, gys, by);
        }
        if (i < c) {
            scal->delta[i] = coef_s;
            scal->delta[c + i] = -gamma * alpha_i;
        }
#ifdef LB_PROFILE_GRAM
        if (lane == 0) {
            ticks[7] = wall_clock64();
            for (int k = 0; k < 9; ++k) scal->delta[40 + k] = (double)(ticks[k] - ticks[0]);
        }
#endif
        if (lane == 0) {
            scal->delta[2 * c] = gamma;
            scal->pairs_used = __popcll(pm);
            if (evaluate_stop) {
                const double pgn = sqrt(red[0]);
                scal->pg2 = pgn;
                scal->pginf = red[1];
                scal->n_fixed = (long long)red[2];
                if (!scal->tol_resolved) {
                    scal->tol_abs = op.tol_relative ? op.tol * fmax(1.0, pgn) : op.tol;
                    scal->tol_resolved = 1;
                }
                if (scal->status == LBFGSB_RUNNING) {
                    if (pgn <= scal->tol_abs) scal->status = LBFGSB_CONVERGED;
                    else if (scal->iters >= op.max_iter) scal->status = LBFGSB_MAX_ITER;
                }
            }
        }
    }
}

void launch_gram(const Dims& dm, const Opts& op, const Geometry& ge, const Buffers& bf, int dbg_inputs,
                 int evaluate_stop, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
    hipExtLaunchKernelGGL(k_gram, dim3(ge.gram_blocks), dim3(kBlock), gram_lds_bytes(dm.m), st, ev0, ev1, 0, dm.n, dm.m,
                          gram_chunk(dm.m), op, bf.x, bf.g, bf.l, bf.u, bf.S, bf.Y, bf.mask, bf.scal, bf.grampart,
                          gram_entries(dm.m), dbg_inputs, evaluate_stop);
}

// Applies a pending update when nothing else is about to (before an evaluation from scratch, and
// before the host reads the scalars).
__global__ void k_commit(Scal* scal, int m) {
    if (threadIdx.x == 0 && blockIdx.x == 0) apply_pending(scal, m);
}
void launch_commit(const Dims& dm, const Buffers& bf, hipStream_t st) {
    hipLaunchKernelGGL(k_commit, dim3(1), dim3(64), 0, st, bf.scal, dm.m);
}

}  // namespace lb
