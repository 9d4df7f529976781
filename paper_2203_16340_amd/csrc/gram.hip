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
//
// Three kernels build G, chosen by the length of the vectors: k_gram (tiles of G per thread, operands staged
// through LDS; a few dozen workgroups, which is what short vectors want), and for n >= 2^17 (even) k_gram_wide
// (m <= 10: element pairs per lane, entries of G divided among the waves) or k_gram_mfma (m > 10: matrix cores).
// All three end in the same recursion on coefficients (recursion_on_coefficients).
#include <cstddef>

#include "common.h"
#include "recursion.h"
#include "wide_close.h"

namespace lb {

namespace {
constexpr int kStageMax = 32;   // vectors one thread stages per chunk
constexpr int kHdr = kGramHdr;   // per-workgroup partial: [0] sum g[S]^2, [1] max KKT residual, [2] #fixed, [3] ||y_new||^2
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
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // one load per wave fetches the integer header of the scalar block (status, ring position, pending
    // update); readlanes hand the fields to every lane
    static_assert(offsetof(Scal, pend_ok) < 64, "header fields must sit in the first 16 ints");
    const int hdr = lane < 16 ? reinterpret_cast<const int*>(scal)[lane] : 0;
    if (__shfl(hdr, offsetof(Scal, status) / 4) != LBFGSB_RUNNING) {
        // a step that finds the solver parked by the short logistic sequence is counted, so that the host can redo it
        if (__shfl(hdr, offsetof(Scal, status) / 4) == kStatusBail && evaluate_stop && !dbg_inputs && blockIdx.x == 0 && tid == 0)
            scal->bail_skipped += 1;
        return;
    }
    int head = __shfl(hdr, offsetof(Scal, head) / 4), c = __shfl(hdr, offsetof(Scal, count) / 4);
    if (__shfl(hdr, offsetof(Scal, pend_valid) / 4)) {          // same rule as effective_ring()
        if (__shfl(hdr, offsetof(Scal, pend_ok) / 4)) { head = (head + 1) % m; c = c < m ? c + 1 : m; }
        else c = 0;
    }
    const double yn_old = prefetch_ynorm2(scal, c, head, m);   // (used by the last workgroup's recursion, fetched now)
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
    if (!arrive_is_last(&scal->counters[kCntGram], &flag)) return;

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
    recursion_on_coefficients(G, Vp, c, head, m, op, scal, red[0], red[1], red[2], red[3], yn_old, alpha_s, dbg_inputs, evaluate_stop);
}


// ---- large n: partial results of many workgroups, added in two levels ---------------------------------------
//
// Every workgroup has written NE doubles at grampart + blockIdx.x * NE (entry 1 is a maximum, all others are
// sums).  The workgroups form at most kGramGroups groups of consecutive indices; the last workgroup of a group
// to finish adds the group's partials in index order into grampart + (gridDim.x + group) * NE, and the last
// group to finish adds the group results, again in index order, into tot[0 .. NE) (LDS).  Returns true in that
// one workgroup (after a barrier), false everywhere else.  No workgroup reads more than kGramGroupMax partials,
// and the order of the additions does not depend on which workgroup finishes last.  Grids of at most
// kGramOneLevelMax workgroups skip the first level (each level costs two fences, an atomic and a dependent round of
// loads: 6-7 us).
constexpr int kGramGroupMax = 32;   // workgroups per group at most: grids of up to kGramGroups * kGramGroupMax

__device__ __forceinline__ bool reduce_partials(double* __restrict__ grampart, int NE, Scal* __restrict__ scal, int* flag,
                                                double* tot) {
    const int tid = threadIdx.x, nwg = gridDim.x;
    if (nwg <= kGramOneLevelMax) {
        // few workgroups: one level, the last one to finish adds all partials in index order
        if (!arrive_is_last(&scal->gram_cnt[kGramGroups], flag, (unsigned)nwg)) return false;
        // 64 partials of an entry at a time, every load of a batch issued before the first is used (one trip to
        // memory per batch; the accumulators' registers are free by now)
        gram_sum_partials_flat(grampart, NE, nwg, tot);
        __syncthreads();
        return true;
    }
    const int gs = (nwg + kGramGroups - 1) / kGramGroups;
    const int ngroups = (nwg + gs - 1) / gs;
    const int grp = blockIdx.x / gs, gfirst = grp * gs;
    const int gsize = nwg - gfirst < gs ? nwg - gfirst : gs;
    if (!arrive_is_last(&scal->gram_cnt[grp], flag, (unsigned)gsize)) return false;
    double* part2 = grampart + (int64_t)(nwg + grp) * NE;
    for (int idx = tid; idx < NE; idx += kBlock) {
        double v[kGramGroupMax];
#pragma unroll
        for (int k = 0; k < kGramGroupMax; ++k) v[k] = k < gsize ? grampart[(int64_t)(gfirst + k) * NE + idx] : 0.0;
        double t = v[0];
        if (idx == 1) {
#pragma unroll
            for (int k = 1; k < kGramGroupMax; ++k) t = fmax(t, v[k]);
        } else {
#pragma unroll
            for (int k = 1; k < kGramGroupMax; ++k) t += v[k];
        }
        part2[idx] = t;
    }
    if (!arrive_is_last(&scal->gram_cnt[kGramGroups], flag, (unsigned)ngroups)) return false;
    for (int idx = tid; idx < NE; idx += kBlock) {
        double v[kGramGroups];
#pragma unroll
        for (int k = 0; k < kGramGroups; ++k) v[k] = k < ngroups ? grampart[(int64_t)(nwg + k) * NE + idx] : 0.0;
        double t = v[0];
        if (idx == 1) {
#pragma unroll
            for (int k = 1; k < kGramGroups; ++k) t = fmax(t, v[k]);
        } else {
#pragma unroll
            for (int k = 1; k < kGramGroups; ++k) t += v[k];
        }
        tot[idx] = t;
    }
    __syncthreads();
    return true;
}

// ---- large n: the Gram matrix on the matrix cores ---------------------------------------------------------
//
// G = B^T B with B = [vectors | n x (2c+1)] masked by the free set is a tall-skinny symmetric rank-n update: a
// dense contraction whose operands stream from memory once.  v_mfma_f64_16x16x4_f64 multiplies a 16 x 4 by a
// 4 x 16 block; lane (i = lane % 16, q = lane / 16) supplies A[i][q] and B[q][i'] -- for a Gram matrix both are
// the same number, vector (16 b + i) at one element, so ONE register per lane feeds both operands and the loads
// go straight from memory into the operand layout (no LDS staging).  A wave takes 64 consecutive elements per
// chunk: lane (i, q) loads, for each of its NB vectors, eight element pairs e0 + 8 s + 2 q + {0,1} (16-byte loads,
// 64 contiguous bytes per vector and instruction) and issues 16 multiply steps; which element a (lane, step)
// holds does not matter for the sum as long as the free-set bit applied to it is that element's.  Lane j of the
// wave evaluates Eq. (ws) for element e0 + j, a ballot turns the 64 results into a bit mask, and step t reads
// bit 8 (t/2) + 2 q + (t%2).  One extra vector slot carries an UNMASKED copy of the newest y, whose diagonal
// entry is the full-vector ||y||^2 the curvature gate needs.
// Result of lane l, register r of a 16 x 16 block: row l/16 + 4 r, column l % 16.

typedef double f64x2 __attribute__((ext_vector_type(2)));
typedef double f64x4 __attribute__((ext_vector_type(4)));

constexpr int64_t kMfmaMinN = 1 << 17;
__host__ __device__ inline int mfma_blocks16(int m) { return (2 * m + 2 + 15) / 16; }   // 2m+1 vectors + unmasked y
__host__ __device__ inline int mfma_nb(int m) { const int b = mfma_blocks16(m); return b <= 1 ? 1 : (b <= 2 ? 2 : 4); }
__host__ __device__ inline int mfma_entries(int nb) { return kHdr + nb * (nb + 1) / 2 * 256; }
// (m <= 10: k_gram_wide.  With 20 pairs and 10^6 variables this kernel takes 181 us per launch where the LDS-tiled
// k_gram takes 457 us on the same data: a 41 x 41 x 10^6 contraction is matrix-core work.)
bool gram_uses_mfma(int64_t n, int m) { return n >= kMfmaMinN && n % 2 == 0 && m > 10; }

template <int NB>
__global__ __launch_bounds__(kBlock) void k_gram_mfma(int64_t n, int m, Opts op, const double* __restrict__ x,
                                                      const double* __restrict__ g, const double* __restrict__ l,
                                                      const double* __restrict__ u, const double* __restrict__ S,
                                                      const double* __restrict__ Y, uint8_t* __restrict__ mask,
                                                      Scal* __restrict__ scal, double* __restrict__ grampart,
                                                      int dbg_inputs, int evaluate_stop) {
    constexpr int NBP = NB * (NB + 1) / 2;
    constexpr int NEM = kHdr + NBP * 256;
    extern __shared__ __align__(16) double dyn[];   // kWaves x NBP x 256 accumulators; later G
    __shared__ double red[kWaves * 4];
    __shared__ double alpha_s[kMaxM + 1];
    __shared__ int flag;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    static_assert(offsetof(Scal, pend_ok) < 64, "header fields must sit in the first 16 ints");
    const int hdr = lane < 16 ? reinterpret_cast<const int*>(scal)[lane] : 0;
    if (__shfl(hdr, offsetof(Scal, status) / 4) != LBFGSB_RUNNING) {
        // a step that finds the solver parked by the short logistic sequence is counted, so that the host can redo it
        if (__shfl(hdr, offsetof(Scal, status) / 4) == kStatusBail && evaluate_stop && !dbg_inputs && blockIdx.x == 0 && tid == 0)
            scal->bail_skipped += 1;
        return;
    }
    int head = __shfl(hdr, offsetof(Scal, head) / 4), c = __shfl(hdr, offsetof(Scal, count) / 4);
    if (__shfl(hdr, offsetof(Scal, pend_valid) / 4)) {          // same rule as effective_ring()
        if (__shfl(hdr, offsetof(Scal, pend_ok) / 4)) { head = (head + 1) % m; c = c < m ? c + 1 : m; }
        else c = 0;
    }
    const double yn_old = prefetch_ynorm2(scal, c, head, m);   // (used by the last workgroup's recursion, fetched now)
    const int V = 2 * c + 1;
    const int Vp = V + 1;
    const int base_slot = c > 0 ? (head - c + 2 * m) % m : 0;   // ring slot of the oldest pair
    auto vec_ptr = [&](int j) -> const double* {
        if (j >= 2 * c) return g;
        const bool is_y = j >= c;
        int sl = base_slot + (is_y ? j - c : j);
        if (sl >= m) sl -= m;
        return (is_y ? Y : S) + (int64_t)sl * n;
    };
    const int nslots = c > 0 ? V + 1 : V;            // slot V: the unmasked copy of the newest y
    const int nbk = (nslots + 15) / 16;              // 16-vector blocks in use (<= NB)
    const int i16 = lane & 15, q = lane >> 4;
    const double* vp[NB];
    int kind[NB];                                    // 0 = unused slot (operand forced to zero), 1 = masked vector, 2 = unmasked
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const int j = 16 * b + i16;
        kind[b] = j < V ? 1 : (j == V && c > 0 ? 2 : 0);
        vp[b] = kind[b] == 1 ? vec_ptr(j) : (kind[b] == 2 ? vec_ptr(2 * c - 1) : g);
    }
    f64x4 acc[NBP];
#pragma unroll
    for (int k = 0; k < NBP; ++k) acc[k] = f64x4{0.0, 0.0, 0.0, 0.0};
    double pginf = 0.0;
    long long nfixed = 0;

    const int64_t nchunks = (n + 63) / 64;
    for (int64_t ch = (int64_t)blockIdx.x * kWaves + wave; ch < nchunks; ch += (int64_t)gridDim.x * kWaves) {
        const int64_t e0 = ch * 64;
        f64x2 v[NB][8];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            if (b < nbk) {
#pragma unroll
                for (int s8 = 0; s8 < 8; ++s8) {
                    int64_t e = e0 + 8 * s8 + 2 * q;
                    if (e > n - 2) e = n - 2;          // past the end (n is even): any in-range pair, zeroed below
                    v[b][s8] = *reinterpret_cast<const f64x2*>(vp[b] + e);
                }
            } else {
#pragma unroll
                for (int s8 = 0; s8 < 8; ++s8) v[b][s8] = f64x2{0.0, 0.0};
            }
        }
        // Eq. (ws) and the KKT residual for element e0 + lane
        const int64_t e = e0 + lane;
        const bool in = e < n;
        const int64_t ec = in ? e : n - 1;
        const double xe = x[ec], ge = g[ec], le = l[ec], ue = u[ec];
        bool fr;
        if (dbg_inputs) {
            fr = mask[ec] != 0;
        } else {
            const bool at_lower = (xe <= le + op.eps) && (ge >= 0.0);
            const bool at_upper = (xe >= ue - op.eps) && (ge <= 0.0);
            fr = !(at_lower || at_upper);
            if (in) mask[e] = (uint8_t)fr;
        }
        if (in) pginf = fmax(pginf, fabs(xe - clampd(xe - ge, le, ue)));
        const unsigned long long bits_in = __ballot(in);
        const unsigned long long bits_free = __ballot(fr && in);
        nfixed += __popcll(bits_in & ~bits_free);
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            const int sh = 8 * (t >> 1) + 2 * q + (t & 1);
            const bool b_free = (bits_free >> sh) & 1ull, b_in = (bits_in >> sh) & 1ull;
            double opnd[NB];
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const double val = (t & 1) ? v[b][t >> 1].y : v[b][t >> 1].x;
                const bool keep = kind[b] == 1 ? b_free : (kind[b] == 2 ? b_in : false);
                opnd[b] = keep ? val : 0.0;
            }
            int k = 0;
#pragma unroll
            for (int a = 0; a < NB; ++a) {
#pragma unroll
                for (int b = a; b < NB; ++b, ++k) {
                    if (b < nbk) acc[k] = __builtin_amdgcn_mfma_f64_16x16x4f64(opnd[a], opnd[b], acc[k], 0, 0, 0);
                }
            }
        }
    }

    // this workgroup's partial: the waves' accumulators added in wave order
#pragma unroll
    for (int k = 0; k < NBP; ++k) {
#pragma unroll
        for (int r = 0; r < 4; ++r) dyn[(wave * NBP + k) * 256 + r * 64 + lane] = acc[k][r];
    }
    double* part = grampart + (int64_t)blockIdx.x * NEM;
    {
        double nf[1] = {lane == 0 ? (double)nfixed : 0.0};
        block_sum<1, kWaves>(nf, red);               // (also the barrier that publishes dyn)
        double mx = wave_max(pginf);
        __syncthreads();
        if (lane == 0) red[wave] = mx;
        __syncthreads();
        if (tid == 0) {
            part[0] = 0.0;
            part[1] = fmax(fmax(red[0], red[1]), fmax(red[2], red[3]));
            part[2] = nf[0];
            part[3] = 0.0;
        }
    }
    for (int idx = tid; idx < NBP * 256; idx += kBlock) {
        double t = 0.0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) t += dyn[w * NBP * 256 + idx];
        part[kHdr + idx] = t;
    }

    double* tot = dyn + 4096;    // totals of the partial entries; G occupies dyn[0 .. 4096)
    if (!reduce_partials(grampart, NEM, scal, &flag, tot)) return;
    double* G = dyn;   // Vp x Vp, row-major
    for (int idx = tid; idx < NBP * 256; idx += kBlock) {
        const double t = tot[kHdr + idx];
        const int pair = idx >> 8, r = (idx >> 6) & 3, ln = idx & 63;
        int a = 0, pb = pair;
        while (pb >= NB - a) { pb -= NB - a; ++a; }      // pair -> blocks (a, a + pb)
        const int b = a + pb;
        const int row = 16 * a + (ln >> 4) + 4 * r, col = 16 * b + (ln & 15);
        if (row < V && col < V) {
            G[row * Vp + col] = t;
            if (a != b) G[col * Vp + row] = t;          // a diagonal block holds both (row, col) and (col, row)
        }
        if (row == V && col == V) red[3] = t;            // ||y_new||^2 over the full vector
        if (row == 2 * c && col == 2 * c) red[0] = t;    // sum over the free set of g^2
    }
    if (tid == 0) { red[1] = tot[1]; red[2] = tot[2]; }
    __syncthreads();
    if (tid == 0) {
        // apply the update the previous kernel left pending, then record the newest pair's norm
        apply_pending(scal, m);
        if (c > 0 && !dbg_inputs) scal->ynorm2[(head - 1 + m) % m] = red[3];
    }
    __syncthreads();
    recursion_on_coefficients(G, Vp, c, head, m, op, scal, red[0], red[1], red[2], red[3], yn_old, alpha_s, dbg_inputs, evaluate_stop);
}


// ---- at most 10 pairs: one element pair per lane, the entries of G divided among the waves -------------------
//
// The fp64 matrix cores of this chip run at the vector rate, and the 16-wide blocks above compute three times
// the entries a 21-vector Gram matrix has.  For m <= 10 the plain vector unit does better: lane l of every wave
// holds elements e0 + 2l, e0 + 2l + 1 of a 128-element chunk (16-byte loads, each instruction a contiguous
// kilobyte of one vector), and the 231 entries of the 21 x 21 matrix over the STATIC slots
//     S ring slots 0..9 | Y ring slots 10..19 | g 20
// are divided among three waves of a workgroup.  With the slots in three groups of seven, a = 0..6, b = 7..13,
// c = 14..20, wave r takes group r among itself and group r times group r + 1 (cyclically):
//     wave 0: a x a (28) + a x b (49)     wave 1: b x b + b x c     wave 2: c x c + c x a
// -- 77 per-lane accumulators and 14 vector loads per chunk each, so the three finish together (an earlier split
// into 66/55/55/55 entries had two waves load 16 vectors and two 10-11, and the workgroup waited 6-9 us for the
// slow pair).  The fourth wave writes the free-set mask and sums the statistics (KKT residual, number of fixed
// variables, full ||y_new||^2).  The waves read the same chunk, so the vectors come from memory once and from the
// cache after that.  Only one operand of a product is masked (the mask is 0 or 1).  Ring slots not in use
// contribute zeros; the last workgroup maps ring slots to the oldest-first order of the recursion.

// Sums 64 per-lane values over the 64 lanes of a wave all at once: on return lane j holds the total of a[j].
// Each step halves the number of values a lane carries (the half it gives away goes to the lane 32, 16, ... 1
// away), so 63 exchanges do what 64 separate butterfly sums would need 384 for.  Fixed order of additions.
template <int D, int N>
__device__ __forceinline__ void transpose_sum_step(double (&a)[N], int lane) {
    const bool upper = (lane & D) != 0;
#pragma unroll
    for (int k = 0; k < D; ++k) {
        const double send = upper ? a[k] : a[k + D];
        const double keep = upper ? a[k + D] : a[k];
        a[k] = keep + __shfl_xor(send, D);
    }
}
__device__ __forceinline__ double transpose_sum64(double (&a)[64]) {
    const int lane = threadIdx.x & 63;
    transpose_sum_step<32>(a, lane);
    transpose_sum_step<16>(a, lane);
    transpose_sum_step<8>(a, lane);
    transpose_sum_step<4>(a, lane);
    transpose_sum_step<2>(a, lane);
    transpose_sum_step<1>(a, lane);
    return a[0];
}

// The same for 16 values: on return every lane l holds the total of a[l % 16].
__device__ __forceinline__ double transpose_sum16(double (&a)[16]) {
    const int lane = threadIdx.x & 63;
    transpose_sum_step<8>(a, lane);
    transpose_sum_step<4>(a, lane);
    transpose_sum_step<2>(a, lane);
    transpose_sum_step<1>(a, lane);
    double t = a[0];                      // total over this row of 16 lanes
    t += __shfl_xor(t, 16);
    t += __shfl_xor(t, 32);
    return t;
}

struct WideCtx {
    int64_t n;
    int m, c, base_slot;
    const double *S, *Y, *g;
    unsigned active;     // bit s: static slot s holds a vector
};

__device__ __forceinline__ const double* wide_ptr(const WideCtx& w, int slot) {
    if (slot < kWideM) return w.S + (int64_t)slot * w.n;
    if (slot < 2 * kWideM) return w.Y + (int64_t)(slot - kWideM) * w.n;
    return w.g;
}

// One wave's share.  ROLE 0..2: the seven slots from P0 among themselves and times the seven from Q0; ROLE 3: the
// free-set mask and the statistics.  Chunks ch0, ch0 + chs, ... of 128 elements.
template <int P0, int Q0, int ROLE, bool UB>
__device__ __forceinline__ void wide_role(const WideCtx& w, const Opts& op, const double* __restrict__ x,
                                          const double* __restrict__ l, const double* __restrict__ u,
                                          uint8_t* __restrict__ mask, int dbg_inputs, double* __restrict__ part,
                                          int offset) {
    constexpr bool STATS = ROLE == 3;
    constexpr int NACC = STATS ? 1 : kWideRole;
    const int lane = threadIdx.x & 63;
    double acc[NACC];
#pragma unroll
    for (int k = 0; k < NACC; ++k) acc[k] = 0.0;
    double pginf = 0.0, ynew = 0.0, nfixed = 0.0;
    const double* yn_ptr = w.c > 0 ? w.Y + (int64_t)((w.base_slot + w.c - 1) % w.m) * w.n : w.g;
    const int64_t nchunks = (w.n + 127) / 128;
    // x, g, l, u (and the given mask) of a chunk decide which lanes load the vectors at all, so they are fetched one
    // chunk ahead: the two dependent round trips of a chunk overlap with the previous chunk's
    auto pair_index = [&](int64_t ch, bool& in) -> int64_t {
        const int64_t e = ch * 128 + 2 * lane;
        in = ch < nchunks && e < w.n;                  // n is even: both elements of the pair, or neither
        return in ? e : w.n - 2;
    };
    bool in_next;
    int64_t ec_next = pair_index(blockIdx.x, in_next);
    // UB: same bounds everywhere, l and u are not streamed (and take no registers)
    f64x2 xn = *reinterpret_cast<const f64x2*>(x + ec_next), gn = *reinterpret_cast<const f64x2*>(w.g + ec_next);
    f64x2 ln = f64x2{op.lo, op.lo}, un = f64x2{op.hi, op.hi};
    if constexpr (!UB) { ln = *reinterpret_cast<const f64x2*>(l + ec_next); un = *reinterpret_cast<const f64x2*>(u + ec_next); }
    unsigned short mkn = dbg_inputs ? *reinterpret_cast<const unsigned short*>(mask + ec_next) : (unsigned short)0;
    for (int64_t ch = blockIdx.x; ch < nchunks; ch += gridDim.x) {
        const bool in = in_next;
        const int64_t ec = ec_next, e = ec_next;
        const f64x2 xe = xn, ge = gn;
        const f64x2 le = UB ? f64x2{op.lo, op.lo} : ln, ue = UB ? f64x2{op.hi, op.hi} : un;
        const unsigned short mk = mkn;
        ec_next = pair_index(ch + gridDim.x, in_next);
        xn = *reinterpret_cast<const f64x2*>(x + ec_next); gn = *reinterpret_cast<const f64x2*>(w.g + ec_next);
        if constexpr (!UB) { ln = *reinterpret_cast<const f64x2*>(l + ec_next); un = *reinterpret_cast<const f64x2*>(u + ec_next); }
        if (dbg_inputs) mkn = *reinterpret_cast<const unsigned short*>(mask + ec_next);
        bool f0, f1;
        if (dbg_inputs) {
            f0 = (mk & 0xffu) != 0;
            f1 = (mk >> 8) != 0;
        } else {
            f0 = !(((xe.x <= le.x + op.eps) && (ge.x >= 0.0)) || ((xe.x >= ue.x - op.eps) && (ge.x <= 0.0)));
            f1 = !(((xe.y <= le.y + op.eps) && (ge.y >= 0.0)) || ((xe.y >= ue.y - op.eps) && (ge.y <= 0.0)));
        }
        if constexpr (STATS) {
            if (in) {
                if (!dbg_inputs)
                    *reinterpret_cast<unsigned short*>(mask + e) = (unsigned short)((f0 ? 1u : 0u) | (f1 ? 0x100u : 0u));
                pginf = fmax(pginf, fmax(fabs(xe.x - clampd(xe.x - ge.x, le.x, ue.x)), fabs(xe.y - clampd(xe.y - ge.y, le.y, ue.y))));
                nfixed += (f0 ? 0.0 : 1.0) + (f1 ? 0.0 : 1.0);
                if (w.c > 0) {
                    const f64x2 yv = *reinterpret_cast<const f64x2*>(yn_ptr + ec);
                    ynew = fma(yv.x, yv.x, ynew);
                    ynew = fma(yv.y, yv.y, ynew);
                }
            }
        } else {
            const double m0 = (in && f0) ? 1.0 : 0.0, m1 = (in && f1) ? 1.0 : 0.0;
            // fixed variables contribute nothing: lanes whose two elements are both fixed (or past the end) load no vector
            if (m0 != 0.0 || m1 != 0.0) {
                f64x2 vp[kWideG], vq[kWideG];
#pragma unroll
                for (int i = 0; i < kWideG; ++i) {
                    vp[i] = f64x2{0.0, 0.0};
                    if ((w.active >> (P0 + i)) & 1u) vp[i] = *reinterpret_cast<const f64x2*>(wide_ptr(w, P0 + i) + ec);
                }
#pragma unroll
                for (int j = 0; j < kWideG; ++j) {
                    vq[j] = f64x2{0.0, 0.0};
                    if ((w.active >> (Q0 + j)) & 1u) vq[j] = *reinterpret_cast<const f64x2*>(wide_ptr(w, Q0 + j) + ec);
                }
#pragma unroll
                for (int i = 0; i < kWideG; ++i) { vp[i].x *= m0; vp[i].y *= m1; }
                int k = 0;
#pragma unroll
                for (int a = 0; a < kWideG; ++a) {
#pragma unroll
                    for (int b = a; b < kWideG; ++b, ++k) {
                        acc[k] = fma(vp[a].x, vp[b].x, acc[k]);
                        acc[k] = fma(vp[a].y, vp[b].y, acc[k]);
                    }
                }
#pragma unroll
                for (int a = 0; a < kWideG; ++a) {
#pragma unroll
                    for (int b = 0; b < kWideG; ++b, ++k) {
                        acc[k] = fma(vp[a].x, vq[b].x, acc[k]);
                        acc[k] = fma(vp[a].y, vq[b].y, acc[k]);
                    }
                }
            }
        }
    }
    if constexpr (STATS) {
        pginf = wave_max(pginf);
        nfixed = wave_sum(nfixed);
        ynew = wave_sum(ynew);
        if (lane == 0) { part[0] = 0.0; part[1] = pginf; part[2] = nfixed; part[3] = ynew; }
    } else {
        // sums over the lanes: 64 accumulators at once (lane j ends up with the total of accumulator j), then the other 13
        double first[64];
#pragma unroll
        for (int k = 0; k < 64; ++k) first[k] = acc[k];
        const double mine = transpose_sum64(first);
        part[kHdr + offset + lane] = mine;
        double rest[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) rest[k] = 64 + k < NACC ? acc[64 + k] : 0.0;
        const double mine2 = transpose_sum16(rest);
        if (lane < NACC - 64) part[kHdr + offset + 64 + lane] = mine2;
    }
}

template <bool UB>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_gram_wide(int64_t n, int m, Opts op, const double* __restrict__ x,
                                                      const double* __restrict__ g, const double* __restrict__ l,
                                                      const double* __restrict__ u, const double* __restrict__ S,
                                                      const double* __restrict__ Y, uint8_t* __restrict__ mask,
                                                      Scal* __restrict__ scal, double* __restrict__ grampart,
                                                      int dbg_inputs, int evaluate_stop, int no_close) {
    __shared__ double Gs[(2 * kWideM + 2) * (2 * kWideM + 2)];
    __shared__ double tot[kWideNE];
    __shared__ double alpha_s[kMaxM + 1];
    __shared__ int flag;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    static_assert(offsetof(Scal, pend_ok) < 64, "header fields must sit in the first 16 ints");
    const int hdr = lane < 16 ? reinterpret_cast<const int*>(scal)[lane] : 0;
    if (__shfl(hdr, offsetof(Scal, status) / 4) != LBFGSB_RUNNING) {
        // a step that finds the solver parked by the short logistic sequence is counted, so that the host can redo it
        if (__shfl(hdr, offsetof(Scal, status) / 4) == kStatusBail && evaluate_stop && !dbg_inputs && blockIdx.x == 0 && tid == 0)
            scal->bail_skipped += 1;
        return;
    }
    int head = __shfl(hdr, offsetof(Scal, head) / 4), c = __shfl(hdr, offsetof(Scal, count) / 4);
    if (__shfl(hdr, offsetof(Scal, pend_valid) / 4)) {          // same rule as effective_ring()
        if (__shfl(hdr, offsetof(Scal, pend_ok) / 4)) { head = (head + 1) % m; c = c < m ? c + 1 : m; }
        else c = 0;
    }
    const double yn_old = prefetch_ynorm2(scal, c, head, m);   // (used by the last workgroup's recursion, fetched now)
    WideCtx w;
    w.n = n; w.m = m; w.c = c; w.S = S; w.Y = Y; w.g = g;
    w.base_slot = c > 0 ? (head - c + 2 * m) % m : 0;           // ring slot of the oldest pair
    w.active = 1u << (2 * kWideM);
    for (int j = 0; j < c; ++j) {
        const int sl = (w.base_slot + j) % m;
        w.active |= (1u << sl) | (1u << (kWideM + sl));
    }
    double* part = grampart + (int64_t)blockIdx.x * kWideNE;
    switch (wave) {
        case 0: wide_role<0, kWideG, 0, UB>(w, op, x, l, u, mask, dbg_inputs, part, 0); break;
        case 1: wide_role<kWideG, 2 * kWideG, 1, UB>(w, op, x, l, u, mask, dbg_inputs, part, kWideRole); break;
        case 2: wide_role<2 * kWideG, 0, 2, UB>(w, op, x, l, u, mask, dbg_inputs, part, 2 * kWideRole); break;
        default: wide_role<0, 0, 3, UB>(w, op, x, l, u, mask, dbg_inputs, part, 0); break;
    }
    if (no_close) return;   // the direction kernel adds the partial sums and does the rest
    if (!reduce_partials(grampart, kWideNE, scal, &flag, tot)) return;
    wide_finish(tot, Gs, alpha_s, scal, m, c, head, w.base_slot, op, yn_old, dbg_inputs, evaluate_stop, true);
}

// (any even n: below 2^17 entries the grid stays small enough for the one-level sum of the partials)
bool gram_uses_wide(int64_t n, int m) { return n % 2 == 0 && m <= kWideM; }
int gram_wide_blocks(int64_t n) {
    const int64_t b = (n + 127) / 128;
    const int64_t cap = n >= kMfmaMinN ? 512 : kGramOneLevelMax;
    return (int)(b > cap ? cap : b);
}

template <int NB>
size_t mfma_lds_bytes() {
    size_t d = (size_t)kWaves * (NB * (NB + 1) / 2) * 256;         // the waves' accumulators
    const size_t fin = 4096 + (size_t)mfma_entries(NB);            // later: G (at most 64 x 64) and the totals
    return (d > fin ? d : fin) * 8;
}

int gram_mfma_blocks(int64_t n) {
    const int64_t b = ((n + 63) / 64 + kWaves - 1) / kWaves;
    return (int)(b > 256 ? 256 : b);
}

int gram_blocks_for(int64_t n, int m) {
    if (gram_uses_wide(n, m)) return gram_wide_blocks(n);
    if (gram_uses_mfma(n, m)) return gram_mfma_blocks(n);
    const int e = gram_chunk(m);
    int64_t b = (n + e - 1) / e;
    return (int)(b < 1 ? 1 : (b > 128 ? 128 : b));
}

size_t gram_partial_bytes(int64_t n, int m) {
    if (gram_uses_wide(n, m)) return (size_t)(gram_wide_blocks(n) + kGramGroups) * kWideNE * 8;
    if (gram_uses_mfma(n, m))
        return (size_t)(gram_mfma_blocks(n) + kGramGroups) * mfma_entries(mfma_nb(m)) * 8;
    return (size_t)gram_blocks_for(n, m) * gram_entries(m) * 8;
}

hipError_t gram_prepare(int64_t n, int m) {
    if (!gram_uses_mfma(n, m) || mfma_nb(m) != 4) return hipSuccess;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gram_mfma<4>), hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)mfma_lds_bytes<4>());
}

template <int NB>
void launch_gram_mfma(const Dims& dm, const Opts& op, const Geometry& ge, const Buffers& bf, int dbg_inputs,
                      int evaluate_stop, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
    hipExtLaunchKernelGGL((k_gram_mfma<NB>), dim3(ge.gram_blocks), dim3(kBlock), mfma_lds_bytes<NB>(), st, ev0, ev1, 0, dm.n,
                          dm.m, op, bf.x, bf.g, bf.l, bf.u, bf.S, bf.Y, bf.mask, bf.scal, bf.grampart, dbg_inputs,
                          evaluate_stop);
}

bool gram_can_skip_close(const Dims& dm, const Geometry& ge) {
    return gram_uses_wide(dm.n, dm.m) && ge.gram_blocks <= kGramOneLevelMax;
}

void launch_gram(const Dims& dm, const Opts& op, const Geometry& ge, const Buffers& bf, int dbg_inputs,
                 int evaluate_stop, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1, int no_close) {
    if (gram_uses_wide(dm.n, dm.m)) {
        if (no_close && !gram_can_skip_close(dm, ge)) no_close = 0;
        if (op.uniform_bounds)
            hipExtLaunchKernelGGL(k_gram_wide<true>, dim3(ge.gram_blocks), dim3(kBlock), 0, st, ev0, ev1, 0, dm.n, dm.m, op, bf.x,
                                  bf.g, bf.l, bf.u, bf.S, bf.Y, bf.mask, bf.scal, bf.grampart, dbg_inputs, evaluate_stop, no_close);
        else
            hipExtLaunchKernelGGL(k_gram_wide<false>, dim3(ge.gram_blocks), dim3(kBlock), 0, st, ev0, ev1, 0, dm.n, dm.m, op, bf.x,
                                  bf.g, bf.l, bf.u, bf.S, bf.Y, bf.mask, bf.scal, bf.grampart, dbg_inputs, evaluate_stop, no_close);
        return;
    }
    if (gram_uses_mfma(dm.n, dm.m)) {
        switch (mfma_nb(dm.m)) {
            case 1: launch_gram_mfma<1>(dm, op, ge, bf, dbg_inputs, evaluate_stop, st, ev0, ev1); break;
            case 2: launch_gram_mfma<2>(dm, op, ge, bf, dbg_inputs, evaluate_stop, st, ev0, ev1); break;
            default: launch_gram_mfma<4>(dm, op, ge, bf, dbg_inputs, evaluate_stop, st, ev0, ev1); break;
        }
        return;
    }
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
