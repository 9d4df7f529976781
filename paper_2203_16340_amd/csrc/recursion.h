// Algorithm 3 (modified two-loop recursion, appendix) carried out on coefficients: shared by the Gram kernels
// (last workgroup) and the single-workgroup resident solver.
#pragma once

#include "common.h"

namespace lb {

// value of v in lane l (l uniform across the wave): a scalar-register read, not a trip through LDS
__device__ __forceinline__ double lane_value(double v, int l) {
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), l);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), l);
    return __hiloint2double(hi, lo);
}

// ||y^i||^2 of the stored pairs for the lane that will own pair i in the recursion (lane i of wave 0).  It does not
// depend on anything the calling kernel computes, so the kernels fetch it when they start, long before it is used.
__device__ __forceinline__ double prefetch_ynorm2(const Scal* __restrict__ scal, int c, int head, int m) {
    const int tid = threadIdx.x;
    return (tid < 64 && tid < c) ? scal->ynorm2[(head - c + tid + 2 * m) % m] : 1.0;
}

constexpr int kRecFast = 10;   // up to this many pairs the recursion keeps its rows of G in registers

// The recursion of Algorithm 3 on coefficients, by one wave (threads 0..63) of the calling workgroup.  G: Vp x Vp (LDS),
// row-major, vectors ordered s^0..s^{c-1}, y^0..y^{c-1}, g.  gg = sum g[S]^2, pginf = max KKT residual, nfixed = #fixed,
// ynew = ||y_new||^2 (full vector), yn_old = prefetch_ynorm2().
__device__ __forceinline__ void recursion_on_coefficients(const double* G, int Vp, int c, int head, int m, const Opts& op,
                                                          Scal* __restrict__ scal, double gg, double pginf, double nfixed,
                                                          double ynew, double yn_old, double* alpha_s, int dbg_inputs,
                                                          int evaluate_stop) {
    const int tid = threadIdx.x, lane = tid & 63;
    if (tid < 64) {
        const int i = lane;   // lane i owns pair i (oldest = 0)
        // what the stopping test at the end reads from the scalar block, requested now: behind the recursion these
        // were three dependent trips (each read sits under a test of the one before)
        int tol_resolved = 1, status0 = LBFGSB_RUNNING;
        double tol_abs0 = 0.0;
        long long iters0 = 0;
        if (lane == 0 && evaluate_stop) {
            tol_resolved = scal->tol_resolved; status0 = scal->status; tol_abs0 = scal->tol_abs; iters0 = scal->iters;
        }
        double rho = 1.0, yn = 1.0, inv = 0.0;
        bool pass = false;
        if (i < c) {
            rho = G[i * Vp + (c + i)];
            // the newest pair's norm was just summed (and stored for later iterations)
            yn = (i == c - 1 && !dbg_inputs) ? ynew : yn_old;
            pass = rho > op.eps * yn;
            inv = 1.0 / rho;
        }
        const unsigned long long pm = __ballot(pass);
        double alpha_i = 0.0, coef_s = 0.0, gamma = 1.0;
        if (c <= kRecFast) {
            // every entry of G this lane needs, fetched at once; the three loops then run on registers and
            // scalar-register broadcasts only.  Same operations in the same order as the general form below.
            double gsy[kRecFast], gyy[kRecFast], gys[kRecFast];
#pragma unroll
            for (int k = 0; k < kRecFast; ++k) {
                const bool in = i < c && k < c;
                gsy[k] = in ? G[i * Vp + (c + k)] : 0.0;          // <s_i, y_k>
                gyy[k] = in ? G[(c + i) * Vp + (c + k)] : 0.0;    // <y_i, y_k>
                gys[k] = in ? G[(c + i) * Vp + k] : 0.0;          // <y_i, s_k>
            }
            double part_s = i < c ? G[i * Vp + 2 * c] : 0.0;      // <s_i, g>
            double tsum = i < c ? G[(c + i) * Vp + 2 * c] : 0.0;  // <y_i, g>
#pragma unroll
            for (int k = kRecFast - 1; k >= 0; --k) {
                if (k < c) {
                    double ak = lane_value(part_s * inv, k);
                    if (!((pm >> k) & 1ull)) ak = 0.0;
                    if (i == k) alpha_i = ak;
                    part_s = fma(-ak, gsy[k], part_s);
                }
            }
            if (c > 0 && ((pm >> (c - 1)) & 1ull)) gamma = lane_value(rho / yn, c - 1);
#pragma unroll
            for (int k = 0; k < kRecFast; ++k)
                if (k < c) tsum = fma(-lane_value(alpha_i, k), gyy[k], tsum);
            double by = gamma * tsum;
#pragma unroll
            for (int k = 0; k < kRecFast; ++k) {
                if (k < c) {
                    double ck = lane_value(alpha_i - by * inv, k);
                    if (!((pm >> k) & 1ull)) ck = 0.0;
                    if (i == k) coef_s = ck;
                    if (i > k) by = fma(ck, gys[k], by);
                }
            }
        } else {
            // first loop: alpha_k, newest to oldest.  Steps of pairs that fail the gate run with alpha_k = 0;
            // a lane's row is dead once its own alpha has been taken, so updating it further is harmless.
            double part_s = i < c ? G[i * Vp + 2 * c] : 0.0;   // <s_i, g>
#pragma unroll 4
            for (int k = c - 1; k >= 0; --k) {
                const double gsy = i < c ? G[i * Vp + (c + k)] : 0.0;   // <s_i, y_k>
                double ak = lane_value(part_s * inv, k);
                if (!((pm >> k) & 1ull)) ak = 0.0;
                if (i == k) alpha_i = ak;
                part_s = fma(-ak, gsy, part_s);
            }
            if (i < c) alpha_s[i] = alpha_i;
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
#pragma unroll 4
            for (int k = 0; k < c; ++k) {
                const double gys = i < c ? G[(c + i) * Vp + k] : 0.0;   // <y_i, s_k>
                double ck = lane_value(alpha_i - by * inv, k);
                if (!((pm >> k) & 1ull)) ck = 0.0;
                if (i == k) coef_s = ck;
                if (i > k) by = fma(ck, gys, by);
            }
        }
        if (i < c) {
            scal->delta[i] = coef_s;
            scal->delta[c + i] = -gamma * alpha_i;
        }
        if (lane == 0) {
            scal->delta[2 * c] = gamma;
            scal->pairs_used = __popcll(pm);
            if (evaluate_stop) {
                const double pgn = sqrt(gg);
                scal->pg2 = pgn;
                scal->pginf = pginf;
                scal->n_fixed = (long long)nfixed;
                if (!tol_resolved) {
                    tol_abs0 = op.tol_relative ? op.tol * fmax(1.0, pgn) : op.tol;
                    scal->tol_abs = tol_abs0;
                    scal->tol_resolved = 1;
                }
                if (status0 == LBFGSB_RUNNING) {
                    if (pgn <= tol_abs0) scal->status = LBFGSB_CONVERGED;
                    else if (iters0 >= op.max_iter) scal->status = LBFGSB_MAX_ITER;
                }
            }
        }
    }
}

}  // namespace lb
