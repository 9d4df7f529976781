// What the wide Gram kernel (gram.hip) and the direction kernel (vec.hip) share: the layout of a workgroup's partial
// sums, their addition in workgroup order, and the closing step -- Gram matrix in the recursion's order, pending
// update, Algorithm 3 on coefficients with the stopping test.  The closing step runs either in the Gram kernel's last
// workgroup on the scalar block itself, or in every workgroup of the direction kernel on a private copy of it.
#pragma once

#include "common.h"
#include "recursion.h"

namespace lb {

constexpr int kGramHdr = 8;   // per-workgroup partial: [0] sum g[S]^2, [1] max KKT residual, [2] #fixed, [3] ||y_new||^2
constexpr int kGramOneLevelMax = 128;   // grids up to this size add their partials in one level

constexpr int kWideM = 10;
constexpr int kWideT = 2 * kWideM + 1;
constexpr int kWideG = 7;                                    // slots per group
constexpr int kWideDiag = kWideG * (kWideG + 1) / 2;         // 28
constexpr int kWideRole = kWideDiag + kWideG * kWideG;       // 77 entries per wave
constexpr int kWideEntries = kWideT * (kWideT + 1) / 2;      // 231 = 3 * 77
constexpr int kWideNE = kGramHdr + kWideEntries;
static_assert(3 * kWideG == kWideT && 3 * kWideRole == kWideEntries, "three groups of seven slots");

// entry index -> static slots (a, b)
__device__ __forceinline__ void wide_entry_slots(int idx, int& a, int& b) {
    const int r = idx / kWideRole;
    int q = idx % kWideRole;
    const int p0 = kWideG * r, q0 = kWideG * ((r + 1) % 3);
    if (q < kWideDiag) {
        int i = 0;
        while (q >= kWideG - i) { q -= kWideG - i; ++i; }
        a = p0 + i;
        b = p0 + i + q;
    } else {
        q -= kWideDiag;
        a = p0 + q / kWideG;
        b = q0 + q % kWideG;
    }
}

// Adds the partials of `nwg` workgroups (NE doubles each; entry 1 is a maximum, the others are sums) in workgroup
// order into tot[0 .. NE): thread idx takes entry idx, 64 partials at a time with every load of a batch issued before
// the first is used.  Called by all kBlock threads; no barrier inside.
__device__ __forceinline__ void gram_sum_partials_flat(const double* __restrict__ grampart, int NE, int nwg, double* tot) {
    constexpr int kBatch = 64;
    for (int idx = threadIdx.x; idx < NE; idx += kBlock) {
        double t = idx == 1 ? -INFINITY : 0.0;
        for (int k0 = 0; k0 < nwg; k0 += kBatch) {
            double v[kBatch];
#pragma unroll
            for (int k = 0; k < kBatch; ++k) v[k] = k0 + k < nwg ? grampart[(int64_t)(k0 + k) * NE + idx] : (idx == 1 ? -INFINITY : 0.0);
            if (idx == 1) {
#pragma unroll
                for (int k = 0; k < kBatch; ++k) t = fmax(t, v[k]);
            } else {
#pragma unroll
                for (int k = 0; k < kBatch; ++k) t += v[k];
            }
        }
        tot[idx] = t;
    }
}

// The closing step from the totals tot[0 .. kWideNE) (LDS, complete: a barrier lies between their last write and this
// call).  c, head: the ring as it will be once the pending update is applied; base_slot: ring slot of the oldest pair.
// Gs: (2 kWideM + 2)^2 doubles, alpha_s: kMaxM + 1 (both LDS).  sc: the scalar block this works on.
__device__ __forceinline__ void wide_finish(const double* tot, double* Gs, double* alpha_s, Scal* sc, int m,
                                            int c, int head, int base_slot, const Opts& op, double yn_old, int dbg_inputs,
                                            int evaluate_stop, bool record) {
    const int tid = threadIdx.x;
    const int V = 2 * c + 1, Vp = V + 1;
    // The update the previous kernel left pending is applied by the last thread while the others put the matrix
    // together: a chain of two dozen dependent accesses that nothing below the barrier has to wait for twice.  (c and
    // head already are the ring as it will be; the recursion reads the iteration count and the status after the barrier.)
    if (tid == kBlock - 1) apply_pending(sc, m, record);
    // static slots -> the recursion's order (s oldest..newest, y oldest..newest, g)
    for (int idx = tid; idx < kWideEntries; idx += kBlock) {
        int a, b;
        wide_entry_slots(idx, a, b);
        auto logical = [&](int slot) -> int {
            if (slot == 2 * kWideM) return 2 * c;
            const int ring = slot < kWideM ? slot : slot - kWideM;
            if (ring >= m) return -1;
            const int j = (ring - base_slot + m) % m;
            if (j >= c) return -1;
            return slot < kWideM ? j : c + j;
        };
        const int row = logical(a), col = logical(b);
        if (row >= 0 && col >= 0) {
            const double t = tot[kGramHdr + idx];
            Gs[row * Vp + col] = t;
            Gs[col * Vp + row] = t;
        }
    }
    __syncthreads();
    const double gg = Gs[(2 * c) * Vp + 2 * c];   // sum over the free set of g^2
    const double ynew = tot[3];                    // ||y_new||^2 over the full vector: kept for later iterations
    if (tid == 0 && c > 0 && !dbg_inputs) sc->ynorm2[(head - 1 + m) % m] = ynew;
    recursion_on_coefficients(Gs, Vp, c, head, m, op, sc, gg, tot[1], tot[2], ynew, yn_old, alpha_s, dbg_inputs, evaluate_stop);
}

}  // namespace lb
