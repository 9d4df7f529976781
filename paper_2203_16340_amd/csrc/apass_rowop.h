// Pieces shared by the two organisations of the A pass: 16-byte loads widened to fp64, the choice
// of the vector A multiplies, and the objective's per-row operation.
#pragma once

#include "common.h"

namespace lb {

template <typename T, int VEC>
struct Loader;
template <>
struct Loader<float, 4> {
    static __device__ __forceinline__ void load(const float* p, double (&o)[4]) {
        const float4 v = *reinterpret_cast<const float4*>(p);
        o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
    }
};
template <>
struct Loader<double, 2> {
    static __device__ __forceinline__ void load(const double* p, double (&o)[2]) {
        const double2 v = *reinterpret_cast<const double2*>(p);
        o[0] = v.x; o[1] = v.y;
    }
};
template <typename T>
struct Loader<T, 1> {
    static __device__ __forceinline__ void load(const T* p, double (&o)[1]) { o[0] = (double)*p; }
};

// Resolves the vector A multiplies: either fixed pointers, or the direction Algorithm 2 selected.
// branch: Algorithm 2's choice when the caller has made it itself (0: read it from the scalar block)
__device__ __forceinline__ void resolve_v(const APassArgs& a, const Scal* scal, int64_t cols, const double*& va,
                                          const double*& vb, int branch = 0) {
    va = a.va;
    vb = a.vb;
    if (a.select_p) {
        va = (branch ? branch : scal->branch) == 1 ? a.p1 : a.p2;
        vb = a.split ? va + cols : nullptr;
    }
}

// The objective's per-row operation on u = a_r . v.  Returns the row's loss contribution.
__device__ __forceinline__ double row_op(int mode, double u, int64_t r, int64_t rows, const double* __restrict__ b,
                                         const double* __restrict__ w, double* __restrict__ row,
                                         double* __restrict__ t, double* __restrict__ psi) {
    switch (mode) {
        case kRowLsqEval: {
            const double res = u - b[r];
            const double wr = w ? w[r] : 1.0;
            row[r] = res;
            psi[r] = wr * res;
            return 0.5 * wr * res * res;
        }
        case kRowDir: {
            const double wr = w ? w[r] : 1.0;
            t[r] = u;
            psi[r] = wr * u;
            return wr * u * u;
        }
        case kRowLogiEval: {
            const double y = b[r];
            const double a = -y * u;
            row[r] = u;
            psi[r] = -y * sigmoid_d(a) / (double)rows;
            return softplus_d(a) / (double)rows;
        }
        case kRowLogiDir:
            t[r] = u;
            return 0.0;
        default:
            return 0.0;   // the QP modes need the row's own entry of v: see k_gemv
    }
}

}  // namespace lb
