// Products with the data matrix A (row-major, rows x cols): the only O(rows*cols) work of an
// iteration, and HBM-bandwidth bound (2 flops per element read).
//
// Two organisations:
//   two-pass : k_gemv  (u = A v, one wave per group of rows, lanes stride over the columns with
//              16-byte loads, fp64 accumulation) applies the per-row operation of the objective
//              and leaves per-row weights psi; k_gemvt (w = A^T psi, threads own columns, row
//              blocks produce partial columns) reads A a second time.
//   fused    : see fused.hip -- a workgroup owns whole rows, keeps them in registers between the
//              row dot product and the transposed accumulation, so A is read once.
// The two-pass kernels serve the shapes the fused kernel does not take (rows wider than its
// registers and LDS hold, unaligned rows), the transposed product after a rejected first trial
// step of the logistic objective (skipped when the fused pass's speculative step was accepted:
// check_status == 2), and the row products of the symmetric quadratic form when forced.
//
// The per-row operations (RowMode) are what "compute f and grad f" of Algorithm 1 means for the
// objectives (least squares with optional per-row weights, L1-split, logistic, the symmetric
// quadratic form with an optional sign vector applied to v), and the t = A p needed by the
// closed-form line search of the quadratic ones.
#include "common.h"
#include "apass_rowop.h"

namespace lb {

template <typename T, int VEC, int R>
__global__ __launch_bounds__(kBlock) void k_gemv(const T* __restrict__ A, int64_t ld, int64_t rows, int64_t cols,
                                                 APassArgs a, const Scal* __restrict__ scal,
                                                 double* __restrict__ row, double* __restrict__ t,
                                                 double* __restrict__ psi, double* __restrict__ losspart) {
    __shared__ double lds[kWaves];
    if (a.check_status && scal->status != LBFGSB_RUNNING) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const double *va, *vb;
    resolve_v(a, scal, cols, va, vb);
    const int64_t nwaves = (int64_t)gridDim.x * kWaves;
    double loss = 0.0;
    for (int64_t r0 = ((int64_t)blockIdx.x * kWaves + wave) * R; r0 < rows; r0 += nwaves * R) {
        double acc[R];
        const T* rp[R];
#pragma unroll
        for (int k = 0; k < R; ++k) {
            acc[k] = 0.0;
            const int64_t rr = r0 + k < rows ? r0 + k : rows - 1;
            rp[k] = A + rr * ld;
        }
#pragma unroll 2
        for (int64_t c = (int64_t)lane * VEC; c < cols; c += 64 * VEC) {
            double v[VEC];
#pragma unroll
            for (int j = 0; j < VEC; ++j) v[j] = va[c + j];
            if (vb) {
#pragma unroll
                for (int j = 0; j < VEC; ++j) v[j] -= vb[c + j];
            }
            if (a.vs) {
#pragma unroll
                for (int j = 0; j < VEC; ++j) v[j] *= a.vs[c + j];
            }
#pragma unroll
            for (int k = 0; k < R; ++k) {
                double e[VEC];
                Loader<T, VEC>::load(rp[k] + c, e);
#pragma unroll
                for (int j = 0; j < VEC; ++j) acc[k] = fma(e[j], v[j], acc[k]);
            }
        }
        double mine = 0.0;   // lane k applies the row operation of row r0 + k
#pragma unroll
        for (int k = 0; k < R; ++k) {
            const double tot = wave_sum(acc[k]);
            if (lane == k) mine = tot;
        }
        if (lane < R && r0 + lane < rows) {
            const int64_t r = r0 + lane;
            if (a.mode == kRowQpEval || a.mode == kRowQpDir) {
                // symmetric quadratic form: the row index is also a column index, v_r = s_r z_r
                const double vr = (va[r] - (vb ? vb[r] : 0.0)) * (a.vs ? a.vs[r] : 1.0);
                if (a.mode == kRowQpEval) { row[r] = mine; loss += 0.5 * vr * mine; }
                else { t[r] = mine; loss += vr * mine; }
            } else {
                loss += row_op(a.mode, mine, r, rows, a.b, a.w, row, t, psi);
            }
        }
    }
    double lv[1] = {loss};
    block_sum<1, kWaves>(lv, lds);
    if (threadIdx.x == 0) losspart[blockIdx.x] = lv[0];
}

// w = A^T psi: threads own VEC adjacent columns, a workgroup covers kBlock*VEC columns and a
// block of rows; partial columns go to wpart[row_block][c] and are summed (in row-block order)
// by the kernel that consumes w.
template <typename T, int VEC>
__global__ __launch_bounds__(kBlock) void k_gemvt(const T* __restrict__ A, int64_t ld, int64_t rows, int64_t cols,
                                                  const double* __restrict__ psi, double* __restrict__ wpart,
                                                  int64_t rows_per_block, const Scal* __restrict__ scal,
                                                  int check_status) {
    if (check_status && scal->status != LBFGSB_RUNNING) return;
    if (check_status == 2 && scal->spec_ok) return;   // the speculative single-read pass already produced these columns
    const int64_t c = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * VEC;
    if (c >= cols) return;
    const int64_t r0 = (int64_t)blockIdx.y * rows_per_block;
    const int64_t r1 = r0 + rows_per_block < rows ? r0 + rows_per_block : rows;
    double acc[VEC];
#pragma unroll
    for (int j = 0; j < VEC; ++j) acc[j] = 0.0;
    const T* p = A + r0 * ld + c;
#pragma unroll 8
    for (int64_t r = r0; r < r1; ++r, p += ld) {
        double e[VEC];
        Loader<T, VEC>::load(p, e);
        const double w = psi[r];
#pragma unroll
        for (int j = 0; j < VEC; ++j) acc[j] = fma(e[j], w, acc[j]);
    }
    double* out = wpart + (int64_t)blockIdx.y * cols + c;
#pragma unroll
    for (int j = 0; j < VEC; ++j) out[j] = acc[j];
}

template <typename T, int VEC>
static void gemv_dispatch(const Dims& dm, const Geometry& ge, const Buffers& bf, const APassArgs& a, hipStream_t st,
                          hipEvent_t ev0, hipEvent_t ev1) {
    hipExtLaunchKernelGGL((k_gemv<T, VEC, 4>), dim3(ge.gemv_blocks), dim3(kBlock), 0, st, ev0, ev1, 0, (const T*)a.A,
                          dm.ld, dm.rows, dm.cols, a, (const Scal*)bf.scal, bf.row, bf.t, bf.psi, bf.losspart);
}

void launch_gemv(const Dims& dm, const Geometry& ge, const Buffers& bf, const APassArgs& a, hipStream_t st,
                 hipEvent_t ev0, hipEvent_t ev1) {
    if (dm.dtype == LBFGSB_F32) {
        if (ge.vec > 1) gemv_dispatch<float, 4>(dm, ge, bf, a, st, ev0, ev1);
        else gemv_dispatch<float, 1>(dm, ge, bf, a, st, ev0, ev1);
    } else {
        if (ge.vec > 1) gemv_dispatch<double, 2>(dm, ge, bf, a, st, ev0, ev1);
        else gemv_dispatch<double, 1>(dm, ge, bf, a, st, ev0, ev1);
    }
}

template <typename T, int VEC>
static void gemvt_dispatch(const Dims& dm, const Geometry& ge, const Buffers& bf, const void* A, const double* psi,
                           int check_status, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
    hipExtLaunchKernelGGL((k_gemvt<T, VEC>), dim3(ge.gemvt_col_tiles, ge.gemvt_row_blocks), dim3(kBlock), 0, st, ev0,
                          ev1, 0, (const T*)A, dm.ld, dm.rows, dm.cols, psi, bf.wpart, ge.gemvt_rows_per_block,
                          (const Scal*)bf.scal, check_status);
}

// psi_src: the per-row weights (bf.psi after an evaluation, bf.t after a direction pass).
void launch_gemvt_from(const Dims& dm, const Geometry& ge, const Buffers& bf, const void* A, const double* psi_src,
                       int check_status, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
    if (dm.dtype == LBFGSB_F32) {
        if (ge.vec > 1) gemvt_dispatch<float, 4>(dm, ge, bf, A, psi_src, check_status, st, ev0, ev1);
        else gemvt_dispatch<float, 1>(dm, ge, bf, A, psi_src, check_status, st, ev0, ev1);
    } else {
        if (ge.vec > 1) gemvt_dispatch<double, 2>(dm, ge, bf, A, psi_src, check_status, st, ev0, ev1);
        else gemvt_dispatch<double, 1>(dm, ge, bf, A, psi_src, check_status, st, ev0, ev1);
    }
}

}  // namespace lb
