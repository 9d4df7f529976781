// Fused single-read A pass for the quadratic objectives.
//
// For f(x) = 0.5*||A v(x) - b||^2 (+ linear terms) one iteration needs t = A v_p and w = A^T t
// (direction pass), and an evaluation needs r = A v - b and A^T r.  Both have the shape
//     u_r = a_r . v,   psi_r = rowop(u_r),   w += a_r * psi_r      for every row r,
// so a workgroup that owns WHOLE rows can keep a row in registers between its dot product and its
// contribution to w, and A is read from HBM exactly once per pass instead of twice.
//
// Layout: a workgroup of NT threads covers all columns; thread `tid` owns the 16-byte chunks
// (k*NT + tid), k = 0..KC-1, of every row (coalesced: a wave reads 1 KiB contiguous per load
// instruction), the matching entries of v and fp64 accumulators for the matching entries of w, all
// in registers.  Rows are dealt to workgroups in contiguous ranges and processed R at a time:
// R*KC loads are issued back to back, the R partial dot products are reduced across the workgroup
// (wave shuffles, then one LDS exchange and one barrier), the row operation is applied, and w is
// updated from the registers.  Each workgroup writes its partial w (summed later in workgroup
// order, so results are bit-reproducible) and one loss partial.
//
// Bytes: rows*cols*sizeof(T) read once, plus G*cols*8 written (G workgroups) and rows*8 for t or r.
#include "common.h"
#include "apass_rowop.h"

namespace lb {

namespace {

template <typename T> struct Raw;
template <> struct Raw<float> { using type = float4; };
template <> struct Raw<double> { using type = double2; };

__device__ __forceinline__ void widen(const float4& r, double (&o)[4]) { o[0] = r.x; o[1] = r.y; o[2] = r.z; o[3] = r.w; }
__device__ __forceinline__ void widen(const double2& r, double (&o)[2]) { o[0] = r.x; o[1] = r.y; }
// Makes the compiler forget what it knows about a loaded fp32 chunk, so that it converts it to fp64
// a second time instead of holding both copies in registers.
__device__ __forceinline__ void keep_raw(float4& r) { asm volatile("" : "+v"(r.x), "+v"(r.y), "+v"(r.z), "+v"(r.w)); }
__device__ __forceinline__ void keep_raw(double2&) {}
__device__ __forceinline__ float4 zero_raw(const float*) { return make_float4(0.f, 0.f, 0.f, 0.f); }
__device__ __forceinline__ double2 zero_raw(const double*) { return make_double2(0.0, 0.0); }

// row operation of the quadratic objectives; every thread computes psi, `writer` also stores the row entry
__device__ __forceinline__ double quad_row_op(int mode, double u, int64_t r, const double* __restrict__ b, bool writer,
                                              double* __restrict__ row, double* __restrict__ t, double& psi) {
    if (mode == kRowDir) {
        psi = u;
        if (writer) t[r] = u;
        return u * u;
    }
    const double res = u - b[r];
    psi = res;
    if (writer) row[r] = res;
    return 0.5 * res * res;
}

template <typename T, int NT, int KC, int R, int WPE>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(WPE, WPE)))
void k_fused(const T* __restrict__ A, int64_t ld, int64_t rows, int64_t cols, int64_t rows_per_wg, APassArgs a,
             const Scal* __restrict__ scal, double* __restrict__ row, double* __restrict__ t,
             double* __restrict__ wpart, double* __restrict__ losspart) {
    using RawT = typename Raw<T>::type;
    constexpr int VEC = 16 / sizeof(T);
    constexpr int NW = NT / 64;
    __shared__ double red[2][R][NW];
    if (a.check_status && scal->status != LBFGSB_RUNNING) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const double *va, *vb;
    resolve_v(a, scal, cols, va, vb);

    // chunk k of this thread starts at column (k*NT + tid)*VEC: a per-thread offset plus a
    // compile-time stride, so the addresses need no registers of their own
    const int64_t c0 = (int64_t)tid * VEC;
    constexpr int64_t kStride = (int64_t)NT * VEC;
    double v[KC][VEC], w[KC][VEC];
#pragma unroll
    for (int k = 0; k < KC; ++k) {
        const bool act = c0 + k * kStride < cols;
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
            double x = 0.0;
            if (act) {
                x = va[c0 + k * kStride + j];
                if (vb) x -= vb[c0 + k * kStride + j];
            }
            v[k][j] = x;
            w[k][j] = 0.0;
        }
    }

    const int64_t r_begin = (int64_t)blockIdx.x * rows_per_wg;
    const int64_t r_end = r_begin + rows_per_wg < rows ? r_begin + rows_per_wg : rows;
    double loss = 0.0;
    int par = 0;
    for (int64_t r0 = r_begin; r0 < r_end; r0 += R) {
        RawT raw[R][KC];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int64_t rr = r0 + r < r_end ? r0 + r : r_end - 1;   // tail rows reload the last row; their psi is 0
            const T* rp = A + rr * ld + c0;
#pragma unroll
            for (int k = 0; k < KC; ++k)
                raw[r][k] = (c0 + k * kStride < cols) ? *reinterpret_cast<const RawT*>(rp + k * kStride)
                                                      : zero_raw((const T*)nullptr);
        }
        double acc[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            double s = 0.0;
#pragma unroll
            for (int k = 0; k < KC; ++k) {
                double e[VEC];
                widen(raw[r][k], e);
#pragma unroll
                for (int j = 0; j < VEC; ++j) s = fma(e[j], v[k][j], s);
            }
            acc[r] = wave_sum(s);
        }
        if (lane == 0) {
#pragma unroll
            for (int r = 0; r < R; ++r) red[par][r][wave] = acc[r];
        }
        __syncthreads();
        double psi[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            double u = 0.0;
#pragma unroll
            for (int q = 0; q < NW; ++q) u += red[par][r][q];
            psi[r] = 0.0;
            if (r0 + r < r_end) loss += quad_row_op(a.mode, u, r0 + r, a.b, tid == 0, row, t, psi[r]);
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
#pragma unroll
            for (int k = 0; k < KC; ++k) {
                keep_raw(raw[r][k]);   // fp32 data is widened again here rather than kept widened across the barrier
                double e[VEC];
                widen(raw[r][k], e);
#pragma unroll
                for (int j = 0; j < VEC; ++j) w[k][j] = fma(e[j], psi[r], w[k][j]);
            }
        }
        par ^= 1;
    }
    double* out = wpart + (int64_t)blockIdx.x * cols + c0;
#pragma unroll
    for (int k = 0; k < KC; ++k) {
        if (c0 + k * kStride < cols) {
#pragma unroll
            for (int j = 0; j < VEC; ++j) out[k * kStride + j] = w[k][j];
        }
    }
    if (tid == 0) losspart[blockIdx.x] = loss;
}

struct Variant {
    int dtype;       // LBFGSB_F64 / LBFGSB_F32
    int nt, kc, r;   // threads, 16-byte chunks per thread and row, rows per stage
    int wgs_per_cu;  // resident workgroups per compute unit the register budget allows
    void (*launch)(const Dims&, int64_t, int, const Buffers&, const APassArgs&, hipStream_t, hipEvent_t, hipEvent_t);
};

template <typename T, int NT, int KC, int R, int WPE>
void launch_variant(const Dims& dm, int64_t rows_per_wg, int blocks, const Buffers& bf, const APassArgs& a,
                    hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
    hipExtLaunchKernelGGL((k_fused<T, NT, KC, R, WPE>), dim3(blocks), dim3(NT), 0, st, ev0, ev1, 0, (const T*)a.A, dm.ld,
                          dm.rows, dm.cols, rows_per_wg, a, (const Scal*)bf.scal, bf.row, bf.t, bf.wpart, bf.losspart);
}

// Ordered by capacity: the first variant whose NT*KC*VEC columns cover the row is used.
const Variant kVariants[] = {
    {LBFGSB_F64, 256, 10, 3, 2, launch_variant<double, 256, 10, 3, 2>},   // cols <=  5120
    {LBFGSB_F64, 512, 10, 2, 1, launch_variant<double, 512, 10, 2, 2>},   // cols <= 10240
    {LBFGSB_F64, 512, 20, 1, 1, launch_variant<double, 512, 20, 1, 2>},   // cols <= 20480
    {LBFGSB_F32, 256, 5, 4, 2, launch_variant<float, 256, 5, 4, 2>},      // cols <=  5120
    {LBFGSB_F32, 512, 5, 4, 1, launch_variant<float, 512, 5, 4, 2>},      // cols <= 10240
    {LBFGSB_F32, 512, 10, 1, 1, launch_variant<float, 512, 10, 1, 2>},    // cols <= 20480
};
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);

int compute_units() {
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess &&
            prop.multiProcessorCount > 0)
            cus = prop.multiProcessorCount;
        else
            cus = 256;   // MI355X; also the answer on a machine without a GPU (sizes only)
        (void)hipGetLastError();
    }
    return cus;
}

int64_t rows_per_wg_for(const Dims& dm, const Variant& v) {
    const int64_t slots = (int64_t)compute_units() * v.wgs_per_cu;
    int64_t rpw = (dm.rows + slots - 1) / slots;
    rpw = (rpw + v.r - 1) / v.r * v.r;
    return rpw < v.r ? v.r : rpw;
}

}  // namespace

bool fused_shape_ok(const Dims& dm, const void* A, int* variant, int* blocks) {
    *variant = -1;
    *blocks = 0;
    if (dm.kind == LBFGSB_OBJ_LOGISTIC_L2) return false;
    const int vec = dm.dtype == LBFGSB_F32 ? 4 : 2;
    if ((uintptr_t)A % 16 != 0 || dm.cols % vec != 0 || dm.ld % vec != 0) return false;   // needs 16-byte loads
    for (int i = 0; i < kNumVariants; ++i) {
        const Variant& v = kVariants[i];
        if (v.dtype != dm.dtype) continue;
        if ((int64_t)v.nt * v.kc * vec < dm.cols) continue;
        const int64_t rpw = rows_per_wg_for(dm, v);
        *variant = i;
        *blocks = (int)((dm.rows + rpw - 1) / rpw);
        return true;
    }
    return false;
}

void launch_fused(const Dims& dm, const Geometry& ge, const Buffers& bf, const APassArgs& a, hipStream_t st,
                  hipEvent_t ev0, hipEvent_t ev1) {
    const Variant& v = kVariants[ge.fused_variant];
    v.launch(dm, rows_per_wg_for(dm, v), ge.fused_blocks, bf, a, st, ev0, ev1);
}

}  // namespace lb
