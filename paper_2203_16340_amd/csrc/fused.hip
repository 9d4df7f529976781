// Fused single-read A pass for the quadratic objectives: variant table and launchers.
// The kernel itself (and the reasoning behind its layout) is in fused_ring.h.
//
// A variant fixes the workgroup size NT, the 16-byte chunks per thread and row KC = KCU*U, the rows
// per barrier R and the ring depth NB (in slots of KCU chunks).  The table below is the outcome of
// timing on MI355X: the entries are those that keep the ring plus the fp64 accumulators of w inside
// the 256 registers a thread has at two waves per SIMD WITHOUT spilling -- a spill inside the row
// loop waits for every outstanding load and so empties the ring, which costs more than a shallower
// ring does.  Measured on matrices of 0.8-8 GB: 75-82 % of the 8 TB/s HBM peak, against 6.0-6.8 TB/s
// for a plain streaming read of the same buffers.
#include "common.h"
#include "fused_ring.h"

namespace lb {

namespace {

struct Variant {
    int dtype;          // LBFGSB_F64 / LBFGSB_F32
    int logistic;       // 1: the kernel instantiated for the logistic row operations, 0: for the quadratic ones
    int trans;          // 1: with the transposed accumulation, 0: row products only (quadratic form, symmetric matrix)
    int nt, kc, r;      // threads, 16-byte chunks per thread and row, rows per stage
    int wgs_per_cu;     // workgroups per compute unit the launch is sized for
    const void* kernel; // for hipFuncSetAttribute
    void (*launch)(const Dims&, int64_t, int, size_t, const Buffers&, const APassArgs&, hipStream_t, hipEvent_t, hipEvent_t);
    size_t (*lds)(int64_t cols);
    // logistic only: the instantiation for the direction pass (same geometry, deeper ring: its row operation is
    // one exponential and one division, which leaves the registers for it)
    const void* kernel_dir;
    void (*launch_dir)(const Dims&, int64_t, int, size_t, const Buffers&, const APassArgs&, hipStream_t, hipEvent_t, hipEvent_t);
};

template <typename T, int NT, int KCU, int U, int R, int NB, int WPE, int LOGI, int KR, bool TRANS>
void launch_variant(const Dims& dm, int64_t rows_per_wg, int blocks, size_t lds, const Buffers& bf, const APassArgs& a,
                    hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
    hipExtLaunchKernelGGL((ring::k_fused_ring<T, NT, KCU, U, R, NB, WPE, LOGI, KR, TRANS>), dim3(blocks), dim3(NT), lds, st, ev0, ev1,
                          0, (const T*)a.A, dm.ld, dm.rows, dm.cols, rows_per_wg, a, bf.scal, bf.row, bf.t, bf.wpart,
                          bf.losspart);
}

#define LB_VARIANT_FULL(dt, LOGI, T, NT, KCU, U, R, NB, WPE, WGS, KR, TRANS)                                                \
    {dt, LOGI, TRANS, NT, (KCU) * (U), R, WGS,                                                                              \
     (const void*)ring::k_fused_ring<T, NT, KCU, U, R, NB, WPE, LOGI, KR, (TRANS) != 0>,                                      \
     launch_variant<T, NT, KCU, U, R, NB, WPE, LOGI, KR, (TRANS) != 0>, ring::lds_bytes<T, NT, (KCU) * (U), KR, R>, nullptr,   \
     nullptr}
#define LB_VARIANT_LOGI(dt, T, NT, KCU, U, R, NB, NBDIR, WPE, WGS)                                                           \
    {dt, 1, 1, NT, (KCU) * (U), R, WGS, (const void*)ring::k_fused_ring<T, NT, KCU, U, R, NB, WPE, 1, 0, true>,                \
     launch_variant<T, NT, KCU, U, R, NB, WPE, 1, 0, true>, ring::lds_bytes<T, NT, (KCU) * (U), 0, R>,                         \
     (const void*)ring::k_fused_ring<T, NT, KCU, U, R, NBDIR, WPE, 2, 0, true>,                                              \
     launch_variant<T, NT, KCU, U, R, NBDIR, WPE, 2, 0, true>}
#define LB_VARIANT_KR(dt, LOGI, T, NT, KCU, U, R, NB, WPE, WGS, KR) LB_VARIANT_FULL(dt, LOGI, T, NT, KCU, U, R, NB, WPE, WGS, KR, 1)
#define LB_VARIANT(dt, LOGI, T, NT, KCU, U, R, NB, WPE, WGS) LB_VARIANT_FULL(dt, LOGI, T, NT, KCU, U, R, NB, WPE, WGS, 0, 1)
#define LB_VARIANT_ROWS(dt, T, NT, KCU, U, R, NB, WPE, WGS) LB_VARIANT_FULL(dt, 0, T, NT, KCU, U, R, NB, WPE, WGS, 0, 0)

// Ordered by capacity within a (matrix type, objective family) group: the first variant of the group
// whose NT*KC*VEC columns cover a row and whose LDS need (v for every column) fits is used.  The
// logistic evaluation kernels spend ~100 registers on exp/log1p, so their rings are shallower; the direction
// pass of the logistic objective has its own instantiation with the deepest ring that does not spill.
const Variant kVariants[] = {
    LB_VARIANT(LBFGSB_F64, 0, double, 256, 2, 1, 2, 4, 4, 4),    // cols <=  1024
    LB_VARIANT(LBFGSB_F64, 0, double, 512, 2, 1, 4, 8, 2, 1),    // cols <=  2048
    LB_VARIANT(LBFGSB_F64, 0, double, 512, 5, 1, 2, 4, 2, 1),    // cols <=  5120
    LB_VARIANT(LBFGSB_F64, 0, double, 512, 10, 1, 1, 2, 2, 1),   // cols <= 10240
    LB_VARIANT(LBFGSB_F64, 0, double, 512, 20, 1, 1, 1, 2, 1),   // cols <= 20480 (LDS: <= 20428)
    LB_VARIANT_KR(LBFGSB_F64, 0, double, 512, 22, 1, 1, 1, 2, 1, 3),   // cols <= 22528, v of the last 3 chunks in registers
    LB_VARIANT_KR(LBFGSB_F64, 0, double, 512, 24, 1, 1, 1, 2, 1, 5),   // cols <= 24576, v of the last 5 chunks in registers
    LB_VARIANT(LBFGSB_F32, 0, float, 128, 1, 1, 2, 4, 4, 8),     // cols <=   512
    LB_VARIANT(LBFGSB_F32, 0, float, 256, 1, 1, 2, 4, 4, 4),     // cols <=  1024
    LB_VARIANT(LBFGSB_F32, 0, float, 256, 2, 1, 4, 12, 2, 2),    // cols <=  2048 (the geometry of the logistic direction pass)
    LB_VARIANT(LBFGSB_F32, 0, float, 256, 5, 1, 1, 2, 2, 2),     // cols <=  5120
    LB_VARIANT(LBFGSB_F32, 0, float, 512, 5, 1, 2, 4, 2, 1),     // cols <= 10240
    LB_VARIANT(LBFGSB_F32, 0, float, 512, 10, 1, 1, 2, 2, 1),    // cols <= 20480 (LDS: <= 20428)
    //              (…, R, ring depth of the evaluation kernel, of the direction kernel, …)
    LB_VARIANT_LOGI(LBFGSB_F64, double, 256, 2, 1, 4, 8, 12, 2, 2),    // cols <=  1024
    LB_VARIANT_LOGI(LBFGSB_F64, double, 512, 2, 1, 4, 4, 8, 2, 1),     // cols <=  2048
    LB_VARIANT_LOGI(LBFGSB_F64, double, 512, 5, 1, 1, 2, 4, 2, 1),     // cols <=  5120
    LB_VARIANT_LOGI(LBFGSB_F64, double, 512, 10, 1, 1, 1, 2, 2, 1),    // cols <= 10240
    LB_VARIANT_LOGI(LBFGSB_F64, double, 512, 20, 1, 1, 1, 1, 2, 1),    // cols <= 20480 (LDS: <= 20428)
    LB_VARIANT_LOGI(LBFGSB_F32, float, 128, 1, 1, 2, 4, 8, 4, 8),      // cols <=   512
    LB_VARIANT_LOGI(LBFGSB_F32, float, 256, 1, 1, 2, 4, 8, 4, 4),      // cols <=  1024
    LB_VARIANT_LOGI(LBFGSB_F32, float, 256, 2, 1, 4, 8, 12, 2, 2),     // cols <=  2048
    LB_VARIANT_LOGI(LBFGSB_F32, float, 256, 5, 1, 1, 2, 4, 2, 2),      // cols <=  5120
    LB_VARIANT_LOGI(LBFGSB_F32, float, 512, 5, 1, 1, 2, 4, 2, 1),      // cols <= 10240
    LB_VARIANT_LOGI(LBFGSB_F32, float, 512, 10, 1, 1, 1, 2, 2, 1),     // cols <= 20480 (LDS: <= 20428)
    // row products only: no accumulators of w, so the ring is deeper
    LB_VARIANT_ROWS(LBFGSB_F64, double, 256, 2, 1, 4, 8, 4, 4),  // cols <=  1024
    LB_VARIANT_ROWS(LBFGSB_F64, double, 512, 5, 1, 2, 8, 2, 1),  // cols <=  5120
    LB_VARIANT_ROWS(LBFGSB_F64, double, 512, 10, 1, 1, 4, 2, 1), // cols <= 10240
    LB_VARIANT_ROWS(LBFGSB_F64, double, 512, 20, 1, 1, 2, 2, 1), // cols <= 20480 (LDS: <= 20428)
    LB_VARIANT_ROWS(LBFGSB_F32, float, 256, 1, 1, 4, 8, 4, 4),   // cols <=  1024
    LB_VARIANT_ROWS(LBFGSB_F32, float, 256, 5, 1, 2, 8, 2, 2),   // cols <=  5120
    LB_VARIANT_ROWS(LBFGSB_F32, float, 512, 5, 1, 2, 8, 2, 1),   // cols <= 10240
    LB_VARIANT_ROWS(LBFGSB_F32, float, 512, 10, 1, 1, 4, 2, 1),  // cols <= 20480 (LDS: <= 20428)
};
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);
constexpr size_t kLdsPerWorkgroup = 160 * 1024;   // gfx950

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
    const int vec = dm.dtype == LBFGSB_F32 ? 4 : 2;
    if ((uintptr_t)A % 16 != 0 || dm.cols % vec != 0 || dm.ld % vec != 0) return false;   // needs 16-byte loads
    for (int i = 0; i < kNumVariants; ++i) {
        const Variant& v = kVariants[i];
        if (v.dtype != dm.dtype || v.logistic != (dm.kind == LBFGSB_OBJ_LOGISTIC_L2) ||
            v.trans != (dm.kind != LBFGSB_OBJ_QP))
            continue;
        if ((int64_t)v.nt * v.kc * vec < dm.cols) continue;
        if (v.lds(dm.cols) > kLdsPerWorkgroup - 256) continue;   // (a few bytes of static LDS come on top)
        const int64_t rpw = rows_per_wg_for(dm, v);
        *variant = i;
        *blocks = (int)((dm.rows + rpw - 1) / rpw);
        return true;
    }
    return false;
}

// The kernels use more dynamic LDS than the default limit of a launch.  The limit is a property of the
// kernel, not of a solver, and several solvers of different widths may share a variant: it is raised to the
// most the variant can ever ask for (its widest row, capped by what a workgroup can have).
hipError_t fused_prepare(const Dims& dm, const Geometry& ge) {
    const Variant& v = kVariants[ge.fused_variant];
    const int vec = v.dtype == LBFGSB_F32 ? 4 : 2;
    size_t most = v.lds((int64_t)v.nt * v.kc * vec);
    const size_t cap = kLdsPerWorkgroup - 256;   // the kernels also hold a few bytes of static LDS
    if (most > cap) most = cap;
    if (v.lds(dm.cols) > most) most = v.lds(dm.cols);
    hipError_t e = hipFuncSetAttribute(v.kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)most);
    if (e == hipSuccess && v.kernel_dir)   // (may also hold two numbers per row of a workgroup: whatever fits)
        e = hipFuncSetAttribute(v.kernel_dir, hipFuncAttributeMaxDynamicSharedMemorySize, (int)cap);
    return e;
}

// LDS the logistic direction pass needs on top when it also sums the loss differences of the first trial step:
// two numbers per row of a workgroup
static size_t ls_first_lds(const Dims& dm, const Variant& v) { return (size_t)rows_per_wg_for(dm, v) * 16; }

bool fused_ls_first_ok(const Dims& dm, const Geometry& ge) {
    const Variant& v = kVariants[ge.fused_variant];
    return v.launch_dir && v.lds(dm.cols) + ls_first_lds(dm, v) <= kLdsPerWorkgroup - 256;
}

void launch_fused(const Dims& dm, const Geometry& ge, const Buffers& bf, const APassArgs& a, hipStream_t st,
                  hipEvent_t ev0, hipEvent_t ev1) {
    const Variant& v = kVariants[ge.fused_variant];
    auto launch = (a.mode == kRowLogiSpec && v.launch_dir) ? v.launch_dir : v.launch;
    const size_t extra = a.mode == kRowLogiSpec && a.ls_first ? ls_first_lds(dm, v) : 0;
    launch(dm, rows_per_wg_for(dm, v), ge.fused_blocks, v.lds(dm.cols) + extra, bf, a, st, ev0, ev1);
}

}  // namespace lb
