// Internal declarations shared by the HIP translation units of libsrigl (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "srigl.h"

namespace srigl {

constexpr int kWave = 64;              // CDNA wavefront width
constexpr int kSegCols = 64;           // columns per entry of the seg table
constexpr size_t kLdsMax = 160 * 1024; // LDS per workgroup on gfx950

struct FwdArgs {
    const void* x;
    int32_t x_bf16;
    int32_t B, d_in;
    const void* W_c;
    const void* idx;     // int32_t, or uint16_t when idx_u16
    int32_t idx_u16;
    const int32_t* active;
    int32_t n_active, K;
    const float* bias;
    int32_t d_out;
    float* y;
    const uint16_t* seg;
    int32_t seg_stride;
    int32_t act;   // srigl_activation applied to every written value (stored and ablated columns alike)
};

// Launch shape of the ROWLANE kernel, decided on the host.
struct RowlanePlan {
    int R, H, NW, NPW, KPRE, C, n_chunks, n_btiles, n_groups;
    size_t lds;
    double cost;  // the planner's estimate for this shape (arbitrary units), to compare shapes
    int out_off;  // word offset of the result tile in LDS (0: it reuses the activation tile after a barrier)
    bool fast;   // x rows allow aligned 4-element loads and d_in is a multiple of 16
    bool ok;
};
constexpr int kStageUnits = 8;   // 16x16 staging units a wavefront holds in registers per chunk
constexpr int kBlock = 16;       // terms per vector load of W_c / idx (one DPP row)
constexpr int rowlane_max_threads(int) { return 1024; }
// stored rows per wavefront the register budget allows without spilling
constexpr int rowlane_max_npw(int R) { return R == 1 ? 6 : 4; }
// blocks of 16 terms per (stored row, chunk) kept in registers, by stored rows per wavefront
constexpr int rowlane_kpre(int npw) { return npw <= 3 ? 3 : (npw <= 4 ? 2 : 1); }
srigl_status launch_rowlane_f32(const FwdArgs& a, const RowlanePlan& p, hipStream_t st);
srigl_status launch_rowlane_bf16(const FwdArgs& a, const RowlanePlan& p, hipStream_t st);
srigl_status launch_rowlane_f32_i16(const FwdArgs& a, const RowlanePlan& p, hipStream_t st);
srigl_status launch_rowlane_bf16_i16(const FwdArgs& a, const RowlanePlan& p, hipStream_t st);

// Each returns SRIGL_OK, SRIGL_ERR_UNSUPPORTED (cannot run these sizes) or SRIGL_ERR_HIP.
srigl_status launch_fwd_generic(const FwdArgs& a, hipStream_t st);
srigl_status launch_fwd_klane(const FwdArgs& a, const srigl_fwd_tuning* t, hipStream_t st);
srigl_status launch_fwd_rowlane(const FwdArgs& a, const srigl_fwd_tuning* t, hipStream_t st);
bool rowlane_supported(const FwdArgs& a, const srigl_fwd_tuning* t);
srigl_fwd_algo choose_fwd_algo(const FwdArgs& a);

// Estimated time (us, operands in cache) of the small-batch forward kernel: a fixed part plus a part per term slot (K rounded
// up to the slots one request of a lane group covers; dearer with one batch row per workgroup, the wide-input setting).
// A fit of timings of 512- to 4096-wide layers at 80-90 % sparsity; used to pick the kernel for batches of 5 to 64 rows and
// by the choice between the condensed and the structured-only form.
inline double klane_estimate_us(int B, int d_in, int n_active, int K) {
    int L = 4;
    while (L < 64 && L * 4 < K) L <<= 1;
    const int req = L * 4;   // term slots one request of a lane group covers (4 terms per lane)
    const double slots = (double)B * n_active * ((K + req - 1) / req * req);
    return 3.2 + 0.0005 * d_in + (d_in <= 1024 ? 0.44e-6 : 0.6e-6) * slots;
}

inline srigl_status hip_ok(hipError_t e) { return e == hipSuccess ? SRIGL_OK : SRIGL_ERR_HIP; }

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

// Activation between the two linear layers of an MLP block: identity, max(v, 0), or v * Phi(v) with the normal
// distribution function Phi (the exact, erf-based GELU).
__device__ __forceinline__ float apply_act(float v, int act) {
    if (act == SRIGL_ACT_RELU) return fmaxf(v, 0.0f);
    if (act == SRIGL_ACT_GELU) return 0.5f * v * (1.0f + erff(v * 0.70710678118654752440f));
    return v;
}

}  // namespace srigl
