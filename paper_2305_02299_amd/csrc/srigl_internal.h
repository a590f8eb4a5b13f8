// Internal declarations shared by the HIP translation units of libsrigl (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <cmath>
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

// The small-batch forward kernel takes its activations either from global memory through the vector caches (a gather:
// no staging pass, no barrier, any d_in) or from rows of x staged in LDS.  Estimated times (us) of both, fits of timings
// (mean of cold and cached operands) of 512- to 4096-wide layers at 80-99 % sparsity and batches of 2 to 256; they pick the
// source of the activations, the kernel for batches of 2 to 2048 rows, and feed the choice between the condensed and the
// structured-only form.  Layers of more than ~1.5 M stored terms no longer sit in one XCD's L2: every pass over
// W_c / idx (one per workgroup row of the batch) then also pays for that stream.
//
// Batch rows per workgroup of the gathering form: a second and a fourth row pay once the pass over W_c / idx they save
// outweighs the longer chain of gathers per lane (measured: from ~1.2 M and ~3.5 M gathered terms).
inline int klane_gather_rows(int B, int n_active, int K) {
    const double work = (double)B * n_active * K;
    int RB = work < 1.2e6 ? 1 : (work < 3.5e6 ? 2 : 4);
    while (RB > 1 && RB > B) RB >>= 1;
    return RB;
}
// Batch rows per workgroup of the staging form (measured: one row up to batch 4 and for wide inputs, where staging two rows
// of x costs more than the second pass over W_c / idx saves; two rows beat four and eight elsewhere).
inline int klane_stage_rows(int B, int d_in) { return (B > 4 && d_in <= 1024) ? 2 : 1; }

// Gathering: a fixed part plus a part per gathered term that grows with the number of distinct 128-byte lines of x a
// wavefront's gather touches (rho = stored terms per line of a row of x: a lane group's consecutive terms share lines
// when rho is large) and with how far the rows of x a workgroup gathers from overflow the vector L1 (the width factor):
// ~1.0 us per million terms at 90 % sparsity, 1.3 at 99 % on 768- to 1024-wide inputs, 2.0 at 99 % on 4096-wide ones.
inline double klane_gather_estimate_us(int B, int d_in, int n_active, int K) {
    const double terms = (double)n_active * K;
    const double rho = 32.0 * K / (d_in > 0 ? d_in : 1);
    const double lines_per_term = rho > 1e-6 ? (1.0 - exp(-rho)) / rho : 1.0;
    const double width = d_in <= 1024 ? 0.4 : (d_in <= 3072 ? 0.7 : 1.0);
    const int RB = klane_gather_rows(B, n_active, K);
    return 2.6 + (0.8 + 1.4 * lines_per_term * width) * 1e-6 * B * terms + (terms > 1.5e6 ? 3.0e-6 * terms * ((B + RB - 1) / RB) : 0.0);
}
// Staging: a fixed part that grows with the row of x every workgroup stages, plus a part per term slot (K rounded up to the
// slots one request of a lane group covers).
inline double klane_stage_estimate_us(int B, int d_in, int n_active, int K) {
    int L = 4;
    while (L < 64 && L * 4 < K) L <<= 1;
    const int req = L * 4;   // term slots one request of a lane group covers (4 terms per lane)
    const double slots = (double)B * n_active * ((K + req - 1) / req * req);
    const double terms = (double)n_active * K;
    const int RB = klane_stage_rows(B, d_in);
    return 3.0 + 0.0007 * d_in + (d_in <= 1024 ? 0.65e-6 : 0.75e-6) * slots + (terms > 1.5e6 ? 3.0e-6 * terms * ((B + RB - 1) / RB) : 0.0);
}
inline bool klane_row_fits_lds(int d_in) { return (size_t)d_in * sizeof(float) <= kLdsMax; }
inline bool klane_gathers(int B, int d_in, int n_active, int K) {
    return !klane_row_fits_lds(d_in) || klane_gather_estimate_us(B, d_in, n_active, K) <= klane_stage_estimate_us(B, d_in, n_active, K);
}
inline double klane_estimate_us(int B, int d_in, int n_active, int K) {
    return klane_gathers(B, d_in, n_active, K) ? klane_gather_estimate_us(B, d_in, n_active, K) : klane_stage_estimate_us(B, d_in, n_active, K);
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
