// Internal declarations shared by the HIP translation units of libsrigl (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <algorithm>
#include <atomic>
#include <cmath>
#include <stdint.h>

#include "srigl.h"

namespace srigl {

constexpr int kWave = 64;              // CDNA wavefront width
constexpr int kSegCols = 64;           // columns per entry of the seg table
constexpr size_t kLdsMax = 160 * 1024; // LDS per workgroup on gfx950

// The streaming copy of the condensed arrays (App. E: values and column indices, n x k each) that srigl_condense and
// srigl_pack_terms write and the forward kernels may read instead of W_c / idx.  Neuron-major and K-interleaved: the weight
// and the column index of a term sit next to each other, terms in row order, rows padded to a multiple of four terms
// (weight bits 0, index 0), so that rows start 16-byte aligned, a lane's four consecutive terms come with one or two
// 16-byte loads, and one 4- or 8-byte load brings both halves of a term:
//   fp32 weights:                  term = w fp32, idx int32                     (8 bytes)
//   bf16 weights, d_in <= 65536:   term = w bf16 (low half), idx uint16 (high)  (4 bytes)
//   bf16 weights, wider inputs:    term = w bf16, 16 zero bits, idx int32       (8 bytes)
struct PackedLayout {
    int terms;        // terms per row, padding included (a multiple of 4)
    int term_bytes;   // 4 or 8
    int w_bytes;      // 4 or 2
    __host__ __device__ size_t row_bytes() const { return (size_t)terms * term_bytes; }
    // term t of a row whose packed copy starts at `row`: weight bits and column
    __device__ void store(unsigned char* row, int t, uint32_t wbits, int col) const {
        if (term_bytes == 4) {
            reinterpret_cast<uint32_t*>(row)[t] = (wbits & 0xffffu) | ((uint32_t)col << 16);
        } else {
            reinterpret_cast<uint2*>(row)[t] = make_uint2(w_bytes == 4 ? wbits : (wbits & 0xffffu), (uint32_t)col);
        }
    }
};
inline PackedLayout packed_layout(int K, int d_in, bool bf16) {
    PackedLayout pl;
    pl.terms = (K + 3) / 4 * 4;
    pl.w_bytes = bf16 ? 2 : 4;
    pl.term_bytes = (bf16 && d_in <= 65536) ? 4 : 8;
    return pl;
}

// One unit of the streaming copy in registers (device side).
// (four consecutive terms; UB = bytes of the four terms: 32, or 16 for bf16 weights beside 16-bit indices)
template <typename XT, int UB> struct PackedUnit;
template <> struct PackedUnit<float, 32> {
    uint4 a, b;   // (w0, i0, w1, i1), (w2, i2, w3, i3)
    __device__ __forceinline__ void load(const unsigned char* __restrict__ u) {
        a = *reinterpret_cast<const uint4*>(u);
        b = *reinterpret_cast<const uint4*>(u + 16);
    }
    __device__ __forceinline__ float weight(int t) const { return __uint_as_float(t == 0 ? a.x : (t == 1 ? a.z : (t == 2 ? b.x : b.z))); }
    __device__ __forceinline__ int col(int t) const { return (int)(t == 0 ? a.y : (t == 1 ? a.w : (t == 2 ? b.y : b.w))); }
};
template <> struct PackedUnit<uint16_t, 16> {
    uint4 v;   // four terms: bf16 weight in the low half, 16-bit index in the high half
    __device__ __forceinline__ void load(const unsigned char* __restrict__ u) { v = *reinterpret_cast<const uint4*>(u); }
    __device__ __forceinline__ uint32_t word(int t) const { return t == 0 ? v.x : (t == 1 ? v.y : (t == 2 ? v.z : v.w)); }
    __device__ __forceinline__ float weight(int t) const { return __uint_as_float(word(t) << 16); }
    __device__ __forceinline__ int col(int t) const { return (int)(word(t) >> 16); }
};
template <> struct PackedUnit<uint16_t, 32> {
    uint4 a, b;   // (w0, i0, w1, i1), (w2, i2, w3, i3), weights as bf16 bits in the low half of their word
    __device__ __forceinline__ void load(const unsigned char* __restrict__ u) {
        a = *reinterpret_cast<const uint4*>(u);
        b = *reinterpret_cast<const uint4*>(u + 16);
    }
    __device__ __forceinline__ float weight(int t) const { return __uint_as_float((t == 0 ? a.x : (t == 1 ? a.z : (t == 2 ? b.x : b.z))) << 16); }
    __device__ __forceinline__ int col(int t) const { return (int)(t == 0 ? a.y : (t == 1 ? a.w : (t == 2 ? b.y : b.w))); }
};

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
    const void* packed;  // the streaming copy of W_c / idx (PackedLayout), or nullptr
    int32_t act;   // srigl_activation applied to every written value (stored and ablated columns alike)
};

// Launch shape of the ROWLANE kernel, decided on the host.
struct RowlanePlan {
    int R, H, NW, NPW, KPRE, C, n_chunks, n_btiles, n_groups;
    int rounds;    // rounds of workgroups on the busiest XCD (32 compute units each)
    int bt_major;  // 1: an XCD owns batch tiles (and runs every group of stored rows on them), 0: it owns groups of stored rows
    size_t lds;
    double cost;  // the planner's estimate for this shape (arbitrary units), to compare shapes
    int out_off;  // word offset of the result tile in LDS (0: it reuses the activation tile after a barrier)
    bool fast;   // x rows allow aligned 4-element loads and d_in is a multiple of 16
    bool pk;     // the terms are read from the streaming copy (forced through the tuning; the default reads W_c / idx)
    int spread;  // 0: a wavefront takes consecutive stored rows; 1: every NW-th of the workgroup's rows in the order of their median
                 // columns; 2 + t: the same in workgroups whose rows' medians lie more than t columns apart
    bool ok;
};
constexpr int kSpanCap = 1024;     // output columns (stored and ablated) a workgroup of the batched kernel writes through its column table
// Words between consecutive columns of the activation tile in LDS (a column holds the tile's BT batch rows).  BT + 4: the
// staging writes of four consecutive columns land in different banks.  Four term slices (16-row tiles): 16, so that the two
// 16-word runs a half-wavefront reads start 0 or 16 banks apart (they collide only when the two columns have the same
// parity) instead of a multiple of 4 banks apart (collide in 7 cases of 8); the staging writes then swap the columns of a
// pair in every other lane group so that they meet in two banks' worth, as with the skew.
// Four rows per lane (16-byte LDS reads): BT with no skew, so that the 16 lanes of a term slice read 256 consecutive bytes,
// all 64 banks once (measured: 4.85 clocks per wavefront read against 8.05 with the skew); the staging writes then stay
// conflict-free through a swizzle of the rows by the column (rowlane_swizzled).
constexpr int rowlane_row_stride(int BT, int H, int R = 1) { return ((H == 4 && BT == 16) || R == 4) ? BT : BT + 4; }
// Row r of column c of the activation tile sits at row position r ^ (((c >> 2) & 3) << 4) of its column.
constexpr bool rowlane_swizzled(int R) { return R == 4; }
constexpr int kStageUnits = 8;   // 16x16 staging units a wavefront holds in registers per chunk
constexpr int kBlock = 16;       // terms per vector load of W_c / idx (one DPP row)
constexpr int rowlane_max_threads(int) { return 1024; }
// stored rows per wavefront the register budget allows without spilling (from six rows on a wavefront keeps one block of
// terms per row in registers; with four rows per lane the 16-byte reads leave room for three)
constexpr int rowlane_max_npw(int R, int H = 2) { return R == 4 ? 3 : 8; }
// blocks of 16 terms per (stored row, chunk) kept in registers, by stored rows per wavefront
constexpr int rowlane_kpre(int npw) { return npw <= 3 ? 3 : (npw <= 4 ? 2 : 1); }
// (two rows per lane with term slices: blocks are 32 or 64 terms, so fewer of them cover the same part of a row)
constexpr int rowlane_kpre_rh(int npw, int R, int H) {
    return R == 4 ? 1 : ((R == 2 && H >= 2) ? (rowlane_kpre(npw) < 2 ? rowlane_kpre(npw) : 2) : rowlane_kpre(npw));
}
srigl_status launch_rowlane_f32(const FwdArgs& a, const RowlanePlan& p, hipStream_t st);
srigl_status launch_rowlane_bf16(const FwdArgs& a, const RowlanePlan& p, hipStream_t st);
srigl_status launch_rowlane_f32_i16(const FwdArgs& a, const RowlanePlan& p, hipStream_t st);
srigl_status launch_rowlane_bf16_i16(const FwdArgs& a, const RowlanePlan& p, hipStream_t st);

// Each returns SRIGL_OK, SRIGL_ERR_UNSUPPORTED (cannot run these sizes) or SRIGL_ERR_HIP.
srigl_status launch_fwd_generic(const FwdArgs& a, hipStream_t st);
srigl_status launch_fwd_klane(const FwdArgs& a, const srigl_fwd_tuning* t, hipStream_t st);
srigl_status launch_fwd_rowlane(const FwdArgs& a, const srigl_fwd_tuning* t, hipStream_t st);
bool rowlane_supported(const FwdArgs& a, const srigl_fwd_tuning* t);
// ROWLOOP (fwd_rowloop.hip): the launch, whether these sizes can run it, its estimated time (us; 1e30 if they cannot) and
// the launch shape for srigl_fwd_plan_query
srigl_status launch_fwd_rowloop(const FwdArgs& a, const srigl_fwd_tuning* t, hipStream_t st);
bool rowloop_supported(const FwdArgs& a, const srigl_fwd_tuning* t);
double rowloop_estimate_us(const FwdArgs& a);
bool rowloop_plan_query(const FwdArgs& a, const srigl_fwd_tuning* t, srigl_fwd_plan* plan);
srigl_fwd_algo choose_fwd_algo(const FwdArgs& a);
// Estimated time (us) of the condensed forward call of these sizes in the kernel the library's own choice takes.
double condensed_estimate_us(int B, int d_in, int n_active, int K, int d_out, bool bf16, bool has_active);

// The small-batch forward kernel takes its activations either from global memory through the vector caches (a gather:
// no staging pass, no barrier, any d_in) or from rows of x staged in LDS.  Estimated times (us) of both: least-squares
// fits (relative error) of the mean of cold and cached timings of 13 layer shapes, 512- to 4096-wide, 80-99 % sparse, at
// batches of 1 to 512 (mean error 7-8 %).  They pick the source of the activations and the kernel for batches of 2 to
// 2048 rows, and feed the choice between the condensed and the structured-only form.  Layers of more than ~1.5 M stored
// terms no longer sit in one XCD's L2: every pass over W_c / idx (one per workgroup row of the batch) then also pays for
// that stream.
//
// Batch rows per workgroup of the gathering form: a second and a fourth row pay once the pass over W_c / idx they save
// outweighs the longer chain of gathers per lane (measured: from ~1.2 M and ~3.5 M gathered terms).
inline int klane_gather_rows(int B, int n_active, int K) {
    const double work = (double)B * n_active * K;
    int RB = work < 1.2e6 ? 1 : (work < 3.5e6 ? 2 : 4);
    while (RB > 1 && RB > B) RB >>= 1;
    return RB;
}
// Batch rows per workgroup of the staging form (measured: two rows for inputs up to 1024 wide from batch 5, else one: on
// wider inputs the second staged row costs more than the saved pass over W_c / idx, four rows always lose).
inline int klane_stage_rows(int B, int d_in) { return (B > 4 && d_in <= 1024) ? 2 : 1; }
// Lanes that share one stored row: enough that a lane has at most ~4 terms, at least 4, at most a wavefront.
inline int klane_lanes(int K) {
    int L = 4;
    while (L < 64 && L * 4 < K) L <<= 1;
    return L;
}

// Gathering: a fixed part plus ~1 us per million gathered terms, more where a wavefront's gather touches many distinct
// 128-byte lines of x (rho = stored terms per line of a row of x; a lane group's consecutive terms share lines when rho
// is large) and the rows gathered from overflow the vector L1 (4096-wide inputs at 99 % sparsity: 2 us per million).
inline double klane_gather_estimate_us(int B, int d_in, int n_active, int K) {
    const double terms = (double)n_active * K;
    const double rho = 32.0 * K / (d_in > 0 ? d_in : 1);
    const double lines_per_term = rho > 1e-6 ? (1.0 - exp(-rho)) / rho : 1.0;
    const double width = d_in <= 1024 ? 0.19 : (d_in <= 3072 ? 0.22 : 0.93);
    const int RB = klane_gather_rows(B, n_active, K);
    return 2.5 + (0.96 + width * lines_per_term) * 1e-6 * B * terms + (terms > 1.5e6 ? 0.31e-6 * terms * ((B + RB - 1) / RB) : 0.0);
}
// Staging: a fixed part, the rows of x every workgroup copies into its LDS (at most 2048 workgroups), and the terms: on
// inputs up to 1024 wide mostly per term slot (K rounded up to the slots one request of a lane group covers), on wider
// ones per stored term.
inline double klane_stage_estimate_us(int B, int d_in, int n_active, int K) {
    const int L = klane_lanes(K), req = L * 4;   // term slots one request of a lane group covers (4 terms per lane)
    const double slots = (double)B * n_active * ((K + req - 1) / req * req);
    const double terms = (double)n_active * K;
    const int RB = klane_stage_rows(B, d_in);
    const double wgs = std::min(2048.0, ceil((double)n_active / (256 / L)) * ((B + RB - 1) / RB));
    const double per_term = d_in <= 1024 ? 0.30e-6 * slots + 0.15e-6 * B * terms : 1.0e-6 * B * terms;
    return 2.7 + 0.00046 * d_in + 4.6e-8 * wgs * RB * d_in * 4.0 + per_term + (terms > 1.5e6 ? 0.40e-6 * terms * ((B + RB - 1) / RB) : 0.0);
}
inline bool klane_row_fits_lds(int d_in) { return (size_t)d_in * sizeof(float) <= kLdsMax; }
inline bool klane_gathers(int B, int d_in, int n_active, int K) {
    return !klane_row_fits_lds(d_in) || klane_gather_estimate_us(B, d_in, n_active, K) <= klane_stage_estimate_us(B, d_in, n_active, K);
}
inline double klane_estimate_us(int B, int d_in, int n_active, int K) {
    return klane_gathers(B, d_in, n_active, K) ? klane_gather_estimate_us(B, d_in, n_active, K) : klane_stage_estimate_us(B, d_in, n_active, K);
}

// Batches of 8 to 32 rows on inputs up to 1024 wide with moderate fan-in and at least 2048 stored rows: the small-batch
// kernel with the rows of x staged in LDS and few lanes per stored row (16 or 32 stored rows per workgroup share one staged
// tile) runs ahead of both the gathering form and the batched kernel, cold and cached: 768 -> 3072 K = 77 at B = 8 / 16 /
// 32: 5.1 / 5.8 / 6.6 us cold against 5.6 / 6.1 / 7.7; K = 39 at B = 16 / 32: 4.8 / 5.6 against 5.6 / 7.0; with 30 % of the
// neurons ablated at B = 32: 7.0 against 9.1; 1024 -> 4096 bf16 K = 102 at B = 8: 5.1 against 6.0.  Not taken where it
// measured behind on operands from HBM: wider inputs (3072 -> 768 at B = 8: 9.1 against 6.1 us; 2048 -> 2048 K = 102: 6.2
// against 5.5), layers of 1024 stored rows (a quarter of the workgroups: 4.7 against 4.1), fan-ins above 128 from B = 16,
// and B x K above ~2500, where the batched kernel is level or ahead.
inline bool klane_few_lanes_staged(int B, int d_in, int n_active, int K, int* L, int* RB) {
    if (d_in > 1024 || d_in % 4 != 0 || n_active < 2048 || B < 8 || B > 32 || K < 32 || (long long)B * K > 2560 || (K > 128 && B > 8))
        return false;
    *L = B >= 16 ? 8 : 16;
    *RB = 2;
    return true;
}

inline srigl_status hip_ok(hipError_t e) { return e == hipSuccess ? SRIGL_OK : SRIGL_ERR_HIP; }

// Kernels that use more than 64 KB of dynamic LDS need the limit raised with hipFuncSetAttribute, which applies to the
// current device only.  One of these per kernel instance (a function-local static): the attribute is set on the first
// launch on each device (a bit per device ordinal) and never per call; safe to use from several host threads.
struct LdsLimit {
    std::atomic<uint64_t> raised{0};
    template <typename Kern>
    srigl_status ensure(Kern kern, size_t bytes) {
        if (bytes <= 64 * 1024) return SRIGL_OK;
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess) return SRIGL_ERR_HIP;
        const uint64_t bit = 1ull << (dev & 63);
        if (dev < 64 && (raised.load(std::memory_order_acquire) & bit)) return SRIGL_OK;
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsMax) != hipSuccess)
            return SRIGL_ERR_HIP;
        if (dev < 64) raised.fetch_or(bit, std::memory_order_release);
        return SRIGL_OK;
    }
};

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

// Activation between the two linear layers of an MLP block: identity, max(v, 0), or v * Phi(v) with the normal
// distribution function Phi (the exact, erf-based GELU).
__device__ __forceinline__ float apply_act(float v, int act) {
    if (act == SRIGL_ACT_RELU) return fmaxf(v, 0.0f);
    if (act == SRIGL_ACT_GELU) return 0.5f * v * (1.0f + erff(v * 0.70710678118654752440f));
    return v;
}

}  // namespace srigl
