// Forward kernels of the condensed constant fan-in linear layer (gfx950).
//
// All of them compute Alg. 1 of arXiv 2305.02299,
//     y[b][active[s]] = bias[active[s]] + sum_k W_c[s][k] * x[b][idx[s][k]],
// and give every column that is not stored (an ablated neuron, Sec. 3.1 step 4) its bias.
// Because `active` is ascending, the columns that are not stored are exactly the gaps between
// consecutive entries; the thread (or wavefront) that owns stored row s also fills the gap in front
// of column active[s], and a virtual row s == n_active fills the tail.
#include "srigl_internal.h"
#include <algorithm>
#include <cmath>
#include <cstring>

namespace srigl {


// ------------------------------------------------------------------------------------------------
// small helpers
// ------------------------------------------------------------------------------------------------
template <typename XT> __device__ __forceinline__ float to_f32(XT v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<uint16_t>(uint16_t v) { return bf16_bits_to_float(v); }

__device__ __forceinline__ float bias_at(const float* __restrict__ bias, int col) { return bias ? bias[col] : 0.0f; }

// ------------------------------------------------------------------------------------------------
// GENERIC: one thread per (batch row, stored row).  Reads x from global memory, clamps indices.
// Correct for any index order; the fallback when nothing better applies.
// ------------------------------------------------------------------------------------------------
template <typename XT, typename IT>
__global__ __launch_bounds__(256) void k_fwd_generic(const XT* __restrict__ x, int B, int d_in, const XT* __restrict__ W_c,
                                                     const IT* __restrict__ idx, const int32_t* __restrict__ active,
                                                     int n_active, int K, const float* __restrict__ bias, int d_out,
                                                     float* __restrict__ y, int act) {
    const int n_slots = active ? n_active + 1 : n_active;   // +1: virtual row that fills the tail gap
    const long long total = (long long)B * n_slots;
    for (long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (long long)gridDim.x * blockDim.x) {
        const int b = (int)(t / n_slots);
        const int s = (int)(t - (long long)b * n_slots);
        float* yr = y + (size_t)b * d_out;
        int col = s, prev = s - 1;
        if (active) {
            col = (s < n_active) ? active[s] : d_out;
            prev = (s > 0) ? active[s - 1] : -1;
            col = min(col, d_out);
            for (int c = max(prev + 1, 0); c < col; ++c) yr[c] = apply_act(bias_at(bias, c), act);
        }
        if (s >= n_active || col < 0 || col >= d_out) continue;
        const XT* xr = x + (size_t)b * d_in;
        const XT* w = W_c + (size_t)s * K;
        const IT* ix = idx + (size_t)s * K;
        float acc = 0.0f;
        for (int k = 0; k < K; ++k) {
            const int j = min(max((int)ix[k], 0), d_in - 1);
            acc = fmaf(to_f32<XT>(w[k]), to_f32<XT>(xr[j]), acc);
        }
        yr[col] = apply_act(acc + bias_at(bias, col), act);
    }
}

// y[b][c] = bias[c] (or 0): the whole forward pass when nothing is stored (n_active == 0 or K == 0).
__global__ __launch_bounds__(256) void k_bias_broadcast(const float* __restrict__ bias, int B, int d_out, float* __restrict__ y, int act) {
    const long long total = (long long)B * d_out;
    for (long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (long long)gridDim.x * blockDim.x)
        y[t] = apply_act(bias_at(bias, (int)(t % d_out)), act);
}

// ------------------------------------------------------------------------------------------------
// KLANE (small batch, online inference).  A workgroup walks over stored rows for RB rows of the batch; L lanes (a power
// of two) share one stored row: lane q takes the terms k = q, q+L, ... so that a wavefront's loads of W_c and idx are
// runs of L contiguous words, and the partial sums are combined with a butterfly of cross-lane shuffles.  The
// activations are gathered from global memory through the vector caches (GATHER), or from RB rows of x the workgroup
// first stages in LDS (fp32, row-major).
// ------------------------------------------------------------------------------------------------
constexpr int kKlaneTerms = 4;   // terms a lane keeps in flight per request

template <int RB, bool GATHER, typename XT, typename IT>
__global__ __launch_bounds__(256) void k_fwd_klane(const XT* __restrict__ x, int B, int d_in, const XT* __restrict__ W_c,
                                                   const IT* __restrict__ idx, const int32_t* __restrict__ active,
                                                   int n_active, int K, const float* __restrict__ bias, int d_out,
                                                   float* __restrict__ y, int log2L, int rows_per_wg, int act) {
    extern __shared__ float xs[];   // [RB][d_in]; unused when GATHER
    const int L = 1 << log2L;
    const int tid = threadIdx.x;
    const int q = tid & (L - 1);                      // lane within the neuron's group
    const int grp = tid >> log2L;                     // group within the workgroup
    const int groups = blockDim.x >> log2L;
    const int b0 = blockIdx.y * RB;
    const int n_slots = active ? n_active + 1 : n_active;
    const int s_begin = blockIdx.x * rows_per_wg;
    const int s_end = min(s_begin + rows_per_wg, n_slots);

    const XT* xrow[RB];                               // rows past B re-read the last row; they are never stored
#pragma unroll
    for (int r = 0; r < RB; ++r) xrow[r] = x + (size_t)min(b0 + r, B - 1) * d_in;
    if (!GATHER) {
        // four loads per thread in flight before the first of them is converted and stored
#pragma unroll
        for (int r = 0; r < RB; ++r)
            for (int j0 = tid; j0 < d_in; j0 += 4 * (int)blockDim.x) {
                XT v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) v[u] = xrow[r][min(j0 + u * (int)blockDim.x, d_in - 1)];
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (j0 + u * (int)blockDim.x < d_in) xs[r * d_in + j0 + u * (int)blockDim.x] = to_f32<XT>(v[u]);
            }
        __syncthreads();
    }

    for (int s = s_begin + grp; s < s_end; s += groups) {
        float acc[RB];
#pragma unroll
        for (int r = 0; r < RB; ++r) acc[r] = 0.0f;
        if (s < n_active) {
            const XT* wrow = W_c + (size_t)s * K;
            const IT* irow = idx + (size_t)s * K;
            for (int k = q; k < K; k += kKlaneTerms * L) {
                XT w[kKlaneTerms];
                int c[kKlaneTerms];
#pragma unroll
                for (int t = 0; t < kKlaneTerms; ++t) {   // unconditional loads (term index clamped into the row)
                    const int kk = min(k + t * L, K - 1);
                    w[t] = wrow[kk];
                    c[t] = (int)irow[kk];
                }
                if (GATHER) {
                    // an index outside [0, d_in) must not become an address outside x (from LDS it only reads a wrong word)
#pragma unroll
                    for (int t = 0; t < kKlaneTerms; ++t) c[t] = min(max(c[t], 0), d_in - 1);
                }
                if (GATHER) {   // a second round trip (the gather needs the indices), all of it in flight at once
                    XT xg[kKlaneTerms][RB];
#pragma unroll
                    for (int t = 0; t < kKlaneTerms; ++t)
#pragma unroll
                        for (int r = 0; r < RB; ++r) xg[t][r] = xrow[r][c[t]];
#pragma unroll
                    for (int t = 0; t < kKlaneTerms; ++t) {
                        if (k + t * L < K) {
                            const float wv = to_f32<XT>(w[t]);
#pragma unroll
                            for (int r = 0; r < RB; ++r) acc[r] = fmaf(wv, to_f32<XT>(xg[t][r]), acc[r]);
                        }
                    }
                } else {
#pragma unroll
                    for (int t = 0; t < kKlaneTerms; ++t) {
                        if (k + t * L < K) {
                            const float wv = to_f32<XT>(w[t]);
#pragma unroll
                            for (int r = 0; r < RB; ++r) acc[r] = fmaf(wv, xs[r * d_in + c[t]], acc[r]);
                        }
                    }
                }
            }
        }
        for (int off = L >> 1; off > 0; off >>= 1) {
#pragma unroll
            for (int r = 0; r < RB; ++r) acc[r] += __shfl_xor(acc[r], off, kWave);
        }
        int col = s, prev = s - 1;
        if (active) {
            col = min((s < n_active) ? active[s] : d_out, d_out);
            prev = (s > 0) ? active[s - 1] : -1;
            // the L lanes of the group share the gap in front of this column
            for (int c = max(prev + 1, 0) + q; c < col; c += L) {
                const float braw = bias_at(bias, c);
                const float bv = act == SRIGL_ACT_NONE ? braw : apply_act(braw, act);
#pragma unroll
                for (int r = 0; r < RB; ++r)
                    if (b0 + r < B) y[(size_t)(b0 + r) * d_out + c] = bv;
            }
        }
        if (q == 0 && s < n_active && col >= 0 && col < d_out) {
            const float bv = bias_at(bias, col);
#pragma unroll
            for (int r = 0; r < RB; ++r)
                if (b0 + r < B) y[(size_t)(b0 + r) * d_out + col] = act == SRIGL_ACT_NONE ? acc[r] + bv : apply_act(acc[r] + bv, act);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// KLANE on the streaming copy of the condensed arrays (PackedLayout).  Same lane mapping and reduction as k_fwd_klane,
// but the four terms a lane has in flight are one unit of the copy: lane q of a row's group takes the units q, q + L, ...
// and gets its four (weight, index) pairs with two 16-byte loads out of one 32-byte piece (one load when a term is 4 bytes:
// bf16 weights beside 16-bit indices) instead of eight 4- or 2-byte loads from two arrays.  The first unit of a
// lane's next stored row is requested before the current row's partial sums are combined; in the staged form the first
// row's unit is requested together with the rows of x, ahead of the barrier, so that both fetches are in flight at once.
// ------------------------------------------------------------------------------------------------
template <int RB, bool GATHER, typename XT, int UB>
__global__ __launch_bounds__(256) void k_fwd_klane_packed(const XT* __restrict__ x, int B, int d_in, const unsigned char* __restrict__ packed,
                                                          int units, const int32_t* __restrict__ active, int n_active, int K,
                                                          const float* __restrict__ bias, int d_out, float* __restrict__ y, int log2L,
                                                          int rows_per_wg, int act) {
    extern __shared__ float xs[];   // [RB][d_in]; unused when GATHER
    const int L = 1 << log2L;
    const int tid = threadIdx.x;
    const int q = tid & (L - 1);
    const int grp = tid >> log2L;
    const int groups = blockDim.x >> log2L;
    const int b0 = blockIdx.y * RB;
    const int n_slots = active ? n_active + 1 : n_active;
    const int s_begin = blockIdx.x * rows_per_wg;
    const int s_end = min(s_begin + rows_per_wg, n_slots);
    const size_t row_bytes = (size_t)units * UB;

    const XT* xrow[RB];
#pragma unroll
    for (int r = 0; r < RB; ++r) xrow[r] = x + (size_t)min(b0 + r, B - 1) * d_in;

    // unit u of stored row s; rows and units past the end re-read the last ones (their terms are never used)
    auto unit_at = [&](int s, int u) {
        return packed + (size_t)min(s, n_active - 1) * row_bytes + (size_t)min(u, units - 1) * UB;
    };
    PackedUnit<XT, UB> first;
    if (!GATHER) {
        XT v[RB][4];
        const int j0 = tid;   // this thread's first column; the loop below strides by 4 * blockDim.x
#pragma unroll
        for (int r = 0; r < RB; ++r)
#pragma unroll
            for (int u = 0; u < 4; ++u) v[r][u] = xrow[r][min(j0 + u * (int)blockDim.x, d_in - 1)];
        first.load(unit_at(s_begin + grp, q));
#pragma unroll
        for (int r = 0; r < RB; ++r)
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (j0 + u * (int)blockDim.x < d_in) xs[r * d_in + j0 + u * (int)blockDim.x] = to_f32<XT>(v[r][u]);
        for (int r = 0; r < RB; ++r)
            for (int j = tid + 4 * (int)blockDim.x; j < d_in; j += (int)blockDim.x) xs[r * d_in + j] = to_f32<XT>(xrow[r][j]);
        __syncthreads();
    } else {
        first.load(unit_at(s_begin + grp, q));
    }

    for (int s = s_begin + grp; s < s_end; s += groups) {
        float acc[RB];
#pragma unroll
        for (int r = 0; r < RB; ++r) acc[r] = 0.0f;
        if (s < n_active) {
            for (int u = q; u < units; u += L) {
                PackedUnit<XT, UB> un;
                if (u == q) un = first; else un.load(unit_at(s, u));
                int c[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) c[t] = GATHER ? min(max(un.col(t), 0), d_in - 1) : un.col(t);
                if (GATHER) {
                    XT xg[4][RB];
#pragma unroll
                    for (int t = 0; t < 4; ++t)
#pragma unroll
                        for (int r = 0; r < RB; ++r) xg[t][r] = xrow[r][c[t]];
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                        if (4 * u + t < K) {
                            const float wv = un.weight(t);
#pragma unroll
                            for (int r = 0; r < RB; ++r) acc[r] = fmaf(wv, to_f32<XT>(xg[t][r]), acc[r]);
                        }
                } else {
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                        if (4 * u + t < K) {
                            const float wv = un.weight(t);
#pragma unroll
                            for (int r = 0; r < RB; ++r) acc[r] = fmaf(wv, xs[r * d_in + c[t]], acc[r]);
                        }
                }
            }
        }
        if (s + groups < s_end) first.load(unit_at(s + groups, q));
        for (int off = L >> 1; off > 0; off >>= 1) {
#pragma unroll
            for (int r = 0; r < RB; ++r) acc[r] += __shfl_xor(acc[r], off, kWave);
        }
        int col = s, prev = s - 1;
        if (active) {
            col = min((s < n_active) ? active[s] : d_out, d_out);
            prev = (s > 0) ? active[s - 1] : -1;
            for (int c = max(prev + 1, 0) + q; c < col; c += L) {
                const float braw = bias_at(bias, c);
                const float bv = act == SRIGL_ACT_NONE ? braw : apply_act(braw, act);
#pragma unroll
                for (int r = 0; r < RB; ++r)
                    if (b0 + r < B) y[(size_t)(b0 + r) * d_out + c] = bv;
            }
        }
        if (q == 0 && s < n_active && col >= 0 && col < d_out) {
            const float bv = bias_at(bias, col);
#pragma unroll
            for (int r = 0; r < RB; ++r)
                if (b0 + r < B) y[(size_t)(b0 + r) * d_out + col] = act == SRIGL_ACT_NONE ? acc[r] + bv : apply_act(acc[r] + bv, act);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// 16-bit copy of the index array (App. E: one index per kept weight).  Eight entries per thread when both arrays
// are 16-byte aligned (two 16-byte loads, one 16-byte store), the tail and unaligned arrays one entry per thread.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t narrow_one(int v, int hi) { return (uint32_t)min(max(v, 0), hi); }

__global__ __launch_bounds__(256) void k_narrow_idx8(const int4* __restrict__ idx, long long n8, int hi, uint4* __restrict__ out) {
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n8; i += (long long)gridDim.x * blockDim.x) {
        const int4 a = idx[2 * i], b = idx[2 * i + 1];
        uint4 o;
        o.x = narrow_one(a.x, hi) | (narrow_one(a.y, hi) << 16);
        o.y = narrow_one(a.z, hi) | (narrow_one(a.w, hi) << 16);
        o.z = narrow_one(b.x, hi) | (narrow_one(b.y, hi) << 16);
        o.w = narrow_one(b.z, hi) | (narrow_one(b.w, hi) << 16);
        out[i] = o;
    }
}

__global__ __launch_bounds__(256) void k_narrow_idx1(const int32_t* __restrict__ idx, long long begin, long long n, int hi,
                                                     uint16_t* __restrict__ out) {
    for (long long i = begin + (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (long long)gridDim.x * blockDim.x)
        out[i] = (uint16_t)narrow_one(idx[i], hi);
}

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------
static int ilog2_floor(int v) { int l = 0; while ((1 << (l + 1)) <= v) ++l; return l; }

srigl_status launch_fwd_generic(const FwdArgs& a, hipStream_t st) {
    const int n_slots = a.active ? a.n_active + 1 : a.n_active;
    const long long total = (long long)a.B * n_slots;
    if (total == 0) return SRIGL_OK;
    long long blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
#define SRIGL_GENERIC(XT, IT)                                                                                              \
    hipLaunchKernelGGL((k_fwd_generic<XT, IT>), dim3((unsigned)blocks), dim3(256), 0, st, (const XT*)a.x, a.B, a.d_in,      \
                       (const XT*)a.W_c, (const IT*)a.idx, a.active, a.n_active, a.K, a.bias, a.d_out, a.y, a.act)
    if (a.x_bf16) { if (a.idx_u16) SRIGL_GENERIC(uint16_t, uint16_t); else SRIGL_GENERIC(uint16_t, int32_t); }
    else { if (a.idx_u16) SRIGL_GENERIC(float, uint16_t); else SRIGL_GENERIC(float, int32_t); }
#undef SRIGL_GENERIC
    return hip_ok(hipGetLastError());
}

template <int RB, bool GATHER, typename XT, typename IT>
static srigl_status launch_klane_t(const FwdArgs& a, int log2L, int rows_per_wg, hipStream_t st) {
    const int n_slots = a.active ? a.n_active + 1 : a.n_active;
    const size_t lds = GATHER ? 0 : (size_t)RB * a.d_in * sizeof(float);
    if (lds > kLdsMax) return SRIGL_ERR_UNSUPPORTED;
    auto kern = k_fwd_klane<RB, GATHER, XT, IT>;
    static LdsLimit lds_limit;
    if (lds_limit.ensure(kern, lds) != SRIGL_OK) return SRIGL_ERR_HIP;
    const unsigned gx = (unsigned)((n_slots + rows_per_wg - 1) / rows_per_wg);
    const unsigned gy = (unsigned)((a.B + RB - 1) / RB);
    if (gy > 65535u) return SRIGL_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(kern, dim3(gx, gy), dim3(256), lds, st, (const XT*)a.x, a.B, a.d_in, (const XT*)a.W_c, (const IT*)a.idx,
                       a.active, a.n_active, a.K, a.bias, a.d_out, a.y, log2L, rows_per_wg, a.act);
    return hip_ok(hipGetLastError());
}

template <int RB, bool GATHER, typename XT, int UB>
static srigl_status launch_klane_packed_t(const FwdArgs& a, int log2L, int rows_per_wg, hipStream_t st) {
    const int n_slots = a.active ? a.n_active + 1 : a.n_active;
    const size_t lds = GATHER ? 0 : (size_t)RB * a.d_in * sizeof(float);
    if (lds > kLdsMax) return SRIGL_ERR_UNSUPPORTED;
    auto kern = k_fwd_klane_packed<RB, GATHER, XT, UB>;
    static LdsLimit lds_limit;
    if (lds_limit.ensure(kern, lds) != SRIGL_OK) return SRIGL_ERR_HIP;
    const unsigned gx = (unsigned)((n_slots + rows_per_wg - 1) / rows_per_wg);
    const unsigned gy = (unsigned)((a.B + RB - 1) / RB);
    if (gy > 65535u) return SRIGL_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(kern, dim3(gx, gy), dim3(256), lds, st, (const XT*)a.x, a.B, a.d_in, static_cast<const unsigned char*>(a.packed),
                       (a.K + 3) / 4, a.active, a.n_active, a.K, a.bias, a.d_out, a.y, log2L, rows_per_wg, a.act);
    return hip_ok(hipGetLastError());
}

// Launch shape of the small-batch kernel, decided on the host.
struct KlanePlan { int L, RB, rows_per_wg, direct; long long workgroups; bool ok; };
static KlanePlan plan_klane(const FwdArgs& a, const srigl_fwd_tuning* t) {
    KlanePlan p{};
    p.ok = false;
    const int n_slots = a.active ? a.n_active + 1 : a.n_active;
    // lanes per stored row: enough that a lane has at most ~4 terms, at least 4, at most 64
    int L = t && t->lanes_per_neuron ? t->lanes_per_neuron : 0;
    // nothing forced: the staged shape with few lanes per stored row where it is ahead
    int few_L = 0, few_RB = 0;
    const bool open_shape = !t || (t->lanes_per_neuron == 0 && t->rows_per_block == 0 && t->direct_gather == 0);
    const bool few = open_shape && klane_few_lanes_staged(a.B, a.d_in, a.n_active, a.K, &few_L, &few_RB) &&
                     (size_t)few_RB * a.d_in * sizeof(float) <= kLdsMax / 2;
    if (few) L = few_L;
    if (L == 0) L = klane_lanes(a.K);
    if (L < 1 || L > 64 || (L & (L - 1)) != 0) return p;
    // activations: gathered from global memory, or staged in LDS (the tuning can force either: 1 = gather, 2 = stage);
    // an input row too long for the LDS is always gathered
    const int dg = t ? t->direct_gather : 0;
    if (dg < 0 || dg > 2) return p;
    p.direct = dg == 1 || (dg == 0 && !few && klane_gathers(a.B, a.d_in, a.n_active, a.K)) ? 1 : 0;
    int RB = t && t->rows_per_block ? t->rows_per_block : (few ? few_RB : 0);
    if (RB != 0 && RB != 1 && RB != 2 && RB != 4 && RB != 8) return p;
    if (RB == 0) RB = p.direct ? klane_gather_rows(a.B, a.n_active, a.K) : klane_stage_rows(a.B, a.d_in);
    if (!p.direct) {
        while (RB > 1 && (size_t)RB * a.d_in * sizeof(float) > kLdsMax / 2) RB >>= 1;
        if ((size_t)RB * a.d_in * sizeof(float) > kLdsMax) return p;   // the staged rows of x must fit the LDS
    }
    if ((a.B + RB - 1) / RB > 65535) return p;                            // the batch is the grid's second dimension
    const int groups = 256 / L;
    // stored rows per workgroup: one pass of all groups, more when that still leaves > 8 workgroups per CU
    int rows_per_wg = groups;
    // (the gathering form has no staging to share between passes: it takes more of them only beyond 32 workgroups per CU)
    const long long max_wgs = p.direct ? 256 * 32 : 256 * 8;
    // (a batch of more row blocks than that limit keeps it out of reach: one pass over all stored rows per workgroup then)
    while (rows_per_wg < n_slots && (long long)((n_slots + rows_per_wg - 1) / rows_per_wg) * ((a.B + RB - 1) / RB) > max_wgs) rows_per_wg += groups;
    p.L = L; p.RB = RB; p.rows_per_wg = rows_per_wg;
    p.workgroups = (long long)((n_slots + rows_per_wg - 1) / rows_per_wg) * ((a.B + RB - 1) / RB);
    p.ok = true;
    return p;
}

srigl_status launch_fwd_klane(const FwdArgs& a, const srigl_fwd_tuning* t, hipStream_t st) {
    const int n_slots = a.active ? a.n_active + 1 : a.n_active;
    if (a.B == 0 || n_slots == 0) return SRIGL_OK;
    const KlanePlan kp = plan_klane(a, t);
    if (!kp.ok || (t && (t->terms_from_copy < 0 || t->terms_from_copy > 1))) return SRIGL_ERR_UNSUPPORTED;
    const int RB = kp.RB, rows_per_wg = kp.rows_per_wg, direct = kp.direct;
    const int log2L = ilog2_floor(kp.L);
    // The streaming copy (same launch shape, a lane's four terms in one unit) when a workgroup holds one batch row: there it
    // is ahead on operands that come from HBM (768->3072: 3.73 against 3.83 us at B = 1; 4096->16384 bf16: 9.5 against 10.6)
    // and level on cached ones.  With two or more rows per workgroup the array kernel is faster (3072->768 at B = 16: 6.4
    // against 9.1 us), so there the copy is read only when the tuning asks for it.  The staged form reads the copy with any
    // number of rows (768 -> 3072 K = 39 at B = 32, two rows per workgroup: 5.3 / 4.5 us against 6.4 / 4.6 on the arrays).
    if (a.packed && !a.idx_u16 && (RB == 1 || !direct || (t && t->terms_from_copy == 1))) {
        const bool narrow = a.x_bf16 && a.d_in <= 65536;
#define SRIGL_KLANE_P(RBV, G)                                                                                        \
    return !a.x_bf16 ? launch_klane_packed_t<RBV, G, float, 32>(a, log2L, rows_per_wg, st)                            \
                     : (narrow ? launch_klane_packed_t<RBV, G, uint16_t, 16>(a, log2L, rows_per_wg, st)              \
                               : launch_klane_packed_t<RBV, G, uint16_t, 32>(a, log2L, rows_per_wg, st))
#define SRIGL_KLANE_PG(RBV)                \
    if (direct) { SRIGL_KLANE_P(RBV, true); } \
    SRIGL_KLANE_P(RBV, false)
        switch (RB) {
            case 1: SRIGL_KLANE_PG(1);
            case 2: SRIGL_KLANE_PG(2);
            case 4: SRIGL_KLANE_PG(4);
            default: SRIGL_KLANE_PG(8);
        }
#undef SRIGL_KLANE_P
#undef SRIGL_KLANE_PG
    }
#define SRIGL_KLANE_G(RBV, G)                                                                           \
    return a.x_bf16 ? (a.idx_u16 ? launch_klane_t<RBV, G, uint16_t, uint16_t>(a, log2L, rows_per_wg, st)  \
                                 : launch_klane_t<RBV, G, uint16_t, int32_t>(a, log2L, rows_per_wg, st))  \
                    : (a.idx_u16 ? launch_klane_t<RBV, G, float, uint16_t>(a, log2L, rows_per_wg, st)     \
                                 : launch_klane_t<RBV, G, float, int32_t>(a, log2L, rows_per_wg, st))
#define SRIGL_KLANE(RBV)                    \
    if (direct) { SRIGL_KLANE_G(RBV, true); } \
    SRIGL_KLANE_G(RBV, false)
    switch (RB) {
        case 1: SRIGL_KLANE(1);
        case 2: SRIGL_KLANE(2);
        case 4: SRIGL_KLANE(4);
        default: SRIGL_KLANE(8);
    }
#undef SRIGL_KLANE_G
#undef SRIGL_KLANE
}

constexpr int kRowlaneTwoRowsMinK = 32;
constexpr int kRowlaneShortRowK = 200;
constexpr int kRowlaneShortRowOneK = 128;
constexpr int kRowlaneTwoRowsFourSlicesMinK = 64;   // blocks of 64 terms: measured 14 % slower than 32 x 2 tiles at a fan-in of 39

// npw_cap: the most stored rows per wavefront the choice may take (0: whatever the tile allows)
static double rowlane_estimate_us(const FwdArgs& a, const RowlanePlan& p, bool whole_blocks = false);
static RowlanePlan plan_rowlane_with(const FwdArgs& a, const srigl_fwd_tuning* t, int npw_cap = 0) {
    // Wavefronts per workgroup, when the tuning leaves them open: 16, or 12 (three per SIMD instead of four) when that takes no
    // more rounds of workgroups, chunks or stored rows per wavefront: the same rows spread over more workgroups, each with a
    // quarter less to do (3072 -> 768 with 538 stored rows at B = 256: 192 workgroups of 16 wavefronts 14.9 us, 240 of 12
    // 13.2 us; 13 or 14 wavefronts load one SIMD like 16 and measured 14.6).
    if (!t || t->waves == 0) {
        srigl_fwd_tuning tw{};
        if (t) tw = *t;
        tw.waves = rowlane_max_threads(tw.rows_per_lane ? tw.rows_per_lane : 1) / kWave;
        const RowlanePlan full = plan_rowlane_with(a, &tw, npw_cap);
        tw.waves = tw.waves * 3 / 4;
        const RowlanePlan fewer = plan_rowlane_with(a, &tw, npw_cap);
        // (with one stored row per wavefront the workgroups are too small for that to pay: 5.4 -> 6.0 us on 768 -> 3072 at B = 32)
        if (full.ok && fewer.ok && full.NPW >= 2 && fewer.rounds <= full.rounds && fewer.NPW <= full.NPW && fewer.n_chunks <= full.n_chunks &&
            fewer.n_groups > full.n_groups)
            return fewer;
        return full.ok ? full : fewer;
    }
    RowlanePlan p{};
    p.ok = false;
    // the kernel indexes x, W_c / idx and seg with 32-bit offsets
    // (term indices are formed for up to 128 slots past the last stored row before they are clamped)
    if ((long long)a.B * a.d_in >= (1LL << 31) || ((long long)a.n_active + 256) * a.K + 4096 >= (1LL << 31) ||
        (long long)a.n_active * a.seg_stride >= (1LL << 31)) return p;
    const int n_slots = a.active ? a.n_active + 1 : a.n_active;
    p.pk = t && t->terms_from_copy == 1 && a.packed != nullptr;
    if (t && (t->terms_from_copy < 0 || t->terms_from_copy > 1)) return p;
    p.R = t && t->rows_per_lane ? t->rows_per_lane : 1;
    p.H = t && t->term_slices ? t->term_slices : 0;
    if (p.R != 1 && p.R != 2 && p.R != 4) return p;
    // fast staging: whole 16-column units, rows aligned for 4-element vector loads
    const size_t xal = (a.x_bf16 ? 2 : 4) * 4;
    p.fast = (a.d_in % 16 == 0) && ((reinterpret_cast<uintptr_t>(a.x) % xal) == 0);
    if (p.H == 0) {
        // A workgroup stages (rows per tile) x d_in activations.  For wide inputs and batches of a few tiles the
        // staging outweighs the arithmetic of the few stored rows a workgroup gets, so the tile gets fewer rows
        // (more term slices); measured on 768- and 3072-wide layers.  Large batches amortise it: 64-row tiles.
        p.H = 1;
        if (p.fast && p.R == 1 && a.B <= 512) p.H = a.d_in <= 1024 ? 1 : (a.d_in <= 2048 ? 2 : 4);
        // batches below one 64-row tile: a tile no taller than the batch keeps every lane on real rows
        // (and up to one 64-row tile two 32-row tiles run faster: twice the workgroups, half the terms per lane)
        if (p.fast && p.R == 1) {
            int hb = a.B <= 16 ? 4 : (a.B <= 64 ? 2 : 1);
            // inputs wider than 1024: 16-row tiles stay ahead up to a batch of 32, and up to 64 when the layer
            // has too few stored rows to fill the GPU otherwise (measured on 1536- and 2048-wide inputs)
            if (a.d_in > 1024 && (a.B <= 32 || (a.B <= 64 && a.n_active <= 1024))) hb = 4;
            if (hb > p.H) p.H = hb;
        }
    }
    if (p.H != 1 && p.H != 2 && p.H != 4) return p;
    if (p.R == 2 && p.H != 1 && p.H != 2 && p.H != 4) return p;
    if (p.R == 4 && p.H != 2 && p.H != 4) return p;   // four rows per lane: 128- or 64-row tiles (whole 64-row groups per term slice)
    if (!p.fast && (p.R != 1 || p.H != 1)) return p;
    const int BT = kWave * p.R / p.H, S = rowlane_row_stride(BT, p.H, p.R);
    if ((long long)(BT + 1) * a.d_in * 4 >= (1LL << 32)) return p;   // a lane's byte offset inside its batch tile is 32-bit
    p.n_btiles = (a.B + BT - 1) / BT;
    const int nw_max = rowlane_max_threads(p.R) / kWave;
    p.NW = t && t->waves ? t->waves : nw_max;
    if (p.NW < 1 || p.NW > nw_max) return p;
    // chunk: a multiple of 64 columns such that (a) the tile plus the all-zero column fits the LDS budget and
    // (b) a wavefront holds a chunk's staging units in registers; chunks of near-equal width
    const size_t budget = 144 * 1024;
    const int d_pad = (a.d_in + kSegCols - 1) / kSegCols * kSegCols;
    const int c_regs = kStageUnits * p.NW * 256 / BT / kSegCols * kSegCols;          // (BT/16)*(C/16) <= units limit
    const int c_lds = (int)(budget / (S * sizeof(float)) - 1) / kSegCols * kSegCols;
    const int c_max = c_lds < c_regs ? c_lds : c_regs;
    int C = t && t->chunk_cols ? t->chunk_cols : 0;
    if (C == 0) {
        if (c_max <= 0) return p;
        const int n = (d_pad + c_max - 1) / c_max;
        C = ((d_pad / kSegCols + n - 1) / n) * kSegCols;
    }
    if (C > d_pad) C = d_pad;
    if (C <= 0 || C % kSegCols != 0 || C > c_max) return p;
    p.C = C;
    p.n_chunks = (a.d_in + C - 1) / C;
    if (p.n_chunks < 1) p.n_chunks = 1;
    if (p.n_chunks > 1 && a.seg == nullptr) return p;   // chunk walking needs ascending rows + seg
    p.lds = (size_t)(C + 1) * S * sizeof(float);
    // stored rows per wavefront: fewest rounds times the cost of a workgroup, a fixed part (staging the tile, barriers,
    // stores) plus a part per stored row of a wavefront.  Rounds are counted per XCD (32 compute units; the kernel gives
    // all batch tiles of a group of stored rows to one XCD): 12 groups are two rounds on four of the eight XCDs even when
    // the launch has fewer than 256 workgroups.  Whole-row tiles (one term slice): in units of one term of a 64-row tile,
    // staging costs 0.15 per column and 64 rows, a term of a 128-row tile 1.3, six rows per wavefront (one block of
    // terms held in registers) a tenth more; with term slices the fixed part is about two stored rows' worth.  Fits of
    // the measured ranking of eight launch shapes each at batches 320..768 of three layers.
    // (two rows per lane in two term slices: the 64-row tile of the whole-row shape, a term at three quarters of its cost)
    const bool r2h2 = (p.R == 2 && p.H >= 2) || p.R == 4;
    const double fixed = p.R == 4 ? 0.15 * a.d_in * (kWave * p.R / p.H) / 64.0 : (r2h2 ? 0.15 * a.d_in : (p.H == 1 ? 0.15 * a.d_in * p.R : 2.0 * a.K));
    const double per_row = (double)a.K * (p.R == 4 ? 0.5 * (kWave * p.R / p.H) / 64.0 : (r2h2 ? 0.75 : (p.H == 1 && p.R == 2 ? 1.3 : 1.0)));
    // which workgroups share an XCD: the order that makes the 8 L2s fetch fewer bytes in all (all of x by each XCD, or
    // all of W_c / idx by each), unless it needs more rounds per XCD; the tuning can force either
    const int xo = t ? t->xcd_order : 0;
    if (xo < 0 || xo > 2) return p;
    const double x_bytes = (double)a.B * a.d_in * (a.x_bf16 ? 2 : 4);
    const double w_bytes = (double)a.n_active * a.K * ((a.x_bf16 ? 2 : 4) + (a.idx_u16 ? 2 : 4));
    auto rounds = [&](long long groups, bool by_tiles) {
        const long long per_xcd = by_tiles ? ((p.n_btiles + 7) / 8) * groups : ((groups + 7) / 8) * p.n_btiles;
        return (per_xcd + 31) / 32;
    };
    auto by_tiles = [&](long long groups) {
        if (xo) return xo == 2;
        // (measured: 3-8 % at 512 rows and more on 3072- and 4096-wide inputs, 20 % at 99 % sparsity; nothing or a loss
        // with fewer than two batch tiles per XCD)
        return x_bytes > w_bytes && p.n_btiles >= 16 && rounds(groups, true) <= rounds(groups, false);
    };
    auto shape_cost = [&](int c) {
        const long long groups = (n_slots + p.NW * c - 1) / (p.NW * c);
        return (double)rounds(groups, by_tiles(groups)) * (fixed + c * per_row) * (p.H == 1 && c >= 6 ? 1.1 : 1.0);
    };
    int npw = t && t->neurons_per_wave ? t->neurons_per_wave : 0;
    if (npw == 0) {
        static const int cand[6] = {1, 2, 3, 4, 6, 8};
        double best = -1.0;
        for (int ci = 0; ci < 6; ++ci) {
            const int c = cand[ci];
            // (six or eight rows with term slices, eight with one row per lane: only as the planner's last shapes)
            if (c > rowlane_max_npw(p.R, p.H) || (npw_cap < 8 && ((p.R == 2 && p.H >= 2 && c > 4) || (p.R == 1 && c > 6)))) break;
            if (npw_cap && c > npw_cap) break;
            const double cost = shape_cost(c);
            if (best < 0 || cost < best) { best = cost; npw = c; }
        }
    }
    if (npw != 1 && npw != 2 && npw != 3 && npw != 4 && npw != 6 && npw != 8) return p;
    if (npw > rowlane_max_npw(p.R, p.H)) return p;
    p.NPW = npw;
    p.cost = shape_cost(npw);
    p.KPRE = rowlane_kpre_rh(npw, p.R, p.H);
    // 32-row tiles of two rows per lane: blocks are 64 terms, and rows shorter than ~200 terms run 4-10 % faster with one
    // block preloaded per stored row and chunk than with two (less fetched beyond the chunk's share of the row), longer
    // ones 4-8 % slower
    if (p.R == 2 && p.H == 4 && a.K < kRowlaneShortRowK) p.KPRE = 1;
    // one row per lane in two or four slices: one block 3-10 % faster at fan-ins up to ~100, 1-5 % slower from 200
    if (p.R == 1 && p.H > 1 && a.K < kRowlaneShortRowOneK) p.KPRE = 1;
    p.n_groups = (n_slots + p.NW * npw - 1) / (p.NW * npw);
    p.bt_major = by_tiles(p.n_groups) ? 1 : 0;
    p.rounds = (int)rounds(p.n_groups, p.bt_major != 0);
    // Rows dealt out by median column: 10-16 % faster on layers whose rows cluster around different columns (4096-wide
    // inputs in 8 or 16 chunks, 2048- and 3072-wide ones at 1024 rows; nothing on 768-wide ones), 0.5-1.5 us per workgroup
    // otherwise (the keys' latency ahead of the first terms, and the barriers of the test).  The library's choice: from four
    // chunks on, where a workgroup is estimated to run for 45 us or more (the test then costs under 2 %), and only in
    // workgroups whose medians lie further apart than those of rows drawn evenly from all columns would (eight standard
    // deviations of such a median).
    const int sp = t ? t->spread_rows : 0;
    if (sp < 0 || sp > 3) return p;
    const int apart = 2 + (int)(4.0 * a.d_in / std::sqrt((double)std::max(a.K, 1)));
    // (rows can be dealt out where the kernel reads W_c / idx with aligned loads and a wavefront holds at least two rows)
    const bool can_spread = npw >= 2 && p.fast && !p.pk && reinterpret_cast<uintptr_t>(a.idx) % 4 == 0;
    const bool long_groups = (rowlane_estimate_us(a, p) - 2.19) / std::max(1, p.rounds) >= 45.0;
    if (sp == 0) p.spread = (p.n_chunks >= 4 && can_spread && a.seg != nullptr && long_groups) ? apart : 0;
    else p.spread = sp == 1 ? 0 : (sp == 2 ? 1 : apart);
    if (p.spread && !can_spread) return p;
    // the result tile sits behind the activation tile when both fit (no barrier between the last term and the
    // transposed write), else it reuses the activation tile's space
    // (with an active list: plus the column table and the bias of the columns the workgroup writes)
    const size_t out_tile = (size_t)BT * (p.NW * npw + 1) * sizeof(float) + (a.active ? (size_t)kSpanCap * 8 : 0);
    if (p.lds + out_tile <= 150 * 1024) { p.out_off = (int)(p.lds / sizeof(float)); p.lds += out_tile; }
    else { p.out_off = 0; if (out_tile > p.lds) p.lds = out_tile; }
    if (p.lds > kLdsMax) return p;
    p.ok = true;
    return p;
}

// Estimated time (us) of the batched kernel in launch shape p: a fixed part, and per round of workgroups (counted on the
// busiest XCD: a second, partly filled round takes as long as a full one) the chunks
// of columns it walks (two barriers and a staging burst each), the bytes of x a workgroup stages, the 16-step blocks of
// terms a wavefront walks (a partly filled block costs a whole one; a step of four term slices costs 1.5 times a step of
// one: its LDS reads collide) and the result tile; large layers also the stream of W_c / idx.  A least-squares fit
// (relative error, mean 5 %) of the mean of cold and cached timings of 260 points: 15 layer shapes, 512- to 4096-wide,
// 80-99 % sparse, at batches 2 to 1024, every term-slice count on seven of them.
// whole_blocks: every row counted in whole blocks of terms, as the comparison with the small-batch kernel was fitted
static double rowlane_estimate_us(const FwdArgs& a, const RowlanePlan& p, bool whole_blocks) {
    const int BT = kWave * p.R / p.H;
    const double rounds = std::max(1, p.rounds);
    // (a row that fits one block of terms is walked in groups of 4 or 8 steps up to its own length, not the whole block:
    // counted so between tile shapes, where whole blocks ranked the sliced tiles 20 % too slow on rows of 16-26 terms:
    // 768 -> 3072 K = 16 at B = 256 9.2 -> 7.7 us, 1024 -> 4096 K = 26 at B = 64 7.3 -> 6.1)
    const int group = p.R >= 2 ? 4 : 8;
    const int short_steps = std::max(group, ((a.K + p.H - 1) / p.H + group - 1) / group * group);
    const double steps = (double)p.NPW * (a.K <= kBlock * p.H && !whole_blocks ? short_steps : ((a.K + kBlock * p.H - 1) / (kBlock * p.H)) * kBlock);
    // (six or eight rows per wavefront keep one block of terms per row: the steps measured 0-40 % slower, longest on long segments)
    // (the same in two slices: 4096 -> 4096 at B = 512 measured 63.5 us with eight rows, 73.1 with four)
    const double many_rows = (p.R == 2 && p.NPW >= 6) ? (p.H == 1 ? 1.15 : 1.2) : 1.0;
    const double per_step = many_rows * (p.R == 2 ? (p.H == 4 ? (a.K < kRowlaneShortRowK ? 0.0345 : 0.0375) : (p.H == 2 ? 0.0337 : 0.0303)) : (p.H == 1 ? 0.0240 : (p.H == 2 ? 0.0279 : 0.0368)));
    const double terms = (double)a.n_active * a.K;
    return 2.19 + rounds * (1.38 * p.n_chunks + 5.90e-6 * BT * a.d_in * 4.0 + per_step * steps + 1.45e-4 * BT * p.NW * p.NPW * 4.0) +
           (terms > 1.5e6 ? 0.29e-6 * terms : 0.0);
}

// The tile: 64 batch rows x 1 term slice, 32 x 2, 16 x 4, or two rows per lane: 128 rows (one 8-byte LDS read feeds
// two rows, but half the workgroups each staging twice the tile), 64 rows in two term slices or 32 rows in four (the
// 64- and 32-row tiles with half the LDS instructions per term: 10-24 % faster than one row per lane from a fan-in of
// ~100, slower below; all need rows long enough for the term loop to matter: slower at fan-in 8).  With nothing forced the library takes the shape with the smallest estimated time; a forced
// part keeps the rules the other part had before the estimate existed.
static RowlanePlan plan_rowlane_by_estimate(const FwdArgs& a, const srigl_fwd_tuning* t) {
    const bool forced = t && (t->rows_per_lane || t->term_slices);
    if (forced) return plan_rowlane_with(a, t);
    RowlanePlan best{};
    best.ok = false;
    double best_us = 0.0;
    // rows per lane, term slices; a later shape must be 5 % ahead of an earlier one (the estimates are good to about that)
    // (the last entry: 128-row tiles with six or eight stored rows per wavefront, half the workgroups of the four-row form;
    // ahead at 1024 rows and more, where it saves a round of workgroups: 768 -> 3072 at B = 1024 36.4 -> 33.0 us)
    // (and the 64-row two-slice tile with six or eight: ahead where that still fills the compute units, 4096 -> 4096 at
    // B = 384 / 512 68.3 / 69.4 -> 62.2 / 63.5 us, 1024 -> 4096 at B = 512 28.8 -> 26.5)
    static const int shapes[8][2] = {{1, 1}, {2, 1}, {1, 2}, {1, 4}, {2, 2}, {2, 4}, {2, 1}, {2, 2}};
    for (int i = 0; i < 8; ++i) {
        // (two rows per lane need rows long enough for the term loop to matter; with six or eight rows per wavefront they are
        // ahead at any fan-in: 1024 -> 4096 K = 26 at B = 1024 39.6 -> 28.8 us, 768 -> 3072 K = 16 22.3 -> 18.3, K = 8 20.3 -> 17.6)
        if (shapes[i][0] == 2 && i < 6 && a.K < kRowlaneTwoRowsMinK) continue;
        if (shapes[i][0] == 2 && shapes[i][1] == 4 && a.K < kRowlaneTwoRowsFourSlicesMinK) continue;
        srigl_fwd_tuning shape{};
        if (t) shape = *t;
        shape.rows_per_lane = shapes[i][0];
        shape.term_slices = shapes[i][1];
        const RowlanePlan p = plan_rowlane_with(a, &shape, i == 1 ? 4 : (i >= 6 ? 8 : 0));
        if (!p.ok || (i >= 6 && p.NPW <= 4)) continue;
        // (inputs wider than 1024 with less than a term per 256 columns: the estimate counts blocks of terms, not the near-empty block every
        // chunk still costs a row, and ranks these shapes ahead of the small-batch kernel where they measured 50-80 % behind
        // it: 4096 -> 4096 K = 12 at B = 512..2048)
        if (i >= 6 && a.K < kRowlaneTwoRowsMinK && a.d_in > 1024 && (long long)a.K * 256 < a.d_in) continue;
        const double us = rowlane_estimate_us(a, p);
        if (!best.ok || us < 0.95 * best_us) { best = p; best_us = us; }
    }
    return best;
}

// A second ranking of the launch shapes, fitted to measurements of every shape (rows per lane x term slices x stored rows
// per wavefront) on 39 layers (768..4096 wide, fan-in 8..410, fp32 and bf16) at up to 14 batches from 48 to 4096, cached operands:
// per launch a constant; per round of workgroups a constant, a cost per chunk, per staged byte and per word of the result
// tile; per stored row and round a cost per step (terms / slices), a cost per chunk that holds terms of the row (the
// expected number for evenly drawn columns), and more per step from six rows per wavefront on (one block of terms in
// registers), the last three per tile shape; and a cost per stored term of layers beyond the L2.  Least squares on the
// relative error (std 8 %) of 17600 launches.  On the first 275 points (fan-in 16 and more, up to 2048 rows) the shape of
// smallest estimate above is 2.0 % slower than the best measured one on average (41 points more than 5 %, 17 more than
// 10 %, worst 25 %), on rows of fewer than 16 terms 4.9 %; the smallest of this ranking 0.9 % on all 489 points (27 beyond
// 5 %, 10 beyond 10 %, worst 22 %), and 1.0 % when the layer in question is left out of the fit.
static double rowlane_model_us(const FwdArgs& a, const RowlanePlan& p) {
    static const double per_shape[6][3] = {{2.1716, 0.93914, 0.27754}, {2.2649, 1.2646, 0.38936}, {2.8034, 2.1405, 0.20622},     // R = 1: H = 1, 2, 4
                                           {2.6393, 0.89263, 0.55438}, {2.8239, 1.3094, 0.56102}, {3.0297, 1.627, 0.67318}};    // R = 2
    if (p.R > 2) return 1e30;
    const int BT = kWave * p.R / p.H, NG = p.NW * p.NPW;
    const double* c = per_shape[(p.R - 1) * 3 + (p.H == 1 ? 0 : (p.H == 2 ? 1 : 2))];
    const double rounds = std::max(1, p.rounds), steps = (double)a.K / p.H;
    const double with_terms = p.n_chunks > 1 ? p.n_chunks * (1.0 - std::pow(1.0 - 1.0 / p.n_chunks, (double)a.K)) : 1.0;
    const double per_row = c[0] * steps * 1e-2 + c[1] * with_terms * 1e-1 + (p.NPW >= 6 ? c[2] * steps * 1e-2 : 0.0);
    const double terms = (double)a.n_active * a.K;
    return 1.4497 + rounds * (1.3486 + 0.39696 * p.n_chunks + 13.5e-6 * BT * a.d_in * 4.0 + 0.38181e-3 * BT * NG + p.NPW * per_row) +
           (terms > 1.5e6 ? 0.89109e-6 * terms : 0.0);
}

// The launch shape of the library's own choice: the one of smallest estimate, unless the fitted ranking has another shape more
// than 5 % ahead of it (mean distance to the best measured shape over the 489 measured points then 0.7 %, 24 points beyond
// 5 %, 8 beyond 10 %).
static RowlanePlan plan_rowlane_ranked(const FwdArgs& a, const srigl_fwd_tuning* t) {
    const RowlanePlan first = plan_rowlane_by_estimate(a, t);
    const bool forced = t && (t->rows_per_lane || t->term_slices || t->neurons_per_wave);
    if (forced || !first.ok) return first;
    const double first_us = rowlane_model_us(a, first);
    RowlanePlan best = first;
    double best_us = first_us;
    static const int rows_per_wave[6] = {1, 2, 3, 4, 6, 8};
    for (int R = 1; R <= 2; ++R)
        for (int H = 1; H <= 4; H *= 2)
            for (int n = 0; n < 6; ++n) {
                srigl_fwd_tuning shape{};
                if (t) shape = *t;
                shape.rows_per_lane = R;
                shape.term_slices = H;
                shape.neurons_per_wave = rows_per_wave[n];
                const RowlanePlan p = plan_rowlane_with(a, &shape, 8);
                if (!p.ok) continue;
                const double us = rowlane_model_us(a, p);
                if (us < best_us) { best = p; best_us = us; }
            }
    return first_us <= 1.05 * best_us ? first : best;
}

// (the ranking walks some hundred candidate shapes: the last few answers are kept per thread, keyed by everything a plan
// depends on, so that a caller that repeats a launch pays for it once)
static RowlanePlan plan_rowlane(const FwdArgs& a, const srigl_fwd_tuning* t) {
    struct Key {
        int32_t B, d_in, n_active, K, d_out, seg_stride, flags;
        srigl_fwd_tuning t;
        bool operator==(const Key& o) const { return std::memcmp(this, &o, sizeof(Key)) == 0; }
    };
    struct Entry { Key key; RowlanePlan plan; bool used; };
    static thread_local Entry cache[8] = {};
    static thread_local int next = 0;
    Key k;
    std::memset(&k, 0, sizeof(k));
    k.B = a.B; k.d_in = a.d_in; k.n_active = a.n_active; k.K = a.K; k.d_out = a.d_out; k.seg_stride = a.seg_stride;
    k.flags = (a.x_bf16 ? 1 : 0) | (a.idx_u16 ? 2 : 0) | (a.active ? 4 : 0) | (a.seg ? 8 : 0) | (a.packed ? 16 : 0) | (a.bias ? 32 : 0) |
              (int)((reinterpret_cast<uintptr_t>(a.x) & 15) << 8) | (int)((reinterpret_cast<uintptr_t>(a.idx) & 3) << 12) | (t ? 64 : 0);
    if (t) k.t = *t;
    for (int i = 0; i < 8; ++i)
        if (cache[i].used && cache[i].key == k) return cache[i].plan;
    const RowlanePlan p = plan_rowlane_ranked(a, t);
    cache[next].key = k; cache[next].plan = p; cache[next].used = true;
    next = (next + 1) & 7;
    return p;
}

bool rowlane_supported(const FwdArgs& a, const srigl_fwd_tuning* t) { return plan_rowlane(a, t).ok; }

srigl_status launch_fwd_rowlane(const FwdArgs& a, const srigl_fwd_tuning* t, hipStream_t st) {
    const int n_slots = a.active ? a.n_active + 1 : a.n_active;
    if (a.B == 0 || n_slots == 0) return SRIGL_OK;
    const RowlanePlan p = plan_rowlane(a, t);
    if (!p.ok) return SRIGL_ERR_UNSUPPORTED;
    if (a.idx_u16) return a.x_bf16 ? launch_rowlane_bf16_i16(a, p, st) : launch_rowlane_f32_i16(a, p, st);
    return a.x_bf16 ? launch_rowlane_bf16(a, p, st) : launch_rowlane_f32(a, p, st);
}

// The library's own choice of kernel: the smallest of the estimated times of the small-batch kernel (gathered or staged
// activations) and of the batched kernel in the launch shape it would take.  A single row always takes the small-batch
// kernel, above 2048 rows the batched kernel always wins.
// The choice between the small-batch kernel, the chunked batched kernel and the fallback.
static srigl_fwd_algo choose_chunked_or_small(const FwdArgs& a) {
    const int B = a.B, d_in = a.d_in, n_active = a.n_active, K = a.K;
    {   // the staged few-lanes shape of the small-batch kernel where it measured ahead of both estimates' kernels
        int few_L = 0, few_RB = 0;
        if (klane_few_lanes_staged(B, d_in, n_active, K, &few_L, &few_RB) && plan_klane(a, nullptr).ok) return SRIGL_FWD_KLANE;
    }
    bool batched = B > 16;
    if (B > 1 && B <= 2048 && d_in % 16 == 0) {
        static_assert(kKlaneTerms == 4, "klane_estimate_us assumes 4 terms per lane and request");
        const RowlanePlan rp = plan_rowlane_by_estimate(a, nullptr);   // (the comparison was fitted with this shape and estimate)
        batched = rp.ok && rowlane_estimate_us(a, rp, true) < klane_estimate_us(B, d_in, n_active, K);
    }
    const bool can_batch = rowlane_supported(a, nullptr);
    if (batched && can_batch) return SRIGL_FWD_ROWLANE;
    if (plan_klane(a, nullptr).ok) return SRIGL_FWD_KLANE;
    return can_batch ? SRIGL_FWD_ROWLANE : SRIGL_FWD_GENERIC;
}

// Estimate (us) of the faster of the small-batch and the chunked batched kernel (above 2048 rows: of the batched one).
static double chunked_or_small_estimate_us(const FwdArgs& a) {
    const RowlanePlan rp = plan_rowlane_by_estimate(a, nullptr);
    const double batched = rp.ok ? rowlane_estimate_us(a, rp, true) : 1e30;
    if (a.B > 2048 && rp.ok) return batched;
    return std::min(batched, klane_estimate_us(a.B, a.d_in, a.n_active, a.K));
}
// The whole-input batched kernel is taken where its estimate is ahead of that one's (5 % behind still counts: over the
// 238 launches its estimate was fitted to, that threshold left the least time on the table, 0.9 % against 7.5 % without
// this kernel); below 32 batch rows never against the staged few-lanes shape of the small-batch kernel, which was placed by
// measurement (at 32 rows this kernel measured ahead of it on rows of 77 terms, 6.1 / 5.4 against 7.5 / 6.4 us, and level on shorter ones).
constexpr double kRowloopMargin = 0.95;
srigl_fwd_algo choose_fwd_algo(const FwdArgs& a) {
    const srigl_fwd_algo base = choose_chunked_or_small(a);
    if (base == SRIGL_FWD_GENERIC || a.B < 2) return base;
    int few_L = 0, few_RB = 0;
    if (base == SRIGL_FWD_KLANE && a.B < 32 && klane_few_lanes_staged(a.B, a.d_in, a.n_active, a.K, &few_L, &few_RB)) return base;
    const double rl = rowloop_estimate_us(a);
    if (rl >= 1e29) return base;
    return rl * kRowloopMargin < chunked_or_small_estimate_us(a) ? SRIGL_FWD_ROWLOOP : base;
}

// stand-ins for the device arrays of a call of these sizes: the planner looks at their alignment and at which ones are
// present, never at their contents
static FwdArgs standin_args(int B, int d_in, int n_active, int K, int d_out, bool bf16, bool has_active, bool has_seg) {
    alignas(64) static const unsigned char aligned[64] = {0};
    FwdArgs a;
    a.x = aligned; a.x_bf16 = bf16; a.B = B; a.d_in = d_in; a.W_c = aligned; a.idx = aligned; a.idx_u16 = 0;
    a.active = has_active ? reinterpret_cast<const int32_t*>(aligned) : nullptr;
    a.n_active = n_active; a.K = K; a.bias = nullptr; a.d_out = d_out; a.y = nullptr;
    a.seg = has_seg ? reinterpret_cast<const uint16_t*>(aligned) : nullptr;
    a.seg_stride = srigl_seg_stride(d_in);
    a.packed = nullptr;
    a.act = SRIGL_ACT_NONE;
    return a;
}

double condensed_estimate_us(int B, int d_in, int n_active, int K, int d_out, bool bf16, bool has_active) {
    if (B <= 0 || n_active <= 0 || K <= 0 || d_in <= 0) return 2.0;
    const FwdArgs a = standin_args(B, d_in, n_active, K, d_out, bf16, has_active, true);
    const double other = chunked_or_small_estimate_us(a), rl = rowloop_estimate_us(a);
    return rl * kRowloopMargin < other ? rl : other;
}

}  // namespace srigl

using namespace srigl;


extern "C" {

static srigl_status fwd_core(const void* x, srigl_dtype x_dtype, int32_t B, int32_t d_in, const void* W_c, srigl_dtype w_dtype,
                             const void* idx, bool idx_u16, const int32_t* active, int32_t n_active, int32_t K, const float* bias,
                             int32_t d_out, float* y, const uint16_t* seg, const void* packed, srigl_fwd_algo algo,
                             const srigl_fwd_tuning* tuning, srigl_activation act, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (act != SRIGL_ACT_NONE && act != SRIGL_ACT_RELU && act != SRIGL_ACT_GELU) return SRIGL_ERR_INVALID_ARG;
    if (B < 0 || d_in < 0 || n_active < 0 || K < 0 || d_out < 0 || K > d_in || n_active > d_out) return SRIGL_ERR_INVALID_ARG;
    if ((x_dtype != SRIGL_F32 && x_dtype != SRIGL_BF16) || (w_dtype != SRIGL_F32 && w_dtype != SRIGL_BF16)) return SRIGL_ERR_INVALID_ARG;
    if (x_dtype != w_dtype) return SRIGL_ERR_UNSUPPORTED;
    if (idx_u16 && d_in > 65536) return SRIGL_ERR_UNSUPPORTED;
    if (seg != nullptr && K > 65535) return SRIGL_ERR_UNSUPPORTED;   // seg entries are 16-bit term counts
    if (packed != nullptr && reinterpret_cast<uintptr_t>(packed) % 16 != 0) return SRIGL_ERR_INVALID_ARG;
    if (active == nullptr && n_active != d_out && n_active != 0) return SRIGL_ERR_INVALID_ARG;
    if (B == 0 || d_out == 0) return SRIGL_OK;
    if (y == nullptr) return SRIGL_ERR_INVALID_ARG;
    if (n_active > 0 && K > 0 && (x == nullptr || W_c == nullptr || idx == nullptr)) return SRIGL_ERR_INVALID_ARG;

    FwdArgs a;
    a.x = x; a.x_bf16 = (x_dtype == SRIGL_BF16); a.B = B; a.d_in = d_in; a.W_c = W_c; a.idx = idx; a.idx_u16 = idx_u16 ? 1 : 0; a.active = active;
    a.n_active = n_active; a.K = K; a.bias = bias; a.d_out = d_out; a.y = y; a.seg = seg;
    a.seg_stride = srigl_seg_stride(d_in);
    a.packed = packed;
    a.act = (int32_t)act;
    if (n_active == 0 || K == 0) {   // nothing is stored: every column holds its bias
        long long blocks = ((long long)B * d_out + 255) / 256;
        if (blocks > 65536) blocks = 65536;
        hipLaunchKernelGGL(k_bias_broadcast, dim3((unsigned)blocks), dim3(256), 0, st, bias, B, d_out, y, a.act);
        return hip_ok(hipGetLastError());
    }
    switch (algo) {
        case SRIGL_FWD_GENERIC: return launch_fwd_generic(a, st);
        case SRIGL_FWD_KLANE: return launch_fwd_klane(a, tuning, st);
        case SRIGL_FWD_ROWLANE: return launch_fwd_rowlane(a, tuning, st);
        case SRIGL_FWD_ROWLOOP: return launch_fwd_rowloop(a, tuning, st);
        case SRIGL_FWD_AUTO: break;
        default: return SRIGL_ERR_INVALID_ARG;
    }
    switch (choose_fwd_algo(a)) {
        case SRIGL_FWD_ROWLANE: return launch_fwd_rowlane(a, nullptr, st);
        case SRIGL_FWD_ROWLOOP: return launch_fwd_rowloop(a, nullptr, st);
        case SRIGL_FWD_KLANE: return launch_fwd_klane(a, nullptr, st);
        default: return launch_fwd_generic(a, st);
    }
}

srigl_status srigl_condensed_linear_fwd_algo(const void* x, srigl_dtype x_dtype, int32_t B, int32_t d_in,
                                             const void* W_c, srigl_dtype w_dtype, const int32_t* idx,
                                             const int32_t* active, int32_t n_active, int32_t K,
                                             const float* bias, int32_t d_out, float* y,
                                             const uint16_t* seg, const void* packed, srigl_fwd_algo algo,
                                             const srigl_fwd_tuning* tuning, void* stream) {
    return fwd_core(x, x_dtype, B, d_in, W_c, w_dtype, idx, false, active, n_active, K, bias, d_out, y, seg, packed, algo, tuning, SRIGL_ACT_NONE, stream);
}

srigl_status srigl_condensed_linear_fwd_act(const void* x, srigl_dtype x_dtype, int32_t B, int32_t d_in,
                                            const void* W_c, srigl_dtype w_dtype, const int32_t* idx,
                                            const int32_t* active, int32_t n_active, int32_t K,
                                            const float* bias, int32_t d_out, float* y,
                                            const uint16_t* seg, const void* packed, srigl_activation act, srigl_fwd_algo algo,
                                            const srigl_fwd_tuning* tuning, void* stream) {
    return fwd_core(x, x_dtype, B, d_in, W_c, w_dtype, idx, false, active, n_active, K, bias, d_out, y, seg, packed, algo, tuning, act, stream);
}

srigl_status srigl_condensed_linear_fwd(const void* x, srigl_dtype x_dtype, int32_t B, int32_t d_in,
                                        const void* W_c, srigl_dtype w_dtype, const int32_t* idx,
                                        const int32_t* active, int32_t n_active, int32_t K,
                                        const float* bias, int32_t d_out, float* y,
                                        const uint16_t* seg, const void* packed, void* stream) {
    return fwd_core(x, x_dtype, B, d_in, W_c, w_dtype, idx, false, active, n_active, K, bias, d_out, y, seg, packed, SRIGL_FWD_AUTO, nullptr,
                    SRIGL_ACT_NONE, stream);
}

srigl_status srigl_condensed_linear_fwd_idx16(const void* x, srigl_dtype x_dtype, int32_t B, int32_t d_in,
                                              const void* W_c, srigl_dtype w_dtype, const uint16_t* idx16,
                                              const int32_t* active, int32_t n_active, int32_t K,
                                              const float* bias, int32_t d_out, float* y,
                                              const uint16_t* seg, srigl_activation act, srigl_fwd_algo algo,
                                              const srigl_fwd_tuning* tuning, void* stream) {
    return fwd_core(x, x_dtype, B, d_in, W_c, w_dtype, idx16, true, active, n_active, K, bias, d_out, y, seg, nullptr, algo, tuning, act, stream);
}

srigl_status srigl_narrow_idx(const int32_t* idx, int64_t n, int32_t d_in, uint16_t* idx16, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (n < 0 || d_in < 0) return SRIGL_ERR_INVALID_ARG;
    if (d_in > 65536) return SRIGL_ERR_UNSUPPORTED;
    if (n == 0) return SRIGL_OK;
    if (idx == nullptr || idx16 == nullptr || d_in == 0) return SRIGL_ERR_INVALID_ARG;
    const int hi = d_in - 1;
    long long done = 0;
    if (reinterpret_cast<uintptr_t>(idx) % 16 == 0 && reinterpret_cast<uintptr_t>(idx16) % 16 == 0 && n >= 8) {
        const long long n8 = n / 8;
        long long blocks = (n8 + 255) / 256;
        if (blocks > 4096) blocks = 4096;
        hipLaunchKernelGGL(k_narrow_idx8, dim3((unsigned)blocks), dim3(256), 0, st, reinterpret_cast<const int4*>(idx), n8, hi,
                           reinterpret_cast<uint4*>(idx16));
        done = n8 * 8;
    }
    if (done < n) {
        long long blocks = (n - done + 255) / 256;
        if (blocks > 4096) blocks = 4096;
        hipLaunchKernelGGL(k_narrow_idx1, dim3((unsigned)blocks), dim3(256), 0, st, idx, done, (long long)n, hi, idx16);
    }
    return hip_ok(hipGetLastError());
}

srigl_status srigl_fwd_plan_query(int32_t B, int32_t d_in, int32_t n_active, int32_t K, int32_t d_out, srigl_dtype dtype,
                                  int32_t has_active, int32_t has_seg, srigl_fwd_plan* plan) {
    return srigl_fwd_plan_query_algo(B, d_in, n_active, K, d_out, dtype, has_active, has_seg, SRIGL_FWD_AUTO, nullptr, plan);
}

srigl_status srigl_fwd_plan_query_algo(int32_t B, int32_t d_in, int32_t n_active, int32_t K, int32_t d_out, srigl_dtype dtype,
                                       int32_t has_active, int32_t has_seg, srigl_fwd_algo forced, const srigl_fwd_tuning* tuning,
                                       srigl_fwd_plan* plan) {
    if (forced != SRIGL_FWD_AUTO && forced != SRIGL_FWD_GENERIC && forced != SRIGL_FWD_KLANE && forced != SRIGL_FWD_ROWLANE &&
        forced != SRIGL_FWD_ROWLOOP)
        return SRIGL_ERR_INVALID_ARG;
    if (plan == nullptr || B < 0 || d_in < 0 || n_active < 0 || K < 0 || d_out < 0 || K > d_in || n_active > d_out)
        return SRIGL_ERR_INVALID_ARG;
    if (dtype != SRIGL_F32 && dtype != SRIGL_BF16) return SRIGL_ERR_INVALID_ARG;
    *plan = srigl_fwd_plan{};
    if (B == 0 || d_out == 0 || n_active == 0 || K == 0) return SRIGL_OK;   // nothing to gather: no forward kernel runs
    const FwdArgs a = standin_args(B, d_in, n_active, K, d_out, dtype == SRIGL_BF16, has_active != 0, has_seg != 0);
    const srigl_fwd_algo algo = forced == SRIGL_FWD_AUTO ? choose_fwd_algo(a) : forced;
    plan->algo = (int32_t)algo;
    if (algo == SRIGL_FWD_ROWLANE) {
        const RowlanePlan p = plan_rowlane(a, tuning);
        if (!p.ok) return SRIGL_ERR_UNSUPPORTED;
        plan->rows_per_lane = p.R; plan->term_slices = p.H; plan->waves = p.NW; plan->neurons_per_wave = p.NPW;
        plan->chunk_cols = p.C; plan->workgroups = (int64_t)p.n_groups * p.n_btiles; plan->xcd_order = p.bt_major ? 2 : 1;
        plan->spread_rows = p.spread == 0 ? 1 : (p.spread == 1 ? 2 : 3);
    } else if (algo == SRIGL_FWD_ROWLOOP) {
        if (!rowloop_plan_query(a, tuning, plan)) return SRIGL_ERR_UNSUPPORTED;
    } else if (algo == SRIGL_FWD_KLANE) {
        const KlanePlan p = plan_klane(a, tuning);
        if (!p.ok) return SRIGL_ERR_UNSUPPORTED;
        plan->lanes_per_neuron = p.L; plan->rows_per_block = p.RB; plan->workgroups = p.workgroups; plan->direct_gather = p.direct;
    }
    return SRIGL_OK;
}

}  // extern "C"
