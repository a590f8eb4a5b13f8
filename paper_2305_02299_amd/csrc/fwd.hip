// Forward kernels of the condensed constant fan-in linear layer (gfx950).
//
// All of them compute Alg. 1 of arXiv 2305.02299,
//     y[b][active[s]] = bias[active[s]] + sum_k W_c[s][k] * x[b][idx[s][k]],
// and give every column that is not stored (an ablated neuron, Sec. 3.1 step 4) its bias.
// Because `active` is ascending, the columns that are not stored are exactly the gaps between
// consecutive entries; the thread (or wavefront) that owns stored row s also fills the gap in front
// of column active[s], and a virtual row s == n_active fills the tail.
#include "srigl_internal.h"

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
template <typename XT>
__global__ __launch_bounds__(256) void k_fwd_generic(const XT* __restrict__ x, int B, int d_in, const XT* __restrict__ W_c,
                                                     const int32_t* __restrict__ idx, const int32_t* __restrict__ active,
                                                     int n_active, int K, const float* __restrict__ bias, int d_out,
                                                     float* __restrict__ y) {
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
            for (int c = max(prev + 1, 0); c < col; ++c) yr[c] = bias_at(bias, c);
        }
        if (s >= n_active || col < 0 || col >= d_out) continue;
        const XT* xr = x + (size_t)b * d_in;
        const XT* w = W_c + (size_t)s * K;
        const int32_t* ix = idx + (size_t)s * K;
        float acc = 0.0f;
        for (int k = 0; k < K; ++k) {
            const int j = min(max(ix[k], 0), d_in - 1);
            acc = fmaf(to_f32<XT>(w[k]), to_f32<XT>(xr[j]), acc);
        }
        yr[col] = acc + bias_at(bias, col);
    }
}

// y[b][c] = bias[c] (or 0): the whole forward pass when nothing is stored (n_active == 0 or K == 0).
__global__ __launch_bounds__(256) void k_bias_broadcast(const float* __restrict__ bias, int B, int d_out, float* __restrict__ y) {
    const long long total = (long long)B * d_out;
    for (long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (long long)gridDim.x * blockDim.x)
        y[t] = bias_at(bias, (int)(t % d_out));
}

// ------------------------------------------------------------------------------------------------
// KLANE (small batch, online inference).  A workgroup stages RB rows of x in LDS (fp32, row-major)
// and walks over stored rows; L lanes (a power of two) share one stored row: lane q takes the terms
// k = q, q+L, ... so that a wavefront's loads of W_c and idx are runs of L contiguous words, and the
// partial sums are combined with a butterfly of cross-lane shuffles.
// ------------------------------------------------------------------------------------------------
template <int RB, typename XT>
__global__ __launch_bounds__(256) void k_fwd_klane(const XT* __restrict__ x, int B, int d_in, const XT* __restrict__ W_c,
                                                   const int32_t* __restrict__ idx, const int32_t* __restrict__ active,
                                                   int n_active, int K, const float* __restrict__ bias, int d_out,
                                                   float* __restrict__ y, int log2L, int rows_per_wg) {
    extern __shared__ float xs[];   // [RB][d_in]
    const int L = 1 << log2L;
    const int tid = threadIdx.x;
    const int q = tid & (L - 1);                      // lane within the neuron's group
    const int grp = tid >> log2L;                     // group within the workgroup
    const int groups = blockDim.x >> log2L;
    const int b0 = blockIdx.y * RB;
    const int n_slots = active ? n_active + 1 : n_active;
    const int s_begin = blockIdx.x * rows_per_wg;
    const int s_end = min(s_begin + rows_per_wg, n_slots);

    // first terms of the first stored row are requested before the staging barrier
    int s = s_begin + grp;
    float w0 = 0.0f;
    int j0 = 0;
    if (s < min(s_end, n_active) && q < K) {
        w0 = to_f32<XT>(W_c[(size_t)s * K + q]);
        j0 = idx[(size_t)s * K + q];
    }

    for (int r = 0; r < RB; ++r) {
        const int b = b0 + r;
        for (int j = tid; j < d_in; j += blockDim.x) xs[r * d_in + j] = (b < B) ? to_f32<XT>(x[(size_t)b * d_in + j]) : 0.0f;
    }
    __syncthreads();

    for (; s < s_end; s += groups) {
        float acc[RB];
#pragma unroll
        for (int r = 0; r < RB; ++r) acc[r] = 0.0f;
        if (s < n_active) {
            const XT* w = W_c + (size_t)s * K;
            const int32_t* ix = idx + (size_t)s * K;
            if (q < K) {
#pragma unroll
                for (int r = 0; r < RB; ++r) acc[r] = w0 * xs[r * d_in + j0];
            }
            for (int k = q + L; k < K; k += L) {
                const float wv = to_f32<XT>(w[k]);
                const int j = ix[k];
#pragma unroll
                for (int r = 0; r < RB; ++r) acc[r] = fmaf(wv, xs[r * d_in + j], acc[r]);
            }
        }
        // next row's first terms: in flight during the reduction and the stores
        const int sn = s + groups;
        if (sn < min(s_end, n_active) && q < K) {
            w0 = to_f32<XT>(W_c[(size_t)sn * K + q]);
            j0 = idx[(size_t)sn * K + q];
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
                const float bv = bias_at(bias, c);
#pragma unroll
                for (int r = 0; r < RB; ++r)
                    if (b0 + r < B) y[(size_t)(b0 + r) * d_out + c] = bv;
            }
        }
        if (q == 0 && s < n_active && col >= 0 && col < d_out) {
            const float bv = bias_at(bias, col);
#pragma unroll
            for (int r = 0; r < RB; ++r)
                if (b0 + r < B) y[(size_t)(b0 + r) * d_out + col] = acc[r] + bv;
        }
    }
}

// ------------------------------------------------------------------------------------------------
// ROWLANE (batched).  Lanes are batch rows: a workgroup owns a tile of 64*R batch rows and a group
// of stored rows, and keeps the activation tile transposed in LDS (xs[column][row], fp32), so that
// for one (stored row, k) the index and the weight are wave-uniform (scalar loads, scalar
// registers) and the gather is one conflict-free LDS read of 64*R consecutive words.  d_in is
// walked in chunks of `C` columns that fit LDS; within a chunk the terms of an ascending row are
// the contiguous range seg[..] gives.  Each wavefront accumulates NPW stored rows in registers
// across the chunks.
//
// LDS row stride S = 64*R + 4 words: the staging pass writes 16 rows x 16 columns per wavefront
// instruction (global reads of 64 contiguous bytes per row) and the +4 skew spreads those writes
// over all banks, while reads of consecutive rows stay conflict-free and 16-byte aligned.
// ------------------------------------------------------------------------------------------------
template <int R> struct RowVec;
template <> struct RowVec<1> { using type = float; };
template <> struct RowVec<2> { using type = float2; };
template <> struct RowVec<4> { using type = float4; };

template <typename XT>
__device__ __forceinline__ void load4(const XT* __restrict__ p, bool vec_ok, int n_valid, float out[4]);

template <>
__device__ __forceinline__ void load4<float>(const float* __restrict__ p, bool vec_ok, int n_valid, float out[4]) {
    if (vec_ok && n_valid >= 4) {
        const float4 v = *reinterpret_cast<const float4*>(p);
        out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) out[i] = (i < n_valid) ? p[i] : 0.0f;
    }
}

template <>
__device__ __forceinline__ void load4<uint16_t>(const uint16_t* __restrict__ p, bool vec_ok, int n_valid, float out[4]) {
    if (vec_ok && n_valid >= 4) {
        const uint2 v = *reinterpret_cast<const uint2*>(p);
        out[0] = __uint_as_float(v.x << 16); out[1] = __uint_as_float(v.x & 0xffff0000u);
        out[2] = __uint_as_float(v.y << 16); out[3] = __uint_as_float(v.y & 0xffff0000u);
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) out[i] = (i < n_valid) ? bf16_bits_to_float(p[i]) : 0.0f;
    }
}

template <int R, int NPW, typename XT>
__global__ __launch_bounds__(1024) void k_fwd_rowlane(const XT* __restrict__ x, int B, int d_in, const XT* __restrict__ W_c,
                                                      const int32_t* __restrict__ idx, const int32_t* __restrict__ active,
                                                      int n_active, int K, const float* __restrict__ bias, int d_out,
                                                      float* __restrict__ y, const uint16_t* __restrict__ seg, int seg_stride,
                                                      int C, int n_chunks, int n_btiles, int n_groups, int vec_ok) {
    extern __shared__ float xs[];   // [C][S]
    constexpr int BT = kWave * R;
    constexpr int S = BT + 4;
    using V = typename RowVec<R>::type;

    // XCD-aware decode: consecutive workgroup ids go to different XCDs (8 of them), so the id modulo 8
    // selects the XCD; all batch tiles of one neuron group are given to the same XCD, whose L2 then
    // holds that group's W_c / idx once.
    const int wg = blockIdx.x;
    const int xcd = wg & 7, inx = wg >> 3;
    const int bt = inx % n_btiles;
    const int g = (inx / n_btiles) * 8 + xcd;
    if (g >= n_groups) return;

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nw = blockDim.x >> 6;
    const int b0 = bt * BT;
    const int n_slots = active ? n_active + 1 : n_active;
    const int s0 = (g * nw + wv) * NPW;   // first stored row of this wavefront

    float acc[NPW][R];
#pragma unroll
    for (int i = 0; i < NPW; ++i)
#pragma unroll
        for (int r = 0; r < R; ++r) acc[i][r] = 0.0f;

    const int segs_per_chunk = C / kSegCols;
    for (int c = 0; c < n_chunks; ++c) {
        const int c0 = c * C;
        const int cw = min(C, d_in - c0);
        if (c > 0) __syncthreads();
        // ---- stage x[b0 .. b0+BT)[c0 .. c0+cw) transposed into xs ----
        {
            const int dq = lane & 3, db = lane >> 2;          // 4 column quads x 16 rows per wavefront pass
            const int col_tiles = (cw + 15) >> 4;
            const int units = (BT / 16) * col_tiles;
            for (int u = wv; u < units; u += nw) {
                const int rt = u / col_tiles, ct = u - rt * col_tiles;
                const int rl = rt * 16 + db;                  // row within the tile
                const int f = ct * 16 + dq * 4;               // column within the chunk
                const int b = b0 + rl;
                float v[4] = {0.0f, 0.0f, 0.0f, 0.0f};
                const int n_valid = min(4, cw - f);
                if (b < B && n_valid > 0) load4<XT>(x + (size_t)b * d_in + c0 + f, vec_ok != 0, n_valid, v);
                if (n_valid > 0) {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (i < n_valid) xs[(f + i) * S + rl] = v[i];
                }
            }
        }
        __syncthreads();
        // ---- accumulate this chunk's terms ----
        const float* xl = xs + lane * R;
#pragma unroll
        for (int i = 0; i < NPW; ++i) {
            const int s = s0 + i;
            if (s < n_active) {
                int k0 = 0, k1 = K;
                if (seg) {
                    const uint16_t* sg = seg + (size_t)s * seg_stride;
                    k0 = sg[c * segs_per_chunk];
                    k1 = sg[min((c + 1) * segs_per_chunk, seg_stride - 1)];
                }
                const XT* w = W_c + (size_t)s * K;
                const int32_t* ix = idx + (size_t)s * K;
#pragma unroll 8
                for (int k = k0; k < k1; ++k) {
                    const float wk = to_f32<XT>(w[k]);
                    const int j = ix[k] - c0;
                    const V xv = *reinterpret_cast<const V*>(xl + j * S);
                    if constexpr (R == 1) {
                        acc[i][0] = fmaf(wk, xv, acc[i][0]);
                    } else if constexpr (R == 2) {
                        acc[i][0] = fmaf(wk, xv.x, acc[i][0]);
                        acc[i][1] = fmaf(wk, xv.y, acc[i][1]);
                    } else {
                        acc[i][0] = fmaf(wk, xv.x, acc[i][0]);
                        acc[i][1] = fmaf(wk, xv.y, acc[i][1]);
                        acc[i][2] = fmaf(wk, xv.z, acc[i][2]);
                        acc[i][3] = fmaf(wk, xv.w, acc[i][3]);
                    }
                }
            }
        }
    }

    // ---- bias, scatter, gaps ----
#pragma unroll
    for (int i = 0; i < NPW; ++i) {
        const int s = s0 + i;
        if (s >= n_slots) break;
        int col = s;
        if (active) {
            col = min((s < n_active) ? active[s] : d_out, d_out);
            const int prev = (s > 0) ? active[s - 1] : -1;
            for (int cc = max(prev + 1, 0); cc < col; ++cc) {
                const float bv = bias_at(bias, cc);
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const int b = b0 + lane * R + r;
                    if (b < B) y[(size_t)b * d_out + cc] = bv;
                }
            }
        }
        if (s < n_active && col >= 0 && col < d_out) {
            const float bv = bias_at(bias, col);
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int b = b0 + lane * R + r;
                if (b < B) y[(size_t)b * d_out + col] = acc[i][r] + bv;
            }
        }
    }
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
    if (a.x_bf16)
        hipLaunchKernelGGL(k_fwd_generic<uint16_t>, dim3((unsigned)blocks), dim3(256), 0, st, (const uint16_t*)a.x, a.B, a.d_in,
                           (const uint16_t*)a.W_c, a.idx, a.active, a.n_active, a.K, a.bias, a.d_out, a.y);
    else
        hipLaunchKernelGGL(k_fwd_generic<float>, dim3((unsigned)blocks), dim3(256), 0, st, (const float*)a.x, a.B, a.d_in,
                           (const float*)a.W_c, a.idx, a.active, a.n_active, a.K, a.bias, a.d_out, a.y);
    return hip_ok(hipGetLastError());
}

template <int RB, typename XT>
static srigl_status launch_klane_t(const FwdArgs& a, int log2L, int rows_per_wg, hipStream_t st) {
    const int n_slots = a.active ? a.n_active + 1 : a.n_active;
    const size_t lds = (size_t)RB * a.d_in * sizeof(float);
    if (lds > kLdsMax) return SRIGL_ERR_UNSUPPORTED;
    auto kern = k_fwd_klane<RB, XT>;
    static size_t lds_allowed = 64 * 1024;   // raised once per kernel instance, not per call
    if (lds > lds_allowed) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsMax) != hipSuccess)
            return SRIGL_ERR_HIP;
        lds_allowed = kLdsMax;
    }
    const unsigned gx = (unsigned)((n_slots + rows_per_wg - 1) / rows_per_wg);
    const unsigned gy = (unsigned)((a.B + RB - 1) / RB);
    if (gy > 65535u) return SRIGL_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(kern, dim3(gx, gy), dim3(256), lds, st, (const XT*)a.x, a.B, a.d_in, (const XT*)a.W_c, a.idx, a.active,
                       a.n_active, a.K, a.bias, a.d_out, a.y, log2L, rows_per_wg);
    return hip_ok(hipGetLastError());
}

srigl_status launch_fwd_klane(const FwdArgs& a, const srigl_fwd_tuning* t, hipStream_t st) {
    const int n_slots = a.active ? a.n_active + 1 : a.n_active;
    if (a.B == 0 || n_slots == 0) return SRIGL_OK;
    // lanes per stored row: enough that a lane has at most ~4 terms, at least 4, at most 64
    int L = t && t->lanes_per_neuron ? t->lanes_per_neuron : 0;
    if (L == 0) { L = 4; while (L < 64 && L * 4 < a.K) L <<= 1; }
    if (L < 1 || L > 64 || (L & (L - 1)) != 0) return SRIGL_ERR_UNSUPPORTED;
    int RB = t && t->rows_per_block ? t->rows_per_block : 0;
    if (RB == 0) { RB = 1; while (RB < 8 && RB < a.B) RB <<= 1; }
    while (RB > 1 && (size_t)RB * a.d_in * sizeof(float) > kLdsMax / 2) RB >>= 1;
    if (RB != 1 && RB != 2 && RB != 4 && RB != 8) return SRIGL_ERR_UNSUPPORTED;
    const int log2L = ilog2_floor(L);
    const int groups = 256 / L;
    // stored rows per workgroup: one pass of all groups, more when that still leaves > 8 workgroups per CU
    int rows_per_wg = groups;
    while ((long long)((n_slots + rows_per_wg - 1) / rows_per_wg) * ((a.B + RB - 1) / RB) > 256 * 8) rows_per_wg += groups;
#define SRIGL_KLANE(RBV)                                                                               \
    return a.x_bf16 ? launch_klane_t<RBV, uint16_t>(a, log2L, rows_per_wg, st) : launch_klane_t<RBV, float>(a, log2L, rows_per_wg, st)
    switch (RB) {
        case 1: SRIGL_KLANE(1);
        case 2: SRIGL_KLANE(2);
        case 4: SRIGL_KLANE(4);
        default: SRIGL_KLANE(8);
    }
#undef SRIGL_KLANE
}

struct RowlanePlan { int R, NW, NPW, C, n_chunks, n_btiles, n_groups; size_t lds; bool ok; };

static RowlanePlan plan_rowlane(const FwdArgs& a, const srigl_fwd_tuning* t) {
    RowlanePlan p{};
    p.ok = false;
    const int n_slots = a.active ? a.n_active + 1 : a.n_active;
    p.R = t && t->rows_per_lane ? t->rows_per_lane : 1;
    if (p.R != 1 && p.R != 2 && p.R != 4) return p;
    const int BT = kWave * p.R, S = BT + 4;
    p.n_btiles = (a.B + BT - 1) / BT;
    // chunk: the largest multiple of 64 columns whose tile fits the LDS budget
    const size_t budget = 144 * 1024;
    int cmax = (int)(budget / (S * sizeof(float))) / kSegCols * kSegCols;
    int C = t && t->chunk_cols ? t->chunk_cols : cmax;
    if (C <= 0 || C % kSegCols != 0 || C > cmax) return p;
    const int d_pad = (a.d_in + kSegCols - 1) / kSegCols * kSegCols;
    if (C > d_pad) C = d_pad;
    p.C = C;
    p.n_chunks = (a.d_in + C - 1) / C;
    if (p.n_chunks < 1) p.n_chunks = 1;
    if (p.n_chunks > 1 && a.seg == nullptr) return p;   // chunk walking needs ascending rows + seg
    p.lds = (size_t)C * S * sizeof(float);
    // workgroup shape: aim at one workgroup per CU over the whole launch
    p.NW = t && t->waves ? t->waves : 16;
    if (p.NW < 1 || p.NW > 16) return p;
    int npw = t && t->neurons_per_wave ? t->neurons_per_wave : 0;
    if (npw == 0) {
        const long long per_cu = ((long long)n_slots * p.n_btiles + 255) / 256;   // (stored row, batch tile) pairs per CU
        npw = (int)((per_cu + p.NW - 1) / p.NW);
        if (npw < 1) npw = 1;
        if (npw > 8) npw = 8;
        if (npw == 5) npw = 6;
        if (npw == 7) npw = 8;
    }
    if (npw != 1 && npw != 2 && npw != 3 && npw != 4 && npw != 6 && npw != 8) return p;
    p.NPW = npw;
    p.n_groups = (n_slots + p.NW * npw - 1) / (p.NW * npw);
    p.ok = true;
    return p;
}

bool rowlane_supported(const FwdArgs& a, const srigl_fwd_tuning* t) { return plan_rowlane(a, t).ok; }

template <int R, int NPW, typename XT>
static srigl_status launch_rowlane_t(const FwdArgs& a, const RowlanePlan& p, hipStream_t st) {
    auto kern = k_fwd_rowlane<R, NPW, XT>;
    static size_t lds_allowed = 64 * 1024;   // raised once per kernel instance, not per call
    if (p.lds > lds_allowed) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsMax) != hipSuccess)
            return SRIGL_ERR_HIP;
        lds_allowed = kLdsMax;
    }
    const long long blocks = 8LL * ((p.n_groups + 7) / 8) * p.n_btiles;
    if (blocks > 0x7fffffffLL) return SRIGL_ERR_UNSUPPORTED;
    const size_t xal = sizeof(XT) * 4;   // bytes of a 4-element vector load
    const int vec_ok = (a.d_in % 4 == 0) && ((reinterpret_cast<uintptr_t>(a.x) % xal) == 0);
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(p.NW * kWave), p.lds, st, (const XT*)a.x, a.B, a.d_in, (const XT*)a.W_c,
                       a.idx, a.active, a.n_active, a.K, a.bias, a.d_out, a.y, a.seg, a.seg_stride, p.C, p.n_chunks, p.n_btiles,
                       p.n_groups, vec_ok);
    return hip_ok(hipGetLastError());
}

template <int R, typename XT>
static srigl_status launch_rowlane_r(const FwdArgs& a, const RowlanePlan& p, hipStream_t st) {
    switch (p.NPW) {
        case 1: return launch_rowlane_t<R, 1, XT>(a, p, st);
        case 2: return launch_rowlane_t<R, 2, XT>(a, p, st);
        case 3: return launch_rowlane_t<R, 3, XT>(a, p, st);
        case 4: return launch_rowlane_t<R, 4, XT>(a, p, st);
        case 6: return launch_rowlane_t<R, 6, XT>(a, p, st);
        default: return launch_rowlane_t<R, 8, XT>(a, p, st);
    }
}

srigl_status launch_fwd_rowlane(const FwdArgs& a, const srigl_fwd_tuning* t, hipStream_t st) {
    const int n_slots = a.active ? a.n_active + 1 : a.n_active;
    if (a.B == 0 || n_slots == 0) return SRIGL_OK;
    const RowlanePlan p = plan_rowlane(a, t);
    if (!p.ok) return SRIGL_ERR_UNSUPPORTED;
    if (a.x_bf16) {
        switch (p.R) {
            case 1: return launch_rowlane_r<1, uint16_t>(a, p, st);
            case 2: return launch_rowlane_r<2, uint16_t>(a, p, st);
            default: return launch_rowlane_r<4, uint16_t>(a, p, st);
        }
    }
    switch (p.R) {
        case 1: return launch_rowlane_r<1, float>(a, p, st);
        case 2: return launch_rowlane_r<2, float>(a, p, st);
        default: return launch_rowlane_r<4, float>(a, p, st);
    }
}

}  // namespace srigl

using namespace srigl;

extern "C" {

srigl_status srigl_condensed_linear_fwd_algo(const void* x, srigl_dtype x_dtype, int32_t B, int32_t d_in,
                                             const void* W_c, srigl_dtype w_dtype, const int32_t* idx,
                                             const int32_t* active, int32_t n_active, int32_t K,
                                             const float* bias, int32_t d_out, float* y,
                                             const uint16_t* seg, srigl_fwd_algo algo,
                                             const srigl_fwd_tuning* tuning, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (B < 0 || d_in < 0 || n_active < 0 || K < 0 || d_out < 0 || K > d_in || n_active > d_out) return SRIGL_ERR_INVALID_ARG;
    if ((x_dtype != SRIGL_F32 && x_dtype != SRIGL_BF16) || (w_dtype != SRIGL_F32 && w_dtype != SRIGL_BF16)) return SRIGL_ERR_INVALID_ARG;
    if (x_dtype != w_dtype) return SRIGL_ERR_UNSUPPORTED;
    if (active == nullptr && n_active != d_out && n_active != 0) return SRIGL_ERR_INVALID_ARG;
    if (B == 0 || d_out == 0) return SRIGL_OK;
    if (y == nullptr) return SRIGL_ERR_INVALID_ARG;
    if (n_active > 0 && K > 0 && (x == nullptr || W_c == nullptr || idx == nullptr)) return SRIGL_ERR_INVALID_ARG;

    FwdArgs a;
    a.x = x; a.x_bf16 = (x_dtype == SRIGL_BF16); a.B = B; a.d_in = d_in; a.W_c = W_c; a.idx = idx; a.active = active;
    a.n_active = n_active; a.K = K; a.bias = bias; a.d_out = d_out; a.y = y; a.seg = seg;
    a.seg_stride = srigl_seg_stride(d_in);
    if (n_active == 0 || K == 0) {   // nothing is stored: every column holds its bias
        long long blocks = ((long long)B * d_out + 255) / 256;
        if (blocks > 65536) blocks = 65536;
        hipLaunchKernelGGL(k_bias_broadcast, dim3((unsigned)blocks), dim3(256), 0, st, bias, B, d_out, y);
        return hip_ok(hipGetLastError());
    }
    switch (algo) {
        case SRIGL_FWD_GENERIC: return launch_fwd_generic(a, st);
        case SRIGL_FWD_KLANE: return launch_fwd_klane(a, tuning, st);
        case SRIGL_FWD_ROWLANE: return launch_fwd_rowlane(a, tuning, st);
        case SRIGL_FWD_AUTO: break;
        default: return SRIGL_ERR_INVALID_ARG;
    }
    if (B >= 32 && rowlane_supported(a, nullptr)) return launch_fwd_rowlane(a, nullptr, st);
    srigl_status s = launch_fwd_klane(a, nullptr, st);
    if (s == SRIGL_ERR_UNSUPPORTED) s = launch_fwd_generic(a, st);
    return s;
}

srigl_status srigl_condensed_linear_fwd(const void* x, srigl_dtype x_dtype, int32_t B, int32_t d_in,
                                        const void* W_c, srigl_dtype w_dtype, const int32_t* idx,
                                        const int32_t* active, int32_t n_active, int32_t K,
                                        const float* bias, int32_t d_out, float* y,
                                        const uint16_t* seg, void* stream) {
    return srigl_condensed_linear_fwd_algo(x, x_dtype, B, d_in, W_c, w_dtype, idx, active, n_active, K, bias, d_out, y, seg,
                                           SRIGL_FWD_AUTO, nullptr, stream);
}

}  // extern "C"
