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
// ROWLANE (batched).  Lanes are batch rows: a workgroup owns a tile of BT = 64*R batch rows and a
// group of stored rows, and keeps the activation tile transposed in LDS (xs[column][row], fp32), so
// that for one term (stored row s, k) the gather x[b][idx[s][k]] of all rows of the tile is one
// conflict-free LDS read of BT consecutive words.
//
// Weights and indices reach the lanes without scalar loads: a wavefront reads 16 consecutive terms
// of a stored row with one vector load (lane l holds term l mod 16, the four 16-lane DPP rows hold
// copies) and every multiply-add takes its weight, and every LDS address its index, through the DPP
// row broadcast (row_newbcast:n) of lane n, which costs no instruction of its own.  Vector loads
// count on vmcnt only, so the terms of the next chunk are in flight while this chunk is computed.
//
// d_in is walked in chunks of C columns, double-buffered in LDS: the global loads of chunk c+1 are
// issued into registers before the arithmetic of chunk c and written to the other buffer after it,
// one barrier per chunk.  Within a chunk the terms of an ascending row are the contiguous range the
// seg table gives; lane j of a per-row register holds boundary j, read with v_readlane.
//
// LDS: row stride S = BT + 4 words.  The staging pass moves 16 rows x 16 columns per wavefront
// instruction (global reads of 64 contiguous bytes per row) and the +4 skew spreads its LDS writes
// over all banks, while reads of consecutive rows stay conflict-free and 16-byte aligned.  Column C
// of each buffer is all zeros: terms that pad a block of 16 carry weight 0 and point there, so that a
// non-finite activation in an unrelated column never meets a padded term.
//
// Results leave through LDS as well: the accumulators are transposed into an out[row][stored row]
// tile so that a wavefront stores runs of consecutive columns of one output row.
// ------------------------------------------------------------------------------------------------
template <int R> struct RowVec;
template <> struct RowVec<1> { using type = float; };
template <> struct RowVec<2> { using type = float2; };
template <> struct RowVec<4> { using type = float4; };

constexpr int kStageUnits = 4;   // 16x16 staging units a wavefront holds in registers per chunk
constexpr int kBlock = 16;       // terms per vector load of W_c / idx (one DPP row)
constexpr int kPre = 2;          // blocks per (stored row, chunk) requested one chunk ahead

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

// lane n of each 16-lane row, seen by every lane of that row (folds into the consuming VALU instruction)
template <int N>
__device__ __forceinline__ int row_bcast(int v) {
    return __builtin_amdgcn_update_dpp(0, v, 0x150 + N, 0xf, 0xf, true);
}

// acc += w[lane n of this row] * x.  The leading s_nop covers the two wait states a DPP read needs after
// a VALU write of `w`; the terms of a block run in order n = 0, 1, ... (they chain through acc).
template <int N>
__device__ __forceinline__ void fmac_row_bcast(float& acc, float w, float x) {
    if constexpr (N == 0)
        asm("s_nop 1\n\tv_fmac_f32_dpp %0, %1, %2 row_newbcast:0 row_mask:0xf bank_mask:0xf bound_ctrl:1" : "+v"(acc) : "v"(w), "v"(x));
    else
        asm("v_fmac_f32_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf bound_ctrl:1" : "+v"(acc) : "v"(w), "v"(x), "n"(N));
}

// one term: every lane adds w[n] * x[its rows][idx[n]]
template <int R, int N>
__device__ __forceinline__ void term(float (&acc)[R], float wv, int ov, const char* __restrict__ xb) {
    using V = typename RowVec<R>::type;
    const V xv = *reinterpret_cast<const V*>(xb + row_bcast<N>(ov));
    if constexpr (R == 1) {
        fmac_row_bcast<N>(acc[0], wv, xv);
    } else if constexpr (R == 2) {
        fmac_row_bcast<N>(acc[0], wv, xv.x);
        fmac_row_bcast<N>(acc[1], wv, xv.y);
    } else {
        fmac_row_bcast<N>(acc[0], wv, xv.x);
        fmac_row_bcast<N>(acc[1], wv, xv.y);
        fmac_row_bcast<N>(acc[2], wv, xv.z);
        fmac_row_bcast<N>(acc[3], wv, xv.w);
    }
}

// n_valid (wave-uniform, 1..16) terms of one block; groups of 8 are skipped when empty
template <int R>
__device__ __forceinline__ void block_terms(float (&acc)[R], float wv, int ov, const char* __restrict__ xb, int n_valid) {
    term<R, 0>(acc, wv, ov, xb); term<R, 1>(acc, wv, ov, xb); term<R, 2>(acc, wv, ov, xb); term<R, 3>(acc, wv, ov, xb);
    term<R, 4>(acc, wv, ov, xb); term<R, 5>(acc, wv, ov, xb); term<R, 6>(acc, wv, ov, xb); term<R, 7>(acc, wv, ov, xb);
    if (n_valid > 8) {
        term<R, 8>(acc, wv, ov, xb); term<R, 9>(acc, wv, ov, xb); term<R, 10>(acc, wv, ov, xb); term<R, 11>(acc, wv, ov, xb);
        term<R, 12>(acc, wv, ov, xb); term<R, 13>(acc, wv, ov, xb); term<R, 14>(acc, wv, ov, xb); term<R, 15>(acc, wv, ov, xb);
    }
}

// 16 consecutive terms of stored row data starting at term index t0 (wave-uniform), n_valid of them real
// (wave-uniform, may be <= 0): lane l holds term l mod 16.  Padding terms get weight 0 and the offset
// of the all-zero column.  Loads are unconditional; the term index is clamped into the arrays.
template <typename XT>
__device__ __forceinline__ void load_terms(const XT* __restrict__ W_c, const int32_t* __restrict__ idx, int t0, int n_valid,
                                           int l16, int t_last, int off_mul, int off_add, int zero_off, float& wv, int& ov) {
    const int t = min(t0 + l16, t_last);
    const float w = to_f32<XT>(W_c[t]);
    const int o = idx[t] * off_mul + off_add;
    const bool real = l16 < n_valid;
    wv = real ? w : 0.0f;
    ov = real ? o : zero_off;
}

template <int R, int NPW, typename XT, bool FAST>
__global__ __launch_bounds__(1024) void k_fwd_rowlane(const XT* __restrict__ x, int B, int d_in, const XT* __restrict__ W_c,
                                                      const int32_t* __restrict__ idx, const int32_t* __restrict__ active,
                                                      int n_active, int K, const float* __restrict__ bias, int d_out,
                                                      float* __restrict__ y, const uint16_t* __restrict__ seg, int seg_stride,
                                                      int C, int n_chunks, int n_btiles, int n_groups) {
    extern __shared__ float lds[];   // x tiles: [1 or 2][C + 1][S]; afterwards out tile [BT][NG + 1]
    constexpr int BT = kWave * R;
    constexpr int S = BT + 4;
    constexpr int S4 = S * 4;

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
    const int l16 = lane & (kBlock - 1);
    const int wv_id = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nw = blockDim.x >> 6;
    const int NG = nw * NPW;                 // stored rows (slots) per workgroup
    const int b0 = bt * BT;
    const int n_slots = active ? n_active + 1 : n_active;
    const int sg0 = g * NG;                  // first slot of the workgroup
    const int s0 = sg0 + wv_id * NPW;        // first slot of this wavefront
    const int buf_words = (C + 1) * S;
    const int zero_off = C * S4;             // byte offset of the all-zero column inside a buffer
    const int segs_per_chunk = C / kSegCols;
    const int t_last = n_active * K - 1;     // the host guarantees n_active * K < 2^31

    // ---- chunk boundaries: lane j of bnd[i] holds the first term of chunk cb + j for slot s0 + i ----
    int bnd[NPW];
    int cb = 0;
#define SRIGL_LOAD_BOUNDS()                                                                                     \
    _Pragma("unroll") for (int i = 0; i < NPW; ++i) {                                                           \
        const int s = min(s0 + i, n_active - 1);                                                                \
        const int j = min(cb + lane, n_chunks);                                                                 \
        int v = (j == 0) ? 0 : K;                                                                               \
        if (seg) v = seg[s * seg_stride + min(j * segs_per_chunk, seg_stride - 1)];                             \
        bnd[i] = v;                                                                                             \
    }
    SRIGL_LOAD_BOUNDS()

    // ---- staging: 16 rows x 16 columns per unit; unit u = wv_id + i * nw -> (row tile, column tile) ----
    const int dq = lane & 3, db = lane >> 2;             // 4 column quads x 16 rows per wavefront pass
    const int col_tiles = C >> 4;                         // C is a multiple of 64
    const int units = (BT / 16) * col_tiles;              // <= kStageUnits * nw (checked by the host)
    int g_off[kStageUnits];                               // element offset into x of this lane's 4 columns (chunk 0)
    int l_off[kStageUnits];                               // word offset into an LDS buffer
    int u_col[kStageUnits];                               // first column of the unit (wave-uniform)
#pragma unroll
    for (int i = 0; i < kStageUnits; ++i) {
        const int u = wv_id + i * nw;
        const int rt = u / col_tiles, ct = u - rt * col_tiles;
        const int rl = rt * 16 + db;
        const int f = ct * 16 + dq * 4;
        // rows past B re-read row B - 1: their lanes compute values that are never stored
        g_off[i] = min(b0 + rl, B - 1) * d_in + f;       // the host guarantees B * d_in < 2^31
        l_off[i] = f * S + rl;
        u_col[i] = (u < units) ? ct * 16 : 0x40000000;   // units past the tile never pass the column test below
    }
    float st[kStageUnits][4];
#define SRIGL_STAGE_LOAD(c)                                                                                     \
    _Pragma("unroll") for (int i = 0; i < kStageUnits; ++i) {                                                   \
        const int c0_ = (c) * C;                                                                                \
        if (FAST) {                                                                                             \
            if (c0_ + u_col[i] < d_in) load4<XT>(x + c0_ + g_off[i], true, 4, st[i]);                           \
        } else {                                                                                                \
            st[i][0] = st[i][1] = st[i][2] = st[i][3] = 0.0f;                                                   \
            const int nv = min(4, d_in - (c0_ + u_col[i] + dq * 4));                                            \
            if (u_col[i] < C && nv > 0) load4<XT>(x + c0_ + g_off[i], false, nv, st[i]);                        \
        }                                                                                                       \
    }
#define SRIGL_STAGE_STORE(buf)                                                                                  \
    _Pragma("unroll") for (int i = 0; i < kStageUnits; ++i) {                                                   \
        if (u_col[i] < C) {                                                                                     \
            float* d_ = (buf) + l_off[i];                                                                       \
            d_[0] = st[i][0]; d_[S] = st[i][1]; d_[2 * S] = st[i][2]; d_[3 * S] = st[i][3];                     \
        }                                                                                                       \
    }

    // ---- terms of the next chunk: first kPre blocks of every slot, requested one chunk ahead ----
    float pw[NPW][kPre];
    int po[NPW][kPre];
#define SRIGL_PRELOAD(c)                                                                                        \
    _Pragma("unroll") for (int i = 0; i < NPW; ++i) {                                                           \
        const int k0_ = __builtin_amdgcn_readlane(bnd[i], (c) - cb);                                            \
        const int k1_ = __builtin_amdgcn_readlane(bnd[i], (c) - cb + 1);                                        \
        const int n_ = (s0 + i < n_active) ? k1_ - k0_ : 0;                                                     \
        _Pragma("unroll") for (int p = 0; p < kPre; ++p)                                                        \
            load_terms<XT>(W_c, idx, (s0 + i) * K + k0_ + p * kBlock, n_ - p * kBlock, l16, t_last, S4,         \
                           -(c) * C * S4, zero_off, pw[i][p], po[i][p]);                                        \
    }

    float acc[NPW][R];
#pragma unroll
    for (int i = 0; i < NPW; ++i)
#pragma unroll
        for (int r = 0; r < R; ++r) acc[i][r] = 0.0f;

    SRIGL_STAGE_LOAD(0)
    SRIGL_PRELOAD(0)
    for (int t = tid; t < S; t += blockDim.x) {           // the all-zero column of both buffers
        lds[C * S + t] = 0.0f;
        if (n_chunks > 1) lds[buf_words + C * S + t] = 0.0f;
    }
    SRIGL_STAGE_STORE(lds)
    __syncthreads();

    for (int c = 0; c < n_chunks; ++c) {
        const char* xb = reinterpret_cast<const char*>(lds + (c & 1) * buf_words) + lane * (R * 4);
        // this chunk's first blocks move to working registers; the next chunk's loads go in flight
        float cw_[NPW][kPre];
        int co_[NPW][kPre];
        int k0s[NPW], k1s[NPW];
#pragma unroll
        for (int i = 0; i < NPW; ++i) {
#pragma unroll
            for (int p = 0; p < kPre; ++p) { cw_[i][p] = pw[i][p]; co_[i][p] = po[i][p]; }
            k0s[i] = __builtin_amdgcn_readlane(bnd[i], c - cb);
            k1s[i] = __builtin_amdgcn_readlane(bnd[i], c - cb + 1);
        }
        if (c + 1 < n_chunks) {
            SRIGL_STAGE_LOAD(c + 1)
            if (c + 2 - cb > kWave - 1) { cb = c + 1; SRIGL_LOAD_BOUNDS() }   // keep boundaries c+1, c+2 in the register
            SRIGL_PRELOAD(c + 1)
        }
#pragma unroll
        for (int i = 0; i < NPW; ++i) {
            const int n_terms = (s0 + i < n_active) ? k1s[i] - k0s[i] : 0;
            if (n_terms > 0) {
                block_terms<R>(acc[i], cw_[i][0], co_[i][0], xb, n_terms);
                if (n_terms > kBlock) block_terms<R>(acc[i], cw_[i][1], co_[i][1], xb, n_terms - kBlock);
                if (n_terms > kPre * kBlock) {            // long ranges: the remaining blocks, each requested one block ahead
                    const int row = (s0 + i) * K;
                    float wn;
                    int on;
                    load_terms<XT>(W_c, idx, row + k0s[i] + kPre * kBlock, n_terms - kPre * kBlock, l16, t_last, S4, -c * C * S4,
                                   zero_off, wn, on);
                    for (int kb = kPre * kBlock; kb < n_terms; kb += kBlock) {
                        const float wc = wn;
                        const int oc = on;
                        if (kb + kBlock < n_terms)
                            load_terms<XT>(W_c, idx, row + k0s[i] + kb + kBlock, n_terms - kb - kBlock, l16, t_last, S4, -c * C * S4,
                                           zero_off, wn, on);
                        block_terms<R>(acc[i], wc, oc, xb, n_terms - kb);
                    }
                }
            }
        }
        if (c + 1 < n_chunks) {
            SRIGL_STAGE_STORE(lds + ((c + 1) & 1) * buf_words)
            __syncthreads();
        }
    }
#undef SRIGL_LOAD_BOUNDS
#undef SRIGL_STAGE_LOAD
#undef SRIGL_STAGE_STORE
#undef SRIGL_PRELOAD

    // ---- results: transpose through LDS, then bias + scatter with row-contiguous stores ----
    __syncthreads();                                       // every wavefront is done reading the x tiles
    const int OS = NG + 1;                                 // odd stride: conflict-free transposed writes
#pragma unroll
    for (int i = 0; i < NPW; ++i)
#pragma unroll
        for (int r = 0; r < R; ++r) lds[(lane * R + r) * OS + wv_id * NPW + i] = acc[i][r];
    __syncthreads();

    // lane <-> slot of the workgroup (two slots per lane cover NG <= 128)
    int colv[2], prevv[2];
    float biasv[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int i = lane + h * kWave;
        const int s = sg0 + i;
        colv[h] = -1;
        prevv[h] = 0;
        biasv[h] = 0.0f;
        if (i < NG && s < n_slots) {
            int col = s, prev = s - 1;
            if (active) {
                col = min((s < n_active) ? active[s] : d_out, d_out);
                prev = (s > 0) ? active[s - 1] : -1;
            }
            prevv[h] = max(prev + 1, 0);                   // first column of the gap in front of this slot
            colv[h] = col;
            if (s < n_active && col >= 0 && col < d_out) biasv[h] = bias_at(bias, col);
        }
    }
    const int n_rows = min(BT, B - b0);
    for (int row = wv_id; row < n_rows; row += nw) {
        float* yr = y + (size_t)(b0 + row) * d_out;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int i = lane + h * kWave;
            const int col = colv[h];
            if (col < 0) continue;
            if (active)
                for (int cc = prevv[h]; cc < col; ++cc) yr[cc] = bias_at(bias, cc);
            if (sg0 + i < n_active && col < d_out) yr[col] = lds[row * OS + i] + biasv[h];
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
    // the kernel indexes x, W_c / idx and seg with 32-bit offsets
    if ((long long)a.B * a.d_in >= (1LL << 31) || (long long)a.n_active * a.K >= (1LL << 31) ||
        (long long)a.n_active * a.seg_stride >= (1LL << 31)) return p;
    const int n_slots = a.active ? a.n_active + 1 : a.n_active;
    p.R = t && t->rows_per_lane ? t->rows_per_lane : 1;
    if (p.R != 1 && p.R != 2 && p.R != 4) return p;
    const int BT = kWave * p.R, S = BT + 4;
    p.n_btiles = (a.B + BT - 1) / BT;
    p.NW = t && t->waves ? t->waves : 16;
    if (p.NW < 1 || p.NW > 16) return p;
    // chunk: a multiple of 64 columns such that (a) two buffers fit the LDS budget (one if the whole
    // of d_in fits a single chunk) and (b) a wavefront holds a chunk's staging units in registers
    const size_t budget = 144 * 1024;
    const int d_pad = (a.d_in + kSegCols - 1) / kSegCols * kSegCols;
    const int c_regs = kStageUnits * p.NW * 256 / BT / kSegCols * kSegCols;          // (BT/16)*(C/16) <= units limit
    const int c_one = (int)(budget / (S * sizeof(float)) - 1) / kSegCols * kSegCols;        // +1: the all-zero column
    const int c_two = (int)(budget / (2 * S * sizeof(float)) - 1) / kSegCols * kSegCols;
    int C = t && t->chunk_cols ? t->chunk_cols : 0;
    if (C == 0) C = (d_pad <= c_one && d_pad <= c_regs) ? d_pad : (c_two < c_regs ? c_two : c_regs);
    if (C > d_pad) C = d_pad;
    if (C <= 0 || C % kSegCols != 0 || C > c_regs) return p;
    p.C = C;
    p.n_chunks = (a.d_in + C - 1) / C;
    if (p.n_chunks < 1) p.n_chunks = 1;
    if (C > (p.n_chunks > 1 ? c_two : c_one)) return p;
    if (p.n_chunks > 1 && a.seg == nullptr) return p;   // chunk walking needs ascending rows + seg
    p.lds = (size_t)(p.n_chunks > 1 ? 2 : 1) * (C + 1) * S * sizeof(float);
    // neurons per wavefront: aim at one workgroup per CU over the whole launch
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
    const size_t out_tile = (size_t)BT * (p.NW * npw + 1) * sizeof(float);   // the result tile reuses the LDS
    if (out_tile > p.lds) p.lds = out_tile;
    if (p.lds > kLdsMax) return p;
    p.ok = true;
    return p;
}

bool rowlane_supported(const FwdArgs& a, const srigl_fwd_tuning* t) { return plan_rowlane(a, t).ok; }

template <int R, int NPW, typename XT, bool FAST>
static srigl_status launch_rowlane_f(const FwdArgs& a, const RowlanePlan& p, hipStream_t st) {
    auto kern = k_fwd_rowlane<R, NPW, XT, FAST>;
    static size_t lds_allowed = 64 * 1024;   // raised once per kernel instance, not per call
    if (p.lds > lds_allowed) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsMax) != hipSuccess)
            return SRIGL_ERR_HIP;
        lds_allowed = kLdsMax;
    }
    const long long blocks = 8LL * ((p.n_groups + 7) / 8) * p.n_btiles;
    if (blocks > 0x7fffffffLL) return SRIGL_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(p.NW * kWave), p.lds, st, (const XT*)a.x, a.B, a.d_in, (const XT*)a.W_c,
                       a.idx, a.active, a.n_active, a.K, a.bias, a.d_out, a.y, a.seg, a.seg_stride, p.C, p.n_chunks, p.n_btiles,
                       p.n_groups);
    return hip_ok(hipGetLastError());
}

template <int R, int NPW, typename XT>
static srigl_status launch_rowlane_t(const FwdArgs& a, const RowlanePlan& p, hipStream_t st) {
    // fast staging: whole 16-column units, rows aligned for 4-element vector loads
    const size_t xal = sizeof(XT) * 4;
    const bool fast = (a.d_in % 16 == 0) && ((reinterpret_cast<uintptr_t>(a.x) % xal) == 0);
    return fast ? launch_rowlane_f<R, NPW, XT, true>(a, p, st) : launch_rowlane_f<R, NPW, XT, false>(a, p, st);
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
