// ROWLANE forward kernel and its launchers, included once per element type (one translation unit each,
// so that the instantiations compile in parallel).
#pragma once
#include <type_traits>

#include "srigl_internal.h"

namespace srigl {

template <typename XT> __device__ __forceinline__ float rl_to_f32(XT v);
template <> __device__ __forceinline__ float rl_to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float rl_to_f32<uint16_t>(uint16_t v) { return bf16_bits_to_float(v); }
// the value lane `byte_addr / 4` holds (every lane names its own source lane)
__device__ __forceinline__ float lane_fetch(float v, int byte_addr) { return __int_as_float(__builtin_amdgcn_ds_bpermute(byte_addr, __float_as_int(v))); }
__device__ __forceinline__ uint16_t lane_fetch(uint16_t v, int byte_addr) { return (uint16_t)__builtin_amdgcn_ds_bpermute(byte_addr, (int)v); }
__device__ __forceinline__ int lane_fetch(int v, int byte_addr) { return __builtin_amdgcn_ds_bpermute(byte_addr, v); }
__device__ __forceinline__ float rl_bias_at(const float* __restrict__ bias, int col) { return bias ? bias[col] : 0.0f; }

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
// count on vmcnt only, so they stay in flight across LDS traffic.
//
// d_in is walked in chunks of C columns (one LDS buffer).  The global loads of chunk c+1 are issued
// into registers before the arithmetic of chunk c, written to LDS after it between two barriers.
// Within a chunk the terms of an ascending row are the contiguous range the seg table gives; lane j
// of a per-row register holds boundary j, read with v_readlane.  The first KPRE blocks of 16 terms
// of the next chunk are requested as soon as the registers of the current chunk's blocks are free.
//
// Terms run in groups of 8: the LDS reads of group g+1 are issued before the multiply-adds of group
// g, so that the LDS latency of one group hides behind the arithmetic of the other.
//
// LDS: row stride S = BT + 4 words (16 with four term slices).  The staging pass moves 16 rows x 16 columns per wavefront
// instruction (global reads of 64 contiguous bytes per row) and the +4 skew spreads its LDS writes
// over all banks, while reads of consecutive rows stay conflict-free and 16-byte aligned.  Column C
// is all zeros: terms that pad a group carry weight 0 and point there, so that a non-finite
// activation in an unrelated column never meets a padded term.
//
// Results leave through LDS as well: the accumulators are transposed into an out[row][stored row]
// tile so that a wavefront stores runs of consecutive columns of one output row.
// ------------------------------------------------------------------------------------------------
template <int R> struct RowVec;
template <> struct RowVec<1> { using type = float; };
template <> struct RowVec<2> { using type = float2; };
template <> struct RowVec<4> { using type = float4; };


// Four consecutive activations of one row as they came from memory.  They are turned into fp32 only when they are
// written to LDS: a conversion right behind the load would make the wavefront wait for the load where it is issued,
// and the loads of the next chunk are issued long before their data is needed.
template <typename XT> struct Staged4;
template <> struct Staged4<float> {
    float v[4];
    __device__ __forceinline__ void clear() { v[0] = v[1] = v[2] = v[3] = 0.0f; }
    __device__ __forceinline__ float get(int k) const { return v[k]; }
};
template <> struct Staged4<uint16_t> {
    uint32_t w[2];   // two bf16 per word, the lower-addressed one in the low half
    __device__ __forceinline__ void clear() { w[0] = w[1] = 0u; }
    __device__ __forceinline__ float get(int k) const {
        return (k & 1) ? __uint_as_float(w[k >> 1] & 0xffff0000u) : __uint_as_float(w[k >> 1] << 16);
    }
};

__device__ __forceinline__ void load4(const float* __restrict__ p, bool vec_ok, int n_valid, Staged4<float>& out) {
    if (vec_ok && n_valid >= 4) {
        const float4 v = *reinterpret_cast<const float4*>(p);
        out.v[0] = v.x; out.v[1] = v.y; out.v[2] = v.z; out.v[3] = v.w;
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) out.v[i] = (i < n_valid) ? p[i] : 0.0f;
    }
}

__device__ __forceinline__ void load4(const uint16_t* __restrict__ p, bool vec_ok, int n_valid, Staged4<uint16_t>& out) {
    if (vec_ok && n_valid >= 4) {
        const uint2 v = *reinterpret_cast<const uint2*>(p);
        out.w[0] = v.x; out.w[1] = v.y;
    } else {
        out.w[0] = out.w[1] = 0u;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (i < n_valid) out.w[i >> 1] |= (uint32_t)p[i] << (16 * (i & 1));
    }
}

// lane n of each 16-lane row, seen by every lane of that row (folds into the consuming VALU instruction)
template <int N>
__device__ __forceinline__ int row_bcast(int v) {
    return __builtin_amdgcn_update_dpp(0, v, 0x150 + N, 0xf, 0xf, true);
}

// (lane n of each 16-lane row) ^ v in one instruction: the LDS address of a term in the swizzled tile
template <int N>
__device__ __forceinline__ int xor_row_bcast(int bcast_src, int v) {
    int r;   // (the s_nop covers the two wait states a DPP read needs after a VALU write of its source, as in fmac_row_bcast)
    if constexpr (N % 4 == 0)
        asm("s_nop 1\n\tv_xor_b32_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf bound_ctrl:1" : "=v"(r) : "v"(bcast_src), "v"(v), "n"(N));
    else
        asm("v_xor_b32_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf bound_ctrl:1" : "=v"(r) : "v"(bcast_src), "v"(v), "n"(N));
    return r;
}

// acc += w[lane n of this row] * x.  The s_nop at the head of every run of 4 covers the two wait states a DPP
// read needs after a VALU write of `w`; the terms of a group run in order (they chain through acc).
template <int N>
__device__ __forceinline__ void fmac_row_bcast(float& acc, float w, float x) {
    if constexpr (N % 4 == 0)
        asm("s_nop 1\n\tv_fmac_f32_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf bound_ctrl:1" : "+v"(acc) : "v"(w), "v"(x), "n"(N));
    else
        asm("v_fmac_f32_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf bound_ctrl:1" : "+v"(acc) : "v"(w), "v"(x), "n"(N));
}

template <int R, int N>
__device__ __forceinline__ void fmac_rows(float (&acc)[R], float wv, const typename RowVec<R>::type& xv) {
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

// Terms run in groups of GS steps: 8 with one row per lane, 4 with more (a row's last group is padded to GS steps, and
// with two rows per lane a step is two multiply-adds: measured 1-2 % faster than groups of 8, 2-5 % in four slices).
template <int R> struct GroupSize { static constexpr int value = (R >= 2) ? 4 : 8; };

// Group Q of a block (terms Q*GS .. Q*GS+GS-1): its LDS reads, and its multiply-adds
// (swizzled tile, R = 4: xb is the tile's base and lanepart the byte offset of the lane's rows, combined by exclusive or)
template <int R, int Q, int J = 0>
__device__ __forceinline__ void group_reads(typename RowVec<R>::type (&xv)[GroupSize<R>::value], int ov, const char* __restrict__ xb,
                                            int lanepart) {
    using V = typename RowVec<R>::type;
    constexpr int GS = GroupSize<R>::value;
    if constexpr (J < GS) {
        if constexpr (rowlane_swizzled(R)) xv[J] = *reinterpret_cast<const V*>(xb + xor_row_bcast<Q * GS + J>(ov, lanepart));
        else xv[J] = *reinterpret_cast<const V*>(xb + row_bcast<Q * GS + J>(ov));
        group_reads<R, Q, J + 1>(xv, ov, xb, lanepart);
    }
}
template <int R, int Q, int J = 0>
__device__ __forceinline__ void group_fmacs(float (&acc)[R], float wv, const typename RowVec<R>::type (&xv)[GroupSize<R>::value]) {
    constexpr int GS = GroupSize<R>::value;
    if constexpr (J < GS) {
        fmac_rows<R, Q * GS + J>(acc, wv, xv[J]);
        group_fmacs<R, Q, J + 1>(acc, wv, xv);
    }
}

// Groups G, G+1, ... of NB blocks held in registers; n = number of real terms (wave-uniform).
// On entry the reads of group G are in flight in `cur`; every path issues the reads of the next group
// before the multiply-adds of this one.
template <int R, int G, int NB>
__device__ __forceinline__ void pipe_groups(float (&acc)[R], const float (&wv)[NB], const int (&ov)[NB], const char* __restrict__ xb,
                                            int lanepart, int n, typename RowVec<R>::type (&cur)[GroupSize<R>::value],
                                            typename RowVec<R>::type (&nxt)[GroupSize<R>::value]) {
    constexpr int GS = GroupSize<R>::value;
    constexpr int GPB = kBlock / GS;   // groups per block
    if constexpr (G + 1 < GPB * NB) {
        if (n > GS * (G + 1)) {
            group_reads<R, (G + 1) % GPB>(nxt, ov[(G + 1) / GPB], xb, lanepart);
            group_fmacs<R, G % GPB>(acc, wv[G / GPB], cur);
            pipe_groups<R, G + 1, NB>(acc, wv, ov, xb, lanepart, n, nxt, cur);
            return;
        }
    }
    group_fmacs<R, G % GPB>(acc, wv[G / GPB], cur);
}

// The same walk with the reads two groups ahead of the multiply-adds (three buffers in rotation): a wavefront's reads then have
// two groups' worth of its own and the other wavefronts' arithmetic to return in, where one group's worth left every
// wavefront of a full compute unit waiting on the LDS queue.  On entry the reads of group G are in flight in `a`, and those
// of group G + 1 in `b` if that group exists.
template <int R, int G, int NB>
__device__ __forceinline__ void pipe_groups2(float (&acc)[R], const float (&wv)[NB], const int (&ov)[NB], const char* __restrict__ xb,
                                             int lanepart, int n, typename RowVec<R>::type (&a)[GroupSize<R>::value],
                                             typename RowVec<R>::type (&b)[GroupSize<R>::value],
                                             typename RowVec<R>::type (&c)[GroupSize<R>::value]) {
    constexpr int GS = GroupSize<R>::value;
    constexpr int GPB = kBlock / GS;
    if constexpr (G + 2 < GPB * NB) {
        if (n > GS * (G + 2)) {
            group_reads<R, (G + 2) % GPB>(c, ov[(G + 2) / GPB], xb, lanepart);
            group_fmacs<R, G % GPB>(acc, wv[G / GPB], a);
            pipe_groups2<R, G + 1, NB>(acc, wv, ov, xb, lanepart, n, b, c, a);
            return;
        }
    }
    group_fmacs<R, G % GPB>(acc, wv[G / GPB], a);
    if constexpr (G + 1 < GPB * NB) {
        if (n > GS * (G + 1)) group_fmacs<R, (G + 1) % GPB>(acc, wv[(G + 1) / GPB], b);
    }
}
// Reads of the first group (and of the second, two ahead), then the walk.  DEPTH = 1 keeps the two-buffer form.
template <int R, int NB, int DEPTH>
__device__ __forceinline__ void walk_groups(float (&acc)[R], const float (&wv)[NB], const int (&ov)[NB], const char* __restrict__ xb,
                                            int lanepart, int n) {
    using V = typename RowVec<R>::type;
    constexpr int GS = GroupSize<R>::value;
    constexpr int GPB = kBlock / GS;
    V a[GS], b[GS];
    group_reads<R, 0>(a, ov[0], xb, lanepart);
    if constexpr (DEPTH == 2 && GPB * NB > 1) {
        V c[GS];
        if (n > GS) group_reads<R, 1 % GPB>(b, ov[1 / GPB], xb, lanepart);
        pipe_groups2<R, 0, NB>(acc, wv, ov, xb, lanepart, n, a, b, c);
    } else {
        pipe_groups<R, 0, NB>(acc, wv, ov, xb, lanepart, n, a, b);
    }
}

// One block of terms of stored-row data starting at term index t0 (wave-uniform): 16 * H consecutive terms, one vector
// load per array.  The lane at position l16 of slice p works on term t0 + tofs, tofs = H * l16 + p (so that a partly
// filled block ends after ceil(n / H) of its 16 steps).  With one slice the lanes load their own terms (16 consecutive
// words, four copies); with 2 or 4 slices that pattern would be a stride of H words across the lanes of a quad, which
// the vector L1 serves as H times the accesses (counters: 5.0 M tag lookups per call on the 3072-wide layer against
// 1.8 M on the 768-wide one), so there lane l loads term t0 + lofs, lofs = l mod 16H (consecutive words), and
// finish_terms() fetches the lane's own term from lane tofs with one cross-lane read per array.  The loads are
// unconditional (the term index is clamped into the arrays) and nothing here consumes their result, so that they stay
// in flight; finish_terms() turns the raw words into a weight and an LDS byte offset when the block is about to be used.
// PKB != 0: the terms come from the streaming copy instead (PKB bytes per term, weight and index side by side): one load per
// block in place of two, t0 then counts terms of the copy's padded rows.
template <typename XT, typename IT, int PKB>
__device__ __forceinline__ void request_terms(const XT* __restrict__ W_c, const IT* __restrict__ idx, const unsigned char* __restrict__ pk,
                                              int t0, int lofs, int t_last, XT& w_raw, int& i_raw) {
    // 32-bit unsigned byte offsets from the (wave-uniform) array bases: one address instruction per load
    const unsigned t = (unsigned)min(t0 + lofs, t_last);
    if constexpr (PKB == 8) {
        const uint2 v = *reinterpret_cast<const uint2*>(pk + t * 8u);
        if constexpr (sizeof(XT) == 4) w_raw = __uint_as_float(v.x); else w_raw = (XT)v.x;
        i_raw = (int)v.y;
    } else if constexpr (PKB == 4) {
        const uint32_t v = *reinterpret_cast<const uint32_t*>(pk + t * 4u);
        w_raw = (XT)(v & 0xffffu);
        i_raw = (int)(v >> 16);
    } else {
        w_raw = *reinterpret_cast<const XT*>(reinterpret_cast<const char*>(W_c) + t * (unsigned)sizeof(XT));
        i_raw = (int)*reinterpret_cast<const IT*>(reinterpret_cast<const char*>(idx) + t * (unsigned)sizeof(IT));
    }
}
// n_valid (wave-uniform, may be <= 0) of the block's terms are real; the others become (weight 0, all-zero column).
// SWZ: the offset also carries the column's swizzle bits (bits 6-7: which 64-byte quarter of the column's first 256 bytes the
// rows 0-15 moved to); off_mul is then a multiple of 256 and off_add moves whole 64-column chunks, which leave those bits alone.
template <typename XT, int H, bool SWZ = false>
__device__ __forceinline__ void finish_terms(XT w_raw, int i_raw, int n_valid, int tofs, int off_mul, int off_add, int zero_off,
                                             float& wv, int& ov, int fetch_ofs = 0) {
    if (H > 1) {   // fetch_ofs: first lane of the block when one load brought two blocks (lanes 0-31 and 32-63)
        w_raw = lane_fetch(w_raw, (tofs + fetch_ofs) * 4);
        i_raw = lane_fetch(i_raw, (tofs + fetch_ofs) * 4);
    }
    const bool real = tofs < n_valid;
    wv = real ? rl_to_f32<XT>(w_raw) : 0.0f;
    ov = real ? i_raw * off_mul + off_add : zero_off;
    if (SWZ) ov = real ? ov | (((i_raw >> 2) & 3) << 6) : ov;
}

// Workgroup barrier that orders LDS accesses only: outstanding vector-memory loads stay in flight across it.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <int R, int H, int NPW, int KPRE, typename XT, bool FAST, typename IT, int PKB = 0, bool SPREAD = false>
__global__ __launch_bounds__(rowlane_max_threads(R)) void k_fwd_rowlane(const XT* __restrict__ x, int B, int d_in, const XT* __restrict__ W_c,
                                                      const IT* __restrict__ idx, const int32_t* __restrict__ active,
                                                      int n_active, int K, const float* __restrict__ bias, int d_out,
                                                      float* __restrict__ y, const uint16_t* __restrict__ seg, int seg_stride,
                                                      int C, int n_chunks, int n_btiles, int n_groups, int out_off, int act, int bt_major,
                                                      const unsigned char* __restrict__ pk, int KS, unsigned div_magic, int spread) {
    extern __shared__ float lds[];   // x tile [C + 1][S]; afterwards out tile [BT][NG + 1]
    constexpr int LR = kWave / H;            // lanes per term slice
    constexpr int BT = LR * R;               // batch rows per tile
    constexpr int S = rowlane_row_stride(BT, H, R);
    constexpr int S4 = S * 4;
    constexpr bool SWZ = rowlane_swizzled(R);
    constexpr int TB = kBlock * H;           // terms per block (16 steps of H terms)
    // Two slices with two preloaded blocks: one 64-lane load brings both blocks (64 consecutive terms, lane l holds term
    // l) instead of two loads of 32 terms twice over; every vector-memory instruction costs the address unit the same
    // 16 clocks whatever it returns, and the loads ahead of the first barrier are what that barrier waits for.
    constexpr bool MERGE = (H == 2 && KPRE == 2);
    // Groups of LDS reads in flight ahead of the multiply-adds: two for 128-row tiles in one slice (measured 5 % faster on the
    // 4096 -> 16384 bf16 layer at B = 2048, 1 % on 768 -> 3072 at B = 1024), one elsewhere (two measured equal on the 64-row
    // two-slice tile and 3 % slower on 16-row tiles; with 16-byte reads a third buffer does not fit the registers)
    constexpr int kReadAhead = (R == 2 && H == 1) ? 2 : 1;
    using V = typename RowVec<R>::type;

    // XCD-aware decode: consecutive workgroup ids go to different XCDs (8 of them), so the id modulo 8 selects the XCD.
    // Either all batch tiles of one group of stored rows are given to the same XCD, whose L2 then holds that group's
    // W_c / idx once while every XCD fetches all of x; or (bt_major) all groups of one batch tile, so that an XCD fetches
    // only its own rows of x and every XCD all of W_c / idx.  The host picks the order that fetches fewer bytes.
    const int wg = blockIdx.x;
    const int xcd = wg & 7, inx = wg >> 3;
    // (the quotient by the host's multiplier, ceil(2^32 / divisor), exact for this launch's ids; 0: plain division)
    const int dec_d = bt_major ? n_groups : n_btiles;
    const int dec_q = dec_d == 1 ? inx : (div_magic ? (int)__umulhi((unsigned)inx, div_magic) : inx / dec_d);
    const int dec_r = inx - dec_q * dec_d;
    int bt, g;
    if (bt_major) {
        g = dec_r;
        bt = dec_q * 8 + xcd;
        if (bt >= n_btiles) return;
    } else {
        bt = dec_r;
        g = dec_q * 8 + xcd;
        if (g >= n_groups) return;
    }

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int rowl = lane & (LR - 1);        // this lane's first row inside the tile is rowl * R
    const int tofs = H * (lane & (kBlock - 1)) + lane / LR;   // this lane's term inside a block
    const int lofs = H == 1 ? tofs : (lane & (kBlock * H - 1));   // the term this lane loads
    const int wv_id = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nw = blockDim.x >> 6;
    const int NG = nw * NPW;                 // stored rows (slots) per workgroup
    const int b0 = bt * BT;
    const int n_slots = active ? n_active + 1 : n_active;
    const int sg0 = g * NG;                  // first slot of the workgroup
    const int s0 = sg0 + wv_id * NPW;        // first slot of this wavefront
    const int zero_off = C * S4;             // byte offset of the all-zero column
    const int segs_per_chunk = C / kSegCols;
    // KS: terms between the starts of consecutive stored rows in the arrays the terms are read from (K, or the padded row of
    // the streaming copy)
    const int t_last = n_active * KS - 1;    // the host guarantees n_active * KS < 2^31 (times the bytes of a term: < 2^32)

    // ---- which stored rows this wavefront takes: NPW consecutive ones, or (spread) every nw-th of the workgroup's rows in
    // the order of their median input column.  Every chunk ends in a barrier, so a chunk costs what its busiest wavefront
    // costs; rows whose columns cluster around the same place are heavy in the same chunks, and dealing them out one
    // to a wavefront evens the chunks out.  Any assignment gives the same sums: a row's terms are still added in order. ----
    // (with six or eight rows per wavefront every use reads the row through an empty asm statement, which keeps the compiler
    // from deriving each row's offsets once for the whole kernel: those live scalar registers spill, and their spill lanes
    // then push vector registers out to scratch; 2-5 % on the shapes that take six or eight rows)
    int slot[NPW];
#pragma unroll
    for (int i = 0; i < NPW; ++i) slot[i] = s0 + i;
    auto slot_of = [&](int i) -> int {
        if constexpr (SPREAD) {
            int v = slot[i];
            if constexpr (NPW >= 6) asm volatile("" : "+s"(v));
            return v;
        } else if constexpr (NPW >= 6) {
            int v = s0;
            asm volatile("" : "+s"(v));
            return v + i;
        } else {
            return s0 + i;
        }
    };
    // ---- chunk boundaries: lane j of bnd[i] holds the first term of chunk cb + j for the i-th row ----
    int bnd[NPW];
    int cb = 0;
#define SRIGL_LOAD_BOUNDS()                                                                                     \
    _Pragma("unroll") for (int i = 0; i < NPW; ++i) {                                                           \
        const int s = min(slot_of(i), n_active - 1);                                                            \
        const int j = min(cb + lane, n_chunks);                                                                 \
        int v = (j == 0) ? 0 : K;                                                                               \
        if (seg) v = seg[(unsigned)(s * seg_stride + min(j * segs_per_chunk, seg_stride - 1))];                 \
        bnd[i] = v;                                                                                             \
    }

    // ---- staging: 16 rows x 16 columns per unit; unit u = wv_id + i * nw -> row tile u % (BT / 16), column tile u / (BT / 16)
    // (BT / 16 is a power of two: the units a wavefront takes walk along its rows, and the split costs a shift) ----
    const int dq = lane & 3, db = lane >> 2;             // 4 column quads x 16 rows per wavefront pass
    const int col_tiles = C >> 4;                         // C is a multiple of 64
    constexpr int RT = BT / 16, RT_LOG2 = RT == 1 ? 0 : (RT == 2 ? 1 : (RT == 4 ? 2 : 3));
    static_assert(RT == 1 || RT == 2 || RT == 4 || RT == 8, "batch tile of 16 .. 128 rows");
    // this lane's bytes are addressed from the tile's first row (a wave-uniform base) with 32-bit offsets: BT rows of x
    const char* const xtile = reinterpret_cast<const char*>(x + (size_t)b0 * d_in);
    unsigned g_off[kStageUnits];                          // byte offset from xtile of this lane's 4 columns (chunk 0)
    int l_off[kStageUnits];                               // word offset into the LDS tile
    int u_col[kStageUnits];                               // first column of the unit (wave-uniform)
#pragma unroll
    for (int i = 0; i < kStageUnits; ++i) {
        const int u = wv_id + i * nw;
        const int rt = u & (RT - 1), ct = u >> RT_LOG2;
        const int rl = rt * 16 + db;
        const int f = ct * 16 + dq * 4;
        // rows past B re-read row B - 1: their lanes compute values that are never stored
        g_off[i] = (unsigned)(min(rl, B - 1 - b0) * d_in + f) * (unsigned)sizeof(XT);   // BT * d_in * 4 < 2^32 (host)
        l_off[i] = f * S + (SWZ ? (rl ^ (((f >> 2) & 3) << 4)) : rl);   // (f .. f + 3 share one swizzle: f is a multiple of 4)
        u_col[i] = (ct < col_tiles) ? ct * 16 : 0x40000000;   // units past the tile never pass the column tests below
    }
    Staged4<XT> st[kStageUnits];
    // live: the chunk exists.  With six or eight stored rows per wavefront (UNC) the aligned form loads unconditionally: a
    // unit past the tile, past d_in, or of a chunk that does not exist reads the tile's first 16 bytes instead and is never
    // used, and the terms behind a row's last chunk are read (clamped into the arrays) and never used.  With loads under
    // branches the compiler waits for every vector-memory operation in flight wherever it needs one of them: a stored row's
    // terms, requested a chunk earlier, then also wait for the next chunk's activations requested a moment ago, six or eight
    // times per chunk.  Measured (cold / cached): 4096->16384 bf16 at batch 2048 887 -> 806 us, 4096->4096 K = 41 at 1024
    // 104 / 88 -> 85 / 74, K = 205 139 / 119 -> 120 / 110; with four rows per wavefront or fewer the spare loads cost more than
    // the counted waits save (3072->768 at batch 64 11.9 -> 12.8), so those shapes keep the branches.
    constexpr bool UNC = NPW >= 6;
#define SRIGL_STAGE_LOAD_UNITS(live, c, u_first, u_last)                                                        \
    _Pragma("unroll") for (int u_ = 0; u_ < kStageUnits; ++u_) {                                                \
        const int c0_ = (c) * C;                                                                                \
        if (u_ >= (u_first) && u_ < (u_last)) {                                                                 \
            if (FAST) {                                                                                         \
                const bool in_ = (live) && c0_ + u_col[u_] < d_in;                                              \
                if (UNC) load4(reinterpret_cast<const XT*>(xtile + (in_ ? g_off[u_] + (unsigned)c0_ * (unsigned)sizeof(XT) : 0u)), true, 4, st[u_]); \
                else if (in_) load4(reinterpret_cast<const XT*>(xtile + (g_off[u_] + (unsigned)c0_ * (unsigned)sizeof(XT))), true, 4, st[u_]); \
            } else if (live) {                                                                                            \
                st[u_].clear();                                                                                 \
                const int nv = min(4, d_in - (c0_ + u_col[u_] + dq * 4));                                       \
                if (u_col[u_] < C && nv > 0) load4(reinterpret_cast<const XT*>(xtile + (g_off[u_] + (unsigned)c0_ * (unsigned)sizeof(XT))), false, nv, st[u_]); \
            }                                                                                                   \
        }                                                                                                       \
    }
#define SRIGL_STAGE_LOAD(c) SRIGL_STAGE_LOAD_UNITS(true, c, 0, kStageUnits)
#define SRIGL_STAGE_STORE()                                                                                     \
    _Pragma("unroll") for (int i = 0; i < kStageUnits; ++i) {                                                   \
        if (u_col[i] < C) {                                                                                     \
            float* d_ = lds + l_off[i];                                                                         \
            if (H == 4 && R == 1) {   /* stride 16: odd column quads write their pairs in the other order (banks 16 apart) */ \
                const bool odd_ = (dq & 1) != 0;                                                                \
                float* p_ = d_ + (odd_ ? S : 0);                                                                \
                float* q_ = d_ + (odd_ ? 0 : S);                                                                \
                const float e0_ = st[i].get(0), e1_ = st[i].get(1), e2_ = st[i].get(2), e3_ = st[i].get(3);     \
                p_[0] = odd_ ? e1_ : e0_;                                                                       \
                q_[0] = odd_ ? e0_ : e1_;                                                                       \
                p_[2 * S] = odd_ ? e3_ : e2_;                                                                   \
                q_[2 * S] = odd_ ? e2_ : e3_;                                                                   \
            } else {                                                                                            \
                d_[0] = st[i].get(0); d_[S] = st[i].get(1); d_[2 * S] = st[i].get(2); d_[3 * S] = st[i].get(3); \
            }                                                                                                   \
        }                                                                                                       \
    }

    // ---- terms: the first KPRE blocks of every slot for one chunk live in registers ----
    XT rw[NPW][KPRE];    // raw words as loaded; finished into (weight, offset) right before use
    int ri[NPW][KPRE];
#define SRIGL_PRELOAD(live, i, c)                                                                               \
    {                                                                                                           \
        const int k0_ = __builtin_amdgcn_readlane(bnd[i], (c) - cb);                                            \
        if (UNC || (live)) {                                                                                    \
            _Pragma("unroll") for (int p = 0; p < (MERGE ? 1 : KPRE); ++p)                                      \
                request_terms<XT, IT, PKB>(W_c, idx, pk, slot_of(i) * KS + k0_ + p * TB, MERGE ? lane : lofs, t_last, rw[i][p], ri[i][p]); \
        }                                                                                                       \
    }

    float acc[NPW][R];
#pragma unroll
    for (int i = 0; i < NPW; ++i)
#pragma unroll
        for (int r = 0; r < R; ++r) acc[i][r] = 0.0f;

    // The activations of chunk 0 go out first: vector loads return in order, and the barrier in front of the first term
    // waits for these only, while the term blocks and the boundaries requested behind them are still in flight.
    // Chunk 0 starts at term 0 of every row, so its blocks are requested before the boundaries are known.
    SRIGL_STAGE_LOAD(0)
    // The keys are read behind the tile's requests, with wave-uniform addresses (scalar loads: they leave the vector-memory
    // counter alone, which the compiler waits to zero once loads sit behind branches, as the tile's do): a wavefront reads
    // those of its NPW consecutive rows, lane i keeps the i-th, and the ranking runs while the tile is on its way.
    if constexpr (SPREAD) {
        int spread_key = 0x7fffffff;                           // rows past the last stored one sort last
        int w_lo = 0x7fffffff, w_hi = -1;                      // smallest and largest key of this wavefront's rows
        const uint32_t* const idx_words = reinterpret_cast<const uint32_t*>(idx);   // (4-byte aligned: the host checks)
#pragma unroll
        for (int i = 0; i < NPW; ++i) {
            if (s0 + i < n_active) {
                const unsigned e = (unsigned)(s0 + i) * (unsigned)K + (unsigned)(K >> 1);   // n_active * K < 2^31 (host)
                int k;
                if constexpr (sizeof(IT) == 4) k = (int)idx_words[e];
                else k = (int)((idx_words[e >> 1] >> ((e & 1u) * 16u)) & 0xffffu);
                if (lane == i) spread_key = k;
                w_lo = min(w_lo, k);
                w_hi = max(w_hi, k);
            }
        }
        // (barriers that wait for this wavefront's LDS traffic only: a __syncthreads would also wait for the tile's loads,
        // and the terms could then be requested only after the tile has arrived)
        // NG <= 128 keys; the NG x NG comparisons of the ranking are split over all threads (part p of the workgroup's
        // 128-thread parts takes every n_parts-th row to compare with)
        int* const keys = reinterpret_cast<int*>(lds);
        int* const ranks = keys + 128;
        int* const place_row = keys + 256;                     // row of the workgroup per place (wavefront, its i-th row)
        int* const wave_lo = keys + 384;
        int* const wave_hi = keys + 400;
        const int t = tid & 127, part = tid >> 7, n_parts = max((int)blockDim.x >> 7, 1);
        if (lane < NPW) keys[wv_id * NPW + lane] = spread_key;
        if (tid < 128) ranks[tid] = 0;
        if (lane == 0) { wave_lo[wv_id] = w_lo; wave_hi[wv_id] = w_hi; }
        if (tid >= nw && tid < 16) { wave_lo[tid] = 0x7fffffff; wave_hi[tid] = -1; }   // (all 16 entries are read below)
        lds_barrier();
        // spread >= 2: only where the medians of this workgroup's rows lie more than spread - 2 columns apart (rows drawn
        // evenly from all columns have their medians close together, and nothing to gain); every wavefront takes the
        // same decision from the same numbers
        bool deal = true;
        if (spread >= 2) {
            int lo = 0x7fffffff, hi = -1;
#pragma unroll
            for (int w = 0; w < 16; w += 4) {                  // four 16-byte reads per array, all in flight together
                const int4 l4 = *reinterpret_cast<const int4*>(wave_lo + w);
                const int4 h4 = *reinterpret_cast<const int4*>(wave_hi + w);
                lo = min(min(lo, min(l4.x, l4.y)), min(l4.z, l4.w));
                hi = max(max(hi, max(h4.x, h4.y)), max(h4.z, h4.w));
            }
            deal = hi >= 0 && hi - lo > spread - 2;
        }
        if (deal) {
            if (t < NG && part < n_parts) {
                const int mine = keys[t];
                int below = 0;
#pragma unroll 8
                for (int u = part; u < NG; u += n_parts) {
                    const int ku = keys[u];
                    below += (ku < mine || (ku == mine && u < t)) ? 1 : 0;
                }
                atomicAdd(&ranks[t], below);
            }
            lds_barrier();
            if (tid < NG) {
                const int rank = ranks[tid];                   // -> wavefront rank % nw, its (rank / nw)-th row
                place_row[(rank % nw) * NPW + rank / nw] = tid;
            }
            lds_barrier();
#pragma unroll
            for (int i = 0; i < NPW; ++i) slot[i] = sg0 + __builtin_amdgcn_readfirstlane(place_row[wv_id * NPW + i]);
        }
        lds_barrier();                                         // the tile is written over this space next
    }
#pragma unroll
    for (int i = 0; i < NPW; ++i)
#pragma unroll
        for (int p = 0; p < (MERGE ? 1 : KPRE); ++p)
            request_terms<XT, IT, PKB>(W_c, idx, pk, slot_of(i) * KS + p * TB, MERGE ? lane : lofs, t_last, rw[i][p], ri[i][p]);
    SRIGL_LOAD_BOUNDS()
    for (int t = tid; t < S; t += blockDim.x) lds[C * S + t] = 0.0f;   // the all-zero column
    SRIGL_STAGE_STORE()
    __syncthreads();

    const int lanepart = rowl * (R * 4);
    const char* xb = reinterpret_cast<const char*>(lds) + (SWZ ? 0 : lanepart);
    for (int c = 0; c < n_chunks; ++c) {
        const bool more = (c + 1 < n_chunks);
        int k0n[NPW], nn[NPW];
#pragma unroll
        for (int i = 0; i < NPW; ++i) {
            k0n[i] = __builtin_amdgcn_readlane(bnd[i], c - cb);
            nn[i] = (slot_of(i) < n_active) ? __builtin_amdgcn_readlane(bnd[i], c - cb + 1) - k0n[i] : 0;
        }
        if (more && c + 2 - cb > kWave - 1) { cb = c + 1; SRIGL_LOAD_BOUNDS() }   // boundaries c+1, c+2 stay in the register
#pragma unroll
        for (int i = 0; i < NPW; ++i) {
            // the next chunk's activations: a share of the staging loads goes out before each stored row's arithmetic,
            // so that the vector-memory queue never takes the whole burst at once
            SRIGL_STAGE_LOAD_UNITS(more, c + 1, (i * kStageUnits) / NPW, ((i + 1) * kStageUnits) / NPW)
            const int n_terms = nn[i];
            if (n_terms > 0) {
                float pw[KPRE];
                int po[KPRE];
#pragma unroll
                for (int p = 0; p < KPRE; ++p)
                    finish_terms<XT, H, SWZ>(rw[i][MERGE ? 0 : p], ri[i][MERGE ? 0 : p], n_terms - p * TB, tofs, S4, -c * C * S4, zero_off, pw[p], po[p],
                                             MERGE ? p * TB : 0);
                walk_groups<R, KPRE, kReadAhead>(acc[i], pw, po, xb, lanepart, (n_terms + H - 1) / H);
                // long ranges: the remaining blocks, one at a time, each requested one block ahead
                if (n_terms > KPRE * TB) {
                    const int row = slot_of(i) * KS + k0n[i];
                    XT wr;
                    int ir;
                    request_terms<XT, IT, PKB>(W_c, idx, pk, row + KPRE * TB, lofs, t_last, wr, ir);
                    for (int kb = KPRE * TB; kb < n_terms; kb += TB) {
                        float wc[1];
                        int oc[1];
                        finish_terms<XT, H, SWZ>(wr, ir, n_terms - kb, tofs, S4, -c * C * S4, zero_off, wc[0], oc[0]);
                        if (kb + TB < n_terms) request_terms<XT, IT, PKB>(W_c, idx, pk, row + kb + TB, lofs, t_last, wr, ir);
                        walk_groups<R, 1, kReadAhead>(acc[i], wc, oc, xb, lanepart, (n_terms - kb + H - 1) / H);
                    }
                }
            }
            SRIGL_PRELOAD(more, i, c + 1)                 // this slot's registers are free: request its next chunk
        }
        if (more) {
            __syncthreads();                              // every wavefront is done reading chunk c
            SRIGL_STAGE_STORE()
            __syncthreads();
        }
    }
#undef SRIGL_LOAD_BOUNDS
#undef SRIGL_STAGE_LOAD
#undef SRIGL_STAGE_LOAD_UNITS
#undef SRIGL_STAGE_STORE
#undef SRIGL_PRELOAD

    // ---- results: transpose through LDS, then bias + scatter with row-contiguous stores ----
    if (out_off == 0) __syncthreads();                     // shared space: every wavefront must be done reading the x tile
    float* const out = lds + out_off;
    const int OS = NG + 1;                                 // odd stride: conflict-free transposed writes
#pragma unroll
    for (int i = 0; i < NPW; ++i)
#pragma unroll
        for (int r = 0; r < R; ++r) {
            float v = acc[i][r];
            if constexpr (H >= 2) v += __shfl_xor(v, LR, kWave);        // the slices hold partial sums of the same rows
            if constexpr (H >= 4) v += __shfl_xor(v, 2 * LR, kWave);
            if (lane < LR) out[(rowl * R + r) * OS + (slot_of(i) - sg0)] = v;
        }
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
            if (s < n_active && col >= 0 && col < d_out) biasv[h] = rl_bias_at(bias, col);
        }
    }
    const int n_rows = min(BT, B - b0);
    if (active) {
        // The stored columns of this workgroup and the ablated ones between them are one run of consecutive columns of
        // y, (active[sg0 - 1], active[last slot]]: a table in LDS says which slot, if any, holds a column, and the lanes
        // write the run left to right (consecutive lanes, consecutive columns) instead of every lane its own column
        // and the gap in front of it.  Runs longer than the table (very few stored neurons) take the loop below.
        const int s_last = min(sg0 + NG, n_slots) - 1;
        const int c0 = sg0 > 0 ? min(active[sg0 - 1] + 1, d_out) : 0;
        const int c1 = s_last < n_active ? min(active[s_last] + 1, d_out) : d_out;
        const int span = c1 - c0;
        if (span > 0 && span <= kSpanCap && c0 >= 0) {
            int* const tab = reinterpret_cast<int*>(out + BT * OS);
            float* const bsp = reinterpret_cast<float*>(tab + kSpanCap);
            for (int c = tid; c < span; c += blockDim.x) {
                tab[c] = -1;
                bsp[c] = rl_bias_at(bias, c0 + c);
            }
            __syncthreads();
            if (wv_id == 0) {
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int i = lane + h * kWave;
                    const int col = colv[h];
                    if (col >= c0 && col < c1 && sg0 + i < n_active) tab[col - c0] = i;
                }
            }
            __syncthreads();
            for (int row = wv_id; row < n_rows; row += nw) {
                float* yr = y + (size_t)(b0 + row) * d_out + c0;
                for (int c = lane; c < span; c += kWave) {
                    const int t = tab[c];
                    const float v = t >= 0 ? out[row * OS + t] + bsp[c] : bsp[c];
                    __builtin_nontemporal_store(act == SRIGL_ACT_NONE ? v : apply_act(v, act), &yr[c]);
                }
            }
            return;
        }
    }
    // the loop exists twice so that the plain forward pass carries no test of the activation code per store
    auto store_rows = [&](auto with_act) {
        for (int row = wv_id; row < n_rows; row += nw) {
            float* yr = y + (size_t)(b0 + row) * d_out;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int i = lane + h * kWave;
                const int col = colv[h];
                if (col < 0) continue;
                if (active)
                    for (int cc = prevv[h]; cc < col; ++cc) {
                        const float bv = rl_bias_at(bias, cc);
                        __builtin_nontemporal_store(decltype(with_act)::value ? apply_act(bv, act) : bv, &yr[cc]);
                    }
                if (sg0 + i < n_active && col < d_out) {
                    const float v = out[row * OS + i] + biasv[h];
                    __builtin_nontemporal_store(decltype(with_act)::value ? apply_act(v, act) : v, &yr[col]);
                }
            }
        }
    };
    if (act == SRIGL_ACT_NONE) store_rows(std::false_type{});
    else store_rows(std::true_type{});
}

// ceil(2^32 / d): workgroup id / 8 divided by d is then one multiply-high, exact while (id / 8) * d < 2^32; 0 = divide
static inline unsigned rowlane_decode_multiplier(long long blocks, int d) {
    if (d <= 1 || (blocks / 8 + 1) * (long long)d >= (1LL << 32)) return 0u;
    return (unsigned)(((1ULL << 32) + (unsigned)d - 1) / (unsigned)d);
}

template <int R, int H, int NPW, int KPRE, typename XT, bool FAST, typename IT, int PKB = 0, bool SPREAD = false>
static srigl_status launch_rowlane_f(const FwdArgs& a, const RowlanePlan& p, hipStream_t st) {
    // (the kernel that deals the rows out is a second instance: with the assignment in registers that the compiler cannot
    // fold into addresses, the consecutive case measured 3-8 % slower inside one kernel that can do both)
    if constexpr (!SPREAD && FAST && PKB == 0 && NPW >= 2) {
        if (p.spread) return launch_rowlane_f<R, H, NPW, KPRE, XT, FAST, IT, PKB, true>(a, p, st);
    }
    if (!SPREAD && p.spread) return SRIGL_ERR_UNSUPPORTED;
    auto kern = k_fwd_rowlane<R, H, NPW, KPRE, XT, FAST, IT, PKB, SPREAD>;
    static LdsLimit lds_limit;
    if (lds_limit.ensure(kern, p.lds) != SRIGL_OK) return SRIGL_ERR_HIP;
    const long long blocks = p.bt_major ? 8LL * ((p.n_btiles + 7) / 8) * p.n_groups : 8LL * ((p.n_groups + 7) / 8) * p.n_btiles;
    if (blocks > 0x7fffffffLL) return SRIGL_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(p.NW * kWave), p.lds, st, (const XT*)a.x, a.B, a.d_in, (const XT*)a.W_c,
                       (const IT*)a.idx, a.active, a.n_active, a.K, a.bias, a.d_out, a.y, a.seg, a.seg_stride, p.C, p.n_chunks, p.n_btiles,
                       p.n_groups, p.out_off, a.act, p.bt_major, static_cast<const unsigned char*>(a.packed), PKB ? (a.K + 3) / 4 * 4 : a.K,
                       rowlane_decode_multiplier(blocks, p.bt_major ? p.n_groups : p.n_btiles), p.spread);
    return hip_ok(hipGetLastError());
}

// The streaming copy is read when the call brings one whose terms this element type can take in one load (fp32: 8 bytes;
// bf16 beside 16-bit indices: 4 bytes) and its byte offsets fit 32 bits.
template <typename XT, typename IT> constexpr int rowlane_packed_term_bytes() { return sizeof(IT) != 4 ? 0 : (sizeof(XT) == 4 ? 8 : 4); }
template <typename XT, typename IT>
static bool rowlane_reads_packed(const FwdArgs& a) {
    constexpr int PKB = rowlane_packed_term_bytes<XT, IT>();
    if (PKB == 0 || a.packed == nullptr) return false;
    if (PKB == 4 && a.d_in > 65536) return false;    // bf16 weights beside 32-bit indices: 8-byte terms, read from the arrays instead
    return ((long long)a.n_active + 256) * ((a.K + 3) / 4 * 4) * PKB + 4096 < (1LL << 32);
}

template <int R, int H, int NPW, typename XT, typename IT>
static srigl_status launch_rowlane_k(const FwdArgs& a, const RowlanePlan& p, hipStream_t st) {
    constexpr int KPRE = rowlane_kpre_rh(NPW, R, H);
    constexpr int PKB = rowlane_packed_term_bytes<XT, IT>();
    const bool pk = p.pk && p.fast && rowlane_reads_packed<XT, IT>(a);
    if constexpr (H > 1 && !(R == 2 && H == 2) && KPRE > 1) {
        // short rows: one preloaded block of 32 or 64 terms per stored row and chunk (the host's choice, by fan-in)
        if (p.KPRE == 1) {
            if (!p.fast) return SRIGL_ERR_UNSUPPORTED;
            if constexpr (PKB != 0) { if (pk) return launch_rowlane_f<R, H, NPW, 1, XT, true, IT, PKB>(a, p, st); }
            return launch_rowlane_f<R, H, NPW, 1, XT, true, IT>(a, p, st);
        }
    }
    if constexpr (PKB != 0) { if (pk) return launch_rowlane_f<R, H, NPW, KPRE, XT, true, IT, PKB>(a, p, st); }
    if (p.fast) return launch_rowlane_f<R, H, NPW, KPRE, XT, true, IT>(a, p, st);
    if constexpr (R == 1 && H == 1) return launch_rowlane_f<R, H, NPW, KPRE, XT, false, IT>(a, p, st);
    return SRIGL_ERR_UNSUPPORTED;   // the planner keeps R = 1, H = 1 when the fast staging does not apply
}

template <int R, int H, typename XT, typename IT>
static srigl_status launch_rowlane_r(const FwdArgs& a, const RowlanePlan& p, hipStream_t st) {
    constexpr int MAXN = rowlane_max_npw(R, H);
    switch (p.NPW) {
        case 1: return launch_rowlane_k<R, H, 1, XT, IT>(a, p, st);
        case 2: return launch_rowlane_k<R, H, 2, XT, IT>(a, p, st);
        case 3: return launch_rowlane_k<R, H, 3, XT, IT>(a, p, st);
        case 4: if constexpr (MAXN >= 4) return launch_rowlane_k<R, H, 4, XT, IT>(a, p, st); else break;
        case 6: if constexpr (MAXN >= 6) return launch_rowlane_k<R, H, 6, XT, IT>(a, p, st); else break;
        case 8: if constexpr (MAXN >= 8) return launch_rowlane_k<R, H, 8, XT, IT>(a, p, st); else break;
        default: break;
    }
    return SRIGL_ERR_UNSUPPORTED;
}

template <typename XT, typename IT>
static srigl_status launch_rowlane_x(const FwdArgs& a, const RowlanePlan& p, hipStream_t st) {
    switch (p.R * 10 + p.H) {
        case 11: return launch_rowlane_r<1, 1, XT, IT>(a, p, st);
        case 12: return launch_rowlane_r<1, 2, XT, IT>(a, p, st);
        case 14: return launch_rowlane_r<1, 4, XT, IT>(a, p, st);
        case 21: return launch_rowlane_r<2, 1, XT, IT>(a, p, st);
        case 22: return launch_rowlane_r<2, 2, XT, IT>(a, p, st);
        case 24: return launch_rowlane_r<2, 4, XT, IT>(a, p, st);
        case 42: return launch_rowlane_r<4, 2, XT, IT>(a, p, st);
        case 44: return launch_rowlane_r<4, 4, XT, IT>(a, p, st);
        default: return SRIGL_ERR_UNSUPPORTED;
    }
}

}  // namespace srigl
