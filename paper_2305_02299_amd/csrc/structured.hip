// Structured-only representation (gfx950): the stored neurons of a layer trained with SRigL keep dense rows
// (ablated neurons removed, fine-grained sparsity not exploited; Sec. 4.4, Fig. 4 and App. H of arXiv
// 2305.02299), and the forward pass is a dense product on the matrix cores,
//     y[b][active[s]] = bias[active[s]] + sum_j Wd[s][j] * x[b][j].
//
// The product is an "NT" GEMM: both operands are K-contiguous (x[b][:], Wd[s][:]).  A workgroup owns a BM x BN
// output tile and walks d_in in stages of SLAB = 128 or 64 bytes per row.  Stages travel from global memory straight
// into a ring of NS LDS stages (global_load_lds_dwordx4: every lane brings 16 bytes, a wavefront fills 1 KB = 1024 / SLAB
// rows of the stage), up to NS - 1 stages ahead of the one being multiplied; one barrier per stage.
// LDS layout of a stage: row r at r * SLAB bytes; its 16-byte piece q sits in slot q ^ ((r >> 1) & 7) for SLAB = 128 and
// q ^ ((r >> 2) & 3) for SLAB = 64: rows that share their banks get different slots, so the 16-byte reads of consecutive
// rows at one q spread over all banks (measured: same rate as a padded pitch, which a direct load cannot produce).  The
// swizzle is applied on the global side: the lane that fills slot s of row r fetches piece s ^ swizzle(r).
// A wavefront owns a (BM/WGM) x (BN/WGN) part of the tile as 32x32 MFMA blocks:
//   bf16: v_mfma_f32_32x32x16_bf16, lane l holds row l%32 and the 8 consecutive k of piece l/32 of the 32-byte step;
//   fp32: v_mfma_f32_32x32x2_f32, lane l holds row l%32, k = l/32; the lane's 16-byte piece carries 4 k, used by 4
//         successive MFMAs (both operands use the same k-to-slot map, so the sum runs over matching k).
// Result block layout: accumulator register e of lane l is row 8*(e/4) + 4*(l/32) + e%4, column l%32.
#include "srigl_internal.h"

namespace srigl {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kXcds = 8;                  // dies with an L2 of their own; workgroup id % 8 selects the die
#ifndef SRIGL_PANEL_N
#define SRIGL_PANEL_N 8
#endif
constexpr int kPanelN = SRIGL_PANEL_N;    // tile columns per panel of the tile order
constexpr int kSlabBytes = 128;   // bytes of K per row and slab = LDS row pitch

__device__ uint4 g_zero16 = {0u, 0u, 0u, 0u};   // source of the pieces past the end of a row

// zero fill, then scatter: two launches so that no ordering inside a wavefront is relied on
__global__ __launch_bounds__(256) void k_fill_zero16(uint4* __restrict__ p, size_t n16) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    const uint4 z = {0u, 0u, 0u, 0u};
    for (; i < n16; i += stride) p[i] = z;
}
__global__ __launch_bounds__(256) void k_fill_zero_bytes(unsigned char* __restrict__ p, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = 0;
}
template <typename T>
__global__ __launch_bounds__(256) void k_scatter_rows(const T* __restrict__ W_c, const int32_t* __restrict__ idx, long long n_terms,
                                                      int K, int d_in, T* __restrict__ Wd) {
    long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long stride = (long long)gridDim.x * blockDim.x;
    for (; t < n_terms; t += stride) {
        const long long s = t / K;
        const int j = idx[t];
        if (j >= 0 && j < d_in) Wd[s * d_in + j] = W_c[t];
    }
}

// Columns that are not stored get their bias (used when no neuron is stored at all; otherwise the product kernel's epilogue
// writes them).  A workgroup takes 256 consecutive columns and kFillRows rows: every thread
// looks its column up in the ascending active list, the ablated ones are gathered into a list in LDS, and the threads then
// walk (row, listed column) pairs so that neighbouring lanes write neighbouring ablated columns of one row.
constexpr int kFillRows = 128;
__global__ __launch_bounds__(256) void k_fill_ablated(const int32_t* __restrict__ active, int n_active, const float* __restrict__ bias,
                                                      int B, int d_out, float* __restrict__ y) {
    __shared__ int list[256];
    __shared__ float list_bias[256];
    __shared__ int wave_count[4];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int c = blockIdx.x * 256 + tid;
    bool ablated = c < d_out;
    if (ablated && n_active > 0) {
        int lo = 0, hi = n_active;   // first position whose entry is >= c
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (active[mid] < c) lo = mid + 1; else hi = mid;
        }
        ablated = !(lo < n_active && active[lo] == c);
    }
    const unsigned long long vote = __ballot(ablated);
    const int before = __builtin_amdgcn_mbcnt_hi((unsigned)(vote >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)vote, 0));
    if (lane == 0) wave_count[wv] = __popcll(vote);
    __syncthreads();
    int base = 0, n_list = 0;
    for (int w = 0; w < 4; ++w) {
        if (w < wv) base += wave_count[w];
        n_list += wave_count[w];
    }
    if (ablated) {
        list[base + before] = c;
        list_bias[base + before] = bias ? bias[c] : 0.0f;
    }
    __syncthreads();
    if (n_list == 0) return;
    const int r0 = blockIdx.y * kFillRows;
    const int rows = min(kFillRows, B - r0);
    for (int idx = tid; idx < rows * n_list; idx += 256) {
        const int r = idx / n_list, k = idx - r * n_list;
        y[(size_t)(r0 + r) * d_out + list[k]] = list_bias[k];
    }
}

// y[r][c] = bias[c] + sum over the parts z (ascending) of part[z][r][s] when column c is stored neuron s, else bias[c].
// One thread per (row r, slot s <= n_active): slot s writes its neuron's column and the ablated columns between the previous
// stored neuron and its own; slot n_active writes the ablated columns after the last stored neuron.  The parts' values are
// requested together (up to kMaxSplits independent loads), so a thread waits for memory twice: the list, then the values.
constexpr int kMaxSplits = 16;
__global__ __launch_bounds__(256) void k_sum_parts(const float* __restrict__ part, int splits, int B, int n_active,
                                                   const int32_t* __restrict__ active, const float* __restrict__ bias, int d_out,
                                                   float* __restrict__ y) {
    const int s = blockIdx.x * 256 + threadIdx.x;
    const int r = blockIdx.y;
    if (s > n_active) return;
    float v[kMaxSplits];
    const size_t plane = (size_t)B * n_active;
    const float* p = part + (size_t)r * n_active + (s < n_active ? s : 0);
#pragma unroll
    for (int z = 0; z < kMaxSplits; ++z) v[z] = (z < splits && s < n_active) ? p[z * plane] : 0.0f;
    int lo, hi;   // ablated columns lo .. hi - 1, then the stored neuron's column hi (none for the last slot)
    if (active == nullptr) {
        lo = hi = s;   // every neuron stored: n_active == d_out
    } else {
        lo = s > 0 ? active[s - 1] + 1 : 0;
        hi = s < n_active ? active[s] : d_out;
    }
    float* yr = y + (size_t)r * d_out;
    for (int c = lo; c < hi; ++c) __builtin_nontemporal_store(bias ? bias[c] : 0.0f, &yr[c]);
    if (s < n_active) {
        float sum = 0.0f;
#pragma unroll
        for (int z = 0; z < kMaxSplits; ++z) sum += v[z];   // parts past `splits` hold zeros
        __builtin_nontemporal_store(sum + (bias ? bias[hi] : 0.0f), &yr[hi]);
    }
}

template <typename T> struct Frag;
template <> struct Frag<uint16_t> { using type = bf16x8_t; };
template <> struct Frag<float> { using type = float4; };

__device__ __forceinline__ void mma_block(f32x16_t& acc, const bf16x8_t& a, const bf16x8_t& b) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
}
__device__ __forceinline__ void mma_block(f32x16_t& acc, const float4& a, const float4& b) {
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b.x, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b.y, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, b.z, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, b.w, acc, 0, 0, 0);
}

// s_waitcnt immediate that waits for the vector-memory counter only (gfx9 encoding: vmcnt in bits 3:0 and 15:14)
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }

using gptr_t = const __attribute__((address_space(1))) void*;
using lptr_t = __attribute__((address_space(3))) void*;

// LDS use of the epilogue: the column table with its bias values and an fp32 tile (pitch BN + 4) of all BM rows when
// that fits, else of the rows of one wavefront row at a time
template <int BM, int BN, int WGM>
struct EpiLayout {
    static constexpr int PITCH = BN + 4;
    static constexpr int TCAP = 1024;   // columns of y per pass
    static constexpr int PHASES = ((size_t)BM * PITCH * 4 + (size_t)TCAP * 8 <= kLdsMax) ? 1 : WGM;
    static constexpr size_t BYTES = (size_t)(BM / PHASES) * PITCH * 4 + (size_t)TCAP * 8;
};

// BM x BN output tile per workgroup of WGM x WGN wavefronts; NS >= 2 LDS stages of SLAB (128 or 64) bytes of K per row.
//
// Schedule of one stage h (KSTEPS = SLAB / 32 MFMA steps): the fragments of step kk + 1 are requested before the MFMAs of
// step kk; before the last step the wavefront waits until its own loads of stage h + 1 have landed and its own reads of
// stage h have returned, meets the others at the barrier (after which stage h + 1 is complete and the slot of stage h is
// free), refills that slot with stage h + NS and requests the first fragments of stage h + 1.  The MFMAs right after
// the barrier have their operands in registers already, so the matrix pipe does not drain at the barrier.
template <typename T, int BM, int BN, int WGM, int WGN, int NS, int SLAB, bool RAGGED>
__global__ __launch_bounds__(WGM * WGN * 64) void k_structured_gemm(const T* __restrict__ x, int B, int d_in, const T* __restrict__ Wd,
                                                                   const int32_t* __restrict__ active, int n_active,
                                                                   const float* __restrict__ bias, int d_out, float* __restrict__ y,
                                                                   int splits, float* __restrict__ part) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];   // [NS][BM + BN rows][SLAB bytes]
    using F = typename Frag<T>::type;
    constexpr int NWAVES = WGM * WGN;
    constexpr int EPS = SLAB / (int)sizeof(T);         // elements of K per stage
    constexpr int EPP = 16 / (int)sizeof(T);           // elements per 16-byte piece
    constexpr int PIECES = SLAB / 16;                  // pieces per row and stage (8 or 4)
    constexpr int KSTEPS = SLAB / 32;                  // MFMA steps per stage (two pieces each)
    constexpr int RPL = 1024 / SLAB;                   // rows one wavefront-wide direct load fills (8 or 16)
    constexpr int SWZ_SHIFT = (SLAB == 128) ? 1 : 2;   // rows 2^shift apart share their banks
    constexpr int WTM = BM / WGM, WTN = BN / WGN;      // wavefront tile
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int ROWS = BM + BN;
    constexpr int STAGE = ROWS * SLAB;
    constexpr int PASSES = ROWS / RPL / NWAVES;        // 1 KB direct loads per wavefront and stage
    static_assert(SLAB == 128 || SLAB == 64, "stage width");
    static_assert(ROWS % (RPL * NWAVES) == 0 && WTM % 32 == 0 && WTN % 32 == 0 && NS >= 2, "tile shape");
    static_assert((NS - 1) * PASSES <= 63, "vmcnt range");
    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);   // wavefront index as a scalar
    const int wm = wv / WGN, wn = wv % WGN;
    // Workgroup -> tile.  Consecutive workgroup ids go round-robin to the 8 XCDs, each with its own L2.  The tiles are put
    // in an order in which neighbours share operands (panels of kPanelN tile columns, row by row inside a panel), that order
    // is cut into 8 equal runs, and XCD c walks run c: the 32 tiles it holds at a time cover about 4 x 8 tiles, which
    // share their rows of x and of Wd through that L2, and every XCD gets the same number of tiles.
    int tile_m, tile_n;
    {
        const int tiles_m = (B + BM - 1) / BM, tiles_n = (n_active + BN - 1) / BN;
        const int total = tiles_m * tiles_n;
        const int per_xcd = (total + kXcds - 1) / kXcds;
        const int id = blockIdx.x;
        const int q = (id % kXcds) * per_xcd + id / kXcds;
        if (id / kXcds >= per_xcd || q >= total) return;   // padding of the last run
        const int full_panel = tiles_m * kPanelN;
        const int panel = q / full_panel, r = q - panel * full_panel;
        const int width = min(kPanelN, tiles_n - panel * kPanelN);
        tile_m = r / width;
        tile_n = panel * kPanelN + r - tile_m * width;
    }
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    // loader: pass p of wavefront wv fills rows RPL * (p * NWAVES + wv) .. + RPL - 1; lane -> (row + lane / PIECES, slot lane % PIECES).
    // The first XP passes are rows of x, the others rows of Wd; a lane keeps one 32-bit byte offset per pass from the tile's
    // first row, the stage advance is scalar.  Rows past the matrix re-read its last row (their results are never stored).
    constexpr int XP = BM / RPL / NWAVES;
    static_assert((BM / RPL) % NWAVES == 0, "a pass is all x rows or all Wd rows");
    uint32_t voff[PASSES];
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        const int row = RPL * (p * NWAVES + wv) + lane / PIECES;
        const int piece = (lane % PIECES) ^ ((row >> SWZ_SHIFT) & (PIECES - 1));
        const int r = (p < XP) ? min(row, B - 1 - m0) : min(row - BM, n_active - 1 - n0);
        voff[p] = (uint32_t)r * (uint32_t)(d_in * (int)sizeof(T)) + piece * 16;
    }
    const unsigned char* xbase = reinterpret_cast<const unsigned char*>(x + (size_t)m0 * d_in);
    const unsigned char* wbase = reinterpret_cast<const unsigned char*>(Wd + (size_t)n0 * d_in);
    // Part blockIdx.y of d_in (splits parts of whole stages, sizes one stage apart at most): stages h_first .. h_first + n_st - 1
    // of the row.  With one part the tile's sums are complete and go to y; with several they go to part[blockIdx.y][B][n_active].
    const int n_st_row = (d_in + EPS - 1) / EPS;
    const int h_first = (int)(((long long)blockIdx.y * n_st_row) / splits);
    const int n_st = (int)(((long long)(blockIdx.y + 1) * n_st_row) / splits) - h_first;
    // RAGGED: d_in is not a multiple of EPS; the pieces of the last stage that lie past the end of the rows come from zeros.
    // A stage index past the end re-issues the last stage (into a slot nobody reads again): the loop body has no branches
    // and the number of loads in flight at each wait is fixed.
    auto issue_stage = [&](int h_unclamped) {
        const int h = h_first + min(h_unclamped, n_st - 1);
        unsigned char* stage = smem + (h_unclamped % NS) * STAGE + 1024 * wv;
        const unsigned char* xs = xbase + (size_t)h * SLAB;
        const unsigned char* ws = wbase + (size_t)h * SLAB;
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            const unsigned char* g = ((p < XP) ? xs : ws) + voff[p];
            if (RAGGED) {
                const int row = RPL * (p * NWAVES + wv) + lane / PIECES;
                const int piece = (lane % PIECES) ^ ((row >> SWZ_SHIFT) & (PIECES - 1));
                if (h * EPS + piece * EPP >= d_in) g = reinterpret_cast<const unsigned char*>(&g_zero16);   // a piece is whole or absent
            }
            __builtin_amdgcn_global_load_lds((gptr_t)g, (lptr_t)(stage + 1024 * NWAVES * p), 16, 0, 0);
        }
    };

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    if (n_st > 0) {
#pragma unroll
        for (int s = 0; s < NS; ++s) issue_stage(s);
    }

    // reader: row l%32 of a block, piece 2*kk + l/32; the swizzle term only depends on the lane (block rows start at multiples of 32)
    const int swz = ((lane & 31) >> SWZ_SHIFT) & (PIECES - 1);
    int frag_off[KSTEPS];
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk) frag_off[kk] = (lane & 31) * SLAB + (((2 * kk + (lane >> 5)) ^ swz) * 16);

    F a[2][TM], b[2][TN];
    auto read_frags = [&](int h, int kk, int set) {
        const unsigned char* buf = smem + (h % NS) * STAGE;
#pragma unroll
        for (int i = 0; i < TM; ++i) a[set][i] = *reinterpret_cast<const F*>(buf + (wm * WTM + i * 32) * SLAB + frag_off[kk]);
#pragma unroll
        for (int j = 0; j < TN; ++j) b[set][j] = *reinterpret_cast<const F*>(buf + (BM + wn * WTN + j * 32) * SLAB + frag_off[kk]);
    };

    if (n_st > 0) {
        __builtin_amdgcn_s_waitcnt(vmcnt_imm((NS - 1) * PASSES));
        __syncthreads();
        read_frags(0, 0, 0);
    }
    for (int h = 0; h < n_st; ++h) {
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
            if (kk + 1 < KSTEPS) {
                read_frags(h, kk + 1, (kk + 1) & 1);
            } else {
                // stages up to h + NS - 1 are on their way; stage h + 1 must have landed.  Every fragment of stage h is in
                // registers by now (the wait before the barrier covers the reads above), so its slot is refilled right away.
                __builtin_amdgcn_s_waitcnt(vmcnt_imm((NS - 2) * PASSES));
                __syncthreads();
                issue_stage(h + NS);
                read_frags(min(h + 1, n_st - 1), 0, 0);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) mma_block(acc[i][j], a[kk & 1][i], b[kk & 1][j]);
        }
    }

    // One part of several: the partial sums of the tile, stored neuron s in column s of this part's [B][n_active] array
    // (bias, ablated columns and the sum over the parts belong to k_sum_parts).
    if (part != nullptr) {
        float* pz = part + (size_t)blockIdx.y * B * n_active;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = n0 + wn * WTN + j * 32 + (lane & 31);
            if (col >= n_active) continue;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int m = m0 + wm * WTM + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                    if (m < B) pz[(size_t)m * n_active + col] = acc[i][j][e];
                }
            }
        }
        return;
    }

    // Epilogue without an active list: stored neuron s is column s; every lane writes its accumulators where they belong
    // (32 neighbouring lanes cover 128 contiguous bytes of a row).
    if (active == nullptr) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = n0 + wn * WTN + j * 32 + (lane & 31);
            if (col >= n_active) continue;
            const float bv = bias ? bias[col] : 0.0f;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int m = m0 + wm * WTM + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                    if (m < B) __builtin_nontemporal_store(acc[i][j][e] + bv, &y[(size_t)m * d_out + col]);   // y is not read again here
                }
            }
        }
        return;
    }

    // Epilogue with an active list.  The stored neurons of this tile and the ablated ones between them cover one contiguous
    // range of columns of y, [c_lo, c_hi].  The range is written row by row with neighbouring lanes on neighbouring columns:
    // a table in LDS says, for each column of the range, which stored neuron of the tile it is (or none: the column is its
    // bias), and the accumulators pass through an LDS tile.  No column of y is touched twice and none is left out.
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));   // the re-issued last stages may still be landing in the ring
    __syncthreads();
    using EL = EpiLayout<BM, BN, WGM>;
    constexpr int NT = NWAVES * 64;
    constexpr int PITCH = EL::PITCH, TCAP = EL::TCAP, EPH = EL::PHASES, PROWS = BM / EPH, WPP = WGM / EPH;
    float* tile = reinterpret_cast<float*>(smem);                         // [PROWS][PITCH]
    int* table = reinterpret_cast<int*>(smem + PROWS * PITCH * 4);        // [TCAP] stored neuron within the tile, or -1
    float* tbias = reinterpret_cast<float*>(table + TCAP);                // [TCAP]
    const int s_cnt = min(BN, n_active - n0);
    const int c_lo = max((n0 > 0) ? active[n0 - 1] + 1 : 0, 0);
    const int c_hi = min((n0 + s_cnt == n_active) ? d_out - 1 : active[n0 + s_cnt - 1], d_out - 1);
    for (int cc = c_lo; cc <= c_hi; cc += TCAP) {
        const int wc = min(TCAP, c_hi - cc + 1);
        if (cc != c_lo) __syncthreads();   // the previous pass is done with the table
        for (int k = tid; k < wc; k += NT) {
            tbias[k] = bias ? bias[cc + k] : 0.0f;
            table[k] = -1;
        }
        __syncthreads();
        for (int s = tid; s < s_cnt; s += NT) {
            const int col = active[n0 + s] - cc;
            if (col >= 0 && col < wc) table[col] = s;
        }
#pragma unroll
        for (int ph = 0; ph < EPH; ++ph) {
            if (ph > 0 || cc != c_lo) __syncthreads();   // tile free again
            if (wm / WPP == ph) {
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
#pragma unroll
                        for (int e = 0; e < 16; ++e)
                            tile[((wm % WPP) * WTM + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3)) * PITCH + wn * WTN + j * 32 + (lane & 31)] =
                                acc[i][j][e];
            }
            __syncthreads();   // tile, table and bias values complete
            const int rows = min(PROWS, B - (m0 + ph * PROWS));
            for (int r = wv; r < rows; r += NWAVES) {
                float* yr = y + (size_t)(m0 + ph * PROWS + r) * d_out + cc;
                for (int k = lane; k < wc; k += 64) {
                    const int tix = table[k];
                    __builtin_nontemporal_store((tix >= 0 ? tile[r * PITCH + tix] : 0.0f) + tbias[k], &yr[k]);
                }
            }
        }
    }
}

template <typename T, int BM, int BN, int WGM, int WGN, int NS, int SLAB, bool RAGGED>
static srigl_status launch_gemm_r(const void* x, int B, int d_in, const void* Wd, const int32_t* active, int n_active, const float* bias,
                                int d_out, float* y, int splits, float* part, hipStream_t st) {
    auto kern = k_structured_gemm<T, BM, BN, WGM, WGN, NS, SLAB, RAGGED>;
    constexpr size_t ring = (size_t)NS * (BM + BN) * SLAB, epi = EpiLayout<BM, BN, WGM>::BYTES;
    constexpr size_t lds = ring > epi ? ring : epi;
    static_assert(lds <= kLdsMax, "LDS");
    static LdsLimit lds_limit;
    if (lds_limit.ensure(kern, lds) != SRIGL_OK) return SRIGL_ERR_HIP;
    const long long tiles_m = (B + BM - 1) / BM, tiles_n = (n_active + BN - 1) / BN;
    const long long n_wg = ((tiles_m * tiles_n + kXcds - 1) / kXcds) * kXcds;   // 8 equal runs of tiles, one per XCD
    if (n_wg > 0x7fffffffLL) return SRIGL_ERR_UNSUPPORTED;
    // every part holds at least one stage
    if (splits < 1 || splits > 65535 || (splits > 1 && (part == nullptr || splits > (d_in * (int)sizeof(T) + SLAB - 1) / SLAB)))
        return SRIGL_ERR_INVALID_ARG;
    if (splits > 1 && B > 65535) return SRIGL_ERR_UNSUPPORTED;   // the sum's grid has one row of workgroups per batch row
    const dim3 grid((unsigned)n_wg, (unsigned)splits);
    // a lane addresses its rows with 32-bit byte offsets from the tile's first row
    if ((long long)(BM > BN ? BM : BN) * d_in * (long long)sizeof(T) >= (1ll << 31)) return SRIGL_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(kern, grid, dim3(WGM * WGN * 64), lds, st, (const T*)x, B, d_in, (const T*)Wd, active, n_active, bias, d_out, y,
                       splits, splits > 1 ? part : nullptr);
    if (splits > 1) {
        hipLaunchKernelGGL(k_sum_parts, dim3((unsigned)(n_active / 256 + 1), (unsigned)B), dim3(256), 0, st, part, splits, B, n_active, active,
                           bias, d_out, y);
    }
    return hip_ok(hipGetLastError());
}

template <typename T, int BM, int BN, int WGM, int WGN, int NS, int SLAB>
static srigl_status launch_gemm(const void* x, int B, int d_in, const void* Wd, const int32_t* active, int n_active, const float* bias,
                                int d_out, float* y, int splits, float* part, hipStream_t st) {
    if (d_in % (SLAB / (int)sizeof(T)) == 0)
        return launch_gemm_r<T, BM, BN, WGM, WGN, NS, SLAB, false>(x, B, d_in, Wd, active, n_active, bias, d_out, y, splits, part, st);
    return launch_gemm_r<T, BM, BN, WGM, WGN, NS, SLAB, true>(x, B, d_in, Wd, active, n_active, bias, d_out, y, splits, part, st);
}

// Tile choice and time estimate: a workgroup needs about ns_per_k nanoseconds per element of d_in for its tile (measured on
// MI355X with every compute unit busy; 64x64 fp32 tiles run slower when a compute unit holds a single workgroup), and the
// tiles take ceil(tiles / 256) rounds over the 256 compute units.
struct TileModel { srigl_gemm_tile tile; int bm, bn; float ns_per_k_bf16, ns_per_k_f32, ns_per_k_f32_single_round; };
static const TileModel kTileModels[] = {
    {SRIGL_TILE_256x256_H, 256, 256, 28.0f, 233.0f, 233.0f},
    {SRIGL_TILE_256x128, 256, 128, 18.0f, 125.0f, 125.0f},
    {SRIGL_TILE_128x128, 128, 128, 12.0f, 70.0f, 70.0f},
    {SRIGL_TILE_64x64, 64, 64, 3.8f, 19.0f, 26.0f},
};

// ns_per_k_out: nanoseconds per element of d_in for the whole product with the chosen tile
static srigl_gemm_tile choose_tile(int B, int n_active, bool f32, double* ns_per_k_out = nullptr) {
    srigl_gemm_tile best = SRIGL_TILE_64x64;
    double best_cost = 0.0;
    for (const TileModel& m : kTileModels) {
        const long long tiles = (long long)((B + m.bm - 1) / m.bm) * ((n_active + m.bn - 1) / m.bn);
        const long long rounds = (tiles + 255) / 256;
        const double cost = (double)rounds * (f32 ? (rounds == 1 ? m.ns_per_k_f32_single_round : m.ns_per_k_f32) : m.ns_per_k_bf16);
        if (best_cost == 0.0 || cost < best_cost) { best_cost = cost; best = m.tile; }
    }
    if (ns_per_k_out) *ns_per_k_out = best_cost;
    return best;
}

// The same choice with d_in cut into parts (the parts' tiles run side by side; their partial sums pass through a workspace
// and a second launch adds them): worth it when the tiles alone reach a fraction of the 256 compute units.  Parts: as many
// as keep the workgroups (8 runs of tiles, padded) within 256, or within 480 for 64x64 tiles, two of which share a compute
// unit and then run about 1.6 times longer each; at most 16, at least 4 stages of 128 bytes each.  Measured on MI355X
// (3072 -> 768 fp32, 538 stored neurons): batch 256 88 us in one part, 21 us in 12; batch 64 69 us and 12 us in 16.
static void choose_tile_and_split(int B, int n_active, int d_in, int d_out, bool f32, srigl_gemm_tile* tile_out, int* splits_out,
                                  double* est_us_out) {
    const int stages = (d_in * (f32 ? 4 : 2) + kSlabBytes - 1) / kSlabBytes;
    srigl_gemm_tile best = SRIGL_TILE_64x64;
    int best_s = 1;
    double best_us = 0.0;
    for (const TileModel& m : kTileModels) {
        const long long tiles = (long long)((B + m.bm - 1) / m.bm) * ((n_active + m.bn - 1) / m.bn);
        const long long padded = (tiles + kXcds - 1) / kXcds * kXcds;
        const long long wg_cap = m.bm == 64 ? 480 : 256;
        int cap = stages / 4 < kMaxSplits ? stages / 4 : kMaxSplits;
        if (cap < 1) cap = 1;
        int s = padded >= wg_cap ? 1 : (int)(wg_cap / padded);
        s = s > cap ? cap : s;
        for (int pass = 0; pass < 2; ++pass) {   // one part, then several
            if (pass == 1 && s == 1) break;
            double us;
            if (pass == 0) {
                const long long rounds = (tiles + 255) / 256;
                const double ns_k = f32 ? (rounds == 1 ? m.ns_per_k_f32_single_round : m.ns_per_k_f32) : m.ns_per_k_bf16;
                us = (double)rounds * ns_k * d_in * 1e-3;
            } else {
                const double ns_k = f32 ? m.ns_per_k_f32 : m.ns_per_k_bf16;
                const double crowd = (m.bm == 64 && padded * s > 256) ? 1.6 : 1.0;
                // 7.0: the second launch and a second pipeline fill; the partial sums are written once and read once
                us = 7.0 + ns_k * crowd * d_in / s * 1e-3 + 8.0 * s * (double)B * n_active / 4.5e6;
            }
            if (best_us == 0.0 || us < best_us) { best_us = us; best = m.tile; best_s = pass == 0 ? 1 : s; }
        }
    }
    if (tile_out) *tile_out = best;
    if (splits_out) *splits_out = best_s;
    if (est_us_out) *est_us_out = 3.5 + best_us + 4.0 * (double)B * d_out / 4.5e6;
}

template <typename T>
static srigl_status launch_structured(int tile, const void* x, int B, int d_in, const void* Wd, const int32_t* active, int n_active,
                                      const float* bias, int d_out, float* y, int splits, float* part, hipStream_t st) {
    if (tile == SRIGL_TILE_AUTO) tile = choose_tile(B, n_active, sizeof(T) == 4);
    switch (tile) {
        case SRIGL_TILE_256x256: return launch_gemm<T, 256, 256, 2, 4, 2, 128>(x, B, d_in, Wd, active, n_active, bias, d_out, y, splits, part, st);
        case SRIGL_TILE_256x256_H: return launch_gemm<T, 256, 256, 2, 4, 5, 64>(x, B, d_in, Wd, active, n_active, bias, d_out, y, splits, part, st);
        case SRIGL_TILE_256x128_W4: return launch_gemm<T, 256, 128, 2, 2, 3, 128>(x, B, d_in, Wd, active, n_active, bias, d_out, y, splits, part, st);
        case SRIGL_TILE_256x128: return launch_gemm<T, 256, 128, 4, 2, 3, 128>(x, B, d_in, Wd, active, n_active, bias, d_out, y, splits, part, st);
        case SRIGL_TILE_128x128: return launch_gemm<T, 128, 128, 2, 2, 4, 128>(x, B, d_in, Wd, active, n_active, bias, d_out, y, splits, part, st);
        case SRIGL_TILE_64x64: return launch_gemm<T, 64, 64, 2, 2, 4, 128>(x, B, d_in, Wd, active, n_active, bias, d_out, y, splits, part, st);
        default: return SRIGL_ERR_INVALID_ARG;
    }
}

}  // namespace srigl

using namespace srigl;

extern "C" {

srigl_status srigl_densify(const void* W_c, srigl_dtype w_dtype, const int32_t* idx, int32_t n_active, int32_t K,
                           int32_t d_in, void* Wd, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (n_active < 0 || K < 0 || d_in < 0 || K > d_in) return SRIGL_ERR_INVALID_ARG;
    if (w_dtype != SRIGL_F32 && w_dtype != SRIGL_BF16) return SRIGL_ERR_INVALID_ARG;
    if (n_active == 0 || d_in == 0) return SRIGL_OK;
    if (Wd == nullptr || (K > 0 && (W_c == nullptr || idx == nullptr))) return SRIGL_ERR_INVALID_ARG;
    const size_t bytes = (size_t)n_active * d_in * (w_dtype == SRIGL_F32 ? 4 : 2);
    if ((reinterpret_cast<uintptr_t>(Wd) & 15) == 0 && (bytes & 15) == 0) {
        size_t blocks = (bytes / 16 + 255) / 256;
        if (blocks > 8192) blocks = 8192;
        hipLaunchKernelGGL(k_fill_zero16, dim3((unsigned)blocks), dim3(256), 0, st, static_cast<uint4*>(Wd), bytes / 16);
    } else {
        size_t blocks = (bytes + 255) / 256;
        if (blocks > 8192) blocks = 8192;
        hipLaunchKernelGGL(k_fill_zero_bytes, dim3((unsigned)blocks), dim3(256), 0, st, static_cast<unsigned char*>(Wd), bytes);
    }
    const long long n_terms = (long long)n_active * K;
    if (n_terms > 0) {
        long long blocks = (n_terms + 255) / 256;
        if (blocks > 8192) blocks = 8192;
        if (w_dtype == SRIGL_F32)
            hipLaunchKernelGGL(k_scatter_rows<uint32_t>, dim3((unsigned)blocks), dim3(256), 0, st, static_cast<const uint32_t*>(W_c), idx,
                               n_terms, K, d_in, static_cast<uint32_t*>(Wd));
        else
            hipLaunchKernelGGL(k_scatter_rows<uint16_t>, dim3((unsigned)blocks), dim3(256), 0, st, static_cast<const uint16_t*>(W_c), idx,
                               n_terms, K, d_in, static_cast<uint16_t*>(Wd));
    }
    return hip_ok(hipGetLastError());
}

// Estimates in microseconds, calibrated on MI355X measurements of both forms (fp32 and bf16 storage, batches 1..2048,
// 512- to 4096-wide layers, 80-99 % sparsity):
//   condensed  = the estimate of the forward kernel the library's own choice takes for these sizes (condensed_estimate_us)
//   structured ~ 3.5 + d_in x (rounds of tiles x nanoseconds per element of d_in of the chosen tile) / 1000 / parts of d_in
//                  + the second launch when d_in is cut into parts (srigl_structured_linear_fwd_split)
//                  + 4 B d_out / 4.5e6              (writing the result at HBM speed)
srigl_representation srigl_choose_representation(int32_t B, int32_t d_in, int32_t n_active, int32_t K, int32_t d_out,
                                                 srigl_dtype dtype, float* est_condensed_us, float* est_structured_us) {
    const double cond = condensed_estimate_us(B, d_in, n_active, K, d_out, dtype == SRIGL_BF16, n_active < d_out);
    const bool f32 = dtype == SRIGL_F32;
    const int elem = f32 ? 4 : 2;
    double stru = 0.0;
    choose_tile_and_split(B > 0 ? B : 1, n_active > 0 ? n_active : 1, d_in, d_out, f32, nullptr, nullptr, &stru);
    if ((d_in * elem) % 16 != 0) stru = 1e30;   // the matrix-core kernel needs rows of whole 16-byte pieces
    if (est_condensed_us) *est_condensed_us = (float)cond;
    if (est_structured_us) *est_structured_us = (float)stru;
    return stru < cond ? SRIGL_REPR_STRUCTURED : SRIGL_REPR_CONDENSED;
}

static srigl_status structured_core(const void* x, srigl_dtype x_dtype, int32_t B, int32_t d_in, const void* Wd, srigl_dtype w_dtype,
                                    const int32_t* active, int32_t n_active, const float* bias, int32_t d_out, float* y, int tile,
                                    int splits, void* workspace, size_t workspace_bytes, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (B < 0 || d_in < 0 || n_active < 0 || d_out < 0 || n_active > d_out) return SRIGL_ERR_INVALID_ARG;
    if ((x_dtype != SRIGL_F32 && x_dtype != SRIGL_BF16) || (w_dtype != SRIGL_F32 && w_dtype != SRIGL_BF16)) return SRIGL_ERR_INVALID_ARG;
    if (x_dtype != w_dtype) return SRIGL_ERR_UNSUPPORTED;
    if (active == nullptr && n_active != d_out && n_active != 0) return SRIGL_ERR_INVALID_ARG;
    if (splits < 0 || splits > kMaxSplits) return SRIGL_ERR_INVALID_ARG;
    if (B == 0 || d_out == 0) return SRIGL_OK;
    if (y == nullptr) return SRIGL_ERR_INVALID_ARG;
    if (n_active > 0 && d_in > 0 && (x == nullptr || Wd == nullptr)) return SRIGL_ERR_INVALID_ARG;
    const int elem = (x_dtype == SRIGL_F32) ? 4 : 2;
    if (n_active > 0 && d_in > 0) {
        if ((d_in * elem) % 16 != 0 || ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(Wd)) & 15) != 0)
            return SRIGL_ERR_UNSUPPORTED;
    }
    if (n_active == 0) {   // nothing is stored: every column is its bias
        const dim3 grid((unsigned)((d_out + 255) / 256), (unsigned)((B + kFillRows - 1) / kFillRows));
        if (grid.y > 65535u) return SRIGL_ERR_UNSUPPORTED;
        hipLaunchKernelGGL(k_fill_ablated, grid, dim3(256), 0, st, active, n_active, bias, B, d_out, y);
        return hip_ok(hipGetLastError());
    }
    if (splits == 0) {   // the library's choice of parts (and of the tile, unless forced)
        srigl_gemm_tile t = SRIGL_TILE_AUTO;
        choose_tile_and_split(B, n_active, d_in, d_out, x_dtype == SRIGL_F32, &t, &splits, nullptr);
        if (tile != SRIGL_TILE_AUTO) splits = 1;   // a forced tile keeps the whole of d_in unless the parts are forced too
        else tile = t;
    }
    if (splits > 1) {
        const size_t need = (size_t)splits * B * n_active * sizeof(float);
        if (workspace == nullptr || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 3) != 0) return SRIGL_ERR_CAPACITY;
    }
    float* part = static_cast<float*>(workspace);
    if (x_dtype == SRIGL_F32) return launch_structured<float>(tile, x, B, d_in, Wd, active, n_active, bias, d_out, y, splits, part, st);
    return launch_structured<uint16_t>(tile, x, B, d_in, Wd, active, n_active, bias, d_out, y, splits, part, st);
}

srigl_status srigl_structured_linear_fwd_tile(const void* x, srigl_dtype x_dtype, int32_t B, int32_t d_in, const void* Wd,
                                              srigl_dtype w_dtype, const int32_t* active, int32_t n_active,
                                              const float* bias, int32_t d_out, float* y, srigl_gemm_tile tile, void* stream) {
    return structured_core(x, x_dtype, B, d_in, Wd, w_dtype, active, n_active, bias, d_out, y, tile, 1, nullptr, 0, stream);
}

srigl_status srigl_structured_linear_fwd(const void* x, srigl_dtype x_dtype, int32_t B, int32_t d_in, const void* Wd,
                                         srigl_dtype w_dtype, const int32_t* active, int32_t n_active,
                                         const float* bias, int32_t d_out, float* y, void* stream) {
    return structured_core(x, x_dtype, B, d_in, Wd, w_dtype, active, n_active, bias, d_out, y, SRIGL_TILE_AUTO, 1, nullptr, 0, stream);
}

srigl_status srigl_structured_split_plan(int32_t B, int32_t d_in, int32_t n_active, int32_t d_out, srigl_dtype dtype, int32_t* splits,
                                         size_t* workspace_bytes) {
    if (B < 0 || d_in < 0 || n_active < 0 || d_out < 0 || (dtype != SRIGL_F32 && dtype != SRIGL_BF16)) return SRIGL_ERR_INVALID_ARG;
    int s = 1;
    if (B > 0 && d_in > 0 && n_active > 0) choose_tile_and_split(B, n_active, d_in, d_out, dtype == SRIGL_F32, nullptr, &s, nullptr);
    if (splits) *splits = s;
    if (workspace_bytes) *workspace_bytes = s > 1 ? (size_t)s * B * n_active * sizeof(float) : 0;
    return SRIGL_OK;
}

srigl_status srigl_structured_linear_fwd_split(const void* x, srigl_dtype x_dtype, int32_t B, int32_t d_in, const void* Wd,
                                               srigl_dtype w_dtype, const int32_t* active, int32_t n_active, const float* bias,
                                               int32_t d_out, float* y, srigl_gemm_tile tile, int32_t splits, void* workspace,
                                               size_t workspace_bytes, void* stream) {
    return structured_core(x, x_dtype, B, d_in, Wd, w_dtype, active, n_active, bias, d_out, y, tile, splits, workspace, workspace_bytes, stream);
}

}  // extern "C"
