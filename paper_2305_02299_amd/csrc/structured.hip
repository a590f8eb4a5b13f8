// Structured-only representation (gfx950): the stored neurons of a layer trained with SRigL keep dense rows
// (ablated neurons removed, fine-grained sparsity not exploited; Sec. 4.4, Fig. 4 and App. H of arXiv
// 2305.02299), and the forward pass is a dense product on the matrix cores,
//     y[b][active[s]] = bias[active[s]] + sum_j Wd[s][j] * x[b][j].
//
// The product is an "NT" GEMM: both operands are K-contiguous (x[b][:], Wd[s][:]).  A workgroup owns a BM x BN
// output tile and walks d_in in slabs of 128 bytes per row (64 bf16 or 32 fp32).  Slabs travel from global memory
// straight into a ring of NS LDS stages (global_load_lds_dwordx4: every lane brings 16 bytes, a wavefront fills 1 KB =
// 8 rows of the stage), NS-1 slabs ahead of the one being multiplied; one barrier per slab.
// LDS layout of a stage: row r at r * 128 bytes; its 16-byte piece q sits in slot q ^ ((r >> 1) & 7).  The 16-byte
// reads of 32 consecutive rows at one q then spread over all banks (measured: same rate as a padded 144-byte pitch,
// which a direct load cannot produce).  The swizzle is applied on the global side: the lane that fills slot s of row
// r fetches piece s ^ ((r >> 1) & 7).
// A wavefront owns a (BM/WGM) x (BN/WGN) part of the tile as 32x32 MFMA blocks:
//   bf16: v_mfma_f32_32x32x16_bf16, lane l holds row l%32 and the 8 consecutive k of piece l/32 of the 32-byte step;
//   fp32: v_mfma_f32_32x32x2_f32, lane l holds row l%32, k = l/32; the lane's 16-byte piece carries 4 k, used by 4
//         successive MFMAs (both operands use the same k-to-slot map, so the sum runs over matching k).
// Result block layout: accumulator register e of lane l is row 8*(e/4) + 4*(l/32) + e%4, column l%32.
#include "srigl_internal.h"

namespace srigl {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

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

// columns that are not stored get their bias (the gaps of the ascending active list)
__global__ __launch_bounds__(256) void k_fill_ablated(const int32_t* __restrict__ active, int n_active, const float* __restrict__ bias,
                                                      int B, int d_out, float* __restrict__ y) {
    const long long total = (long long)B * (n_active + 1);
    for (long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (long long)gridDim.x * blockDim.x) {
        const int b = (int)(t / (n_active + 1));
        const int s = (int)(t - (long long)b * (n_active + 1));
        const int col = min((s < n_active) ? active[s] : d_out, d_out);
        const int prev = (s > 0) ? active[s - 1] : -1;
        for (int c = max(prev + 1, 0); c < col; ++c) y[(size_t)b * d_out + c] = bias ? bias[c] : 0.0f;
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

// BM x BN output tile per workgroup of WGM x WGN wavefronts, NS LDS stages
template <typename T, int BM, int BN, int WGM, int WGN, int NS>
__global__ __launch_bounds__(WGM * WGN * 64) void k_structured_gemm(const T* __restrict__ x, int B, int d_in, const T* __restrict__ Wd,
                                                                   const int32_t* __restrict__ active, int n_active,
                                                                   const float* __restrict__ bias, int d_out, float* __restrict__ y) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];   // [NS][BM + BN rows][128 bytes]
    using F = typename Frag<T>::type;
    constexpr int NWAVES = WGM * WGN;
    constexpr int EPS = kSlabBytes / (int)sizeof(T);   // elements of K per slab
    constexpr int EPP = 16 / (int)sizeof(T);           // elements per 16-byte piece
    constexpr int WTM = BM / WGM, WTN = BN / WGN;      // wavefront tile
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int ROWS = BM + BN;
    constexpr int STAGE = ROWS * kSlabBytes;
    constexpr int PASSES = ROWS / 8 / NWAVES;          // 1 KB direct loads per wavefront and slab
    static_assert(ROWS % (8 * NWAVES) == 0 && WTM % 32 == 0 && WTN % 32 == 0 && NS >= 2, "tile shape");
    static_assert((NS - 2) * PASSES <= 63, "vmcnt range");
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int wm = wv / WGN, wn = wv % WGN;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;

    // loader: pass p of wavefront wv fills rows 8 * (p * NWAVES + wv) .. + 7; lane -> (row + lane / 8, slot lane % 8)
    const unsigned char* src[PASSES];
    int piece[PASSES];
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        const int row = 8 * (p * NWAVES + wv) + (lane >> 3);
        piece[p] = (lane & 7) ^ ((row >> 1) & 7);
        const T* base = (row < BM) ? x + (size_t)min(m0 + row, B - 1) * d_in : Wd + (size_t)min(n0 + row - BM, n_active - 1) * d_in;
        src[p] = reinterpret_cast<const unsigned char*>(base + piece[p] * EPP);
    }
    const int n_slabs = (d_in + EPS - 1) / EPS;
    auto issue_slab = [&](int sl) {
        unsigned char* stage = smem + (sl % NS) * STAGE;
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            const bool in = sl * EPS + piece[p] * EPP < d_in;   // d_in is a multiple of EPP: a piece is whole or absent
            const unsigned char* g = in ? src[p] + (size_t)sl * kSlabBytes : reinterpret_cast<const unsigned char*>(&g_zero16);
            __builtin_amdgcn_global_load_lds((gptr_t)g, (lptr_t)(stage + 1024 * (p * NWAVES + wv)), 16, 0, 0);
        }
    };

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

#pragma unroll
    for (int s = 0; s < NS - 1; ++s)
        if (s < n_slabs) issue_slab(s);

    // reader: row l%32 of a block, piece 2*kk + l/32; the swizzle term only depends on the lane (block rows start at multiples of 32)
    const int swz = ((lane & 31) >> 1) & 7;
    int frag_off[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) frag_off[kk] = (lane & 31) * kSlabBytes + (((2 * kk + (lane >> 5)) ^ swz) * 16);

    for (int sl = 0; sl < n_slabs; ++sl) {
        if (sl + NS - 2 < n_slabs) __builtin_amdgcn_s_waitcnt(vmcnt_imm((NS - 2) * PASSES));
        else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
        __syncthreads();   // slab sl is in LDS for every wavefront; everyone is done reading the stage refilled next
        if (sl + NS - 1 < n_slabs) issue_slab(sl + NS - 1);
        const unsigned char* buf = smem + (sl % NS) * STAGE;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            F a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) a[i] = *reinterpret_cast<const F*>(buf + (wm * WTM + i * 32) * kSlabBytes + frag_off[kk]);
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = *reinterpret_cast<const F*>(buf + (BM + wn * WTN + j * 32) * kSlabBytes + frag_off[kk]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) mma_block(acc[i][j], a[i], b[j]);
        }
    }

    // epilogue: bias and scatter to the stored neurons' columns
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int s = n0 + wn * WTN + j * 32 + (lane & 31);
        if (s >= n_active) continue;
        const int col = active ? active[s] : s;
        if (col < 0 || col >= d_out) continue;
        const float bv = bias ? bias[col] : 0.0f;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int m = m0 + wm * WTM + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                if (m < B) y[(size_t)m * d_out + col] = acc[i][j][e] + bv;
            }
        }
    }
}

template <typename T, int BM, int BN, int WGM, int WGN, int NS>
static srigl_status launch_gemm(const void* x, int B, int d_in, const void* Wd, const int32_t* active, int n_active, const float* bias,
                                int d_out, float* y, hipStream_t st) {
    auto kern = k_structured_gemm<T, BM, BN, WGM, WGN, NS>;
    const size_t lds = (size_t)NS * (BM + BN) * kSlabBytes;
    static_assert((size_t)NS * (BM + BN) * kSlabBytes <= kLdsMax, "LDS");
    static bool raised = false;
    if (lds > 64 * 1024 && !raised) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return SRIGL_ERR_HIP;
        raised = true;
    }
    const dim3 grid((unsigned)((n_active + BN - 1) / BN), (unsigned)((B + BM - 1) / BM));
    if (grid.y > 65535u) return SRIGL_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(kern, grid, dim3(WGM * WGN * 64), lds, st, (const T*)x, B, d_in, (const T*)Wd, active, n_active, bias, d_out, y);
    return hip_ok(hipGetLastError());
}

static long long n_tiles(int B, int n_active, int bm, int bn) { return (long long)((B + bm - 1) / bm) * ((n_active + bn - 1) / bn); }

template <typename T>
static srigl_status launch_structured(int tile, const void* x, int B, int d_in, const void* Wd, const int32_t* active, int n_active,
                                      const float* bias, int d_out, float* y, hipStream_t st) {
    if (tile == SRIGL_TILE_AUTO) {
        // the largest tile that still gives every compute unit work
        if (n_tiles(B, n_active, 256, 256) >= 256) tile = SRIGL_TILE_256x256;
        else if (n_tiles(B, n_active, 128, 128) >= 256) tile = SRIGL_TILE_128x128;
        else tile = SRIGL_TILE_64x64;
    }
    switch (tile) {
        case SRIGL_TILE_256x256: return launch_gemm<T, 256, 256, 2, 4, 2>(x, B, d_in, Wd, active, n_active, bias, d_out, y, st);
        case SRIGL_TILE_256x256_W4: return launch_gemm<T, 256, 256, 2, 2, 2>(x, B, d_in, Wd, active, n_active, bias, d_out, y, st);
        case SRIGL_TILE_256x128: return launch_gemm<T, 256, 128, 2, 2, 3>(x, B, d_in, Wd, active, n_active, bias, d_out, y, st);
        case SRIGL_TILE_128x128: return launch_gemm<T, 128, 128, 2, 2, 2>(x, B, d_in, Wd, active, n_active, bias, d_out, y, st);
        case SRIGL_TILE_128x128_S4: return launch_gemm<T, 128, 128, 2, 2, 4>(x, B, d_in, Wd, active, n_active, bias, d_out, y, st);
        case SRIGL_TILE_64x64: return launch_gemm<T, 64, 64, 2, 2, 4>(x, B, d_in, Wd, active, n_active, bias, d_out, y, st);
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

srigl_status srigl_structured_linear_fwd_tile(const void* x, srigl_dtype x_dtype, int32_t B, int32_t d_in, const void* Wd,
                                              srigl_dtype w_dtype, const int32_t* active, int32_t n_active,
                                              const float* bias, int32_t d_out, float* y, srigl_gemm_tile tile, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (B < 0 || d_in < 0 || n_active < 0 || d_out < 0 || n_active > d_out) return SRIGL_ERR_INVALID_ARG;
    if ((x_dtype != SRIGL_F32 && x_dtype != SRIGL_BF16) || (w_dtype != SRIGL_F32 && w_dtype != SRIGL_BF16)) return SRIGL_ERR_INVALID_ARG;
    if (x_dtype != w_dtype) return SRIGL_ERR_UNSUPPORTED;
    if (active == nullptr && n_active != d_out && n_active != 0) return SRIGL_ERR_INVALID_ARG;
    if (B == 0 || d_out == 0) return SRIGL_OK;
    if (y == nullptr) return SRIGL_ERR_INVALID_ARG;
    if (n_active > 0 && d_in > 0 && (x == nullptr || Wd == nullptr)) return SRIGL_ERR_INVALID_ARG;
    const int elem = (x_dtype == SRIGL_F32) ? 4 : 2;
    if (n_active > 0 && d_in > 0) {
        if ((d_in * elem) % 16 != 0 || ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(Wd)) & 15) != 0)
            return SRIGL_ERR_UNSUPPORTED;
    }
    // ablated columns (and everything, when nothing is stored)
    if (active != nullptr || n_active == 0) {
        long long blocks = ((long long)B * (n_active + 1) + 255) / 256;
        if (blocks > 65536) blocks = 65536;
        hipLaunchKernelGGL(k_fill_ablated, dim3((unsigned)blocks), dim3(256), 0, st, active, n_active, bias, B, d_out, y);
    }
    if (n_active == 0) return hip_ok(hipGetLastError());
    if (x_dtype == SRIGL_F32) return launch_structured<float>(tile, x, B, d_in, Wd, active, n_active, bias, d_out, y, st);
    return launch_structured<uint16_t>(tile, x, B, d_in, Wd, active, n_active, bias, d_out, y, st);
}

srigl_status srigl_structured_linear_fwd(const void* x, srigl_dtype x_dtype, int32_t B, int32_t d_in, const void* Wd,
                                         srigl_dtype w_dtype, const int32_t* active, int32_t n_active,
                                         const float* bias, int32_t d_out, float* y, void* stream) {
    return srigl_structured_linear_fwd_tile(x, x_dtype, B, d_in, Wd, w_dtype, active, n_active, bias, d_out, y, SRIGL_TILE_AUTO, stream);
}

}  // extern "C"
