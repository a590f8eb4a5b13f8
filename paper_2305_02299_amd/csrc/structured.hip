// Structured-only representation (gfx950): the stored neurons of a layer trained with SRigL keep dense rows
// (ablated neurons removed, fine-grained sparsity not exploited; Sec. 4.4, Fig. 4 and App. H of arXiv
// 2305.02299), and the forward pass is a dense product on the matrix cores,
//     y[b][active[s]] = bias[active[s]] + sum_j Wd[s][j] * x[b][j].
//
// The product is an "NT" GEMM: both operands are K-contiguous (x[b][:], Wd[s][:]).  A workgroup of 4
// wavefronts owns a BM x BN output tile and walks d_in in slabs of 128 bytes per row (64 bf16 or 32 fp32),
// double-buffered in LDS: the next slab's global loads are issued into registers before the MFMAs of the current
// one.  LDS rows are 144 bytes apart (128 + 16): the 16-byte reads of 16 consecutive rows then fall on disjoint
// bank groups.  A wavefront owns (BM/2) x (BN/2) of the tile as 32x32 MFMA blocks:
//   bf16: v_mfma_f32_32x32x16_bf16, lane l holds row l%32 and the 8 consecutive k of group l/32;
//   fp32: v_mfma_f32_32x32x2_f32, lane l holds row l%32, k = l/32; the lane's 16-byte read carries 4 consecutive k
//         of its group, used by 4 successive MFMAs (both operands use the same k-to-slot map, so the sum is over
//         matching k whatever the order).
// Result block layout: accumulator register i of lane l is row 8*(i/4) + 4*(l/32) + i%4, column l%32.
#include "srigl_internal.h"

namespace srigl {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kSlabBytes = 128;           // bytes of K per row and slab
constexpr int kRowBytes = kSlabBytes + 16; // LDS row pitch

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

// BM x BN output tile per workgroup (256 threads = 2 x 2 wavefronts), TM = BM/64, TN = BN/64 MFMA blocks per wavefront and side
template <typename T, int BM, int BN>
__global__ __launch_bounds__(256) void k_structured_gemm(const T* __restrict__ x, int B, int d_in, const T* __restrict__ Wd,
                                                         const int32_t* __restrict__ active, int n_active,
                                                         const float* __restrict__ bias, int d_out, float* __restrict__ y) {
    extern __shared__ unsigned char smem[];   // [2][(BM + BN) rows][kRowBytes]
    using F = typename Frag<T>::type;
    constexpr int EPS = kSlabBytes / (int)sizeof(T);   // elements of K per slab
    constexpr int TM = BM / 64, TN = BN / 64;
    constexpr int ROWS = BM + BN;
    constexpr int PASSES = ROWS * 8 / 256;             // 16-byte vectors per thread and slab (8 per row)
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int wm = wv >> 1, wn = wv & 1;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;

    // staging map: vector v = tid + 256 * p -> (row v / 8, 16-byte column v % 8); rows < BM come from x, the rest from Wd;
    // rows past the matrix re-read its last row (their results are never stored)
    const T* src[PASSES];
    int dst[PASSES];
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        const int v = tid + 256 * p;
        const int row = v >> 3, c16 = v & 7;
        const T* base = (row < BM) ? x + (size_t)min(m0 + row, B - 1) * d_in : Wd + (size_t)min(n0 + row - BM, n_active - 1) * d_in;
        src[p] = base + c16 * (16 / (int)sizeof(T));
        dst[p] = row * kRowBytes + c16 * 16;
    }
    const int n_slabs = (d_in + EPS - 1) / EPS;
    uint4 st[PASSES];
    auto load_slab = [&](int sl) {
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            const int c16 = (tid + 256 * p) & 7;
            const int k = sl * EPS + c16 * (16 / (int)sizeof(T));
            st[p] = (k < d_in) ? *reinterpret_cast<const uint4*>(src[p] + (size_t)sl * EPS) : uint4{0u, 0u, 0u, 0u};   // d_in is a multiple of 16 bytes
        }
    };
    auto store_slab = [&](int buf) {
#pragma unroll
        for (int p = 0; p < PASSES; ++p) *reinterpret_cast<uint4*>(smem + (size_t)buf * ROWS * kRowBytes + dst[p]) = st[p];
    };

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    load_slab(0);
    store_slab(0);
    __syncthreads();
    const int frag_off = (lane & 31) * kRowBytes + (lane >> 5) * 16;
    for (int sl = 0; sl < n_slabs; ++sl) {
        const unsigned char* buf = smem + (size_t)(sl & 1) * ROWS * kRowBytes;
        if (sl + 1 < n_slabs) load_slab(sl + 1);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            F a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) a[i] = *reinterpret_cast<const F*>(buf + (wm * (BM / 2) + i * 32) * kRowBytes + frag_off + kk * 32);
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = *reinterpret_cast<const F*>(buf + (BM + wn * (BN / 2) + j * 32) * kRowBytes + frag_off + kk * 32);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) mma_block(acc[i][j], a[i], b[j]);
        }
        if (sl + 1 < n_slabs) {
            store_slab((sl + 1) & 1);   // the other buffer: its last readers passed the barrier of the previous iteration
            __syncthreads();
        }
    }

    // epilogue: bias and scatter to the stored neurons' columns
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int s = n0 + wn * (BN / 2) + j * 32 + (lane & 31);
        if (s >= n_active) continue;
        const int col = active ? active[s] : s;
        if (col < 0 || col >= d_out) continue;
        const float bv = bias ? bias[col] : 0.0f;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int m = m0 + wm * (BM / 2) + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                if (m < B) y[(size_t)m * d_out + col] = acc[i][j][e] + bv;
            }
        }
    }
}

template <typename T, int BM, int BN>
static srigl_status launch_gemm(const void* x, int B, int d_in, const void* Wd, const int32_t* active, int n_active, const float* bias,
                                int d_out, float* y, hipStream_t st) {
    auto kern = k_structured_gemm<T, BM, BN>;
    const size_t lds = (size_t)2 * (BM + BN) * kRowBytes;
    static bool raised = false;
    if (lds > 64 * 1024 && !raised) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return SRIGL_ERR_HIP;
        raised = true;
    }
    const dim3 grid((unsigned)((n_active + BN - 1) / BN), (unsigned)((B + BM - 1) / BM));
    if (grid.y > 65535u) return SRIGL_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, st, (const T*)x, B, d_in, (const T*)Wd, active, n_active, bias, d_out, y);
    return hip_ok(hipGetLastError());
}

template <typename T>
static srigl_status launch_structured(const void* x, int B, int d_in, const void* Wd, const int32_t* active, int n_active,
                                      const float* bias, int d_out, float* y, hipStream_t st) {
    // large tiles when they still give every CU a workgroup, small ones otherwise
    const long long big = (long long)((n_active + 127) / 128) * ((B + 127) / 128);
    if (big >= 256) return launch_gemm<T, 128, 128>(x, B, d_in, Wd, active, n_active, bias, d_out, y, st);
    return launch_gemm<T, 64, 64>(x, B, d_in, Wd, active, n_active, bias, d_out, y, st);
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

srigl_status srigl_structured_linear_fwd(const void* x, srigl_dtype x_dtype, int32_t B, int32_t d_in, const void* Wd,
                                         srigl_dtype w_dtype, const int32_t* active, int32_t n_active,
                                         const float* bias, int32_t d_out, float* y, void* stream) {
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
    if (x_dtype == SRIGL_F32) return launch_structured<float>(x, B, d_in, Wd, active, n_active, bias, d_out, y, st);
    return launch_structured<uint16_t>(x, B, d_in, Wd, active, n_active, bias, d_out, y, st);
}

}  // extern "C"
