// The unstructured comparison of Sec. 4.4 / Fig. 4 of arXiv 2305.02299 on the same GPU: the layer's kept weights in
// compressed sparse row form, y[b][r] = bias[r] + sum over row r's entries of value * x[b][column].  The kernel has the
// shape of the small-batch condensed kernel (activations gathered from global memory or from RB rows of x staged in LDS,
// by the same rule; L lanes share one row of the matrix and take its entries L apart, partial sums meet in a butterfly of
// cross-lane shuffles); what differs is what the format forces: a row's extent comes from row_ptr (one more dependent
// load per row) and rows differ in length.
#include "srigl_internal.h"
#include <algorithm>

namespace srigl {

template <typename XT> __device__ __forceinline__ float csr_to_f32(XT v);
template <> __device__ __forceinline__ float csr_to_f32<float>(float v) { return v; }

constexpr int kCsrTerms = 4;   // entries a lane keeps in flight per request

template <int RB, bool GATHER, typename XT>
__global__ __launch_bounds__(256) void k_fwd_csr(const XT* __restrict__ x, int B, int d_in, const XT* __restrict__ values,
                                                 const int32_t* __restrict__ col_idx, const int32_t* __restrict__ row_ptr,
                                                 const float* __restrict__ bias, int d_out, float* __restrict__ y, int log2L,
                                                 int rows_per_wg, int act) {
    extern __shared__ float xs[];   // [RB][d_in]; unused when GATHER
    const int L = 1 << log2L;
    const int tid = threadIdx.x;
    const int q = tid & (L - 1);
    const int grp = tid >> log2L;
    const int groups = blockDim.x >> log2L;
    const int b0 = blockIdx.y * RB;
    const int s_begin = blockIdx.x * rows_per_wg;
    const int s_end = min(s_begin + rows_per_wg, d_out);
    int s = s_begin + grp;
    int beg = 0, end = 0;
    if (s < s_end) { beg = row_ptr[s]; end = row_ptr[s + 1]; }   // in flight while x is staged

    if (!GATHER) {
        for (int r = 0; r < RB; ++r) {
            const XT* xr = x + (size_t)min(b0 + r, B - 1) * d_in;   // rows past B re-read the last row; they are never stored
            for (int j0 = tid; j0 < d_in; j0 += 4 * (int)blockDim.x) {   // four loads in flight before the first is stored
                XT v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) v[u] = xr[min(j0 + u * (int)blockDim.x, d_in - 1)];
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (j0 + u * (int)blockDim.x < d_in) xs[r * d_in + j0 + u * (int)blockDim.x] = csr_to_f32<XT>(v[u]);
            }
        }
        __syncthreads();
    }

    for (; s < s_end; s += groups) {
        float acc[RB];
#pragma unroll
        for (int r = 0; r < RB; ++r) acc[r] = 0.0f;
        const int sn = s + groups;
        int nbeg = 0, nend = 0;
        if (sn < s_end) { nbeg = row_ptr[sn]; nend = row_ptr[sn + 1]; }   // the next row's extent, ahead of its use
        for (int t = beg + q; t < end; t += kCsrTerms * L) {
            XT w[kCsrTerms];
            int c[kCsrTerms];
#pragma unroll
            for (int j = 0; j < kCsrTerms; ++j) {        // unconditional loads (entry index clamped into the row)
                const int tt = min(t + j * L, end - 1);
                w[j] = values[tt];
                c[j] = col_idx[tt];
            }
            if (GATHER) {
                // a column outside [0, d_in) must not become an address outside x
#pragma unroll
                for (int j = 0; j < kCsrTerms; ++j) c[j] = min(max(c[j], 0), d_in - 1);
                XT xg[kCsrTerms][RB];
#pragma unroll
                for (int j = 0; j < kCsrTerms; ++j)
#pragma unroll
                    for (int r = 0; r < RB; ++r) xg[j][r] = x[(size_t)min(b0 + r, B - 1) * d_in + c[j]];
#pragma unroll
                for (int j = 0; j < kCsrTerms; ++j) {
                    if (t + j * L < end) {
                        const float wv = csr_to_f32<XT>(w[j]);
#pragma unroll
                        for (int r = 0; r < RB; ++r) acc[r] = fmaf(wv, csr_to_f32<XT>(xg[j][r]), acc[r]);
                    }
                }
            } else {
#pragma unroll
                for (int j = 0; j < kCsrTerms; ++j) {
                    if (t + j * L < end) {
                        const float wv = csr_to_f32<XT>(w[j]);
#pragma unroll
                        for (int r = 0; r < RB; ++r) acc[r] = fmaf(wv, xs[r * d_in + c[j]], acc[r]);
                    }
                }
            }
        }
        for (int off = L >> 1; off > 0; off >>= 1) {
#pragma unroll
            for (int r = 0; r < RB; ++r) acc[r] += __shfl_xor(acc[r], off, kWave);
        }
        if (q == 0) {
            const float bv = bias ? bias[s] : 0.0f;
#pragma unroll
            for (int r = 0; r < RB; ++r)
                if (b0 + r < B) y[(size_t)(b0 + r) * d_out + s] = apply_act(acc[r] + bv, act);
        }
        beg = nbeg;
        end = nend;
    }
}

template <int RB, bool GATHER, typename XT>
static srigl_status launch_csr(const void* x, int B, int d_in, const void* values, const int32_t* col_idx, const int32_t* row_ptr,
                               const float* bias, int d_out, float* y, int log2L, int act, hipStream_t st) {
    const size_t lds = GATHER ? 0 : (size_t)RB * d_in * sizeof(float);
    if (lds > kLdsMax) return SRIGL_ERR_UNSUPPORTED;
    auto kern = k_fwd_csr<RB, GATHER, XT>;
    static LdsLimit lds_limit;
    if (lds_limit.ensure(kern, lds) != SRIGL_OK) return SRIGL_ERR_HIP;
    const int groups = 256 >> log2L;
    const int gy = (B + RB - 1) / RB;
    if (gy > 65535) return SRIGL_ERR_UNSUPPORTED;
    // rows per workgroup: one pass of all groups, more when that still leaves > 8 (gathering: 32) workgroups per CU
    int rows_per_wg = groups;
    // (a batch of more row blocks than that keeps the limit out of reach: one pass over all rows per workgroup then)
    while (rows_per_wg < d_out && (long long)((d_out + rows_per_wg - 1) / rows_per_wg) * gy > 256 * (GATHER ? 32 : 8)) rows_per_wg += groups;
    const unsigned gx = (unsigned)((d_out + rows_per_wg - 1) / rows_per_wg);
    hipLaunchKernelGGL(kern, dim3(gx, (unsigned)gy), dim3(256), lds, st, (const XT*)x, B, d_in, (const XT*)values, col_idx, row_ptr,
                       bias, d_out, y, log2L, rows_per_wg, act);
    return hip_ok(hipGetLastError());
}

}  // namespace srigl

using namespace srigl;

extern "C" srigl_status srigl_csr_linear_fwd(const void* x, srigl_dtype x_dtype, int32_t B, int32_t d_in, const void* values,
                                             srigl_dtype w_dtype, const int32_t* col_idx, const int32_t* row_ptr, int64_t nnz,
                                             const float* bias, int32_t d_out, float* y, srigl_activation act, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (act != SRIGL_ACT_NONE && act != SRIGL_ACT_RELU && act != SRIGL_ACT_GELU) return SRIGL_ERR_INVALID_ARG;
    if (B < 0 || d_in < 0 || d_out < 0 || nnz < 0 || nnz > (int64_t)d_out * d_in || nnz >= (1ll << 31)) return SRIGL_ERR_INVALID_ARG;
    if ((x_dtype != SRIGL_F32 && x_dtype != SRIGL_BF16) || (w_dtype != SRIGL_F32 && w_dtype != SRIGL_BF16)) return SRIGL_ERR_INVALID_ARG;
    if (x_dtype != SRIGL_F32 || w_dtype != SRIGL_F32) return SRIGL_ERR_UNSUPPORTED;   // the comparison is timed in fp32 only
    if (B > 65535) return SRIGL_ERR_UNSUPPORTED;
    if (B == 0 || d_out == 0) return SRIGL_OK;
    if (y == nullptr || row_ptr == nullptr || (d_in > 0 && x == nullptr)) return SRIGL_ERR_INVALID_ARG;
    if (nnz > 0 && (values == nullptr || col_idx == nullptr)) return SRIGL_ERR_INVALID_ARG;
    // lanes per row from the mean row length: a lane has about 4 entries, at least 4 lanes, at most a wavefront
    const long long mean = (nnz + d_out - 1) / d_out;
    int L = 4, log2L = 2;
    while (L < 64 && (long long)L * kCsrTerms < mean) { L <<= 1; ++log2L; }
    // source of the activations and batch rows per workgroup: the rules of the condensed small-batch kernel, with the mean
    // row length in the place of K
    const int K_mean = (int)std::min<long long>(mean, d_in);
    const int direct = klane_gathers(B, d_in, d_out, K_mean) ? 1 : 0;
    const int RB = direct ? klane_gather_rows(B, d_out, K_mean) : klane_stage_rows(B, d_in);
#define SRIGL_CSR(RBV)                                                                                                        \
    return direct ? launch_csr<RBV, true, float>(x, B, d_in, values, col_idx, row_ptr, bias, d_out, y, log2L, (int)act, st)    \
                  : launch_csr<RBV, false, float>(x, B, d_in, values, col_idx, row_ptr, bias, d_out, y, log2L, (int)act, st)
    if (RB == 4) SRIGL_CSR(4);
    if (RB == 2) SRIGL_CSR(2);
    SRIGL_CSR(1);
#undef SRIGL_CSR
}
