// Width reduction of an MLP block (gfx950).  Neuron ablation reduces the width of a layer (Sec. 3.1 of arXiv 2305.02299):
// when the first linear layer of a block has ablated neurons, their outputs are the constants act(bias), and the second
// layer can read the compact vector of the stored neurons' outputs instead of the full-width one.  srigl_fold_ablated_inputs
// rewrites the second layer's condensed arrays for that: an index naming stored neuron active1[p] becomes p, a term on an
// ablated neuron moves into the bias of its row's neuron, and the row is filled up to K2 entries again with the smallest
// positions it does not use, weight zero, in ascending order: it stays a constant fan-in row (App. E layout).
#include "srigl_internal.h"

namespace srigl {

constexpr size_t kFoldLdsBudget = 144 * 1024;

__global__ __launch_bounds__(256) void k_copy_f32(const float* __restrict__ src, float* __restrict__ dst, int n) {
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) dst[i] = src ? src[i] : 0.0f;
}

// The first layer of a folded pair writes its stored neurons only, next to each other: position p holds neuron active1[p],
// bias_compact[p] = bias1[active1[p]] (zero at the padding positions p >= n_active1), active_compact[p] = p.
__global__ __launch_bounds__(256) void k_compact_hidden(const float* __restrict__ bias1, const int32_t* __restrict__ active1, int n_active1,
                                                        int d_hidden, int width, float* __restrict__ bias_compact,
                                                        int32_t* __restrict__ active_compact) {
    for (int p = blockIdx.x * blockDim.x + threadIdx.x; p < width; p += gridDim.x * blockDim.x) {
        float b = 0.0f;
        if (p < n_active1 && bias1) {
            const int j = active1 ? active1[p] : p;
            if (j >= 0 && j < d_hidden) b = bias1[j];
        }
        if (bias_compact) bias_compact[p] = b;
        if (active_compact && p < n_active1) active_compact[p] = p;
    }
}

// One wavefront per stored row of the second layer; all LDS traffic stays inside the wavefront.
// LDS per wavefront: V[K2] (compact positions of the kept terms, ascending), Wv[K2] (their weight bits),
// Io[K2] / Wo[K2] (the output row).
template <typename T>
__global__ void k_fold_rows(const int32_t* __restrict__ idx2, const T* __restrict__ W_c2, const float* __restrict__ bias2,
                            const int32_t* __restrict__ active2, int n2, int K2, int d_out2, const int32_t* __restrict__ active1,
                            int n_active1, int d_hidden, const float* __restrict__ bias1, int act, int32_t* __restrict__ idx_out,
                            T* __restrict__ W_out, float* __restrict__ bias_out) {
    extern __shared__ int32_t fold_lds[];
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x >> 6;
    const int n = blockIdx.x * (blockDim.x >> 6) + wv;
    if (n >= n2) return;
    int32_t* V = fold_lds + (size_t)wv * 4 * K2;
    uint32_t* Wv = reinterpret_cast<uint32_t*>(V + K2);
    int32_t* Io = V + 2 * K2;
    uint32_t* Wo = reinterpret_cast<uint32_t*>(V + 3 * K2);
    const size_t row = (size_t)n * K2;

    // kept terms -> (position among the stored neurons, weight bits), compacted in order; the others add to the constant
    int m = 0;
    float constant = 0.0f;
    for (int k0 = 0; k0 < K2; k0 += kWave) {
        const int k = k0 + lane;
        bool kept = false;
        int p = -1;
        uint32_t bits = 0;
        if (k < K2) {
            const int j = idx2[row + k];
            bits = (uint32_t)W_c2[row + k];
            if (j >= 0 && j < d_hidden) {
                if (active1 == nullptr) {
                    kept = true;
                    p = j;
                } else {
                    int lo = 0, hi = n_active1;   // first entry >= j
                    while (lo < hi) {
                        const int mid = (lo + hi) >> 1;
                        if (active1[mid] < j) lo = mid + 1; else hi = mid;
                    }
                    kept = lo < n_active1 && active1[lo] == j;
                    p = lo;
                }
                if (!kept) {
                    const float w = sizeof(T) == 4 ? __uint_as_float(bits) : bf16_bits_to_float(bits);
                    constant = fmaf(w, apply_act(bias1 ? bias1[j] : 0.0f, act), constant);
                }
            }
        }
        const unsigned long long vote = __ballot(kept);
        if (kept) {
            const int at = m + __builtin_amdgcn_mbcnt_hi((unsigned)(vote >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)vote, 0));
            V[at] = p;
            Wv[at] = bits;
        }
        m += __popcll(vote);
    }
    for (int off = kWave / 2; off > 0; off >>= 1) constant += __shfl_xor(constant, off, kWave);
    if (lane == 0) {
        const int col = active2 ? active2[n] : n;
        if (col >= 0 && col < d_out2) bias_out[col] = (bias2 ? bias2[col] : 0.0f) + constant;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();

    // f fillers are needed: the f smallest positions not in V.  With r* = the first rank whose entry has at least f
    // unused positions below it (V[r] - r >= f; V[r] - r never decreases), the largest filler is G = f - 1 + r*, and the
    // output row is 0, 1, ..., G followed by V[r*], V[r* + 1], ...
    const int f = K2 - m;
    int rstar = m;
    for (int r0 = 0; r0 < m && rstar == m; r0 += kWave) {
        const int r = r0 + lane;
        const bool hit = r < m && V[r] - r >= f;
        const unsigned long long vote = __ballot(hit);
        if (vote) rstar = r0 + __builtin_ctzll(vote);
    }
    const int G = f - 1 + rstar;
    for (int p = lane; p <= G; p += kWave) { Io[p] = p; Wo[p] = 0u; }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    for (int r = lane; r < rstar; r += kWave) Wo[V[r]] = Wv[r];           // kept terms inside the prefix
    for (int r = rstar + lane; r < m; r += kWave) {                       // kept terms past the prefix
        Io[G + 1 + (r - rstar)] = V[r];
        Wo[G + 1 + (r - rstar)] = Wv[r];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    for (int k = lane; k < K2; k += kWave) {
        idx_out[row + k] = Io[k];
        W_out[row + k] = (T)Wo[k];
    }
}

// ------------------------------------------------------------------------------------------------
// Both linear layers of an MLP block in one launch, for online inference and very small batches (App. H's block:
// linear, activation, linear).  256 workgroups, all resident at once.  Phase 1: every workgroup computes its share of
// layer 1's neurons (small-batch kernel on the streaming copy: L lanes per stored row, four terms per lane and unit) and
// writes them to the hidden vector in global memory.  Grid barrier.  Phase 2: its share of layer 2 from the hidden vector.
//
// The hidden vector crosses compute units and XCDs inside one launch, so it is written and read with agent-scope
// accesses (they go past the per-XCD L2), every wavefront waits for its own stores before the workgroup arrives at the
// barrier, and the barrier is one counter in device memory: an arrival adds 1 and waits until the count reaches the next
// multiple of the grid size (every launch adds exactly the grid size, so the counter is never reset).  The wait is
// bounded: after spin_limit polls a workgroup gives up, flags the call as failed and goes on, so every wavefront exits.
// ------------------------------------------------------------------------------------------------
constexpr int kMlpGrid = 256;
static __device__ unsigned int g_mlp_arrivals;   // arrivals of all launches so far on this device

__device__ __forceinline__ float load_agent(const float* p) {
    return __uint_as_float(__hip_atomic_load(reinterpret_cast<const unsigned int*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}
__device__ __forceinline__ void store_agent(float* p, float v) {
    __hip_atomic_store(reinterpret_cast<unsigned int*>(p), __float_as_uint(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Slots [s_begin, s_end) of one layer (a slot is a stored row plus the gap of ablated columns in front of it; slot n_active
// is the tail gap) for RB batch rows.  ACROSS: the input was written by other workgroups of this launch / the output is read
// by them.
template <int RB, bool IN_ACROSS, bool OUT_ACROSS>
__device__ __forceinline__ void mlp_layer_slots(const float* __restrict__ xin, int B, int d_in, const unsigned char* __restrict__ packed,
                                                int K, const int32_t* __restrict__ active, int n_active, const float* __restrict__ bias,
                                                int d_out, float* __restrict__ yout, int log2L, int s_begin, int s_end, int act) {
    const int L = 1 << log2L;
    const int q = threadIdx.x & (L - 1), grp = threadIdx.x >> log2L, groups = blockDim.x >> log2L;
    const int units = (K + 3) / 4;
    const size_t row_bytes = (size_t)units * 32;
    auto put = [&](int b, int c, float v) {
        if (OUT_ACROSS) store_agent(yout + (size_t)b * d_out + c, v); else yout[(size_t)b * d_out + c] = v;
    };
    for (int s = s_begin + grp; s < s_end; s += groups) {
        float acc[RB];
#pragma unroll
        for (int r = 0; r < RB; ++r) acc[r] = 0.0f;
        if (s < n_active) {
            const unsigned char* row = packed + (size_t)s * row_bytes;
            for (int u = q; u < units; u += L) {
                PackedUnit<float, 32> un;
                un.load(row + (size_t)u * 32);
                float xg[4][RB];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int c = min(max(un.col(t), 0), d_in - 1);
#pragma unroll
                    for (int r = 0; r < RB; ++r) {
                        const float* px = xin + (size_t)min(r, B - 1) * d_in + c;
                        xg[t][r] = IN_ACROSS ? load_agent(px) : *px;
                    }
                }
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    if (4 * u + t < K) {
                        const float wv = un.weight(t);
#pragma unroll
                        for (int r = 0; r < RB; ++r) acc[r] = fmaf(wv, xg[t][r], acc[r]);
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
            for (int c = max(prev + 1, 0) + q; c < col; c += L) {
                const float bv = apply_act(bias ? bias[c] : 0.0f, act);
#pragma unroll
                for (int r = 0; r < RB; ++r)
                    if (r < B) put(r, c, bv);
            }
        }
        if (q == 0 && s < n_active && col >= 0 && col < d_out) {
            const float bv = bias ? bias[col] : 0.0f;
#pragma unroll
            for (int r = 0; r < RB; ++r)
                if (r < B) put(r, col, apply_act(acc[r] + bv, act));
        }
    }
}

template <int RB>
__global__ __launch_bounds__(256) void k_mlp_fused(const float* __restrict__ x, int B, int d_in, const unsigned char* __restrict__ packed1, int K1,
                                                   const int32_t* __restrict__ active1, int n1, const float* __restrict__ bias1, int d_hidden,
                                                   float* __restrict__ hidden, int act, const unsigned char* __restrict__ packed2, int K2,
                                                   const int32_t* __restrict__ active2, int n2, const float* __restrict__ bias2, int d_out,
                                                   float* __restrict__ y, int log2L1, int log2L2, int spin_limit, int32_t* __restrict__ status) {
    __shared__ int s_ok;
    const int wg = blockIdx.x;
    {   // phase 1: an equal share of layer 1's slots per workgroup
        const int n_slots = active1 ? n1 + 1 : n1;
        const int per = (n_slots + kMlpGrid - 1) / kMlpGrid;
        mlp_layer_slots<RB, false, true>(x, B, d_in, packed1, K1, active1, n1, bias1, d_hidden, hidden, log2L1, wg * per,
                                         min((wg + 1) * per, n_slots), act);
    }
    // every wavefront: its stores of the hidden vector have completed before the workgroup arrives
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned int t = __hip_atomic_fetch_add(&g_mlp_arrivals, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const unsigned int target = (t / kMlpGrid + 1u) * kMlpGrid;
        int ok = 1, polls = 0;
        while ((int)(__hip_atomic_load(&g_mlp_arrivals, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - target) < 0) {
            if (++polls > spin_limit) { ok = 0; break; }
            __builtin_amdgcn_s_sleep(2);
        }
        s_ok = ok;
        if (!ok && status) __hip_atomic_store(status, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    (void)s_ok;   // a workgroup that gave up still computes its share (from whatever the hidden vector holds) and exits
    {   // phase 2
        const int n_slots = active2 ? n2 + 1 : n2;
        const int per = (n_slots + kMlpGrid - 1) / kMlpGrid;
        mlp_layer_slots<RB, true, false>(hidden, B, d_hidden, packed2, K2, active2, n2, bias2, d_out, y, log2L2, wg * per,
                                         min((wg + 1) * per, n_slots), SRIGL_ACT_NONE);
    }
}

}  // namespace srigl

using namespace srigl;

extern "C" {

srigl_status srigl_fold_ablated_inputs(const int32_t* idx2, const void* W_c2, srigl_dtype w_dtype, const float* bias2,
                                       const int32_t* active2, int32_t n2, int32_t K2, int32_t d_out2, const int32_t* active1,
                                       int32_t n_active1, int32_t d_hidden, const float* bias1, srigl_activation act,
                                       int32_t* idx_out, void* W_out, float* bias_out, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (n2 < 0 || K2 < 0 || d_out2 < 0 || n_active1 < 0 || d_hidden < 0 || n2 > d_out2 || n_active1 > d_hidden) return SRIGL_ERR_INVALID_ARG;
    if (w_dtype != SRIGL_F32 && w_dtype != SRIGL_BF16) return SRIGL_ERR_INVALID_ARG;
    if (act != SRIGL_ACT_NONE && act != SRIGL_ACT_RELU && act != SRIGL_ACT_GELU) return SRIGL_ERR_INVALID_ARG;
    if (active1 == nullptr && n_active1 != d_hidden) return SRIGL_ERR_INVALID_ARG;
    if (active2 == nullptr && n2 != d_out2 && n2 != 0) return SRIGL_ERR_INVALID_ARG;
    if (d_out2 > 0 && bias_out == nullptr) return SRIGL_ERR_INVALID_ARG;
    if (n2 > 0 && K2 > 0 && (idx2 == nullptr || W_c2 == nullptr || idx_out == nullptr || W_out == nullptr)) return SRIGL_ERR_INVALID_ARG;
    if (K2 > n_active1) return SRIGL_ERR_UNSUPPORTED;   // no room for K2 distinct positions
    if (d_out2 > 0) {
        int blocks = (d_out2 + 255) / 256;
        if (blocks > 4096) blocks = 4096;
        hipLaunchKernelGGL(k_copy_f32, dim3(blocks), dim3(256), 0, st, bias2, bias_out, d_out2);
    }
    if (n2 == 0 || K2 == 0) return hip_ok(hipGetLastError());
    const size_t per_wave = (size_t)16 * K2;
    if (per_wave > kFoldLdsBudget) return SRIGL_ERR_UNSUPPORTED;
    int waves = (int)(kFoldLdsBudget / per_wave);
    if (waves > 4) waves = 4;
    const size_t lds = per_wave * waves;
    const unsigned blocks = (unsigned)((n2 + waves - 1) / waves);
    if (w_dtype == SRIGL_F32) {
        auto kern = k_fold_rows<uint32_t>;
        if (lds > 64 * 1024 && hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)kFoldLdsBudget) != hipSuccess)
            return SRIGL_ERR_HIP;
        hipLaunchKernelGGL(kern, dim3(blocks), dim3(waves * kWave), lds, st, idx2, static_cast<const uint32_t*>(W_c2), bias2, active2, n2, K2,
                           d_out2, active1, n_active1, d_hidden, bias1, (int)act, idx_out, static_cast<uint32_t*>(W_out), bias_out);
    } else {
        auto kern = k_fold_rows<uint16_t>;
        if (lds > 64 * 1024 && hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)kFoldLdsBudget) != hipSuccess)
            return SRIGL_ERR_HIP;
        hipLaunchKernelGGL(kern, dim3(blocks), dim3(waves * kWave), lds, st, idx2, static_cast<const uint16_t*>(W_c2), bias2, active2, n2, K2,
                           d_out2, active1, n_active1, d_hidden, bias1, (int)act, idx_out, static_cast<uint16_t*>(W_out), bias_out);
    }
    return hip_ok(hipGetLastError());
}

srigl_status srigl_compact_hidden_layer(const float* bias1, const int32_t* active1, int32_t n_active1, int32_t d_hidden, int32_t width,
                                        float* bias_compact, int32_t* active_compact, void* stream) {
    if (n_active1 < 0 || d_hidden < 0 || width < n_active1 || n_active1 > d_hidden) return SRIGL_ERR_INVALID_ARG;
    if (active1 == nullptr && n_active1 != d_hidden) return SRIGL_ERR_INVALID_ARG;
    if (width == 0 || (bias_compact == nullptr && active_compact == nullptr)) return SRIGL_OK;
    int blocks = (width + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(k_compact_hidden, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream), bias1, active1, n_active1, d_hidden,
                       width, bias_compact, active_compact);
    return hip_ok(hipGetLastError());
}

srigl_status srigl_condensed_mlp_fwd(const float* x, int32_t B, int32_t d_in, const void* packed1, const int32_t* active1, int32_t n_active1,
                                     int32_t K1, const float* bias1, int32_t d_hidden, srigl_activation act, float* hidden,
                                     const void* packed2, const int32_t* active2, int32_t n_active2, int32_t K2, const float* bias2,
                                     int32_t d_out, float* y, int32_t spin_limit, int32_t* status_dev, void* stream) {
    if (B < 0 || d_in < 0 || n_active1 < 0 || K1 < 0 || d_hidden < 0 || n_active2 < 0 || K2 < 0 || d_out < 0) return SRIGL_ERR_INVALID_ARG;
    if (K1 > d_in || K2 > d_hidden || n_active1 > d_hidden || n_active2 > d_out) return SRIGL_ERR_INVALID_ARG;
    if (act != SRIGL_ACT_NONE && act != SRIGL_ACT_RELU && act != SRIGL_ACT_GELU) return SRIGL_ERR_INVALID_ARG;
    if ((active1 == nullptr && n_active1 != d_hidden && n_active1 != 0) || (active2 == nullptr && n_active2 != d_out && n_active2 != 0))
        return SRIGL_ERR_INVALID_ARG;
    if (B > 8) return SRIGL_ERR_UNSUPPORTED;                    // larger batches: two calls of the batched kernel
    if (B == 0 || d_out == 0) return SRIGL_OK;
    if (n_active1 == 0 || K1 == 0 || n_active2 == 0 || K2 == 0 || d_hidden == 0) return SRIGL_ERR_UNSUPPORTED;   // a layer without terms: two calls
    if (x == nullptr || packed1 == nullptr || packed2 == nullptr || hidden == nullptr || y == nullptr) return SRIGL_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(packed1) | reinterpret_cast<uintptr_t>(packed2)) % 16 != 0) return SRIGL_ERR_INVALID_ARG;
    if (spin_limit <= 0) spin_limit = 1 << 20;
    auto log2_lanes = [](int K) { int L = klane_lanes(K), l = 0; while ((1 << (l + 1)) <= L) ++l; return l; };
    hipStream_t st = static_cast<hipStream_t>(stream);
#define SRIGL_MLP(RBV)                                                                                                          \
    hipLaunchKernelGGL(k_mlp_fused<RBV>, dim3(kMlpGrid), dim3(256), 0, st, x, B, d_in, static_cast<const unsigned char*>(packed1), K1, \
                       active1, n_active1, bias1, d_hidden, hidden, (int)act, static_cast<const unsigned char*>(packed2), K2, active2, \
                       n_active2, bias2, d_out, y, log2_lanes(K1), log2_lanes(K2), spin_limit, status_dev)
    if (B == 1) SRIGL_MLP(1); else if (B == 2) SRIGL_MLP(2); else if (B <= 4) SRIGL_MLP(4); else SRIGL_MLP(8);
#undef SRIGL_MLP
    return hip_ok(hipGetLastError());
}

}  // extern "C"
