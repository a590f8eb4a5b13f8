// One SRigL connectivity update of a layer on the GPU (gfx950): Sec. 3.1 of arXiv 2305.02299, steps 1-7 (prune / grow
// criteria, salient weights per neuron, neuron ablation with threshold gamma_sal, new fan-in k', layer-wide pruning, per-neuron
// regrowth), fp32 weights and gradients, dense [d_out][d_in] storage with a byte mask.  Readings of the text are listed in
// include/srigl.h next to srigl_mask_update.
//
// Every ranking is a selection of the K largest of unique 64-bit keys, (magnitude bits, position): equal magnitudes are
// ordered by position, so the selected set is unique and no sort is needed.  Layer-wide selections (steps 3 and 6) find the
// K-th largest key by a most-significant-digit-first radix walk: 8 passes of (histogram of one byte over the elements that
// match the prefix found so far, pick the byte).  Row-wise selections (step 7) do the same walk inside one workgroup per row.
#include "srigl_internal.h"

namespace srigl {

struct SelState {
    unsigned long long threshold;   // after the walk: the K-th largest key (select key >= threshold)
    unsigned long long k_rem;       // how many of the keys with the current prefix are still wanted
    unsigned long long total;       // number of candidate keys
    int done;                       // the threshold is final (nothing wanted: ~0; everything wanted: 0; or 8 passes walked)
    int pad;
};

struct UpdateScratch {              // head of the workspace
    unsigned int hist[256];
    SelState sel[3];                // 0: smallest kept weights of the layer, 1: largest gradients at pruned positions,
                                    // 2: smallest kept weights of the remaining neurons
    long long k_new, n_remaining, n_ablated_now, n_pruned;
};

__device__ __forceinline__ unsigned int mag_bits(float v) { return __float_as_uint(v) & 0x7fffffffu; }
// larger key = smaller magnitude, then lower position
__device__ __forceinline__ unsigned long long key_small_first(unsigned int mag, unsigned int pos) {
    return ((unsigned long long)(0x7fffffffu - mag) << 32) | (0xffffffffu - pos);
}
// larger key = larger magnitude, then lower position
__device__ __forceinline__ unsigned long long key_large_first(unsigned int mag, unsigned int pos) {
    return ((unsigned long long)mag << 32) | (0xffffffffu - pos);
}

__global__ void k_update_init(UpdateScratch* s, long long K_upd) {
    const int t = threadIdx.x;
    if (t < 256) s->hist[t] = 0;
    if (t < 3) {
        s->sel[t].threshold = 0;
        s->sel[t].k_rem = (unsigned long long)K_upd;
        s->sel[t].total = 0;
        s->sel[t].done = 0;
    }
}

// MODE 0: kept weights, key_small_first(|w|);  1: pruned positions, key_large_first(|grad|);
// MODE 2: kept weights of remaining neurons, key_small_first(|w|)
template <int MODE>
__device__ __forceinline__ bool layer_key(const float* __restrict__ W, const uint8_t* __restrict__ mask, const float* __restrict__ grad,
                                          const int* __restrict__ remains, unsigned int i, int d_in, unsigned long long& key) {
    const bool kept = mask[i] != 0;
    if (MODE == 1) {
        if (kept) return false;
        key = key_large_first(mag_bits(grad[i]), i);
        return true;
    }
    if (!kept) return false;
    if (MODE == 2 && !remains[i / (unsigned)d_in]) return false;
    key = key_small_first(mag_bits(W[i]), i);
    return true;
}

template <int MODE>
__global__ __launch_bounds__(256) void k_layer_hist(const float* __restrict__ W, const uint8_t* __restrict__ mask,
                                                    const float* __restrict__ grad, const int* __restrict__ remains, unsigned int N,
                                                    int d_in, int pass, UpdateScratch* __restrict__ s) {
    __shared__ unsigned int h[256];
    if (s->sel[MODE].done) return;
    h[threadIdx.x] = 0;
    __syncthreads();
    const int shift = 56 - 8 * pass;
    const unsigned long long prefix = s->sel[MODE].threshold;   // the bytes found so far, right-aligned
    for (unsigned long long i = (unsigned long long)blockIdx.x * 256 + threadIdx.x; i < N; i += (unsigned long long)gridDim.x * 256) {
        unsigned long long key;
        if (!layer_key<MODE>(W, mask, grad, remains, (unsigned int)i, d_in, key)) continue;
        if (pass > 0 && (key >> (shift + 8)) != prefix) continue;
        atomicAdd(&h[(unsigned int)(key >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (h[threadIdx.x]) atomicAdd(&s->hist[threadIdx.x], h[threadIdx.x]);
}

// One workgroup of 256 threads: picks the byte of this pass from the histogram and clears it.
__global__ __launch_bounds__(256) void k_layer_pick(int which, int pass, UpdateScratch* __restrict__ s) {
    __shared__ unsigned long long suffix[257];
    const int t = threadIdx.x;
    SelState& st = s->sel[which];
    if (st.done) { s->hist[t] = 0; return; }
    const unsigned int mine = s->hist[t];
    s->hist[t] = 0;
    suffix[t] = mine;
    if (t == 0) suffix[256] = 0;
    __syncthreads();
    // suffix[d] = number of keys whose byte is >= d (Hillis-Steele from the top)
    for (int off = 1; off < 256; off <<= 1) {
        const unsigned long long add = (t + off < 256) ? suffix[t + off] : 0ull;
        __syncthreads();
        suffix[t] += add;
        __syncthreads();
    }
    const unsigned long long want = st.k_rem;
    if (pass == 0 && t == 0) st.total = suffix[0];
    if (pass == 0 && (want == 0 || suffix[0] < want)) {
        __syncthreads();
        if (t == 0) {
            st.threshold = (want == 0) ? ~0ull : 0ull;   // nothing / everything
            st.done = 1;
        }
        return;
    }
    // the byte d with suffix[d] >= want > suffix[d + 1]
    if (suffix[t] >= want && suffix[t + 1] < want) {
        st.threshold = (pass == 0 ? 0ull : (st.threshold << 8)) | (unsigned long long)t;
        st.k_rem = want - suffix[t + 1];
        if (pass == 7) st.done = 1;
    }
}

// Steps 3 and the start of 4: per neuron, how many weights it holds and how many salient ones.  One wavefront per row.
__global__ __launch_bounds__(256) void k_row_salient(const float* __restrict__ W, const uint8_t* __restrict__ mask,
                                                     const float* __restrict__ grad, int d_out, int d_in,
                                                     const UpdateScratch* __restrict__ s, int* __restrict__ held, int* __restrict__ salient) {
    const int lane = threadIdx.x & 63;
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= d_out) return;
    const unsigned long long t_small = s->sel[0].threshold, t_grad = s->sel[1].threshold;
    int h = 0, sal = 0;
    for (int c = lane; c < d_in; c += 64) {
        const unsigned int i = (unsigned int)r * d_in + c;
        if (mask[i]) {
            ++h;
            if (key_small_first(mag_bits(W[i]), i) < t_small) ++sal;    // survives the layer-wide pruning
        } else if (key_large_first(mag_bits(grad[i]), i) >= t_grad) {
            ++sal;                                                        // would be grown
        }
    }
    for (int off = 32; off > 0; off >>= 1) { h += __shfl_xor(h, off, 64); sal += __shfl_xor(sal, off, 64); }
    if (lane == 0) { held[r] = h; salient[r] = sal; }
}

// Steps 4 and 5.  One workgroup.
__global__ __launch_bounds__(1024) void k_decide(const int* __restrict__ held, const int* __restrict__ salient, int d_out, int d_in, int k,
                                                 int gamma_percent, long long budget, int* __restrict__ remains,
                                                 UpdateScratch* __restrict__ s) {
    __shared__ int n_rem, n_abl;
    if (threadIdx.x == 0) { n_rem = 0; n_abl = 0; }
    __syncthreads();
    int rem = 0, abl = 0;
    for (int r = threadIdx.x; r < d_out; r += blockDim.x) {
        int stays = 0;
        if (held[r] > 0) {
            const long long sal = salient[r];
            const bool too_few = sal < 1 || sal * 100 < (long long)gamma_percent * k;
            if (too_few) ++abl; else { stays = 1; ++rem; }
        }
        remains[r] = stays;
    }
    if (rem) atomicAdd(&n_rem, rem);
    if (abl) atomicAdd(&n_abl, abl);
    __syncthreads();
    if (threadIdx.x == 0) {
        long long k_new = n_rem > 0 ? budget / n_rem : 0;
        if (k_new > d_in) k_new = d_in;
        s->k_new = k_new;
        s->n_remaining = n_rem;
        s->n_ablated_now = n_abl;
    }
}

// Radix walk inside one workgroup: the threshold of the `want` largest keys among the row's candidates.
// key_of(c, key) returns whether column c is a candidate.  want >= 1 and at most the number of candidates.
template <typename KeyOf>
__device__ unsigned long long row_select(int d_in, unsigned long long want, KeyOf key_of, unsigned int* h, unsigned long long* suffix,
                                         unsigned long long* shared2) {
    const int t = threadIdx.x;
    unsigned long long prefix = 0;
    for (int pass = 0; pass < 8; ++pass) {
        const int shift = 56 - 8 * pass;
        h[t] = 0;
        __syncthreads();
        for (int c = t; c < d_in; c += 256) {
            unsigned long long key;
            if (!key_of(c, key)) continue;
            if (pass > 0 && (key >> (shift + 8)) != prefix) continue;
            atomicAdd(&h[(unsigned int)(key >> shift) & 255u], 1u);
        }
        __syncthreads();
        suffix[t] = h[t];
        if (t == 0) suffix[256] = 0;
        __syncthreads();
        for (int off = 1; off < 256; off <<= 1) {
            const unsigned long long add = (t + off < 256) ? suffix[t + off] : 0ull;
            __syncthreads();
            suffix[t] += add;
            __syncthreads();
        }
        if (suffix[t] >= want && suffix[t + 1] < want) {
            shared2[0] = (prefix << 8) | (unsigned long long)t;
            shared2[1] = want - suffix[t + 1];
        }
        __syncthreads();
        prefix = shared2[0];
        want = shared2[1];
        __syncthreads();
    }
    return prefix;
}

// Steps 6 (applied) and 7.  One workgroup of 256 threads per row.
__global__ __launch_bounds__(256) void k_row_update(const float* __restrict__ W, const uint8_t* __restrict__ mask,
                                                    const float* __restrict__ grad, int d_in, const int* __restrict__ remains,
                                                    const UpdateScratch* __restrict__ s, uint8_t* __restrict__ mask_out,
                                                    float* __restrict__ W_out) {
    __shared__ unsigned int h[256];
    __shared__ unsigned long long suffix[257];
    __shared__ unsigned long long shared2[2];
    __shared__ int n_kept;
    const int r = blockIdx.x, t = threadIdx.x;
    const unsigned int row0 = (unsigned int)r * d_in;
    if (!remains[r]) {
        for (int c = t; c < d_in; c += 256) { mask_out[row0 + c] = 0; W_out[row0 + c] = 0.0f; }
        return;
    }
    const unsigned long long t_prune = s->sel[2].threshold;
    const long long k_new = s->k_new;
    auto survives = [&](int c) { return mask[row0 + c] != 0 && key_small_first(mag_bits(W[row0 + c]), row0 + c) < t_prune; };
    if (t == 0) n_kept = 0;
    __syncthreads();
    int mine = 0;
    for (int c = t; c < d_in; c += 256) mine += survives(c) ? 1 : 0;
    if (mine) atomicAdd(&n_kept, mine);
    __syncthreads();
    const long long kept = n_kept;
    unsigned long long t_keep = 0;       // keep a surviving weight iff its key >= t_keep
    unsigned long long t_grow = ~0ull;   // grow a free position iff its key >= t_grow
    if (kept > k_new) {
        if (k_new == 0) t_keep = ~0ull;
        else t_keep = row_select(d_in, (unsigned long long)k_new, [&](int c, unsigned long long& key) {
            if (!survives(c)) return false;
            key = key_large_first(mag_bits(W[row0 + c]), (unsigned int)c);
            return true;
        }, h, suffix, shared2);
    } else if (kept < k_new) {
        t_grow = row_select(d_in, (unsigned long long)(k_new - kept), [&](int c, unsigned long long& key) {
            if (survives(c)) return false;
            key = key_large_first(mag_bits(grad[row0 + c]), (unsigned int)c);
            return true;
        }, h, suffix, shared2);
    }
    for (int c = t; c < d_in; c += 256) {
        uint8_t m = 0;
        float w = 0.0f;
        if (survives(c)) {
            if (key_large_first(mag_bits(W[row0 + c]), (unsigned int)c) >= t_keep) { m = 1; w = W[row0 + c]; }
        } else if (key_large_first(mag_bits(grad[row0 + c]), (unsigned int)c) >= t_grow) {
            m = 1;   // grown: the weight starts at zero
        }
        mask_out[row0 + c] = m;
        W_out[row0 + c] = w;
    }
}

__global__ void k_update_report(const UpdateScratch* __restrict__ s, long long K_upd, long long* __restrict__ report) {
    if (threadIdx.x == 0) {
        report[0] = s->k_new;
        report[1] = s->n_remaining;
        report[2] = s->n_ablated_now;
        const unsigned long long cand = s->sel[2].total;
        report[3] = (long long)((unsigned long long)K_upd < cand ? (unsigned long long)K_upd : cand);
    }
}

template <int MODE>
static void layer_select(const float* W, const uint8_t* mask, const float* grad, const int* remains, unsigned int N, int d_in,
                         UpdateScratch* s, hipStream_t st) {
    unsigned int blocks = (N + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    for (int pass = 0; pass < 8; ++pass) {
        hipLaunchKernelGGL(k_layer_hist<MODE>, dim3(blocks), dim3(256), 0, st, W, mask, grad, remains, N, d_in, pass, s);
        hipLaunchKernelGGL(k_layer_pick, dim3(1), dim3(256), 0, st, MODE, pass, s);
    }
}

}  // namespace srigl

using namespace srigl;

extern "C" {

size_t srigl_mask_update_workspace_bytes(int32_t d_out) {
    const size_t rows = d_out > 0 ? (size_t)d_out : 0;
    return ((sizeof(UpdateScratch) + 255) / 256) * 256 + 3 * rows * sizeof(int32_t);
}

srigl_status srigl_mask_update(const float* W, const uint8_t* mask, const float* grad, int32_t d_out, int32_t d_in, int32_t k,
                               int64_t K_upd, int32_t gamma_percent, int64_t budget, uint8_t* mask_out, float* W_out,
                               void* workspace, size_t workspace_bytes, int64_t* report_dev, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (d_out < 0 || d_in < 0 || k < 0 || k > d_in || K_upd < 0 || gamma_percent < 0 || budget < 0 || report_dev == nullptr)
        return SRIGL_ERR_INVALID_ARG;
    if ((long long)d_out * d_in >= (1ll << 32)) return SRIGL_ERR_UNSUPPORTED;   // positions are ranked as 32-bit numbers
    if (workspace == nullptr) return SRIGL_ERR_INVALID_ARG;
    if (workspace_bytes < srigl_mask_update_workspace_bytes(d_out)) return SRIGL_ERR_CAPACITY;
    const unsigned int N = (unsigned int)((long long)d_out * d_in);
    if (N > 0 && (W == nullptr || mask == nullptr || grad == nullptr || mask_out == nullptr || W_out == nullptr)) return SRIGL_ERR_INVALID_ARG;
    UpdateScratch* s = static_cast<UpdateScratch*>(workspace);
    int* held = reinterpret_cast<int*>(static_cast<unsigned char*>(workspace) + ((sizeof(UpdateScratch) + 255) / 256) * 256);
    int* salient = held + d_out;
    int* remains = salient + d_out;
    hipLaunchKernelGGL(k_update_init, dim3(1), dim3(256), 0, st, s, (long long)K_upd);
    if (N > 0) {
        layer_select<0>(W, mask, grad, remains, N, d_in, s, st);
        layer_select<1>(W, mask, grad, remains, N, d_in, s, st);
        hipLaunchKernelGGL(k_row_salient, dim3((d_out + 3) / 4), dim3(256), 0, st, W, mask, grad, d_out, d_in, s, held, salient);
    }
    hipLaunchKernelGGL(k_decide, dim3(1), dim3(1024), 0, st, held, salient, d_out, d_in, k, gamma_percent, (long long)budget, remains, s);
    if (N > 0) {
        layer_select<2>(W, mask, grad, remains, N, d_in, s, st);
        hipLaunchKernelGGL(k_row_update, dim3(d_out), dim3(256), 0, st, W, mask, grad, d_in, remains, s, mask_out, W_out);
    }
    hipLaunchKernelGGL(k_update_report, dim3(1), dim3(64), 0, st, s, (long long)K_upd, reinterpret_cast<long long*>(report_dev));
    return hip_ok(hipGetLastError());
}

}  // extern "C"
