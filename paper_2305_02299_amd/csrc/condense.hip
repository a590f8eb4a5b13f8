// check_fanin and condense kernels (gfx950).
//
// Constant fan-in invariant: Fig. 1a / Sec. 3.1 of arXiv 2305.02299 (every neuron that is not
// ablated keeps exactly K incoming weights).  Condensed form: App. E (an [n][k] array of values and
// an [n][k] array of column indices), with ablated neurons dropped (Sec. 4.4).
//
// All three steps are bandwidth work over the mask (1 byte per weight) and, for the compaction, the
// dense weights: one wavefront owns one row, lanes read 4 consecutive mask bytes each so that a
// wavefront covers 256 contiguous columns per iteration, and positions inside the row come from
// ballots and prefix popcounts (no LDS, no atomics).
#include "srigl_internal.h"

#include <mutex>

// Scratch of srigl_condense_static (the condense call for callers that cannot allocate): the per-row counts and slots that
// srigl_condense takes from its workspace argument.  One copy per GPU, held until the process ends.  The name is a host-side
// stand-in: kernels get the device address that hipGetSymbolAddress returns for the current device.
static __device__ __align__(256) unsigned char scratch[2 * sizeof(int32_t) * (size_t)SRIGL_STATIC_MAX_ROWS + 256];

namespace srigl {

constexpr int kRowsPerBlock = 4;   // 4 wavefronts of 64 lanes, one row each

__device__ __forceinline__ uint32_t lanes_below(uint64_t ballot) {
    // number of set bits of `ballot` that belong to lanes below this one
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(ballot >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)ballot, 0u));
}

// 4 mask bytes of row `m` starting at column `col` (bytes past d_in read as 0), one byte per 8 bits.
__device__ __forceinline__ uint32_t load_mask4(const uint8_t* __restrict__ m, int col, int d_in, bool aligned4) {
    if (col + 4 <= d_in) {
        if (aligned4) return *reinterpret_cast<const uint32_t*>(m + col);
        return (uint32_t)m[col] | ((uint32_t)m[col + 1] << 8) | ((uint32_t)m[col + 2] << 16) | ((uint32_t)m[col + 3] << 24);
    }
    uint32_t v = 0;
    for (int p = 0; p < 4; ++p)
        if (col + p < d_in) v |= (uint32_t)m[col + p] << (8 * p);
    return v;
}

// per-byte non-zero flags of a 32-bit word: bit 7 of each byte
__device__ __forceinline__ uint32_t nonzero_bytes(uint32_t w) {
    return (((w & 0x7f7f7f7fu) + 0x7f7f7f7fu) | w) & 0x80808080u;
}

// counts[r] = number of non-zero mask bytes in row r
__global__ __launch_bounds__(kRowsPerBlock* kWave) void k_row_count(const uint8_t* __restrict__ mask, int n_rows,
                                                                  int d_in, int32_t* __restrict__ counts) {
    const int lane = threadIdx.x & (kWave - 1);
    const int r = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
    if (r >= n_rows) return;
    const uint8_t* m = mask + (size_t)r * d_in;
    const bool aligned4 = ((reinterpret_cast<uintptr_t>(m) & 3) == 0);
    int c = 0;
    for (int col = lane * 4; col < d_in; col += kWave * 4) c += __popc(nonzero_bytes(load_mask4(m, col, d_in, aligned4)));
    for (int off = 32; off > 0; off >>= 1) c += __shfl_xor(c, off, kWave);
    if (lane == 0) counts[r] = c;
}

// Index mode: counts[r] = K if row r of idx is in range and strictly ascending, else -1; seg rows.
__global__ __launch_bounds__(kRowsPerBlock* kWave) void k_check_idx(const int32_t* __restrict__ idx, int n_rows, int K,
                                                                  int d_in, int32_t* __restrict__ counts,
                                                                  uint16_t* __restrict__ seg, int seg_stride) {
    const int lane = threadIdx.x & (kWave - 1);
    const int r = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
    if (r >= n_rows) return;
    const int32_t* row = idx + (size_t)r * K;
    bool ok = true;
    for (int k = lane; k < K; k += kWave) {
        int32_t cur = row[k];
        if (cur < 0 || cur >= d_in) ok = false;
        if (k > 0 && row[k - 1] >= cur) ok = false;
    }
    const bool row_ok = (__ballot(!ok) == 0ull);
    if (lane == 0) counts[r] = row_ok ? K : -1;
    if (seg == nullptr) return;
    uint16_t* sg = seg + (size_t)r * seg_stride;
    if (!row_ok || K == 0) {
        for (int c = lane; c < seg_stride; c += kWave) sg[c] = 0;
        return;
    }
    // ascending row: seg[c] = position of the first index >= 64*c.  The lane that owns position k
    // fills the entries c in (prev/64, cur/64]; the tail entries hold K.
    for (int k = lane; k < K; k += kWave) {
        const int cur = row[k];
        const int lo = (k == 0) ? 0 : row[k - 1] / kSegCols + 1;
        const int hi = cur / kSegCols;
        for (int c = lo; c <= hi; ++c) sg[c] = (uint16_t)k;
    }
    const int last = row[K - 1] / kSegCols + 1;
    for (int c = last + lane; c < seg_stride; c += kWave) sg[c] = (uint16_t)K;
}

// One workgroup.  Reads counts[], decides K, numbers the stored rows, writes slot[], active[], report.
// index_mode: counts hold K (valid) or -1 (bad); every valid row is "stored" even when K == 0.
__global__ __launch_bounds__(1024) void k_scan_rows(const int32_t* __restrict__ counts, int n_rows, int K_expected,
                                                    int index_mode, int cap_rows, int32_t* __restrict__ slot,
                                                    int32_t* __restrict__ active, srigl_report* __restrict__ report) {
    __shared__ int s_wave[16];
    __shared__ int s_k, s_base, s_min;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid >> 6;
    const int nthreads = blockDim.x, nwaves = nthreads >> 6;

    if (tid == 0) { s_min = 0x7fffffff; s_base = 0; }
    __syncthreads();
    int K = K_expected;
    if (K_expected < 0) {   // fan-in of the first non-empty row
        int first = 0x7fffffff;
        for (int r = tid; r < n_rows; r += nthreads)
            if (counts[r] > 0) { first = r; break; }
        for (int off = 32; off > 0; off >>= 1) first = min(first, __shfl_xor(first, off, kWave));
        if (lane == 0 && first != 0x7fffffff) atomicMin(&s_min, first);
        __syncthreads();
        if (tid == 0) s_k = (s_min == 0x7fffffff) ? 0 : counts[s_min];
        __syncthreads();
        K = s_k;
        __syncthreads();
        if (tid == 0) s_min = 0x7fffffff;
        __syncthreads();
    }

    // Every thread takes a run of consecutive rows: it counts its stored rows, the workgroup turns the counts into each thread's
    // first slot (one scan inside every wavefront, one over the 16 wavefront totals), and the thread numbers its rows from there.
    int n_bad = 0, first_bad = 0x7fffffff;
    const int per_thread = (n_rows + nthreads - 1) / nthreads;
    const int r0 = tid * per_thread, r1 = min(n_rows, r0 + per_thread);
    auto classify = [&](int r, bool& stored, bool& bad) {
        const int c = counts[r];
        if (index_mode) { stored = (c == K); bad = (c != K); }
        else            { stored = (c == K) && (c > 0); bad = (c != 0) && (c != K); }
    };
    int mine = 0;
    for (int r = r0; r < r1; ++r) {
        bool stored, bad;
        classify(r, stored, bad);
        mine += stored ? 1 : 0;
        if (bad) { ++n_bad; first_bad = min(first_bad, r); }
    }
    int incl = mine;   // inclusive scan over the lanes of this wavefront
    for (int off = 1; off < kWave; off <<= 1) {
        const int up = __shfl_up(incl, off, kWave);
        if (lane >= off) incl += up;
    }
    if (lane == kWave - 1) s_wave[wv] = incl;
    __syncthreads();
    int my = incl - mine;
    for (int w = 0; w < wv; ++w) my += s_wave[w];
    if (tid == nthreads - 1) s_base = my + mine;   // the last thread's end is the number of stored rows
    for (int r = r0; r < r1; ++r) {
        bool stored, bad;
        classify(r, stored, bad);
        if (slot) slot[r] = stored ? my : -1;
        if (stored && active && my < cap_rows) active[my] = r;
        my += stored ? 1 : 0;
    }
    __syncthreads();
    for (int off = 32; off > 0; off >>= 1) {
        n_bad += __shfl_xor(n_bad, off, kWave);
        first_bad = min(first_bad, __shfl_xor(first_bad, off, kWave));
    }
    if (lane == 0) s_wave[wv] = n_bad;
    if (lane == 0 && first_bad != 0x7fffffff) atomicMin(&s_min, first_bad);
    __syncthreads();
    if (tid == 0) {
        int t = 0;
        for (int w = 0; w < nwaves; ++w) t += s_wave[w];
        report->K = K;
        report->n_active = s_base;
        report->n_bad_rows = t;
        report->first_bad_row = (s_min == 0x7fffffff) ? -1 : s_min;
        int st = SRIGL_OK;
        if (t > 0) st = index_mode ? SRIGL_ERR_INDEX_RANGE : SRIGL_ERR_FANIN;
        else if (active && s_base > cap_rows) st = SRIGL_ERR_CAPACITY;
        report->status = st;
        report->reserved[0] = report->reserved[1] = report->reserved[2] = 0;
    }
}

// One wavefront per row: ordered stream compaction of the kept columns.
// T = bit container of one weight (uint32_t for fp32, uint16_t for bf16).
// With `packed` the same pass also writes the streaming copy (see PackedLayout): term `pos` of stored row s next to its
// index, and the places behind the K-th term up to the next multiple of four get weight bits 0 and index 0.
template <typename T>
__global__ __launch_bounds__(kRowsPerBlock* kWave) void k_compact_rows(const T* __restrict__ W, const uint8_t* __restrict__ mask,
                                                                     int d_out, int d_in, int K, int cap_rows,
                                                                     const int32_t* __restrict__ slot, T* __restrict__ W_c,
                                                                     int32_t* __restrict__ idx, uint16_t* __restrict__ seg,
                                                                     int seg_stride, unsigned char* __restrict__ packed, PackedLayout pl) {
    const int lane = threadIdx.x & (kWave - 1);
    const int r = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
    if (r >= d_out) return;
    const int s = slot[r];
    if (s < 0 || s >= cap_rows) return;   // ablated, invalid, or no room
    const uint8_t* m = mask + (size_t)r * d_in;
    const T* w = W + (size_t)r * d_in;
    const bool aligned4 = ((reinterpret_cast<uintptr_t>(m) & 3) == 0);
    T* wc = W_c + (size_t)s * K;
    int32_t* ix = idx + (size_t)s * K;
    uint16_t* sg = seg ? seg + (size_t)s * seg_stride : nullptr;
    unsigned char* pk = packed ? packed + (size_t)s * pl.row_bytes() : nullptr;

    int base = 0;   // kept columns seen in earlier iterations (same in every lane)
    int chunk = 0;  // index of the next seg entry; one iteration covers 256 columns = 4 entries
    for (int col0 = 0; col0 < d_in; col0 += kWave * 4, chunk += 4) {
        const int col = col0 + lane * 4;
        const uint32_t nz = (col < d_in) ? nonzero_bytes(load_mask4(m, col, d_in, aligned4)) : 0u;
        uint64_t bal[4];
        int before = 0, total = 0;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            bal[p] = __ballot((nz >> (8 * p + 7)) & 1u);
            before += (int)lanes_below(bal[p]);
            total += __popcll(bal[p]);
        }
        if (sg && lane < 4 && chunk + lane < seg_stride) {
            // entry for columns col0 + 64*lane ...: kept columns in the 16*lane lanes before it
            const uint64_t lo = (lane == 0) ? 0ull : ((1ull << (16 * lane)) - 1ull);
            int cnt = 0;
#pragma unroll
            for (int p = 0; p < 4; ++p) cnt += __popcll(bal[p] & lo);
            sg[chunk + lane] = (uint16_t)(base + cnt);
        }
        int pos = base + before;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            if ((nz >> (8 * p + 7)) & 1u) {
                if (pos < K) {
                    const T wbits = w[col + p];
                    ix[pos] = col + p;
                    wc[pos] = wbits;
                    if (pk) pl.store(pk, pos, (uint32_t)wbits, col + p);
                }
                ++pos;
            }
        }
        base += total;
    }
    if (sg)
        for (int c = chunk + lane; c < seg_stride; c += kWave) sg[c] = (uint16_t)base;
    if (pk)
        for (int t = K + lane; t < pl.terms; t += kWave) pl.store(pk, t, 0u, 0);
}

// The streaming copy from the canonical arrays: one thread per term, padding included.
__global__ __launch_bounds__(256) void k_pack_terms(const void* __restrict__ W_c, const int32_t* __restrict__ idx, int n_rows, int K,
                                                    unsigned char* __restrict__ packed, PackedLayout pl) {
    const long long places = (long long)n_rows * pl.terms;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < places; i += (long long)gridDim.x * blockDim.x) {
        const int s = (int)(i / pl.terms), t = (int)(i - (long long)s * pl.terms);
        uint32_t wbits = 0u;
        int col = 0;
        if (t < K) {
            const size_t e = (size_t)s * K + t;
            wbits = pl.w_bytes == 4 ? static_cast<const uint32_t*>(W_c)[e] : (uint32_t)static_cast<const uint16_t*>(W_c)[e];
            col = idx[e];
        }
        pl.store(packed + (size_t)s * pl.row_bytes(), t, wbits, col);
    }
}

__global__ void k_empty() {}

__global__ __launch_bounds__(256) void k_copy16(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace srigl

using namespace srigl;

extern "C" {

size_t srigl_workspace_bytes(int32_t n_rows) {
    if (n_rows < 0) n_rows = 0;
    return 2 * sizeof(int32_t) * (size_t)n_rows + 256;
}

int32_t srigl_seg_stride(int32_t d_in) {
    if (d_in < 0) d_in = 0;
    return (d_in + kSegCols - 1) / kSegCols + 1;
}

srigl_status srigl_check_fanin(const uint8_t* mask, const int32_t* idx, int32_t n_rows, int32_t d_in,
                               int32_t K_expected, uint16_t* seg, void* workspace, size_t workspace_bytes,
                               srigl_report* report_dev, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if ((mask == nullptr) == (idx == nullptr)) return SRIGL_ERR_INVALID_ARG;
    if (n_rows < 0 || d_in < 0 || report_dev == nullptr) return SRIGL_ERR_INVALID_ARG;
    if (idx && (K_expected < 0 || K_expected > d_in)) return SRIGL_ERR_INVALID_ARG;
    if (mask && K_expected > d_in) return SRIGL_ERR_INVALID_ARG;
    if (idx && seg && K_expected > 65535) return SRIGL_ERR_UNSUPPORTED;
    if (n_rows > 0 && workspace == nullptr) return SRIGL_ERR_INVALID_ARG;
    if (workspace_bytes < srigl_workspace_bytes(n_rows)) return SRIGL_ERR_CAPACITY;
    int32_t* counts = static_cast<int32_t*>(workspace);
    const int blocks = (n_rows + kRowsPerBlock - 1) / kRowsPerBlock;
    if (n_rows > 0) {
        if (mask) hipLaunchKernelGGL(k_row_count, dim3(blocks), dim3(kRowsPerBlock * kWave), 0, st, mask, n_rows, d_in, counts);
        else      hipLaunchKernelGGL(k_check_idx, dim3(blocks), dim3(kRowsPerBlock * kWave), 0, st, idx, n_rows, K_expected, d_in, counts, seg, srigl_seg_stride(d_in));
    }
    hipLaunchKernelGGL(k_scan_rows, dim3(1), dim3(1024), 0, st, counts, n_rows, K_expected, idx ? 1 : 0, n_rows,
                       (int32_t*)nullptr, (int32_t*)nullptr, report_dev);
    return hip_ok(hipGetLastError());
}

static srigl_status condense_core(const void* W, srigl_dtype w_dtype, const uint8_t* mask, int32_t d_out, int32_t d_in, int32_t K,
                                  int32_t cap_rows, void* W_c, int32_t* idx, int32_t* active, uint16_t* seg, void* packed,
                                  size_t packed_bytes, void* workspace, srigl_report* report_dev, hipStream_t st) {
    if (d_out < 0 || d_in < 0 || K < 0 || K > d_in || cap_rows < 0 || report_dev == nullptr) return SRIGL_ERR_INVALID_ARG;
    if (w_dtype != SRIGL_F32 && w_dtype != SRIGL_BF16) return SRIGL_ERR_INVALID_ARG;
    if (d_out > 0 && d_in > 0 && (W == nullptr || mask == nullptr)) return SRIGL_ERR_INVALID_ARG;
    if (cap_rows > 0 && (active == nullptr || (K > 0 && (W_c == nullptr || idx == nullptr)))) return SRIGL_ERR_INVALID_ARG;
    if (seg && K > 65535) return SRIGL_ERR_UNSUPPORTED;
    if (d_out > 0 && workspace == nullptr) return SRIGL_ERR_INVALID_ARG;
    const PackedLayout pl = packed_layout(K, d_in, w_dtype == SRIGL_BF16);
    if (packed) {
        if (reinterpret_cast<uintptr_t>(packed) % 16 != 0) return SRIGL_ERR_INVALID_ARG;
        if (packed_bytes < srigl_packed_bytes(cap_rows, K, d_in, w_dtype)) return SRIGL_ERR_CAPACITY;
    }
    int32_t* counts = static_cast<int32_t*>(workspace);
    int32_t* slot = counts + d_out;
    const int blocks = (d_out + kRowsPerBlock - 1) / kRowsPerBlock;
    if (d_out > 0) hipLaunchKernelGGL(k_row_count, dim3(blocks), dim3(kRowsPerBlock * kWave), 0, st, mask, d_out, d_in, counts);
    hipLaunchKernelGGL(k_scan_rows, dim3(1), dim3(1024), 0, st, counts, d_out, K, 0, cap_rows, slot, active, report_dev);
    if (d_out > 0 && cap_rows > 0 && K > 0) {
        const int ss = srigl_seg_stride(d_in);
        if (w_dtype == SRIGL_F32)
            hipLaunchKernelGGL(k_compact_rows<uint32_t>, dim3(blocks), dim3(kRowsPerBlock * kWave), 0, st,
                               static_cast<const uint32_t*>(W), mask, d_out, d_in, K, cap_rows, slot,
                               static_cast<uint32_t*>(W_c), idx, seg, ss, static_cast<unsigned char*>(packed), pl);
        else
            hipLaunchKernelGGL(k_compact_rows<uint16_t>, dim3(blocks), dim3(kRowsPerBlock * kWave), 0, st,
                               static_cast<const uint16_t*>(W), mask, d_out, d_in, K, cap_rows, slot,
                               static_cast<uint16_t*>(W_c), idx, seg, ss, static_cast<unsigned char*>(packed), pl);
    }
    return hip_ok(hipGetLastError());
}

srigl_status srigl_condense(const void* W, srigl_dtype w_dtype, const uint8_t* mask, int32_t d_out,
                            int32_t d_in, int32_t K, int32_t cap_rows, void* W_c, int32_t* idx,
                            int32_t* active, uint16_t* seg, void* packed, size_t packed_bytes, void* workspace,
                            size_t workspace_bytes, srigl_report* report_dev, void* stream) {
    if (d_out >= 0 && workspace_bytes < srigl_workspace_bytes(d_out)) return SRIGL_ERR_CAPACITY;
    return condense_core(W, w_dtype, mask, d_out, d_in, K, cap_rows, W_c, idx, active, seg, packed, packed_bytes, workspace,
                         report_dev, static_cast<hipStream_t>(stream));
}

// Device address of `scratch` on the current device, looked up once per device.
static srigl_status scratch_on_current_device(void** out) {
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void* ptr[kMaxDevices] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return SRIGL_ERR_HIP;
    if (dev < 0 || dev >= kMaxDevices) return SRIGL_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(mu);
    if (ptr[dev] == nullptr) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return SRIGL_ERR_HIP;
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return SRIGL_OK;
}

srigl_status srigl_condense_static(const void* W, srigl_dtype w_dtype, const uint8_t* mask, int32_t d_out, int32_t d_in, int32_t K,
                                   int32_t cap_rows, void* W_c, int32_t* idx, int32_t* active, uint16_t* seg, void* packed,
                                   size_t packed_bytes, srigl_report* report_dev, void* stream) {
    if (d_out > SRIGL_STATIC_MAX_ROWS) return SRIGL_ERR_CAPACITY;   // more rows than the built-in scratch holds
    void* ws = nullptr;
    const srigl_status st = scratch_on_current_device(&ws);
    if (st != SRIGL_OK) return st;
    // every count and slot of rows [0, d_out) is written by the first two kernels before anything reads it, so what an
    // earlier call left in the scratch is never seen and nothing has to be cleared
    return condense_core(W, w_dtype, mask, d_out, d_in, K, cap_rows, W_c, idx, active, seg, packed, packed_bytes, ws, report_dev,
                         static_cast<hipStream_t>(stream));
}

size_t srigl_packed_bytes(int32_t n_rows, int32_t K, int32_t d_in, srigl_dtype w_dtype) {
    if (n_rows <= 0 || K <= 0 || d_in <= 0 || (w_dtype != SRIGL_F32 && w_dtype != SRIGL_BF16)) return 0;
    return (size_t)n_rows * packed_layout(K, d_in, w_dtype == SRIGL_BF16).row_bytes();
}

srigl_status srigl_pack_terms(const void* W_c, srigl_dtype w_dtype, const int32_t* idx, int32_t n_rows, int32_t K, int32_t d_in,
                              void* packed, size_t packed_bytes, void* stream) {
    if (n_rows < 0 || K < 0 || d_in < 0 || K > d_in || (w_dtype != SRIGL_F32 && w_dtype != SRIGL_BF16)) return SRIGL_ERR_INVALID_ARG;
    if (n_rows == 0 || K == 0) return SRIGL_OK;
    if (W_c == nullptr || idx == nullptr || packed == nullptr || reinterpret_cast<uintptr_t>(packed) % 16 != 0) return SRIGL_ERR_INVALID_ARG;
    if (packed_bytes < srigl_packed_bytes(n_rows, K, d_in, w_dtype)) return SRIGL_ERR_CAPACITY;
    const PackedLayout pl = packed_layout(K, d_in, w_dtype == SRIGL_BF16);
    long long blocks = ((long long)n_rows * pl.terms + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(k_pack_terms, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream), W_c, idx, n_rows, K,
                       static_cast<unsigned char*>(packed), pl);
    return hip_ok(hipGetLastError());
}

srigl_status srigl_launch_empty(void* stream) {
    hipLaunchKernelGGL(k_empty, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream));
    return hip_ok(hipGetLastError());
}

srigl_status srigl_copy_bytes(const void* src, void* dst, size_t n_bytes, void* stream) {
    if (n_bytes == 0) return SRIGL_OK;
    if (src == nullptr || dst == nullptr || (n_bytes & 15) != 0) return SRIGL_ERR_INVALID_ARG;
    if (((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15) != 0) return SRIGL_ERR_INVALID_ARG;
    const size_t n16 = n_bytes / 16;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(k_copy16, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4*>(src), static_cast<uint4*>(dst), n16);
    return hip_ok(hipGetLastError());
}

const char* srigl_status_str(srigl_status s) {
    switch (s) {
        case SRIGL_OK: return "ok";
        case SRIGL_ERR_INVALID_ARG: return "invalid argument";
        case SRIGL_ERR_FANIN: return "a row holds neither 0 nor K kept weights";
        case SRIGL_ERR_CAPACITY: return "buffer too small";
        case SRIGL_ERR_INDEX_RANGE: return "index out of range or row not strictly ascending";
        case SRIGL_ERR_UNSUPPORTED: return "unsupported configuration";
        case SRIGL_ERR_HIP: return "HIP call failed";
    }
    return "unknown status";
}

}  // extern "C"
