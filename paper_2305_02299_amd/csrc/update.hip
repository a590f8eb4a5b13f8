// One SRigL connectivity update of a layer on the GPU (gfx950): Sec. 3.1 of arXiv 2305.02299, steps 1-7 (prune / grow
// criteria, salient weights per neuron, neuron ablation with threshold gamma_sal, new fan-in k', layer-wide pruning, per-neuron
// regrowth), fp32 weights and gradients, dense [d_out][d_in] storage with a byte mask.  Readings of the text are listed in
// include/srigl.h next to srigl_mask_update.
//
// Every ranking is a selection of the K largest of unique 64-bit keys, (magnitude bits, position): equal magnitudes are
// ordered by position, so the selected set is unique and no sort is needed.  Layer-wide selections (steps 3 and 6) find the
// K-th largest key by a most-significant-digit-first radix walk: passes of (histogram of one digit over the elements that
// match the prefix found so far, then the digit that holds the K-th key), ended as soon as every key of the chosen digit is
// wanted.  The top bit of every key is zero, so the digits are bits 62-55, 54-47, ..., 14-7 and 6-0: two passes fix the
// exponent and 8 mantissa bits of the threshold; the third pass also copies the keys that match those 16 bits (a fraction
// of a percent of a layer with real-valued contents) into a candidate list, and the remaining passes read that list
// instead of the layer (a list that would overflow is dropped and the passes stay on the layer).  The two selections of step 3 share their passes, and every workgroup of a pass picks the previous pass's byte for
// itself from that pass's own counters (no pick launches, no device-wide fences); step 6 reuses step 3's answer when no
// neuron was ablated.  Row-wise selections (step 7) do the same walk inside one workgroup per row, on keys held in registers.
#include "srigl_internal.h"

namespace srigl {

struct SelState {
    unsigned long long prefix;      // the bytes of the K-th largest key found so far (right-aligned); at the end: the key itself
    unsigned long long k_rem;       // how many of the keys with this prefix are still wanted
    unsigned long long total;       // number of candidate keys
    int done;                       // the threshold is final (nothing wanted: ~0; everything wanted: 0; or the walk has ended)
    int pad;
};

// Head of the workspace.  Selections: 0 = smallest kept weights of the layer, 1 = largest gradients at pruned positions,
// 2 = smallest kept weights of the remaining neurons.  Pass p of a walk adds into hist[sel][p]; the launch of pass p + 1
// reads it (every workgroup picks the byte of pass p for itself), so no launch reads and clears the same counters, and no
// device-wide fence is needed (on this multi-die GPU such a fence costs about 0.1 ms per launch).
// slot[sel][p & 1] = the walk's state before pass p (written by workgroup 0 of the launch of pass p, read by the next launch).
// The launch after a walk's eighth pass takes the last digit for itself (finished_walk): select key >= its prefix.
// Copies of every layer-wide histogram: a pass ends with one atomic per non-empty digit and workgroup, and 2048 workgroups
// adding to the same 256 counters took longer than reading a 2.4-million-element layer (43 us of a 167 us update).  Every
// workgroup of the next pass reads all copies, which costs too: 4 copies measured best (1, 2, 8: 2-5 % slower; 32: 50 %).
constexpr int kHistCopies = 4;
constexpr int kCountCopies = 64;
struct UpdateScratch {
    unsigned int hist[3][8][kHistCopies][256];   // workgroup w adds into copy w % kHistCopies
    SelState slot[3][2];
    SelState fin[2];                    // the finished selections of step 3 (written by k_row_salient for the launches after it)
    // steps 4-5: neurons that stay / are ablated now (sums of the copies: one per lane of the wavefront that reads them; a
    // workgroup of the per-neuron kernel adds into copy w % 64, so a 16384-row layer sends 64 atomics to an address, not 1024)
    unsigned int cnt_remaining[kCountCopies], cnt_ablated[kCountCopies];
    unsigned long long cand_count[3];   // keys in the selection's candidate list; above the capacity: the list is not valid
};

// Pass p of a walk decides `pass_bits(p)` bits of the key, found at `pass_shift(p)`; before pass p the top
// `bits_done(p)` bits are fixed (the always-zero top bit counts as fixed from the start).
__host__ __device__ constexpr int pass_shift(int p) { return p < 7 ? 55 - 8 * p : 0; }
__host__ __device__ constexpr int pass_bits(int p) { return p < 7 ? 8 : 7; }
__host__ __device__ constexpr int bits_done(int p) { return p < 8 ? 1 + 8 * p : 64; }
constexpr int kCompactPass = 2;      // the pass that also writes the candidate lists
constexpr int kBlockList = 1024;     // candidate keys a workgroup collects in LDS before it appends them

__device__ __forceinline__ unsigned int mag_bits(float v) { return __float_as_uint(v) & 0x7fffffffu; }
// larger key = smaller magnitude, then lower position
__device__ __forceinline__ unsigned long long key_small_first(unsigned int mag, unsigned int pos) {
    return ((unsigned long long)(0x7fffffffu - mag) << 32) | (0xffffffffu - pos);
}
// larger key = larger magnitude, then lower position
__device__ __forceinline__ unsigned long long key_large_first(unsigned int mag, unsigned int pos) {
    return ((unsigned long long)mag << 32) | (0xffffffffu - pos);
}

__global__ __launch_bounds__(256) void k_update_init(UpdateScratch* s, long long K_upd) {
    const int t = threadIdx.x;
    const int n = 3 * 8 * kHistCopies * 256;
    for (int i = blockIdx.x * 256 + t; i < n; i += gridDim.x * 256) (&s->hist[0][0][0][0])[i] = 0;
    if (blockIdx.x == 0 && t < 3) {
        SelState z;
        z.prefix = 0; z.k_rem = (unsigned long long)K_upd; z.total = 0; z.done = 0; z.pad = 0;
        s->slot[t][0] = z;
        s->slot[t][1] = z;
        if (t < 2) s->fin[t] = z;
        s->cand_count[t] = 0;
    }
    if (blockIdx.x == 0 && t < kCountCopies) { s->cnt_remaining[t] = 0; s->cnt_ablated[t] = 0; }
}

// From a 256-bin histogram (lane l reads bins 4l .. 4l + 3), for one wavefront: the byte d with suffix(d) >= want >
// suffix(d + 1), suffix(d) = number of keys whose byte is >= d; `above` = suffix(d + 1), `in_bin` = keys with byte d, `total`
// = suffix(0).  The results are the same on every lane.
__device__ __forceinline__ void pick_from(const unsigned long long (&v)[4], unsigned long long want, int lane, unsigned long long& digit,
                                          unsigned long long& above, unsigned long long& in_bin, unsigned long long& total) {
    unsigned long long part[5];
    part[4] = 0;
#pragma unroll
    for (int j = 3; j >= 0; --j) part[j] = part[j + 1] + v[j];
    unsigned long long incl = part[0];   // becomes the sum over this lane and the lanes above it
    for (int off = 1; off < 64; off <<= 1) {
        const unsigned long long up = __shfl_down(incl, off, 64);
        if (lane + off < 64) incl += up;
    }
    const unsigned long long excl = incl - part[0];
    total = __shfl(incl, 0, 64);
    bool found = false;
    digit = 0; above = 0; in_bin = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if (excl + part[j] >= want && excl + part[j + 1] < want) {
            found = true;
            digit = 4 * lane + j;
            above = excl + part[j + 1];
            in_bin = v[j];
        }
    }
    const unsigned long long owner = __ballot(found);
    const int src = owner ? __builtin_ctzll(owner) : 0;
    digit = __shfl(digit, src, 64);
    above = __shfl(above, src, 64);
    in_bin = __shfl(in_bin, src, 64);
}
// Over the sum of COPIES sub-histograms (lane l reads bins 4l .. 4l + 3 of each); copy c keeps the count of digit d at index (d + TURN * c) mod 256 (in LDS a
// turn of kCopyTurn puts equal digits of different copies in different banks)
constexpr int kCopyTurn = 16;
template <int COPIES, int TURN>
__device__ __forceinline__ void sum_byte_copies(const unsigned int (*h)[256], int lane, unsigned long long (&v)[4]) {
    v[0] = v[1] = v[2] = v[3] = 0;
#pragma unroll
    for (int c = 0; c < COPIES; ++c) {
        const uint4 q = *reinterpret_cast<const uint4*>(&h[c][(4 * lane + TURN * c) & 255]);
        v[0] += q.x; v[1] += q.y; v[2] += q.z; v[3] += q.w;
    }
}
template <int COPIES, int TURN>
__device__ __forceinline__ void pick_byte_copies(const unsigned int (*h)[256], unsigned long long want, int lane, unsigned long long& digit,
                                                 unsigned long long& above, unsigned long long& in_bin, unsigned long long& total) {
    unsigned long long v[4];
    sum_byte_copies<COPIES, TURN>(h, lane, v);
    pick_from(v, want, lane, digit, above, in_bin, total);
}

// The state of a layer-wide walk before pass `pass` (1..8), from the state before pass - 1 and the histogram of pass - 1.
// Called by one whole wavefront; the result is the same on every lane.
// advance_from: with the counters of pass - 1 already summed (lane l holds digits 4l .. 4l + 3); advance requests them
// before the state is looked at, so that the two reads from memory do not wait for each other.
__device__ SelState advance_from(const SelState& before, const unsigned long long (&v)[4], int pass, int lane) {
    SelState st = before;
    if (st.done) return st;
    unsigned long long digit, above, in_bin, total;
    pick_from(v, st.k_rem == 0 ? 1 : st.k_rem, lane, digit, above, in_bin, total);
    if (pass == 1) {
        st.total = total;
        if (st.k_rem == 0 || total < st.k_rem) {
            st.prefix = (st.k_rem == 0) ? ~0ull : 0ull;   // nothing / everything
            st.done = 1;
            return st;
        }
    }
    st.prefix = (st.prefix << pass_bits(pass - 1)) | digit;
    st.k_rem -= above;
    // every key of the chosen digit is wanted (always so once the keys under the prefix are down to one): the walk is over,
    // the threshold is the smallest key with this prefix
    if (pass == 8 || st.k_rem == in_bin) {
        if (pass < 8) st.prefix <<= 64 - bits_done(pass);
        st.done = 1;
    }
    return st;
}
__device__ SelState advance(const SelState& before, const unsigned int (*hist_prev)[256], int pass, int lane) {
    unsigned long long v[4];
    sum_byte_copies<kHistCopies, 0>(hist_prev, lane, v);
    return advance_from(before, v, pass, lane);
}

// The finished selection `sel` for the launch that follows its eighth pass: the last digit from that pass's counters.
// Called by one whole wavefront; the result is the same on every lane.
__device__ __forceinline__ SelState finished_walk(const UpdateScratch* __restrict__ s, int sel, int lane) {
    return advance(s->slot[sel][1], s->hist[sel][7], 8, lane);
}
// Sum of the 64 copies of a neuron counter.  Called by one whole wavefront; the result is the same on every lane.
__device__ __forceinline__ unsigned int sum_copies(const unsigned int (&c)[kCountCopies], int lane) {
    unsigned int n = c[lane];
    for (int off = 32; off > 0; off >>= 1) n += __shfl_xor(n, off, 64);
    return n;
}

// One pass of the walk.  PAIR: selections 0 (kept weights, smallest first) and 1 (pruned positions, largest gradient first)
// together: every element belongs to exactly one of them, so one read of the layer serves both.  Otherwise selection 2
// (kept weights of the remaining neurons).  kCopies sub-histograms spread the LDS atomics of equal digits.
// COMPACT (the launch of pass kCompactPass): every key that matches the prefix is also appended to the selection's candidate
// list (collected per workgroup in LDS, one counter update per workgroup); a workgroup that meets more than kBlockList of
// them, or a list longer than `cap`, leaves the counter above `cap`, and the later passes then keep reading the layer.
// VEC (d_in a multiple of 4, 16-byte aligned arrays): four consecutive elements per thread and step, moved with one 4-byte
// and two 16-byte loads that do not wait for each other (a line of W or grad is fetched for almost every run of 32 elements
// anyway, so reading both arrays in full costs no extra traffic).
constexpr int kCopies = 8;
constexpr int kPassThreads = 256;   // threads per workgroup of a layer-wide pass (512 and 1024 measured no faster)
template <bool PAIR, bool COMPACT, bool VEC>
__global__ __launch_bounds__(kPassThreads) void k_layer_hist(const float* __restrict__ W, const uint8_t* __restrict__ mask,
                                                    const float* __restrict__ grad, const int* __restrict__ remains, unsigned int N,
                                                    int d_in, int pass, UpdateScratch* __restrict__ s,
                                                    unsigned long long* __restrict__ candA, unsigned long long* __restrict__ candB,
                                                    unsigned long long cap) {
    __shared__ unsigned int h[2][kCopies][256];
    __shared__ SelState cur[2];
    __shared__ unsigned long long keep[COMPACT ? 2 : 1][COMPACT ? kBlockList : 1];
    __shared__ unsigned int keep_n[2];
    __shared__ unsigned long long keep_base[2];
    const int t = threadIdx.x;
    const int selA = PAIR ? 0 : 2;
    const SelState before_a = s->slot[selA][(pass + 1) & 1], before_b = s->slot[1][(pass + 1) & 1];
    // walks that had ended before the previous pass: nothing to count
    if (pass > 0 && before_a.done != 0 && (!PAIR || before_b.done != 0)) {
        if (blockIdx.x == 0 && t == 0) {
            s->slot[selA][pass & 1] = before_a;
            if (PAIR) s->slot[1][pass & 1] = before_b;
        }
        return;
    }
    if (t < 64) {
        SelState a = before_a, b = before_b;
        if (pass > 0) {
            a = advance(a, s->hist[selA][pass - 1], pass, t);
            if (PAIR) b = advance(b, s->hist[1][pass - 1], pass, t);
            if (blockIdx.x == 0 && t == 0) {
                s->slot[selA][pass & 1] = a;
                if (PAIR) s->slot[1][pass & 1] = b;
            }
        } else {
            a = s->slot[selA][0];
            b = s->slot[1][0];
            // step 6 with no neuron ablated in step 4: same candidates, same count, so step 3's walk already has the answer
            if (!PAIR && sum_copies(s->cnt_ablated, t) == 0) {
                a = s->fin[0];
                if (blockIdx.x == 0 && t == 0) s->slot[2][0] = a;
            }
        }
        if (t == 0) { cur[0] = a; cur[1] = b; }
    }
    for (int i = t; i < 2 * kCopies * 256; i += kPassThreads) (&h[0][0][0])[i] = 0;
    if (t < 2) keep_n[t] = 0;
    __syncthreads();
    const bool doneA = cur[0].done != 0, doneB = PAIR ? cur[1].done != 0 : true;
    if (doneA && doneB) return;
    const int shift = pass_shift(pass);
    const unsigned int dmask = (1u << pass_bits(pass)) - 1u;
    const int pshift = 64 - bits_done(pass);   // pass > 0: a key is still in the walk iff key >> pshift == prefix
    const unsigned long long prefixA = cur[0].prefix, prefixB = cur[1].prefix;
    const int copy = t & (kCopies - 1);
    const bool lists = !COMPACT && pass > kCompactPass && cap > 0;
    const unsigned long long countA = lists ? s->cand_count[selA] : 0, countB = (lists && PAIR) ? s->cand_count[1] : 0;
    const bool listA = lists && countA <= cap, listB = lists && PAIR && countB <= cap;
    const bool scanA = !doneA && !listA, scanB = PAIR && !doneB && !listB;
    // one element: position ii, mask byte m, weight w, gradient g, whether its neuron remains (selection 2 only)
    auto element = [&](unsigned int ii, unsigned int m, float w, float g, bool rem) {
        if (m != 0) {
            if (!scanA || (!PAIR && !rem)) return;
            const unsigned long long key = key_small_first(mag_bits(w), ii);
            if (pass > 0 && (key >> pshift) != prefixA) return;
            atomicAdd(&h[0][copy][(unsigned int)(key >> shift) & dmask], 1u);
            if (COMPACT) {
                const unsigned int slot = atomicAdd(&keep_n[0], 1u);
                if (slot < (unsigned)kBlockList) keep[0][slot] = key;
            }
        } else if (scanB) {
            const unsigned long long key = key_large_first(mag_bits(g), ii);
            if (pass > 0 && (key >> pshift) != prefixB) return;
            atomicAdd(&h[1][copy][(unsigned int)(key >> shift) & dmask], 1u);
            if (COMPACT) {
                const unsigned int slot = atomicAdd(&keep_n[1], 1u);
                if (slot < (unsigned)kBlockList) keep[1][slot] = key;
            }
        }
    };
    if ((scanA || scanB) && VEC) {
        const unsigned int N4 = N / 4;   // d_in is a multiple of 4, so N is, and a run of 4 stays inside one row
        for (unsigned long long i = (unsigned long long)blockIdx.x * kPassThreads + t; i < N4; i += (unsigned long long)gridDim.x * kPassThreads) {
            const unsigned int base = 4u * (unsigned int)i;
            const uint32_t m4 = *reinterpret_cast<const uint32_t*>(mask + base);
            float4 w4 = make_float4(0.0f, 0.0f, 0.0f, 0.0f), g4 = w4;
            if (scanA) w4 = *reinterpret_cast<const float4*>(W + base);
            if (scanB) g4 = *reinterpret_cast<const float4*>(grad + base);
            const bool rem = (PAIR || m4 == 0) ? true : remains[base / (unsigned)d_in] != 0;
            element(base + 0, m4 & 0xffu, w4.x, g4.x, rem);
            element(base + 1, (m4 >> 8) & 0xffu, w4.y, g4.y, rem);
            element(base + 2, (m4 >> 16) & 0xffu, w4.z, g4.z, rem);
            element(base + 3, m4 >> 24, w4.w, g4.w, rem);
        }
    } else if (scanA || scanB) {
        for (unsigned long long i = (unsigned long long)blockIdx.x * kPassThreads + t; i < N; i += (unsigned long long)gridDim.x * kPassThreads) {
            const unsigned int ii = (unsigned int)i;
            const unsigned int m = mask[ii];
            if (m != 0) {
                if (scanA) element(ii, m, W[ii], 0.0f, PAIR ? true : remains[ii / (unsigned)d_in] != 0);
            } else if (scanB) {
                element(ii, 0u, 0.0f, grad[ii], true);
            }
        }
    }
    if (!doneA && listA) {
        for (unsigned long long i = (unsigned long long)blockIdx.x * kPassThreads + t; i < countA; i += (unsigned long long)gridDim.x * kPassThreads) {
            const unsigned long long key = candA[i];
            if ((key >> pshift) == prefixA) atomicAdd(&h[0][copy][(unsigned int)(key >> shift) & dmask], 1u);
        }
    }
    if (PAIR && !doneB && listB) {
        for (unsigned long long i = (unsigned long long)blockIdx.x * kPassThreads + t; i < countB; i += (unsigned long long)gridDim.x * kPassThreads) {
            const unsigned long long key = candB[i];
            if ((key >> pshift) == prefixB) atomicAdd(&h[1][copy][(unsigned int)(key >> shift) & dmask], 1u);
        }
    }
    __syncthreads();
    unsigned int a = 0, b = 0;
    if (t < 256) {
#pragma unroll
        for (int c = 0; c < kCopies; ++c) { a += h[0][c][t]; b += h[1][c][t]; }
        if (a) atomicAdd(&s->hist[selA][pass][blockIdx.x % kHistCopies][t], a);
        if (PAIR && b) atomicAdd(&s->hist[1][pass][blockIdx.x % kHistCopies][t], b);
    }
    if (COMPACT) {
        if (t < 2) {
            const unsigned int n = keep_n[t];
            // more keys than the workgroup can hold: the counter goes past `cap` for good, the list is not used
            keep_base[t] = n ? atomicAdd(&s->cand_count[t == 0 ? selA : 1], n > (unsigned)kBlockList ? cap + 1ull : (unsigned long long)n) : 0ull;
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const unsigned int n = keep_n[q];
            unsigned long long* __restrict__ dst = q == 0 ? candA : candB;
            if (n == 0 || n > (unsigned)kBlockList || keep_base[q] + n > cap) continue;
            for (unsigned int e = t; e < n; e += kPassThreads) dst[keep_base[q] + e] = keep[q][e];
        }
    }
}

// Steps 3 to 5 up to the counts: per neuron, how many weights it holds and how many salient ones, whether it stays
// (remains[r]; a neuron without weights stays ablated), and the layer's numbers of staying and newly ablated neurons (one
// atomic per workgroup and counter, spread over copies; read by the launches after this one).  One wavefront per row.
// VEC as in k_layer_hist: a lane takes runs of 4 columns.
template <bool VEC>
__global__ __launch_bounds__(256) void k_row_salient(const float* __restrict__ W, const uint8_t* __restrict__ mask,
                                                     const float* __restrict__ grad, int d_out, int d_in, int k, int gamma_percent,
                                                     UpdateScratch* __restrict__ s, int* __restrict__ remains) {
    __shared__ int wg_stay, wg_ablated;
    const int lane = threadIdx.x & 63;
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (threadIdx.x == 0) { wg_stay = 0; wg_ablated = 0; }
    // the row's first kAhead steps are requested before the thresholds are (they do not depend on them)
    constexpr int kAhead = 2;
    uint32_t pm[kAhead];
    float4 pw[kAhead], pg[kAhead];
    if (VEC && r < d_out) {
#pragma unroll
        for (int u = 0; u < kAhead; ++u) {
            const int c = 4 * lane + 256 * u;
            const unsigned int i = (unsigned int)r * d_in + (c < d_in ? c : 0);
            pm[u] = *reinterpret_cast<const uint32_t*>(mask + i);
            pw[u] = *reinterpret_cast<const float4*>(W + i);
            pg[u] = *reinterpret_cast<const float4*>(grad + i);
        }
    }
    const SelState fa = finished_walk(s, 0, lane), fb = finished_walk(s, 1, lane);
    if (blockIdx.x == 0 && threadIdx.x == 0) { s->fin[0] = fa; s->fin[1] = fb; }
    __syncthreads();
    const unsigned long long t_small = fa.prefix, t_grad = fb.prefix;
    int h = 0, sal = 0;
    auto element = [&](unsigned int i, unsigned int m, float w, float g) {
        if (m) {
            ++h;
            if (key_small_first(mag_bits(w), i) < t_small) ++sal;    // survives the layer-wide pruning
        } else if (key_large_first(mag_bits(g), i) >= t_grad) {
            ++sal;                                                    // would be grown
        }
    };
    if (r < d_out) {
        if (VEC) {
#pragma unroll
            for (int u = 0; u < kAhead; ++u) {
                const int c = 4 * lane + 256 * u;
                if (c >= d_in) break;
                const unsigned int i = (unsigned int)r * d_in + c;
                element(i + 0, pm[u] & 0xffu, pw[u].x, pg[u].x);
                element(i + 1, (pm[u] >> 8) & 0xffu, pw[u].y, pg[u].y);
                element(i + 2, (pm[u] >> 16) & 0xffu, pw[u].z, pg[u].z);
                element(i + 3, pm[u] >> 24, pw[u].w, pg[u].w);
            }
            for (int c = 4 * lane + 256 * kAhead; c < d_in; c += 256) {
                const unsigned int i = (unsigned int)r * d_in + c;
                const uint32_t m4 = *reinterpret_cast<const uint32_t*>(mask + i);
                const float4 w4 = *reinterpret_cast<const float4*>(W + i);
                const float4 g4 = *reinterpret_cast<const float4*>(grad + i);
                element(i + 0, m4 & 0xffu, w4.x, g4.x);
                element(i + 1, (m4 >> 8) & 0xffu, w4.y, g4.y);
                element(i + 2, (m4 >> 16) & 0xffu, w4.z, g4.z);
                element(i + 3, m4 >> 24, w4.w, g4.w);
            }
        } else {
            for (int c = lane; c < d_in; c += 64) {
                const unsigned int i = (unsigned int)r * d_in + c;
                const unsigned int m = mask[i];
                element(i, m, m ? W[i] : 0.0f, m ? 0.0f : grad[i]);
            }
        }
        for (int off = 32; off > 0; off >>= 1) { h += __shfl_xor(h, off, 64); sal += __shfl_xor(sal, off, 64); }
        if (lane == 0) {
            int stays = 0;
            if (h > 0) {
                const bool too_few = sal < 1 || (long long)sal * 100 < (long long)gamma_percent * k;
                if (too_few) atomicAdd(&wg_ablated, 1); else { stays = 1; atomicAdd(&wg_stay, 1); }
            }
            remains[r] = stays;
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        if (wg_stay) atomicAdd(&s->cnt_remaining[blockIdx.x % kCountCopies], (unsigned int)wg_stay);
        if (wg_ablated) atomicAdd(&s->cnt_ablated[blockIdx.x % kCountCopies], (unsigned int)wg_ablated);
    }
}

// Radix walk inside one workgroup of 256 threads: the threshold of the `want` largest keys among the row's candidates.
// key_of(j, key): whether the thread's j-th column is a candidate, and its key.  1 <= want <= number of candidates.
// Same digits as the layer-wide walk (the top bit of a key is zero).  One barrier per pass: the histograms rotate through
// three buffers (a pass adds into one, clears the next; the one before may still be read by a wavefront that is late), and
// every wavefront sums the kRowCopies sub-histograms and picks the digit for itself, so nothing is handed round.
constexpr int kRowCopies = 4;
template <int CPT, typename KeyOf>
__device__ unsigned long long row_select(unsigned long long want, KeyOf key_of, unsigned int (*h)[kRowCopies][256]) {
    const int t = threadIdx.x, lane = t & 63;
    const int copy = t & (kRowCopies - 1);
    unsigned long long prefix = 0;
#pragma unroll
    for (int c = 0; c < kRowCopies; ++c) h[0][c][t] = 0;
    __syncthreads();
#pragma unroll 1
    for (int pass = 0; pass < 8; ++pass) {
        const int cur = pass % 3, nxt = (pass + 1) % 3;
        const int shift = pass_shift(pass);
        const unsigned int dmask = (1u << pass_bits(pass)) - 1u;
        const int pshift = 64 - bits_done(pass);
#pragma unroll
        for (int c = 0; c < kRowCopies; ++c) h[nxt][c][t] = 0;
#pragma unroll
        for (int j = 0; j < CPT; ++j) {
            unsigned long long key;
            if (!key_of(j, key)) continue;
            if (pass > 0 && (key >> pshift) != prefix) continue;
            atomicAdd(&h[cur][copy][(((unsigned int)(key >> shift) & dmask) + kCopyTurn * copy) & 255u], 1u);
        }
        __syncthreads();
        unsigned long long digit, above, in_bin, total;
        pick_byte_copies<kRowCopies, kCopyTurn>(h[cur], want, lane, digit, above, in_bin, total);
        prefix = (prefix << pass_bits(pass)) | digit;
        want -= above;
        // every key of this digit is wanted: the walk is over, the threshold is the smallest key with this prefix
        if (want == in_bin && pass < 7) return prefix << (64 - bits_done(pass + 1));
    }
    return prefix;
}

// Steps 6 (applied) and 7.  One workgroup of 256 threads per row; a thread holds CPT columns of the row (d_in <= 256 CPT):
// whether the weight survives step 6, and the one key the column can be ranked by (its weight magnitude if it survives,
// else its gradient magnitude), so the walks read registers only.  VEC (d_in a multiple of 4, 16-byte aligned arrays): a
// thread's columns are runs of 4, moved with 16-byte loads and stores; otherwise column t + 256 j, one element at a time.
template <int CPT, bool VEC>
__global__ __launch_bounds__(256, CPT <= 16 ? 5 : 2) void k_row_update(const float* __restrict__ W, const uint8_t* __restrict__ mask,
                                                    const float* __restrict__ grad, int d_in, const int* __restrict__ remains,
                                                    const UpdateScratch* __restrict__ s, long long K_upd, long long budget,
                                                    uint8_t* __restrict__ mask_out, float* __restrict__ W_out,
                                                    long long* __restrict__ report) {
    __shared__ __align__(16) unsigned int h[3][kRowCopies][256];
    __shared__ int n_kept;
    __shared__ unsigned long long prune_threshold;
    __shared__ long long new_fan_in;
    const int r = blockIdx.x, t = threadIdx.x;
    const unsigned int row0 = (unsigned int)r * d_in;
    // rows of up to 4096 columns: the thread's columns are requested before the selection's state is (neither waits for the other)
    constexpr bool kEarly = VEC && CPT <= 16;
    float4 pw[kEarly ? CPT / 4 : 1], pg[kEarly ? CPT / 4 : 1];
    uint32_t pm[kEarly ? CPT / 4 : 1];
    if (kEarly) {
#pragma unroll
        for (int q = 0; q < CPT / 4; ++q) {
            const int c0 = 4 * (t + 256 * q);
            const unsigned int i = row0 + (c0 < d_in ? c0 : 0);
            pw[q] = *reinterpret_cast<const float4*>(W + i);
            pg[q] = *reinterpret_cast<const float4*>(grad + i);
            pm[q] = *reinterpret_cast<const uint32_t*>(mask + i);
        }
    }
    // step 5: the new fan-in from the count of staying neurons; step 6's finished selection (its last digit is taken here)
    if (t < 64) {
        const long long n_remaining = sum_copies(s->cnt_remaining, t);
        const long long n_ablated = sum_copies(s->cnt_ablated, t);
        long long k = n_remaining > 0 ? budget / n_remaining : 0;
        if (k > d_in) k = d_in;
        const SelState f2 = finished_walk(s, 2, t);
        if (t == 0) {
            prune_threshold = f2.prefix;
            new_fan_in = k;
            if (r == 0) {
                report[0] = k;
                report[1] = n_remaining;
                report[2] = n_ablated;
                report[3] = (long long)((unsigned long long)K_upd < f2.total ? (unsigned long long)K_upd : f2.total);
            }
        }
    }
    // column of the thread's j-th element
    auto col_of = [&](int j) { return VEC ? 4 * (t + 256 * (j >> 2)) + (j & 3) : t + 256 * j; };
    if (!remains[r]) {
        if (VEC) {
            for (int c = 4 * t; c < d_in; c += 1024) {
                *reinterpret_cast<uint32_t*>(mask_out + row0 + c) = 0u;
                *reinterpret_cast<float4*>(W_out + row0 + c) = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            }
        } else {
            for (int c = t; c < d_in; c += 256) { mask_out[row0 + c] = 0; W_out[row0 + c] = 0.0f; }
        }
        return;
    }
    unsigned long long key[CPT];
    unsigned int survives = 0, valid = 0;   // bit j: the thread's j-th column
    if (t == 0) n_kept = 0;
    __syncthreads();
    const unsigned long long t_prune = prune_threshold;
    const long long k_new = new_fan_in;
    auto take = [&](int j, int c, float w, float g, uint8_t m) {
        valid |= 1u << j;
        const unsigned int i = row0 + c;
        if (m != 0 && key_small_first(mag_bits(w), i) < t_prune) {
            survives |= 1u << j;
            key[j] = key_large_first(mag_bits(w), (unsigned int)c);
        } else {
            key[j] = key_large_first(mag_bits(g), (unsigned int)c);
        }
    };
#pragma unroll
    for (int j = 0; j < CPT; ++j) key[j] = 0;
    if (VEC) {
#pragma unroll
        for (int q = 0; q < CPT / 4; ++q) {
            const int c0 = 4 * (t + 256 * q);
            if (c0 < d_in) {
                // all three loads go out at once (the lines are fetched either way)
                const float4 w4 = kEarly ? pw[kEarly ? q : 0] : *reinterpret_cast<const float4*>(W + row0 + c0);
                const float4 g4 = kEarly ? pg[kEarly ? q : 0] : *reinterpret_cast<const float4*>(grad + row0 + c0);
                const uint32_t m4 = kEarly ? pm[kEarly ? q : 0] : *reinterpret_cast<const uint32_t*>(mask + row0 + c0);
                take(4 * q + 0, c0 + 0, w4.x, g4.x, (uint8_t)(m4 & 0xffu));
                take(4 * q + 1, c0 + 1, w4.y, g4.y, (uint8_t)((m4 >> 8) & 0xffu));
                take(4 * q + 2, c0 + 2, w4.z, g4.z, (uint8_t)((m4 >> 16) & 0xffu));
                take(4 * q + 3, c0 + 3, w4.w, g4.w, (uint8_t)(m4 >> 24));
            }
        }
    } else {
#pragma unroll
        for (int j = 0; j < CPT; ++j) {
            const int c = t + 256 * j;
            if (c < d_in) {
                const unsigned int i = row0 + c;
                const float w = W[i], g = grad[i];
                const uint8_t m = mask[i];
                take(j, c, w, g, m);
            }
        }
    }
    if (survives) atomicAdd(&n_kept, __popc(survives));
    __syncthreads();
    const long long kept = n_kept;
    unsigned long long t_keep = 0;       // keep a surviving weight iff its key >= t_keep
    unsigned long long t_grow = ~0ull;   // grow a free position iff its key >= t_grow
    if (kept > k_new) {
        if (k_new == 0) t_keep = ~0ull;
        else t_keep = row_select<CPT>((unsigned long long)k_new, [&](int j, unsigned long long& k_out) {
            k_out = key[j];
            return ((survives >> j) & 1u) != 0;
        }, h);
    } else if (kept < k_new) {
        t_grow = row_select<CPT>((unsigned long long)(k_new - kept), [&](int j, unsigned long long& k_out) {
            k_out = key[j];
            return ((valid >> j) & 1u) != 0 && ((survives >> j) & 1u) == 0;
        }, h);
    }
    // column j of the thread: kept (its weight is copied), grown (weight zero) or free
    auto kept_j = [&](int j) { return ((survives >> j) & 1u) != 0 && key[j] >= t_keep; };
    auto grown_j = [&](int j) { return ((valid >> j) & 1u) != 0 && ((survives >> j) & 1u) == 0 && key[j] >= t_grow; };
    if (VEC) {
#pragma unroll
        for (int q = 0; q < CPT / 4; ++q) {
            const int c0 = 4 * (t + 256 * q);
            if (c0 >= d_in) continue;
            const bool k0 = kept_j(4 * q), k1 = kept_j(4 * q + 1), k2 = kept_j(4 * q + 2), k3 = kept_j(4 * q + 3);
            float4 w4 = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            if (k0 || k1 || k2 || k3) w4 = *reinterpret_cast<const float4*>(W + row0 + c0);
            const uint32_t m4 = (uint32_t)(k0 || grown_j(4 * q)) | ((uint32_t)(k1 || grown_j(4 * q + 1)) << 8) |
                                ((uint32_t)(k2 || grown_j(4 * q + 2)) << 16) | ((uint32_t)(k3 || grown_j(4 * q + 3)) << 24);
            *reinterpret_cast<uint32_t*>(mask_out + row0 + c0) = m4;
            *reinterpret_cast<float4*>(W_out + row0 + c0) = make_float4(k0 ? w4.x : 0.0f, k1 ? w4.y : 0.0f, k2 ? w4.z : 0.0f, k3 ? w4.w : 0.0f);
        }
    } else {
#pragma unroll
        for (int j = 0; j < CPT; ++j) {
            const int c = t + 256 * j;
            if (c >= d_in) continue;
            const bool kj = kept_j(j);
            mask_out[row0 + c] = (uint8_t)(kj || grown_j(j));
            W_out[row0 + c] = kj ? W[row0 + c] : 0.0f;
        }
    }
}

// A layer without elements: nothing stays, nothing is pruned.
__global__ void k_update_report_empty(long long* __restrict__ report) {
    if (threadIdx.x < 4) report[threadIdx.x] = 0;
}

template <bool PAIR>
static void layer_select(const float* W, const uint8_t* mask, const float* grad, const int* remains, unsigned int N, int d_in,
                         UpdateScratch* s, unsigned long long* candA, unsigned long long* candB, unsigned long long cap, hipStream_t st) {
    const bool vec = d_in % 4 == 0 && reinterpret_cast<uintptr_t>(W) % 16 == 0 && reinterpret_cast<uintptr_t>(grad) % 16 == 0 &&
                     reinterpret_cast<uintptr_t>(mask) % 4 == 0;
    // a thread takes 1 or 4 elements per step and at least 8 steps (every workgroup ends with up to 512 atomics), at most
    // four workgroups per compute unit
    const unsigned int per_step = (vec ? 4u : 1u) * kPassThreads;
    unsigned int blocks = (N / 8 + per_step - 1) / per_step;
    if (blocks > 1024) blocks = 1024;
    if (blocks == 0) blocks = 1;
#define SRIGL_HIST(COMPACT, VEC)                                                                                                   \
    hipLaunchKernelGGL((k_layer_hist<PAIR, COMPACT, VEC>), dim3(blocks), dim3(kPassThreads), 0, st, W, mask, grad, remains, N, d_in, pass, s, \
                       candA, candB, cap)
    for (int pass = 0; pass < 8; ++pass) {
        if (pass == kCompactPass && cap > 0) { if (vec) SRIGL_HIST(true, true); else SRIGL_HIST(true, false); }
        else { if (vec) SRIGL_HIST(false, true); else SRIGL_HIST(false, false); }
    }
#undef SRIGL_HIST
}

// Keys per candidate list: a sixteenth of the layer, at least 4096 (a list holds the keys that share 16 leading bits with
// the threshold: a fraction of a percent of real-valued contents; constant contents overflow it and do without).
static size_t cand_capacity(int32_t d_out, int32_t d_in) {
    const size_t n = (d_out > 0 && d_in > 0) ? (size_t)d_out * (size_t)d_in : 0;
    const size_t c = n / 16;
    return c < 4096 ? 4096 : c;
}
static size_t update_head_bytes(int32_t d_out) {
    const size_t rows = d_out > 0 ? (size_t)d_out : 0;
    return ((sizeof(UpdateScratch) + rows * sizeof(int32_t) + 255) / 256) * 256;
}

}  // namespace srigl

using namespace srigl;

extern "C" {

size_t srigl_mask_update_workspace_bytes(int32_t d_out, int32_t d_in) {
    return update_head_bytes(d_out) + 2 * cand_capacity(d_out, d_in) * sizeof(unsigned long long);
}

srigl_status srigl_mask_update(const float* W, const uint8_t* mask, const float* grad, int32_t d_out, int32_t d_in, int32_t k,
                               int64_t K_upd, int32_t gamma_percent, int64_t budget, uint8_t* mask_out, float* W_out,
                               void* workspace, size_t workspace_bytes, int64_t* report_dev, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (d_out < 0 || d_in < 0 || k < 0 || k > d_in || K_upd < 0 || gamma_percent < 0 || budget < 0 || report_dev == nullptr)
        return SRIGL_ERR_INVALID_ARG;
    if ((long long)d_out * d_in >= (1ll << 32)) return SRIGL_ERR_UNSUPPORTED;   // positions are ranked as 32-bit numbers
    if (d_in > 8192) return SRIGL_ERR_UNSUPPORTED;                              // a row is held in the registers of one workgroup
    if (workspace == nullptr) return SRIGL_ERR_INVALID_ARG;
    if (workspace_bytes < srigl_mask_update_workspace_bytes(d_out, d_in)) return SRIGL_ERR_CAPACITY;
    const unsigned int N = (unsigned int)((long long)d_out * d_in);
    if (N > 0 && (W == nullptr || mask == nullptr || grad == nullptr || mask_out == nullptr || W_out == nullptr)) return SRIGL_ERR_INVALID_ARG;
    UpdateScratch* s = static_cast<UpdateScratch*>(workspace);
    int* remains = reinterpret_cast<int*>(static_cast<unsigned char*>(workspace) + sizeof(UpdateScratch));
    const unsigned long long cap = cand_capacity(d_out, d_in);
    unsigned long long* candA = reinterpret_cast<unsigned long long*>(static_cast<unsigned char*>(workspace) + update_head_bytes(d_out));
    unsigned long long* candB = candA + cap;
    long long* report = reinterpret_cast<long long*>(report_dev);
    if (N == 0) {
        hipLaunchKernelGGL(k_update_report_empty, dim3(1), dim3(64), 0, st, report);
        return hip_ok(hipGetLastError());
    }
    // 19 launches, each reading what the one before it counted: the state, 8 passes of steps 1-3, the per-neuron counts of
    // steps 3-5, 8 passes of step 6, and step 7 (which also writes the report)
    hipLaunchKernelGGL(k_update_init, dim3(48), dim3(256), 0, st, s, (long long)K_upd);
    layer_select<true>(W, mask, grad, remains, N, d_in, s, candA, candB, cap, st);
    const bool vec_in = d_in % 4 == 0 && reinterpret_cast<uintptr_t>(W) % 16 == 0 && reinterpret_cast<uintptr_t>(grad) % 16 == 0 &&
                        reinterpret_cast<uintptr_t>(mask) % 4 == 0;
    if (vec_in) hipLaunchKernelGGL(k_row_salient<true>, dim3((d_out + 3) / 4), dim3(256), 0, st, W, mask, grad, d_out, d_in, k, gamma_percent, s, remains);
    else hipLaunchKernelGGL(k_row_salient<false>, dim3((d_out + 3) / 4), dim3(256), 0, st, W, mask, grad, d_out, d_in, k, gamma_percent, s, remains);
    layer_select<false>(W, mask, grad, remains, N, d_in, s, candA, candB, cap, st);
    // 16-byte moves need rows that start on 16-byte (mask: 4-byte) boundaries
    const bool vec = vec_in && reinterpret_cast<uintptr_t>(W_out) % 16 == 0 && reinterpret_cast<uintptr_t>(mask_out) % 4 == 0;
#define SRIGL_ROW_UPDATE(CPT)                                                                                                      \
    if (vec) hipLaunchKernelGGL((k_row_update<CPT, true>), dim3(d_out), dim3(256), 0, st, W, mask, grad, d_in, remains, s,         \
                                (long long)K_upd, (long long)budget, mask_out, W_out, report);                                     \
    else hipLaunchKernelGGL((k_row_update<CPT, false>), dim3(d_out), dim3(256), 0, st, W, mask, grad, d_in, remains, s,            \
                            (long long)K_upd, (long long)budget, mask_out, W_out, report)
    if (d_in <= 1024) { SRIGL_ROW_UPDATE(4); }
    else if (d_in <= 4096) { SRIGL_ROW_UPDATE(16); }
    else { SRIGL_ROW_UPDATE(32); }
#undef SRIGL_ROW_UPDATE
    return hip_ok(hipGetLastError());
}

}  // extern "C"
