// CPU oracle for the condensed constant fan-in sparse linear layer.
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, plain-loop statement of what
// the GPU library must compute.  It shares no code, header, table or helper with
// the HIP path, and nothing in the product imports it: only tests/, the smoke
// check and the benchmark's cpu_baseline leg call it.
//
// What each function follows (paper: arXiv 2305.02299):
//   * oracle_dense_masked_fwd_*  -- the definition: the ordinary matrix-vector
//     product of App. E, first equation, with W replaced by W (.) M, plus bias
//     (Sec. 4.4 extracts "weights and bias" of the layer).
//   * oracle_fwd_*               -- Alg. 1 (condensed forward), three nested
//     loops b, n, k in the paper's order: every stored weight of neuron n times the
//     input column its index names, summed into output (b, n).
//     Readings where Alg. 1 is silent: a bias is added; the output has the full
//     layer width and the s-th stored neuron writes column active[s]; every
//     column of a neuron that is not stored (ablated, Sec. 3.1 step 4: all of
//     its incoming weights are pruned) holds its bias only.
//   * oracle_condense            -- App. E, last paragraph: two n x k arrays, one
//     with the values of the non-zeros of W and one with their column indices;
//     Sec. 4.4: ablated neurons are dropped.  Reading: which entries are
//     "non-zero" is decided by the mask, not by the value; columns appear in
//     ascending order; stored neurons appear in ascending order.
//   * oracle_densify / oracle_structured_fwd_* -- the structured-only representation of Sec. 4.4 /
//     Fig. 4: ablated neurons removed, the remaining neurons' rows kept dense.
//   * oracle_check_fanin_*       -- the constant fan-in invariant (Fig. 1a, Sec.
//     3.1): every neuron that is not ablated has exactly k unmasked weights.
//
// Floating point: accumulation in double in ascending k, one rounding to float
// at the end.  Parity status: every function here is pinned by the CPU tests
// (hand-worked fixture, dense definition by a library matmul, K == d_in special
// case, one-hot inputs, integer-exact inputs, round trip through the mask).

#include <cmath>
#include <cstdint>
#include <algorithm>
#include <cstring>
#include <utility>
#include <vector>
#ifdef _OPENMP
#include <omp.h>
#endif

extern "C" {

// report[0]=K, [1]=n_active, [2]=n_bad_rows, [3]=first_bad_row (-1 if none)
// A row is "bad" when its count of non-zero mask bytes is neither 0 nor K.
// K_expected < 0: K is the count of the first non-empty row (0 if all rows empty).
int oracle_check_fanin_mask(const uint8_t* mask, int n_rows, int d_in, int K_expected, int32_t* report) {
    int K = K_expected;
    if (K < 0) {
        K = 0;
        for (int r = 0; r < n_rows && K == 0; ++r) {
            int c = 0;
            for (int j = 0; j < d_in; ++j) c += mask[(size_t)r * d_in + j] != 0;
            K = c;
        }
    }
    int n_active = 0, n_bad = 0, first_bad = -1;
    for (int r = 0; r < n_rows; ++r) {
        int c = 0;
        for (int j = 0; j < d_in; ++j) c += mask[(size_t)r * d_in + j] != 0;
        if (c == 0) continue;
        if (c == K) { ++n_active; continue; }
        ++n_bad;
        if (first_bad < 0) first_bad = r;
    }
    report[0] = K; report[1] = n_active; report[2] = n_bad; report[3] = first_bad;
    return n_bad == 0 ? 0 : 2;
}

// Condensed-form check: every row of idx[n_rows][K] in [0, d_in) and strictly
// ascending (hence distinct, App. E: j_alpha != j_alpha').
int oracle_check_fanin_idx(const int32_t* idx, int n_rows, int K, int d_in, int32_t* report) {
    int n_bad = 0, first_bad = -1;
    for (int r = 0; r < n_rows; ++r) {
        bool ok = true;
        for (int k = 0; k < K; ++k) {
            int32_t j = idx[(size_t)r * K + k];
            if (j < 0 || j >= d_in) ok = false;
            if (k > 0 && j <= idx[(size_t)r * K + k - 1]) ok = false;
        }
        if (!ok) { ++n_bad; if (first_bad < 0) first_bad = r; }
    }
    report[0] = K; report[1] = n_rows - n_bad; report[2] = n_bad; report[3] = first_bad;
    return n_bad == 0 ? 0 : 2;
}

// W: d_out x d_in elements of elem_bytes bytes each (4 = fp32, 2 = bf16), copied bit for bit.
// Outputs sized for d_out rows.  Returns 0, or 2 if some row count is neither 0 nor K
// (then *first_bad_row names it and the outputs are not meaningful).
int oracle_condense(const void* W, int elem_bytes, const uint8_t* mask, int d_out, int d_in, int K,
                    void* W_c, int32_t* idx, int32_t* active, int32_t* n_active, int32_t* first_bad_row) {
    const unsigned char* w = static_cast<const unsigned char*>(W);
    unsigned char* wc = static_cast<unsigned char*>(W_c);
    int slot = 0;
    *first_bad_row = -1;
    for (int r = 0; r < d_out; ++r) {
        int c = 0;
        for (int j = 0; j < d_in; ++j) c += mask[(size_t)r * d_in + j] != 0;
        if (c == 0) continue;                       // ablated neuron: dropped
        if (c != K) { *first_bad_row = r; *n_active = slot; return 2; }
        active[slot] = r;
        int t = 0;
        for (int j = 0; j < d_in; ++j) {
            if (mask[(size_t)r * d_in + j] == 0) continue;
            idx[(size_t)slot * K + t] = j;
            std::memcpy(wc + ((size_t)slot * K + t) * elem_bytes, w + ((size_t)r * d_in + j) * elem_bytes, elem_bytes);
            ++t;
        }
        ++slot;
    }
    *n_active = slot;
    return 0;
}

static inline float bf16_to_float(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    std::memcpy(&f, &u, 4);
    return f;
}

// Alg. 1 with bias and the active-neuron scatter.  active == NULL means the s-th
// stored neuron is column s.  bias == NULL means zero bias (Alg. 1 verbatim).
// scale (optional, B x d_out doubles): |bias| + sum_k |w * x| per output, the size
// of the terms that were added, against which a relative error is measured.
static void fwd_generic(const float* xf, const uint16_t* xh, int B, int d_in,
                        const float* wf, const uint16_t* wh, const int32_t* idx, const int32_t* active,
                        int n_active, int K, const float* bias, int d_out, float* y, double* scale) {
    for (int b = 0; b < B; ++b)
        for (int r = 0; r < d_out; ++r) {
            float bv = bias ? bias[r] : 0.0f;
            y[(size_t)b * d_out + r] = bv;
            if (scale) scale[(size_t)b * d_out + r] = std::fabs((double)bv);
        }
    for (int b = 0; b < B; ++b) {
        for (int n = 0; n < n_active; ++n) {
            double acc = 0.0, mag = 0.0;
            for (int k = 0; k < K; ++k) {   // Alg. 1: the k-th stored weight of neuron n meets the input column it names
                const size_t t = (size_t)n * K + k;
                const size_t j = (size_t)b * d_in + idx[t];
                const double xv = xf ? (double)xf[j] : (double)bf16_to_float(xh[j]);
                const double wv = wf ? (double)wf[t] : (double)bf16_to_float(wh[t]);
                acc += xv * wv;
                mag += std::fabs(xv * wv);
            }
            int col = active ? active[n] : n;
            double bv = bias ? (double)bias[col] : 0.0;
            y[(size_t)b * d_out + col] = (float)(acc + bv);
            if (scale) scale[(size_t)b * d_out + col] = mag + std::fabs(bv);
        }
    }
}

void oracle_fwd_f32(const float* x, int B, int d_in, const float* W_c, const int32_t* idx,
                    const int32_t* active, int n_active, int K, const float* bias, int d_out,
                    float* y, double* scale) {
    fwd_generic(x, nullptr, B, d_in, W_c, nullptr, idx, active, n_active, K, bias, d_out, y, scale);
}

void oracle_fwd_bf16(const uint16_t* x, int B, int d_in, const uint16_t* W_c, const int32_t* idx,
                     const int32_t* active, int n_active, int K, const float* bias, int d_out,
                     float* y, double* scale) {
    fwd_generic(nullptr, x, B, d_in, nullptr, W_c, idx, active, n_active, K, bias, d_out, y, scale);
}

// The definition: y[b][r] = bias[r] + sum_j M[r][j] W[r][j] x[b][j], all d_in terms visited.
void oracle_dense_masked_fwd_f32(const float* x, int B, int d_in, const float* W, const uint8_t* mask,
                                 const float* bias, int d_out, float* y) {
    for (int b = 0; b < B; ++b)
        for (int r = 0; r < d_out; ++r) {
            double acc = 0.0;
            for (int j = 0; j < d_in; ++j)
                if (mask[(size_t)r * d_in + j] != 0)
                    acc += (double)W[(size_t)r * d_in + j] * (double)x[(size_t)b * d_in + j];
            y[(size_t)b * d_out + r] = (float)(acc + (bias ? (double)bias[r] : 0.0));
        }
}

// The unstructured comparison of Sec. 4.4 / Fig. 4 (the same weights in compressed sparse row form): row r holds the
// entries values[row_ptr[r] .. row_ptr[r+1]) at columns col_idx[...]; y[b][r] = bias[r] + sum over the row's entries of
// value * x[b][column].  A row without entries outputs its bias.  fp32 storage, fp64 accumulation; scale as in fwd.
void oracle_csr_fwd_f32(const float* x, int B, int d_in, const float* values, const int32_t* col_idx, const int32_t* row_ptr,
                        const float* bias, int d_out, float* y, double* scale) {
    (void)d_in;
    for (int b = 0; b < B; ++b)
        for (int r = 0; r < d_out; ++r) {
            double acc = 0.0, mag = 0.0;
            for (int t = row_ptr[r]; t < row_ptr[r + 1]; ++t) {
                const double term = (double)values[t] * (double)x[(size_t)b * d_in + col_idx[t]];
                acc += term;
                mag += std::fabs(term);
            }
            const double bv = bias ? (double)bias[r] : 0.0;
            y[(size_t)b * d_out + r] = (float)(acc + bv);
            if (scale) scale[(size_t)b * d_out + r] = mag + std::fabs(bv);
        }
}

// Structured-only representation (Sec. 4.4, Fig. 4 and App. H: the same layer with the ablated neurons removed and
// the sparsity inside the remaining rows left unused): the stored neurons keep dense rows.
// densify: Wd[s][j] = W_c[s][t] where idx[s][t] == j, zero elsewhere (elements copied bit for bit).
void oracle_densify(const void* W_c, int elem_bytes, const int32_t* idx, int n_active, int K, int d_in, void* Wd) {
    const unsigned char* wc = static_cast<const unsigned char*>(W_c);
    unsigned char* wd = static_cast<unsigned char*>(Wd);
    std::memset(wd, 0, (size_t)n_active * d_in * elem_bytes);
    for (int s = 0; s < n_active; ++s)
        for (int t = 0; t < K; ++t)
            std::memcpy(wd + ((size_t)s * d_in + idx[(size_t)s * K + t]) * elem_bytes, wc + ((size_t)s * K + t) * elem_bytes, elem_bytes);
}

// y[b][active[s]] = bias + sum over ALL j of Wd[s][j] * x[b][j]; other columns hold their bias.
static void structured_generic(const float* xf, const uint16_t* xh, int B, int d_in, const float* wf, const uint16_t* wh,
                               const int32_t* active, int n_active, const float* bias, int d_out, float* y) {
    for (int b = 0; b < B; ++b)
        for (int r = 0; r < d_out; ++r) y[(size_t)b * d_out + r] = bias ? bias[r] : 0.0f;
    for (int b = 0; b < B; ++b)
        for (int s = 0; s < n_active; ++s) {
            double acc = 0.0;
            for (int j = 0; j < d_in; ++j) {
                double xv = xf ? (double)xf[(size_t)b * d_in + j] : (double)bf16_to_float(xh[(size_t)b * d_in + j]);
                double wv = wf ? (double)wf[(size_t)s * d_in + j] : (double)bf16_to_float(wh[(size_t)s * d_in + j]);
                acc += xv * wv;
            }
            const int col = active ? active[s] : s;
            y[(size_t)b * d_out + col] = (float)(acc + (bias ? (double)bias[col] : 0.0));
        }
}
void oracle_structured_fwd_f32(const float* x, int B, int d_in, const float* Wd, const int32_t* active, int n_active,
                               const float* bias, int d_out, float* y) {
    structured_generic(x, nullptr, B, d_in, Wd, nullptr, active, n_active, bias, d_out, y);
}
void oracle_structured_fwd_bf16(const uint16_t* x, int B, int d_in, const uint16_t* Wd, const int32_t* active, int n_active,
                                const float* bias, int d_out, float* y) {
    structured_generic(nullptr, x, B, d_in, nullptr, Wd, active, n_active, bias, d_out, y);
}

// Activation between the two linear layers of an MLP block (App. H times one linear of a ViT MLP block): 0 identity,
// 1 max(v, 0), 2 the erf-form GELU v * Phi(v), Phi the normal distribution function.  In place, evaluated in double.
static double activation_f64(double v, int act) {
    if (act == 1) return v > 0.0 ? v : 0.0;
    if (act == 2) return 0.5 * v * (1.0 + std::erf(v / std::sqrt(2.0)));
    return v;
}

void oracle_activate(float* y, long long n, int act) {
    for (long long i = 0; i < n; ++i) y[i] = (float)activation_f64((double)y[i], act);
}

// Width reduction (Sec. 3.1: ablating neurons reduces the width of a layer).  Layer 1 has d_hidden neurons of which
// active1[0..n_active1) are stored; an ablated neuron r outputs the constant act(bias1[r]).  Layer 2 (n2 stored rows of
// fan-in K2 over the d_hidden outputs of layer 1) is rewritten to read the compact vector of the n_active1 stored
// outputs: an index that names stored neuron active1[p] becomes p; a term on an ablated neuron is a constant and moves
// into the bias of that row's neuron; the row is filled up to K2 entries again with the smallest positions it does not use yet, weight zero,
// and sorted ascending, so that it is a constant fan-in row like any other.  Returns 0, or 1 if K2 > n_active1 (no
// room for K2 distinct positions).  Weights are fp32 (elem_bytes 4) or bf16 bit patterns (2), copied bit for bit.
// bias2 / bias_out have d_out2 entries; stored row n of layer 2 is column active2[n] (n itself if active2 == NULL).
int oracle_fold_ablated_inputs(const int32_t* idx2, const void* W_c2, int elem_bytes, const float* bias2, const int32_t* active2,
                               int n2, int K2, int d_out2, const int32_t* active1, int n_active1, int d_hidden,
                               const float* bias1, int act, int32_t* idx_out, void* W_out, float* bias_out) {
    if (K2 > n_active1) return 1;
    for (int c = 0; c < d_out2; ++c) bias_out[c] = bias2 ? bias2[c] : 0.0f;
    std::vector<int32_t> position(d_hidden, -1);
    for (int p = 0; p < n_active1; ++p) position[active1[p]] = p;
    const unsigned char* w_in = static_cast<const unsigned char*>(W_c2);
    unsigned char* w_out = static_cast<unsigned char*>(W_out);
    for (int n = 0; n < n2; ++n) {
        std::vector<std::pair<int32_t, int>> entries;   // (new index, source k or -1 for a filler)
        std::vector<char> used(n_active1, 0);
        double constant = 0.0;
        for (int k = 0; k < K2; ++k) {
            const int32_t j = idx2[(size_t)n * K2 + k];
            const int32_t p = position[j];
            if (p >= 0) {
                entries.push_back({p, k});
                used[p] = 1;
            } else {
                double w;
                if (elem_bytes == 4) { float f; std::memcpy(&f, w_in + ((size_t)n * K2 + k) * 4, 4); w = f; }
                else { uint16_t h; std::memcpy(&h, w_in + ((size_t)n * K2 + k) * 2, 2); w = bf16_to_float(h); }
                constant += w * activation_f64(bias1 ? (double)bias1[j] : 0.0, act);
            }
        }
        for (int g = 0; (int)entries.size() < K2; ++g)
            if (!used[g]) entries.push_back({g, -1});
        std::sort(entries.begin(), entries.end());
        for (int k = 0; k < K2; ++k) {
            idx_out[(size_t)n * K2 + k] = entries[k].first;
            unsigned char* dst = w_out + ((size_t)n * K2 + k) * elem_bytes;
            if (entries[k].second >= 0) std::memcpy(dst, w_in + ((size_t)n * K2 + entries[k].second) * elem_bytes, elem_bytes);
            else std::memset(dst, 0, elem_bytes);
        }
        const int col = active2 ? active2[n] : n;
        bias_out[col] = (float)((bias2 ? (double)bias2[col] : 0.0) + constant);
    }
    return 0;
}

// One SRigL connectivity update of one layer (Sec. 3.1, steps 1-7), fp32 weights and gradients, in the paper's order.
// mask: d_out x d_in bytes, every row holds 0 (ablated) or k kept weights.  Readings where the text leaves a choice:
//  * step 3: salient by the prune criterion = a kept weight that is not among the K_upd smallest-magnitude kept weights of
//    the layer (it would survive the pruning); salient by the growth criterion = a pruned position among the K_upd
//    largest-magnitude gradients at pruned positions of the layer (it would be grown); a neuron's count is how many of
//    both lie in its row.  (Taking "top-K" of the magnitudes literally would leave no salient weight, hence no neuron,
//    once the update fraction has annealed to zero.)
//  * step 4: a neuron that holds weights is ablated if its count is below max(gamma * k, 1), gamma = gamma_percent / 100
//    (the appendix on tuning gamma_sal, caption of its figure of minimum salient weights per ResNet-50 layer: the
//    minimum is one whenever gamma * k is below one); a neuron without weights on entry stays ablated;
//  * step 5: k' = min(d_in, budget / number of remaining neurons) in integers (the layer keeps its weight budget);
//  * step 6: the K_upd smallest-magnitude kept weights of the remaining neurons are pruned, layer-wide;
//  * step 7: each remaining neuron keeps its unpruned weights (its k' largest, should it hold more than k') and grows the
//    positions it does not keep in order of decreasing gradient magnitude until it holds k';
//  * equal magnitudes are ordered by position (lower flat index / column first in every ranking);
//  * grown weights start at zero, pruned weights are set to zero (as in RigL).
// out4: {k', remaining neurons, neurons ablated by this update, weights pruned in step 6}.
struct Ranked { uint32_t key; int64_t pos; };
static uint32_t magnitude_bits(float v) { uint32_t u; std::memcpy(&u, &v, 4); return u & 0x7fffffffu; }

void oracle_mask_update(const float* W, const uint8_t* mask, const float* grad, int d_out, int d_in, int k, long long K_upd,
                        int gamma_percent, long long budget, uint8_t* mask_out, float* W_out, long long* out4) {
    const int64_t N = (int64_t)d_out * d_in;
    // steps 1-3
    std::vector<Ranked> kept, pruned;
    for (int64_t i = 0; i < N; ++i) {
        if (mask[i]) kept.push_back({magnitude_bits(W[i]), i});
        else pruned.push_back({magnitude_bits(grad[i]), i});
    }
    auto larger_first = [](const Ranked& a, const Ranked& b) { return a.key != b.key ? a.key > b.key : a.pos < b.pos; };
    auto smaller_first = [](const Ranked& a, const Ranked& b) { return a.key != b.key ? a.key < b.key : a.pos < b.pos; };
    std::sort(kept.begin(), kept.end(), smaller_first);
    std::sort(pruned.begin(), pruned.end(), larger_first);
    std::vector<long long> salient(d_out, 0), held(d_out, 0);
    for (int64_t t = 0; t < (int64_t)kept.size(); ++t) {
        ++held[kept[t].pos / d_in];
        if (t >= K_upd) ++salient[kept[t].pos / d_in];
    }
    for (int64_t t = 0; t < (int64_t)pruned.size() && t < K_upd; ++t) ++salient[pruned[t].pos / d_in];
    // step 4
    std::vector<char> remains(d_out, 0);
    long long n_remaining = 0, n_ablated_now = 0;
    for (int r = 0; r < d_out; ++r) {
        if (held[r] == 0) continue;
        const bool too_few = salient[r] < 1 || salient[r] * 100 < (long long)gamma_percent * k;
        if (too_few) ++n_ablated_now;
        else { remains[r] = 1; ++n_remaining; }
    }
    // step 5
    long long k_new = n_remaining > 0 ? budget / n_remaining : 0;
    if (k_new > d_in) k_new = d_in;
    // step 6
    std::vector<Ranked> candidates;
    for (const Ranked& e : kept)
        if (remains[e.pos / d_in]) candidates.push_back(e);
    std::sort(candidates.begin(), candidates.end(), smaller_first);
    std::vector<char> keep(N, 0);
    long long n_pruned = 0;
    for (int64_t t = 0; t < (int64_t)candidates.size(); ++t) {
        if (t < K_upd) ++n_pruned;
        else keep[candidates[t].pos] = 1;
    }
    // step 7
    for (int64_t i = 0; i < N; ++i) { mask_out[i] = 0; W_out[i] = 0.0f; }
    for (int r = 0; r < d_out; ++r) {
        if (!remains[r]) continue;
        std::vector<Ranked> mine, others;
        for (int c = 0; c < d_in; ++c) {
            const int64_t i = (int64_t)r * d_in + c;
            if (keep[i]) mine.push_back({magnitude_bits(W[i]), (int64_t)c});
            else others.push_back({magnitude_bits(grad[i]), (int64_t)c});
        }
        std::sort(mine.begin(), mine.end(), larger_first);
        std::sort(others.begin(), others.end(), larger_first);
        long long have = 0;
        for (const Ranked& e : mine) {
            if (have == k_new) break;
            mask_out[(int64_t)r * d_in + e.pos] = 1;
            W_out[(int64_t)r * d_in + e.pos] = W[(int64_t)r * d_in + e.pos];
            ++have;
        }
        for (const Ranked& e : others) {
            if (have == k_new) break;
            mask_out[(int64_t)r * d_in + e.pos] = 1;   // grown: weight starts at zero
            ++have;
        }
    }
    out4[0] = k_new; out4[1] = n_remaining; out4[2] = n_ablated_now; out4[3] = n_pruned;
}

// Timing companion of oracle_fwd_f32 (not used for parity): the same three loops of Alg. 1 with fp32
// accumulation and the batch x neuron iterations spread over the host cores with OpenMP.  It exists so that
// the benchmark can say what all host cores do with the plain loops; nothing else is changed or tuned.
void oracle_fwd_f32_allcores(const float* x, int B, int d_in, const float* W_c, const int32_t* idx,
                             const int32_t* active, int n_active, int K, const float* bias, int d_out, float* y) {
#pragma omp parallel for schedule(static)
    for (int b = 0; b < B; ++b)
        for (int r = 0; r < d_out; ++r) y[(size_t)b * d_out + r] = bias ? bias[r] : 0.0f;
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < B; ++b) {
        for (int n = 0; n < n_active; ++n) {
            float acc = 0.0f;
            for (int k = 0; k < K; ++k) acc += x[(size_t)b * d_in + idx[(size_t)n * K + k]] * W_c[(size_t)n * K + k];
            const int col = active ? active[n] : n;
            y[(size_t)b * d_out + col] = acc + (bias ? bias[col] : 0.0f);
        }
    }
}

int oracle_num_threads() {
#ifdef _OPENMP
    int n = 1;
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
    return n;
#else
    return 1;
#endif
}

}  // extern "C"
