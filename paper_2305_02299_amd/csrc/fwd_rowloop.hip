// ROWLOOP forward kernel (gfx950): the batched formulation of fwd_rowlane.inl (lanes are batch rows, the activation
// tile transposed in LDS, weights and LDS offsets through DPP row broadcasts; Alg. 1 of arXiv 2305.02299 with the bias of
// Sec. 4.4 and the ablated neurons of Sec. 3.1 step 4) for inputs narrow enough that a batch tile holds *every* column of x.
//
// With all of d_in in LDS there is no walk over column chunks: a stored row's K terms are one contiguous range, no partial
// sum has to live across a chunk boundary, and so a wavefront is not limited to the handful of stored rows whose
// accumulators fit its registers.  It walks any number of rows one after the other and parks each finished row in a
// result tile in LDS.  A workgroup can therefore own as many stored rows as the result tile has room for (hundreds), and
// the batch tile of x, which every workgroup of the chunked kernel stages again for every 16-128 stored rows, is staged
// once per several hundred: at 1024 batch rows on a 768-wide input 8 groups of stored rows instead of 24.
//
// Tile: two batch rows per lane in H = 4 (32-row tile) or 2 (64-row tile) term slices; row stride BT + 4 words.
// Terms: a term slice takes a run of ceil(K / H) consecutive terms of the row, 16 to a block, one vector load per array and
// block, requested two rows ahead; the group walk (LDS reads one group ahead of the multiply-adds) is the chunked kernel's.
#include "fwd_rowlane.inl"
#include <type_traits>

namespace srigl {

constexpr int kRowloopReadAhead = 2;   // groups of LDS reads in flight ahead of the multiply-adds (walk_groups)
struct RowloopPlan {
    int H, NW, NG, KPRE, n_btiles, n_groups, out_off, span_cap, bt_major;
    int rounds;
    size_t lds;
    bool ok;
};

template <int R, int H, int KPRE, typename XT, typename IT>
__global__ __launch_bounds__(1024) void k_fwd_rowloop(const XT* __restrict__ x, int B, int d_in, const XT* __restrict__ W_c,
                                                      const IT* __restrict__ idx, const int32_t* __restrict__ active, int n_active,
                                                      int K, const float* __restrict__ bias, int d_out, float* __restrict__ y,
                                                      int NG, int n_btiles, int n_groups, int out_off, int span_cap, int act, int bt_major) {
    extern __shared__ float lds[];   // x tile [d_in + 1][S]; result tile [BT][NG | 1]; bias [NG], or bias and column table [span_cap] each
    constexpr int LR = kWave / H;            // lanes per term slice
    constexpr int BT = LR * R;               // batch rows per tile
    constexpr int S = rowlane_row_stride(BT, H, R);
    constexpr int S4 = S * 4;
    static_assert(R == 2 && (H == 2 || H == 4) && !rowlane_swizzled(R), "two rows per lane in two or four term slices");

    // consecutive workgroup ids go to different XCDs (one L2 each): either all batch tiles of a group of stored rows share an
    // XCD (its L2 fetches that group's W_c / idx once and all of x), or (bt_major) all groups of a batch tile (its own rows of
    // x, which every workgroup waits for at its start, and all of W_c / idx, which streams in behind the arithmetic)
    const int wg = blockIdx.x;
    const int xcd = wg & 7, inx = wg >> 3;
    const int dec_d = bt_major ? n_groups : n_btiles;
    const int dec_q = inx / dec_d, dec_r = inx - dec_q * dec_d;
    const int bt = bt_major ? dec_q * 8 + xcd : dec_r;
    const int g = bt_major ? dec_r : dec_q * 8 + xcd;
    if (g >= n_groups || bt >= n_btiles) return;

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int rowl = lane & (LR - 1);
    const int wv_id = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nw = blockDim.x >> 6;
    const int b0 = bt * BT;
    const int sg0 = g * NG;
    const int ng = min(NG, n_active - sg0);   // > 0: n_groups = ceil(n_active / NG)
    const int C = d_in;                        // a multiple of 16 (host)
    const int zero_off = C * S4;
    const int t_last = n_active * K - 1;

    // ---- the tile: units of 16 rows x 16 columns, eight per wavefront in flight ----
    const int dq = lane & 3, db = lane >> 2;
    constexpr int RT = BT / 16, RT_LOG2 = RT == 2 ? 1 : 2;
    static_assert(RT == 2 || RT == 4, "32- or 64-row tiles");
    const int n_units = RT * (C >> 4);
    const char* const xtile = reinterpret_cast<const char*>(x + (size_t)b0 * d_in);

    // Terms.  Slice p of the lanes takes the p-th run of Q = ceil(K / H) consecutive terms of a row, 16 steps to a block: the
    // lane at position l16 of its 16-lane DPP row loads term p * Q + 16 * block + l16 (16 consecutive words per slice and
    // block) and that is also the term its DPP row broadcasts at step l16 of the block, so no cross-lane fetch is needed.
    // D = 2 rows are in flight ahead of the one being walked (D buffers in turn; three and four measured 1-4 % slower, from HBM
    // and cached, also once the waits for a row's terms were counted ones).
    const int Q = (K + H - 1) / H;
    const int slice = lane / LR, l16 = lane & (kBlock - 1);
    const int t_lane = slice * Q + l16;       // this lane's term of block 0, counted from the row's first term
    constexpr int D = 2;
    XT rw[D][KPRE];
    int ri[D][KPRE];
    auto request_row = [&](int j, XT (&w)[KPRE], int (&i)[KPRE]) {
        const unsigned base = (unsigned)(sg0 + j) * (unsigned)K + (unsigned)t_lane;
#pragma unroll
        for (int p = 0; p < KPRE; ++p) {
            const unsigned t = min(base + (unsigned)(kBlock * p), (unsigned)t_last);   // (n_active + 256) * K * 4 < 2^31 (host)
            w[p] = *reinterpret_cast<const XT*>(reinterpret_cast<const char*>(W_c) + t * (unsigned)sizeof(XT));
            i[p] = (int)*reinterpret_cast<const IT*>(reinterpret_cast<const char*>(idx) + t * (unsigned)sizeof(IT));
        }
    };
    // block `blk` of the lane's run: a real term becomes (weight, byte offset of its column in the tile), the others
    // (past the run, or past the row) weight 0 on the all-zero column
    auto finish = [&](XT w_raw, int i_raw, int blk, float& wv, int& ov) {
        const int pos = kBlock * blk + l16;
        const bool real = pos < Q && slice * Q + pos < K;
        wv = real ? rl_to_f32<XT>(w_raw) : 0.0f;
        ov = real ? i_raw * S4 : zero_off;
    };

    // What the stores at the end need besides the sums is requested behind the tile and parked in LDS before the first barrier,
    // so that the epilogue reads LDS only (its loads used to cost it two dependent trips to the L2, about a microsecond):
    // without an active list the bias of the workgroup's columns; with one, the run of consecutive columns [c0, c1) that the
    // workgroup writes (the columns behind the previous group's last stored one up to this group's last; the last group also
    // takes the ablated columns up to d_out), the bias of that run and, per column of it, which row of the result tile holds
    // it, if any.  TP entries per thread wait in registers behind the tile's requests; what is beyond goes through a loop.
    constexpr int TP = 4;
    const int nthreads = blockDim.x;
    float* const out = lds + out_off;
    const int OS = NG | 1;                    // odd stride: conflict-free transposed writes
    float* const bsp = out + BT * OS;         // bias of the workgroup's columns
    int* const tab = reinterpret_cast<int*>(bsp + (active ? span_cap : NG));
    int c0 = 0, c1 = 0, span = 0;
    bool tabled = false;
    if (active != nullptr) {
        c0 = sg0 > 0 ? min(max(active[sg0 - 1] + 1, 0), d_out) : 0;
        c1 = (g == n_groups - 1) ? d_out : min(max(active[sg0 + ng - 1] + 1, c0), d_out);
        span = c1 - c0;
        tabled = span <= span_cap;
    }
    const int n_bias = active ? (tabled ? span : 0) : ng;      // bias entries parked, counted from column (active ? c0 : sg0)
    const int bias0 = active ? c0 : sg0;
    float e_bias[TP];
    int e_col[TP];

    // A pass stages kStageUnits units per wavefront.  Every load of a pass is unconditional (a unit, row or entry past the
    // end re-reads the last one and is dropped afterwards) and the first pass, which is the only one with 16 wavefronts, is
    // straight-line code: with loads under branches, or in a loop whose registers a load of the last turn may still own, the
    // compiler waits for every load in flight before the next one is issued (measured on the staging of this kernel: the
    // six tile loads of a wavefront went out one round trip after the other).
    const float* const bias_src = bias ? bias : reinterpret_cast<const float*>(x);   // never used: entries are 0 without a bias
    auto stage_pass = [&](int ub, auto first) {
        Staged4<XT> st[kStageUnits];
        int l_off[kStageUnits];
#pragma unroll
        for (int i = 0; i < kStageUnits; ++i) {
            const int u = min(ub + wv_id + i * nw, n_units - 1);
            const int rt = u & (RT - 1), ct = u >> RT_LOG2;
            const int rl = rt * 16 + db;
            const int f = ct * 16 + dq * 4;
            // rows past B re-read row B - 1: their lanes compute values that are never stored
            const unsigned off = (unsigned)(min(rl, B - 1 - b0) * d_in + f) * (unsigned)sizeof(XT);   // BT * d_in * 4 < 2^32 (host)
            load4(reinterpret_cast<const XT*>(xtile + off), true, 4, st[i]);
            l_off[i] = f * S + rl;
        }
        if constexpr (decltype(first)::value) {
            // behind the tile's first requests: the first rows' terms (vector loads return in order, and the tile's stores
            // into LDS wait for the tile only), and, behind those, what the epilogue needs
#pragma unroll
            for (int d = 0; d < D; ++d) request_row(min(wv_id + d * nw, ng - 1), rw[d], ri[d]);
#pragma unroll
            for (int q = 0; q < TP; ++q) {
                const int e = tid + q * nthreads;
                // (raw values: whether an entry counts is decided where it is written to LDS, so that nothing here waits)
                e_bias[q] = bias_src[bias ? min(bias0 + min(e, max(n_bias - 1, 0)), d_out - 1) : 0];
                e_col[q] = active != nullptr ? active[sg0 + min(e, ng - 1)] : -1;
            }
            if (tabled)
                for (int c = tid; c < span; c += nthreads) tab[c] = -1;
        }
#pragma unroll
        for (int i = 0; i < kStageUnits; ++i) {
            if (ub + wv_id + i * nw < n_units) {
                float* d = lds + l_off[i];
                d[0] = st[i].get(0); d[S] = st[i].get(1); d[2 * S] = st[i].get(2); d[3 * S] = st[i].get(3);
            }
        }
    };
    stage_pass(0, std::true_type{});
    for (int ub = kStageUnits * nw; ub < n_units; ub += kStageUnits * nw) stage_pass(ub, std::false_type{});
    for (int t = tid; t < S; t += blockDim.x) lds[C * S + t] = 0.0f;   // the all-zero column that padding terms point at
#pragma unroll
    for (int q = 0; q < TP; ++q) {
        const int e = tid + q * nthreads;
        if (e < n_bias) bsp[e] = bias ? e_bias[q] : 0.0f;
    }
    for (int e = tid + TP * nthreads; e < n_bias; e += nthreads) bsp[e] = rl_bias_at(bias, bias0 + e);
    if (tabled) {
        lds_barrier();   // every thread's part of the table is cleared (LDS only: the tile's loads stay in flight)
#pragma unroll
        for (int q = 0; q < TP; ++q) {
            const int col = e_col[q];
            if (tid + q * nthreads < ng && col >= c0 && col < c1) tab[col - c0] = tid + q * nthreads;
        }
        for (int e = tid + TP * nthreads; e < ng; e += nthreads) {
            const int col = active[sg0 + e];
            if (col >= c0 && col < c1) tab[col - c0] = e;
        }
    }
    __syncthreads();

    // ---- the rows of this wavefront, one after the other ----
    const int lanepart = rowl * (R * 4);
    const char* const xb = reinterpret_cast<const char*>(lds) + lanepart;
    auto walk_row = [&](int j, XT (&w)[KPRE], int (&i)[KPRE]) {
        float acc[R];
#pragma unroll
        for (int r = 0; r < R; ++r) acc[r] = 0.0f;
        float pw[KPRE];
        int po[KPRE];
#pragma unroll
        for (int p = 0; p < KPRE; ++p) finish(w[p], i[p], p, pw[p], po[p]);
        // the buffer is free: the row D rows on goes out now, with the arithmetic of D rows to return in (unconditional, as in
        // the prologue: past the workgroup's last row the last one is read again and never walked; under a branch the wait
        // for the next row's terms would become a wait for everything in flight, these included)
        request_row(min(j + D * nw, ng - 1), w, i);
        walk_groups<R, KPRE, kRowloopReadAhead>(acc, pw, po, xb, lanepart, Q);
        if (Q > KPRE * kBlock) {   // long rows: the remaining blocks, each requested one block ahead
            const unsigned base = (unsigned)(sg0 + j) * (unsigned)K + (unsigned)t_lane;
            auto fetch = [&](int blk, XT& wr, int& ir) {
                const unsigned t = min(base + (unsigned)(kBlock * blk), (unsigned)t_last);
                wr = *reinterpret_cast<const XT*>(reinterpret_cast<const char*>(W_c) + t * (unsigned)sizeof(XT));
                ir = (int)*reinterpret_cast<const IT*>(reinterpret_cast<const char*>(idx) + t * (unsigned)sizeof(IT));
            };
            XT wr;
            int ir;
            fetch(KPRE, wr, ir);
            for (int blk = KPRE; blk * kBlock < Q; ++blk) {
                float wc[1];
                int oc[1];
                finish(wr, ir, blk, wc[0], oc[0]);
                if ((blk + 1) * kBlock < Q) fetch(blk + 1, wr, ir);
                walk_groups<R, 1, 1>(acc, wc, oc, xb, lanepart, Q - blk * kBlock);
            }
        }
        // The slices hold partial sums of the same batch rows.  Swapping the upper half of the first row's register with the
        // lower half of the second's and adding leaves the first row's sums over the halves in lanes 0-31 and the second row's
        // in lanes 32-63; with four slices the same between the odd and even 16-lane rows of two copies of that.
        const auto h = __builtin_amdgcn_permlane32_swap(__float_as_uint(acc[0]), __float_as_uint(acc[1]), false, false);
        float v = __uint_as_float(h[0]) + __uint_as_float(h[1]);
        if constexpr (H == 4) {
            const auto q = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
            v = __uint_as_float(q[0]) + __uint_as_float(q[1]);
        }
        if (H == 2 || (lane & 16) == 0) out[(rowl * R + (lane >> 5)) * OS + j] = v;
    };
    int j = wv_id;
    for (; j + (D - 1) * nw < ng; j += D * nw) {   // whole turns of the D buffers: straight-line
#pragma unroll
        for (int d = 0; d < D; ++d) walk_row(j + d * nw, rw[d], ri[d]);
    }
#pragma unroll
    for (int d = 0; d < D - 1; ++d)                 // the rows of a last, partial turn
        if (j + d * nw < ng) walk_row(j + d * nw, rw[d], ri[d]);
    __syncthreads();

    // ---- results: row-contiguous stores of the workgroup's run of columns ----
    const int n_rows = min(BT, B - b0);
    if (active == nullptr) {
        for (int row = wv_id; row < n_rows; row += nw) {
            float* yr = y + (size_t)(b0 + row) * d_out + sg0;
            for (int c = lane; c < ng; c += kWave) {
                const float v = out[row * OS + c] + bsp[c];
                __builtin_nontemporal_store(act == SRIGL_ACT_NONE ? v : apply_act(v, act), &yr[c]);
            }
        }
        return;
    }
    if (tabled) {
        // lanes write the run left to right
        for (int row = wv_id; row < n_rows; row += nw) {
            float* yr = y + (size_t)(b0 + row) * d_out + c0;
            for (int c = lane; c < span; c += kWave) {
                const int t = tab[c];
                const float bv = bsp[c];
                const float v = t >= 0 ? out[row * OS + t] + bv : bv;
                __builtin_nontemporal_store(act == SRIGL_ACT_NONE ? v : apply_act(v, act), &yr[c]);
            }
        }
        return;
    }
    // runs longer than the table (few stored neurons among many ablated ones): every lane writes its stored column and the
    // ablated columns in front of it; the last group's first lane also writes the columns behind the last stored one
    for (int row = wv_id; row < n_rows; row += nw) {
        float* yr = y + (size_t)(b0 + row) * d_out;
        for (int j = lane; j < ng; j += kWave) {
            const int col = active[sg0 + j];
            const int prev = sg0 + j > 0 ? max(active[sg0 + j - 1] + 1, 0) : 0;
            for (int cc = prev; cc < min(col, d_out); ++cc) {
                const float bv = rl_bias_at(bias, cc);
                __builtin_nontemporal_store(act == SRIGL_ACT_NONE ? bv : apply_act(bv, act), &yr[cc]);
            }
            if (col >= 0 && col < d_out) {
                const float v = out[row * OS + j] + rl_bias_at(bias, col);
                __builtin_nontemporal_store(act == SRIGL_ACT_NONE ? v : apply_act(v, act), &yr[col]);
            }
        }
        if (g == n_groups - 1 && lane == 0) {
            for (int cc = max(active[n_active - 1] + 1, 0); cc < d_out; ++cc) {
                const float bv = rl_bias_at(bias, cc);
                __builtin_nontemporal_store(act == SRIGL_ACT_NONE ? bv : apply_act(bv, act), &yr[cc]);
            }
        }
    }
}

// Estimated time (us) of a launch shape, used to rank the shapes of this kernel among themselves.  Per round of workgroups
// on the busiest XCD: the tile (bytes through the vector L1), the rows a wavefront walks (a step of H terms x BT rows on a
// full compute unit, plus a fixed part per row: the requests, the cross-lane fetch, the slices' sum) and the result tile.
static double rowloop_shape_us(const FwdArgs& a, const RowloopPlan& p) {
    const int BT = kWave * 2 / p.H;
    const double rows_per_wave = (double)((p.NG + p.NW - 1) / p.NW);
    const double steps = (double)((a.K + p.H - 1) / p.H);
    const double per_step = (p.H == 4 ? 0.030 : 0.027) * p.NW / 16.0;
    const double terms = (double)a.n_active * a.K;
    return 1.6 + p.rounds * (1.0 + 9.0e-6 * BT * a.d_in * 4.0 + rows_per_wave * (steps * per_step + 0.12) + 1.2e-4 * BT * p.NG) +
           (terms > 1.5e6 ? 0.29e-6 * terms : 0.0);
}

// Estimated time (us) of the shape the ranking above has taken, to compare this kernel with the others: the same terms,
// with an extra one for the bytes of y, fitted (least squares of the relative error, standard deviation 5.7 %) to the mean of the
// cold and cached timings of 238 launches: 17 layers 256 to 1024 wide, fan-ins 8 to 231, up to 70 % of the neurons ablated,
// at 14 batches from 16 to 4096.
static double rowloop_compare_us(const FwdArgs& a, const RowloopPlan& p) {
    const int BT = kWave * 2 / p.H;
    const double rows_per_wave = (double)((p.NG + p.NW - 1) / p.NW);
    const double steps = (double)((a.K + p.H - 1) / p.H);
    const double per_step = 0.0336 * p.NW / 16.0;
    const double terms = (double)a.n_active * a.K;
    return 1.86 + p.rounds * (2.41 + 7.3e-6 * BT * a.d_in * 4.0 + rows_per_wave * (steps * per_step + 0.059)) +
           1.75e-6 * a.B * a.d_out + (terms > 1.5e6 ? 0.29e-6 * terms : 0.0);
}

static RowloopPlan plan_rowloop(const FwdArgs& a, const srigl_fwd_tuning* t) {
    RowloopPlan p{};
    p.ok = false;
    if (a.B <= 0 || a.n_active <= 0 || a.K <= 0) return p;
    if (t && t->rows_per_lane != 0 && t->rows_per_lane != 2) return p;
    p.H = t && t->term_slices ? t->term_slices : 4;
    if (p.H != 2 && p.H != 4) return p;
    // whole 16-column units, rows aligned for 4-element vector loads; 32-bit term and tile offsets
    const size_t xal = (a.x_bf16 ? 2 : 4) * 4;
    if (a.d_in % 16 != 0 || reinterpret_cast<uintptr_t>(a.x) % xal != 0) return p;
    if (((long long)a.n_active + 256) * a.K + 4096 >= (1LL << 29)) return p;
    const int BT = kWave * 2 / p.H, S = rowlane_row_stride(BT, p.H, 2);
    if ((long long)(BT + 1) * a.d_in * 4 >= (1LL << 32)) return p;
    p.NW = t && t->waves ? t->waves : 16;
    if (p.NW < 1 || p.NW > 16) return p;
    const size_t tile = (size_t)(a.d_in + 1) * S * sizeof(float);
    if (tile + (size_t)BT * (p.NW + 1) * sizeof(float) > kLdsMax) return p;
    const size_t rem = kLdsMax - tile;
    // rows per workgroup the result tile (and, with an active list, a column table of twice as many columns) has room for
    const size_t per_row = (size_t)BT * sizeof(float) + (a.active ? 2 * (sizeof(int) + sizeof(float)) : sizeof(float));
    long long ng_max = (long long)(rem / per_row) - 2;
    if (ng_max < p.NW) return p;
    if (ng_max > 4096) ng_max = 4096;
    p.n_btiles = (a.B + BT - 1) / BT;
    const int xo = t ? t->xcd_order : 0;
    if (xo < 0 || xo > 2) return p;
    const double x_bytes = (double)a.B * a.d_in * (a.x_bf16 ? 2 : 4);
    const double term_bytes = (double)a.n_active * a.K * ((a.x_bf16 ? 2 : 4) + (a.idx_u16 ? 2 : 4));
    auto shape = [&](int NG) {
        RowloopPlan q = p;
        q.NG = NG;
        q.n_groups = (a.n_active + NG - 1) / NG;
        const long long by_groups = (long long)((q.n_groups + 7) / 8) * q.n_btiles, by_tiles = (long long)((q.n_btiles + 7) / 8) * q.n_groups;
        // batch tiles to XCDs when that takes no more rounds, every XCD gets a tile and x is the larger operand: an XCD's L2
        // then fetches its own rows of x and all of W_c / idx; else groups of stored rows (all of x, its groups' W_c / idx)
        q.bt_major = xo ? (xo == 2) : (q.n_btiles >= 8 && by_tiles <= by_groups && x_bytes >= term_bytes);
        q.rounds = (int)(((q.bt_major ? by_tiles : by_groups) + 31) / 32);
        return q;
    };
    if (t && t->neurons_per_wave) {
        if (t->neurons_per_wave < 0 || (long long)t->neurons_per_wave * p.NW > ng_max) return p;
        p = shape(t->neurons_per_wave * p.NW);
    } else {
        // as many groups as fill the compute units, fewer rows per workgroup where that costs no round
        RowloopPlan best{};
        double best_us = 0.0;
        for (int rpw = 1; (long long)rpw * p.NW <= ng_max; ++rpw) {
            const RowloopPlan q = shape(rpw * p.NW);
            const double us = rowloop_shape_us(a, q);
            if (!best.ok || us < best_us) { best = q; best.ok = true; best_us = us; }
            if (q.n_groups == 1) break;
        }
        if (!best.ok) return p;
        p = best;
    }
    {   // blocks of 16 steps a row's terms are preloaded in (up to four; longer rows walk the rest one block at a time)
        const int blocks = ((a.K + p.H - 1) / p.H + kBlock - 1) / kBlock;
        p.KPRE = blocks < 4 ? blocks : 4;
    }
    const int OS = p.NG | 1;
    p.out_off = (a.d_in + 1) * S;
    // behind the result tile: the bias of the workgroup's columns; with an active list the bias and the column table of a run
    // of up to span_cap columns
    const size_t used = tile + (size_t)BT * OS * sizeof(float) + (a.active ? 0 : (size_t)p.NG * sizeof(float));
    if (used > kLdsMax) return p;
    p.span_cap = a.active ? (int)std::min<size_t>((kLdsMax - used) / (sizeof(int) + sizeof(float)), 1u << 20) : 0;
    p.lds = used + (size_t)p.span_cap * (sizeof(int) + sizeof(float));
    if (8LL * ((p.n_groups + 7) / 8) * ((p.n_btiles + 7) / 8 * 8) > 0x7fffffffLL) return p;
    p.ok = true;
    return p;
}

template <int H, int KPRE, typename XT, typename IT>
static srigl_status launch_rowloop_f(const FwdArgs& a, const RowloopPlan& p, hipStream_t st) {
    auto kern = k_fwd_rowloop<2, H, KPRE, XT, IT>;
    static LdsLimit lds_limit;
    if (lds_limit.ensure(kern, p.lds) != SRIGL_OK) return SRIGL_ERR_HIP;
    const long long blocks = p.bt_major ? 8LL * ((p.n_btiles + 7) / 8) * p.n_groups : 8LL * ((p.n_groups + 7) / 8) * p.n_btiles;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(p.NW * kWave), p.lds, st, (const XT*)a.x, a.B, a.d_in, (const XT*)a.W_c,
                       (const IT*)a.idx, a.active, a.n_active, a.K, a.bias, a.d_out, a.y, p.NG, p.n_btiles, p.n_groups, p.out_off,
                       p.span_cap, a.act, p.bt_major);
    return hip_ok(hipGetLastError());
}

template <typename XT, typename IT>
static srigl_status launch_rowloop_x(const FwdArgs& a, const RowloopPlan& p, hipStream_t st) {
    switch (p.H * 10 + p.KPRE) {
        case 41: return launch_rowloop_f<4, 1, XT, IT>(a, p, st);
        case 42: return launch_rowloop_f<4, 2, XT, IT>(a, p, st);
        case 43: return launch_rowloop_f<4, 3, XT, IT>(a, p, st);
        case 44: return launch_rowloop_f<4, 4, XT, IT>(a, p, st);
        case 21: return launch_rowloop_f<2, 1, XT, IT>(a, p, st);
        case 22: return launch_rowloop_f<2, 2, XT, IT>(a, p, st);
        case 23: return launch_rowloop_f<2, 3, XT, IT>(a, p, st);
        case 24: return launch_rowloop_f<2, 4, XT, IT>(a, p, st);
        default: return SRIGL_ERR_UNSUPPORTED;
    }
}

bool rowloop_supported(const FwdArgs& a, const srigl_fwd_tuning* t) { return plan_rowloop(a, t).ok; }

double rowloop_estimate_us(const FwdArgs& a) {
    const RowloopPlan p = plan_rowloop(a, nullptr);
    return p.ok ? rowloop_compare_us(a, p) : 1e30;
}

bool rowloop_plan_query(const FwdArgs& a, const srigl_fwd_tuning* t, srigl_fwd_plan* plan) {
    const RowloopPlan p = plan_rowloop(a, t);
    if (!p.ok) return false;
    plan->rows_per_lane = 2; plan->term_slices = p.H; plan->waves = p.NW; plan->neurons_per_wave = (p.NG + p.NW - 1) / p.NW;
    plan->chunk_cols = a.d_in; plan->workgroups = (int64_t)p.n_groups * p.n_btiles; plan->xcd_order = p.bt_major ? 2 : 1; plan->spread_rows = 1;
    return true;
}

srigl_status launch_fwd_rowloop(const FwdArgs& a, const srigl_fwd_tuning* t, hipStream_t st) {
    if (a.B == 0 || a.n_active == 0) return SRIGL_OK;
    const RowloopPlan p = plan_rowloop(a, t);
    if (!p.ok) return SRIGL_ERR_UNSUPPORTED;
    if (a.idx_u16) return a.x_bf16 ? launch_rowloop_x<uint16_t, uint16_t>(a, p, st) : launch_rowloop_x<float, uint16_t>(a, p, st);
    return a.x_bf16 ? launch_rowloop_x<uint16_t, int32_t>(a, p, st) : launch_rowloop_x<float, int32_t>(a, p, st);
}

}  // namespace srigl
