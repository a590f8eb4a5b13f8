/* srigl.h -- C ABI of the condensed constant fan-in sparse linear layer for AMD MI355X (gfx950).
 *
 * The layer is the inference form of a network trained with SRigL (arXiv 2305.02299): every
 * neuron that is not ablated keeps exactly K incoming weights (constant fan-in, Fig. 1a, Sec. 3.1),
 * so the sparse weight matrix is stored as two dense [n_active][K] arrays, the kept values W_c and
 * their column indices idx (App. E), and the forward pass is the triple loop of Alg. 1:
 *
 *     y[b][active[s]] = bias[active[s]] + sum_{k<K} W_c[s][k] * x[b][ idx[s][k] ]
 *     y[b][r]         = bias[r]                      for every neuron r that is not stored (ablated)
 *
 * General conventions
 *   - Every data pointer is a DEVICE pointer on the current HIP device unless marked "host".
 *   - The caller owns every buffer.  The library never allocates, frees or keeps a pointer.
 *   - All matrices are row-major and dense: x[B][d_in], y[B][d_out], W[d_out][d_in],
 *     mask[d_out][d_in], W_c[rows][K], idx[rows][K].
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the default stream) and
 *     the call returns without synchronising.
 *   - The return value reports what the host can see (NULL pointers, negative sizes, K > d_in,
 *     workspace too small, launch failure).  What only the data can show (a row with a wrong
 *     fan-in, an index out of range, too few output rows) is written to the device-side
 *     srigl_report, which the caller reads after its own synchronisation.
 *   - Empty problems (B == 0, d_out == 0, n_rows == 0) are valid and do nothing; K == 0 or
 *     n_active == 0 makes the forward pass a bias broadcast.
 *   - Calls that share a workspace or an output buffer must be ordered by the caller (same stream
 *     or explicit dependencies).
 */
#ifndef SRIGL_H_
#define SRIGL_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SRIGL_OK = 0,
    SRIGL_ERR_INVALID_ARG = 1, /* NULL where data is required, negative size, K > d_in, bad enum   */
    SRIGL_ERR_FANIN = 2,       /* device-side: some row holds neither 0 nor K kept weights          */
    SRIGL_ERR_CAPACITY = 3,    /* workspace too small (host) / more stored rows than cap_rows (dev) */
    SRIGL_ERR_INDEX_RANGE = 4, /* device-side: an index outside [0, d_in) or a row not ascending    */
    SRIGL_ERR_UNSUPPORTED = 5, /* dtype combination or algorithm not available for these sizes      */
    SRIGL_ERR_HIP = 6          /* a HIP call failed                                                 */
} srigl_status;

typedef enum { SRIGL_F32 = 0, SRIGL_BF16 = 1 } srigl_dtype;

/* Forward algorithms.  AUTO picks by batch size and shape. */
typedef enum {
    SRIGL_FWD_AUTO = 0,
    SRIGL_FWD_GENERIC = 1,  /* one thread per output, activations read from global memory; any index order */
    SRIGL_FWD_KLANE = 2,    /* small batch: lanes split one neuron's K terms, cross-lane reduction          */
    SRIGL_FWD_ROWLANE = 3,  /* batched: lanes are batch rows, activation tile transposed in LDS             */
    SRIGL_FWD_ROWLOOP = 4   /* batched, inputs narrow enough that a 32-row tile holds every column of x: a wavefront
                               walks any number of stored rows, so a workgroup owns hundreds of them per staged tile */
} srigl_fwd_algo;

/* 32 bytes, lives in device memory, written by check_fanin / condense. */
typedef struct {
    int32_t K;             /* fan-in that was checked against (given, or inferred)        */
    int32_t n_active;      /* rows holding exactly K kept weights (mask mode) / valid rows */
    int32_t n_bad_rows;    /* rows that violate the invariant                              */
    int32_t first_bad_row; /* smallest such row, -1 if none                                */
    int32_t status;        /* SRIGL_OK, SRIGL_ERR_FANIN, SRIGL_ERR_INDEX_RANGE, SRIGL_ERR_CAPACITY */
    int32_t reserved[3];
} srigl_report;

/* Bytes of device scratch that check_fanin / condense need for n_rows rows. */
size_t srigl_workspace_bytes(int32_t n_rows);

/* Number of uint16 entries per stored row in the optional `seg` table: d_in/64 rounded up, plus 1. */
int32_t srigl_seg_stride(int32_t d_in);

/* srigl_check_fanin -- the constant fan-in invariant (Fig. 1a; Sec. 3.1: every neuron that is not
 * ablated has the same number of unmasked incoming weights).
 *
 * Mask mode (idx == NULL): mask[n_rows][d_in], uint8, non-zero = kept.  A row is valid when it
 *   holds 0 (ablated) or K kept weights.  K_expected < 0: K is taken from the first non-empty row.
 * Index mode (mask == NULL): idx[n_rows][K_expected] must lie in [0, d_in) and be strictly
 *   ascending within each row (distinct columns, App. E).  If seg != NULL it receives, per row,
 *   srigl_seg_stride(d_in) uint16 entries: seg[r][c] = number of indices of row r below 64*c
 *   (the forward pass uses it to walk a row chunk by chunk); rows that fail the check get
 *   all-zero entries so that a later forward pass reads nothing for them.
 * Exactly one of mask / idx must be non-NULL.  workspace: srigl_workspace_bytes(n_rows) bytes.
 * report_dev receives {K, n_active, n_bad_rows, first_bad_row, status}.
 */
srigl_status srigl_check_fanin(const uint8_t* mask, const int32_t* idx, int32_t n_rows, int32_t d_in,
                               int32_t K_expected, uint16_t* seg, void* workspace, size_t workspace_bytes,
                               srigl_report* report_dev, void* stream);

/* srigl_condense -- dense weights plus constant fan-in mask to the condensed form (App. E, last
 * paragraph: one [n][k] array of values, one of column indices; Sec. 4.4: ablated neurons and
 * masked weights are removed).
 *
 * W[d_out][d_in] of w_dtype, mask[d_out][d_in] uint8.  For the s-th row r (ascending) that holds
 * exactly K kept weights: active[s] = r, idx[s][0..K) = its kept columns ascending,
 * W_c[s][t] = W[r][idx[s][t]] copied bit for bit (the mask decides, not the value).
 * Rows s >= n_active of the outputs are left untouched.  cap_rows = rows available in W_c / idx /
 * active / seg; if n_active > cap_rows only the first cap_rows stored rows are written and
 * report.status = SRIGL_ERR_CAPACITY.  Rows whose count is neither 0 nor K are skipped and
 * reported (status = SRIGL_ERR_FANIN); the other outputs are then not meaningful.
 * seg (optional, may be NULL): [cap_rows][srigl_seg_stride(d_in)] uint16 as in check_fanin.
 * K > 65535 with seg != NULL is SRIGL_ERR_UNSUPPORTED.
 * packed (optional, may be NULL): receives the streaming copy of the first min(n_active, cap_rows) stored rows (see
 * srigl_packed_bytes); 16-byte aligned, packed_bytes >= srigl_packed_bytes(cap_rows, K, d_in, w_dtype), else
 * SRIGL_ERR_INVALID_ARG / SRIGL_ERR_CAPACITY.  W_c and idx stay the result that defines the layer; the copy is derived.
 */
srigl_status srigl_condense(const void* W, srigl_dtype w_dtype, const uint8_t* mask, int32_t d_out,
                            int32_t d_in, int32_t K, int32_t cap_rows, void* W_c, int32_t* idx,
                            int32_t* active, uint16_t* seg, void* packed, size_t packed_bytes, void* workspace,
                            size_t workspace_bytes, srigl_report* report_dev, void* stream);

/* The streaming copy of a condensed layer.  App. E's representation is the two n x k arrays; how they lie in memory
 * for the forward pass is free, and W_c / idx as separate row-major arrays of K = 77, 205, 307 ... words per row leave
 * every row at another alignment, so a lane can fetch only one 4-byte (2-byte) word per load.  The copy holds the same
 * terms neuron-major in units of four consecutive terms of a row, the four weights of a unit next to its four column
 * indices (rows padded to whole units with weight 0 / index 0; 16-bit indices beside bf16 weights when d_in <= 65536),
 * so that one or two 16-byte loads bring a lane its four terms and a lane group reads consecutive units.  The layout
 * belongs to the library: callers size the buffer with srigl_packed_bytes, have srigl_condense or srigl_pack_terms fill
 * it, and hand it to the forward call together with W_c / idx.  It must describe the same rows as W_c / idx.
 *
 * srigl_packed_bytes: bytes for n_rows stored rows (0 when any size is not positive).
 * srigl_pack_terms: the copy from W_c[n_rows][K] / idx[n_rows][K] (for layers that did not come out of srigl_condense,
 * e.g. the folded second layer of an MLP block).  Index values are copied as they are (the 16-bit form keeps their low
 * 16 bits: validate with srigl_check_fanin first).  Device pointers, `packed` 16-byte aligned, asynchronous on `stream`. */
size_t srigl_packed_bytes(int32_t n_rows, int32_t K, int32_t d_in, srigl_dtype w_dtype);

srigl_status srigl_pack_terms(const void* W_c, srigl_dtype w_dtype, const int32_t* idx, int32_t n_rows, int32_t K, int32_t d_in,
                              void* packed, size_t packed_bytes, void* stream);

/* srigl_condense for callers that cannot allocate device memory or pass scratch of their own: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and errors as srigl_condense
 * without `workspace`: the per-row counts and slots live in an array inside the library (8 bytes per row of W,
 * SRIGL_STATIC_MAX_ROWS rows: 512 KiB per GPU, held until the process ends).  d_out > SRIGL_STATIC_MAX_ROWS returns
 * SRIGL_ERR_CAPACITY and launches nothing.  The call allocates and frees nothing (the first call on a device looks the
 * array's address up, which is not an allocation).  Every call on a GPU uses that GPU's one array: calls that may
 * overlap on one GPU (different streams without an order between them) race and must be ordered by the caller; calls
 * in order need no clearing in between (each call writes what it reads). */
#define SRIGL_STATIC_MAX_ROWS 65536
srigl_status srigl_condense_static(const void* W, srigl_dtype w_dtype, const uint8_t* mask, int32_t d_out, int32_t d_in, int32_t K,
                                   int32_t cap_rows, void* W_c, int32_t* idx, int32_t* active, uint16_t* seg, void* packed,
                                   size_t packed_bytes, srigl_report* report_dev, void* stream);

/* srigl_condensed_linear_fwd -- Alg. 1 (condensed linear layer forward) plus bias and the scatter of
 * stored neurons to their columns.
 *
 * x[B][d_in] of x_dtype; W_c[n_active][K] of w_dtype (both F32 or both BF16); idx[n_active][K]
 * int32 in [0, d_in) (not checked here: validate once with srigl_check_fanin in index mode);
 * active[n_active] strictly ascending columns in [0, d_out), or NULL when n_active == d_out
 * (the s-th stored neuron is column s) or n_active == 0; bias[d_out] fp32 or NULL (= zero, Alg. 1 verbatim);
 * y[B][d_out] fp32, fully overwritten.  Accumulation is fp32 (bf16 products are exact in fp32).
 * seg: the table written by condense / check_fanin for these idx, or NULL.  Whenever seg is passed every row of idx
 * must be strictly ascending (the library cannot see an unsorted row: validate once with srigl_check_fanin in index
 * mode, which also writes seg; with unsorted rows and a seg table the batched kernel returns wrong sums without an
 * error).  With seg == NULL only algorithms that do not depend on the order are used, and any in-range order, repeats
 * included, is summed as Alg. 1 does.  seg != NULL with K > 65535 is SRIGL_ERR_UNSUPPORTED (its entries are 16 bits).
 * packed: the streaming copy of these W_c / idx rows (srigl_condense, srigl_pack_terms), 16-byte aligned, or NULL.  The
 * kernels that can stream it read it in place of W_c / idx (which must still be passed: other kernels read them); the
 * same terms are summed, possibly in another order (same tolerance).
 * Out-of-range entries of `active` are skipped, never written.
 */
srigl_status srigl_condensed_linear_fwd(const void* x, srigl_dtype x_dtype, int32_t B, int32_t d_in,
                                        const void* W_c, srigl_dtype w_dtype, const int32_t* idx,
                                        const int32_t* active, int32_t n_active, int32_t K,
                                        const float* bias, int32_t d_out, float* y,
                                        const uint16_t* seg, const void* packed, void* stream);

/* Launch-shape knobs of the forward kernels (host struct).  0 in a field = the library's default.
 * Values the kernels cannot run are rejected with SRIGL_ERR_UNSUPPORTED, never launched.
 * SRIGL_FWD_ROWLOOP reads rows_per_lane (2 only), term_slices (4: 32-row tile, inputs up to about 1100 columns wide;
 * 2: 64-row tile, up to about 600), waves (1..16), neurons_per_wave (stored rows a wavefront walks, any number the result
 * tile in LDS has room for) and xcd_order; d_in must be a multiple of 16; the index order within a row is free. */
typedef struct {
    int32_t rows_per_lane;    /* ROWLANE: batch rows per lane, 1, 2 or 4 (4: with 2 or 4 term slices only)  */
    int32_t waves;            /* ROWLANE: wavefronts per workgroup, 1..16                                  */
    int32_t neurons_per_wave; /* ROWLANE: stored neurons accumulated per wavefront, 1..8                   */
    int32_t chunk_cols;       /* ROWLANE: activation columns per LDS tile, multiple of 64                  */
    int32_t lanes_per_neuron; /* KLANE: lanes that share one neuron, power of two 1..64                    */
    int32_t rows_per_block;   /* KLANE: batch rows per workgroup, 1, 2, 4 or 8                             */
    int32_t term_slices;      /* ROWLANE: 1, 2 or 4 groups of lanes that work on different terms of a stored
                                 row at once (batch tile = 64 * rows_per_lane / term_slices rows)           */
    int32_t direct_gather;    /* KLANE: 1 = gather activations from global memory, 2 = stage rows of x in LDS     */
    int32_t xcd_order;        /* ROWLANE: which workgroups share an XCD (one L2): 1 = all batch tiles of a group of
                                 stored rows (W_c / idx fetched once, x by every XCD), 2 = all groups of a batch tile */
    int32_t terms_from_copy;  /* 1 = read the terms from the streaming copy wherever the call brings one.  The default, 0:
                                 ROWLANE reads W_c / idx (one load per block of terms instead of two measured no faster);
                                 KLANE reads the copy when a workgroup holds one batch row and W_c / idx when it holds
                                 more (measured faster that way round)                                              */
    int32_t spread_rows;      /* ROWLANE: how a workgroup's stored rows are shared out among its wavefronts: 1 = consecutive
                                 rows to a wavefront, 2 = dealt out in the order of their median input column, so that rows
                                 whose indices cluster in the same columns do not meet in one wavefront (every column chunk
                                 ends in a barrier and costs what its busiest wavefront costs), 3 = dealt out in the
                                 workgroups whose rows' medians lie far apart, consecutive in the others; 0 = the library's
                                 choice (3 from four chunks per row on, else 1)                                          */
} srigl_fwd_tuning;

/* Same, with the algorithm and launch shape forced (for tests and measurements).  tuning may be
 * NULL.  SRIGL_ERR_UNSUPPORTED if the algorithm cannot run these sizes (e.g. ROWLANE without seg
 * when d_in does not fit one LDS tile). */
srigl_status srigl_condensed_linear_fwd_algo(const void* x, srigl_dtype x_dtype, int32_t B, int32_t d_in,
                                             const void* W_c, srigl_dtype w_dtype, const int32_t* idx,
                                             const int32_t* active, int32_t n_active, int32_t K,
                                             const float* bias, int32_t d_out, float* y,
                                             const uint16_t* seg, const void* packed, srigl_fwd_algo algo,
                                             const srigl_fwd_tuning* tuning, void* stream);

/* What the library's own choice (SRIGL_FWD_AUTO) would launch for a forward call of these sizes: the kernel and its
 * launch shape.  Host arithmetic only (no GPU call, no device pointers: has_active / has_seg say whether the call would
 * pass an active list / a seg table; arrays are taken to be 16-byte aligned).  All fields are 0 when no forward kernel
 * would run (B, d_out, n_active or K zero).  For tests of the planner and for users who want to know. */
typedef struct {
    int32_t algo;             /* srigl_fwd_algo: SRIGL_FWD_GENERIC, _KLANE, _ROWLANE or _ROWLOOP             */
    int32_t rows_per_lane, term_slices, waves, neurons_per_wave, chunk_cols;   /* ROWLANE, ROWLOOP (chunk_cols = d_in), else 0 */
    int32_t lanes_per_neuron, rows_per_block;                                 /* KLANE, else 0            */
    int64_t workgroups;       /* workgroups that do work                                                    */
    int32_t direct_gather;    /* KLANE: 1 = activations gathered from global memory, 0 = rows of x staged in LDS */
    int32_t xcd_order;        /* ROWLANE: 1 or 2 as in srigl_fwd_tuning                                     */
    int32_t spread_rows;      /* ROWLANE: 1, 2 or 3 as in srigl_fwd_tuning                                  */
} srigl_fwd_plan;
srigl_status srigl_fwd_plan_query(int32_t B, int32_t d_in, int32_t n_active, int32_t K, int32_t d_out, srigl_dtype dtype,
                                  int32_t has_active, int32_t has_seg, srigl_fwd_plan* plan);
/* Same for a forced algorithm and launch shape (algo and tuning as in srigl_condensed_linear_fwd_algo; tuning may be NULL;
 * SRIGL_FWD_AUTO is the call above): SRIGL_ERR_UNSUPPORTED where that forward call would return it. */
srigl_status srigl_fwd_plan_query_algo(int32_t B, int32_t d_in, int32_t n_active, int32_t K, int32_t d_out, srigl_dtype dtype,
                                       int32_t has_active, int32_t has_seg, srigl_fwd_algo algo, const srigl_fwd_tuning* tuning,
                                       srigl_fwd_plan* plan);

/* ---- MLP block: activation in the epilogue, width reduction -------------------------------------------
 * Sec. 3.1 (neuron ablation reduces the width of a layer) and App. H (the timed layer is one linear of a ViT MLP
 * block: linear, GELU, linear).  srigl_condensed_linear_fwd_act is the forward call with an activation applied to
 * every written value, stored and ablated columns alike (an ablated neuron outputs act(bias)); SRIGL_ACT_GELU is
 * v * Phi(v) with the normal distribution function (erf form). */
typedef enum srigl_activation { SRIGL_ACT_NONE = 0, SRIGL_ACT_RELU = 1, SRIGL_ACT_GELU = 2 } srigl_activation;

srigl_status srigl_condensed_linear_fwd_act(const void* x, srigl_dtype x_dtype, int32_t B, int32_t d_in,
                                            const void* W_c, srigl_dtype w_dtype, const int32_t* idx,
                                            const int32_t* active, int32_t n_active, int32_t K,
                                            const float* bias, int32_t d_out, float* y,
                                            const uint16_t* seg, const void* packed, srigl_activation act, srigl_fwd_algo algo,
                                            const srigl_fwd_tuning* tuning, void* stream);

/* Width reduction.  Layer 1 has d_hidden neurons of which active1[0..n_active1) are stored (NULL: all of them); an
 * ablated neuron outputs the constant act(bias1).  Layer 2 (n2 stored rows of fan-in K2 over layer 1's d_hidden outputs;
 * stored row n is neuron active2[n] of d_out2, NULL: n) is rewritten to read the compact vector of the n_active1 stored
 * outputs: idx_out / W_out [n2][K2] (same element type as W_c2, bit copies; fillers are zero bits; rows ascending and
 * without repeats, entries in [0, n_active1)), bias_out[d_out2] = bias2 plus, for each stored row, the terms that named
 * ablated neurons.  All pointers are device memory; outputs must not alias inputs.  SRIGL_ERR_UNSUPPORTED if
 * K2 > n_active1 (no room for K2 distinct positions) or K2 > 9216.  idx2 entries outside [0, d_hidden) are dropped. */
srigl_status srigl_fold_ablated_inputs(const int32_t* idx2, const void* W_c2, srigl_dtype w_dtype, const float* bias2,
                                       const int32_t* active2, int32_t n2, int32_t K2, int32_t d_out2, const int32_t* active1,
                                       int32_t n_active1, int32_t d_hidden, const float* bias1, srigl_activation act,
                                       int32_t* idx_out, void* W_out, float* bias_out, void* stream);

/* The first layer of such a pair as it is run: it writes its n_active1 stored neurons next to each other into a hidden
 * vector of `width` >= n_active1 columns (the caller may pad the width, e.g. to a multiple of 16; padding columns are
 * neurons nobody reads).  bias_compact[width]: bias1[active1[p]] at position p < n_active1, zero behind; active_compact
 * [n_active1]: p at position p (the active list of the compact layer when width > n_active1).  Either output may be NULL;
 * bias1 == NULL is a zero bias, active1 == NULL means n_active1 == d_hidden.  Device pointers, asynchronous on `stream`.
 *
 * What a caller of the folded pair must know: the zero-weight fillers of a folded row sit at positions of real hidden
 * neurons.  Alg. 1 multiplies them like any other term, so a hidden value that is not finite turns 0 * inf into NaN in
 * rows that never named that neuron in the unfolded layer (srigl_densify + the dense product behave the same way: stored
 * zeros times x).  The unfolded condensed call has no such term. */
srigl_status srigl_compact_hidden_layer(const float* bias1, const int32_t* active1, int32_t n_active1, int32_t d_hidden, int32_t width,
                                        float* bias_compact, int32_t* active_compact, void* stream);

/* Both layers of an MLP block in one launch, for online inference and batches of up to 8 rows (App. H: the timed layer is
 * one linear of a ViT block: linear, GELU, linear; Sec. 3.1: layer 1's ablation is layer 2's width reduction):
 *   hidden[b][c] = act(bias1[c] + sum_k W1[s][k] x[b][idx1[s][k]]) for stored neuron s of layer 1 at column c = active1[s]
 *                  (other columns: act(bias1[c])),   y = bias2 + layer 2 applied to hidden (ablated columns: bias2).
 * Both layers fp32, each given by its streaming copy (packed1: n_active1 rows of fan-in K1 over d_in columns; packed2:
 * n_active2 rows of fan-in K2 over d_hidden columns), its active list (NULL: every neuron stored) and bias (NULL: zero).
 * x[B][d_in], hidden[B][d_hidden] (scratch of the caller, fully overwritten), y[B][d_out].  One launch of 256 workgroups with
 * a barrier across them between the layers (a counter inside the library, one per GPU: calls that may overlap on one GPU
 * must be ordered by the caller, and the 256 workgroups must be able to be resident together, which they are on an idle
 * MI355X).  A workgroup that polls the counter more than spin_limit times (<= 0: about a million) stops waiting, the call's
 * result is then wrong and *status_dev (device int32, may be NULL; set it to 0 before the call) becomes 1: every wavefront
 * exits either way.  SRIGL_ERR_UNSUPPORTED for B > 8 or a layer without terms (use two forward calls). */
srigl_status srigl_condensed_mlp_fwd(const float* x, int32_t B, int32_t d_in, const void* packed1, const int32_t* active1, int32_t n_active1,
                                     int32_t K1, const float* bias1, int32_t d_hidden, srigl_activation act, float* hidden,
                                     const void* packed2, const int32_t* active2, int32_t n_active2, int32_t K2, const float* bias2,
                                     int32_t d_out, float* y, int32_t spin_limit, int32_t* status_dev, void* stream);

/* ---- narrow column indices ------------------------------------------------------------------------------
 * App. E: the condensed layer stores one column index per kept weight; that index array is all the representation
 * adds to the weights themselves.  A layer with d_in <= 65536 can hold it in 16 bits (half the index bytes; with
 * bf16 weights the whole representation is then 4 bytes per weight instead of 6).
 *
 * srigl_narrow_idx: idx16[i] = idx[i] for i in [0, n); device pointers, distinct arrays.  Entries must lie in
 * [0, d_in) as srigl_condense writes them (others are clamped into that range).  SRIGL_ERR_UNSUPPORTED if
 * d_in > 65536, SRIGL_ERR_INVALID_ARG on negative sizes or NULL pointers with n > 0.
 *
 * srigl_condensed_linear_fwd_idx16: srigl_condensed_linear_fwd_act with idx16[n_active][K] in place of idx; every
 * other argument, the result and the errors are the same (same kernels, same order of additions: the output is
 * bit-identical to the 32-bit call on the same arrays without a streaming copy).  d_in > 65536 is SRIGL_ERR_UNSUPPORTED. */
srigl_status srigl_narrow_idx(const int32_t* idx, int64_t n, int32_t d_in, uint16_t* idx16, void* stream);

srigl_status srigl_condensed_linear_fwd_idx16(const void* x, srigl_dtype x_dtype, int32_t B, int32_t d_in,
                                              const void* W_c, srigl_dtype w_dtype, const uint16_t* idx16,
                                              const int32_t* active, int32_t n_active, int32_t K,
                                              const float* bias, int32_t d_out, float* y,
                                              const uint16_t* seg, srigl_activation act, srigl_fwd_algo algo,
                                              const srigl_fwd_tuning* tuning, void* stream);

/* ---- unstructured comparison: the same weights in compressed sparse row form ------------------------------
 * Sec. 4.4 / Fig. 4 and App. H time the condensed layer against the layer's kept weights held as an unstructured sparse
 * matrix.  srigl_csr_linear_fwd is that comparison on this GPU, built like the small-batch condensed kernel:
 * y[b][r] = act(bias[r] + sum over t in [row_ptr[r], row_ptr[r+1]) of values[t] * x[b][col_idx[t]]), r in [0, d_out).
 * x[B][d_in] and values[nnz] fp32 (x_dtype == w_dtype == SRIGL_F32; BF16 is SRIGL_ERR_UNSUPPORTED), col_idx[nnz] int32 in [0, d_in) (not checked),
 * row_ptr[d_out + 1] int32 ascending with row_ptr[0] == 0 and row_ptr[d_out] == nnz (not checked; nnz is passed so that
 * the launch shape can follow the mean row length), bias[d_out] fp32 or NULL, y[B][d_out] fp32, fully overwritten
 * (a row without entries outputs act(bias)).  Device pointers, caller's stream, no allocation.
 * SRIGL_ERR_UNSUPPORTED if B > 65535. */
srigl_status srigl_csr_linear_fwd(const void* x, srigl_dtype x_dtype, int32_t B, int32_t d_in, const void* values,
                                  srigl_dtype w_dtype, const int32_t* col_idx, const int32_t* row_ptr, int64_t nnz,
                                  const float* bias, int32_t d_out, float* y, srigl_activation act, void* stream);

/* ---- one SRigL connectivity update of a layer ------------------------------------------------------------
 * Sec. 3.1, steps 1-7 (with the minimum of one salient weight stated in the appendix on tuning gamma_sal).  W, grad: fp32 [d_out][d_in]; mask: bytes, every
 * row holds 0 (ablated) or k kept weights; K_upd: the number of weights pruned and grown in this update (step 2, chosen
 * by the caller's schedule); gamma_percent: the ablation threshold gamma_sal in percent; budget: the number of weights the
 * layer may hold (normally k times its neurons that hold weights).  Outputs: mask_out (every row 0 or k' ones), W_out (kept
 * weights copied, everything else zero: grown weights start at zero), report_dev[4] = {k', neurons that remain, neurons
 * ablated by this update, weights pruned in step 6}.  All buffers are device memory, caller-owned; outputs must not alias
 * inputs; workspace of srigl_mask_update_workspace_bytes(d_out, d_in) bytes (counters, three integers per neuron and two
 * candidate lists of d_out * d_in / 16 eight-byte keys each, at least 4096), 256-byte aligned.  Asynchronous on `stream`.
 * Readings: a kept weight is salient if it is not among the K_upd smallest-magnitude kept weights of the layer, a pruned
 * position if its gradient is among the K_upd largest at pruned positions; a neuron is ablated if it holds weights and
 * its salient count is below max(gamma k, 1); a neuron without weights stays ablated; k' = min(d_in, budget / remaining
 * neurons); step 6 prunes among the remaining neurons' weights; step 7 keeps a neuron's unpruned weights (its k' largest
 * if it holds more) and grows free positions by decreasing gradient magnitude; equal magnitudes rank by position (lower
 * first).  d_out * d_in must be below 2^32 and d_in at most 8192, else SRIGL_ERR_UNSUPPORTED. */
size_t srigl_mask_update_workspace_bytes(int32_t d_out, int32_t d_in);

srigl_status srigl_mask_update(const float* W, const uint8_t* mask, const float* grad, int32_t d_out, int32_t d_in, int32_t k,
                               int64_t K_upd, int32_t gamma_percent, int64_t budget, uint8_t* mask_out, float* W_out,
                               void* workspace, size_t workspace_bytes, int64_t* report_dev, void* stream);

/* ---- structured-only representation -----------------------------------------------------------------
 * Sec. 4.4 / Fig. 4 / App. H compare the condensed layer with the same layer sped up by neuron ablation alone
 * (the sparsity inside the remaining rows is not used): the stored neurons keep dense rows, and the paper finds
 * it faster at larger batch and modest sparsity, from the same set of weights.
 *
 * srigl_densify: Wd[n_active][d_in] (w_dtype) <- the condensed rows scattered to their columns, zero
 * elsewhere (bit copies).  idx as in the forward call (in range; not checked here).
 *
 * srigl_structured_linear_fwd: y[b][active[s]] = bias[active[s]] + sum_j Wd[s][j] * x[b][j] on the matrix
 * cores (fp32 MFMA for F32 storage; bf16 MFMA with fp32 accumulate for BF16 storage), other columns = bias.
 * Same argument conventions as srigl_condensed_linear_fwd.  x and Wd must be 16-byte aligned and d_in a
 * multiple of 16 bytes' worth of elements (4 for F32, 8 for BF16), else SRIGL_ERR_UNSUPPORTED.
 */
srigl_status srigl_densify(const void* W_c, srigl_dtype w_dtype, const int32_t* idx, int32_t n_active, int32_t K,
                           int32_t d_in, void* Wd, void* stream);

srigl_status srigl_structured_linear_fwd(const void* x, srigl_dtype x_dtype, int32_t B, int32_t d_in, const void* Wd,
                                         srigl_dtype w_dtype, const int32_t* active, int32_t n_active,
                                         const float* bias, int32_t d_out, float* y, void* stream);

/* The same call with the workgroup tile forced (tests and tuning); SRIGL_TILE_AUTO is the library's own choice. */
typedef enum srigl_gemm_tile {
    SRIGL_TILE_AUTO = 0,
    SRIGL_TILE_256x256 = 1,     /* 8 wavefronts of 128x64, 2 LDS stages of 128 bytes of K per row */
    SRIGL_TILE_256x256_H = 2,   /* 8 wavefronts of 128x64, 5 LDS stages of 64 bytes */
    SRIGL_TILE_256x128_W4 = 3,  /* 4 wavefronts of 128x64, 3 LDS stages of 128 bytes */
    SRIGL_TILE_256x128 = 4,     /* 8 wavefronts of 64x64, 3 LDS stages of 128 bytes */
    SRIGL_TILE_128x128 = 5,     /* 4 wavefronts of 64x64, 4 LDS stages of 128 bytes */
    SRIGL_TILE_64x64 = 6        /* 4 wavefronts of 32x32, 4 LDS stages of 128 bytes */
} srigl_gemm_tile;

srigl_status srigl_structured_linear_fwd_tile(const void* x, srigl_dtype x_dtype, int32_t B, int32_t d_in, const void* Wd,
                                              srigl_dtype w_dtype, const int32_t* active, int32_t n_active,
                                              const float* bias, int32_t d_out, float* y, srigl_gemm_tile tile, void* stream);

/* The same product with d_in cut into parts (Sec. 4.4 / Fig. 4, structured-only form at small batch or few stored neurons:
 * the output tiles alone then reach a fraction of the compute units).  Every part's tiles run side by side and write
 * partial sums to workspace[part][B][n_active] (fp32); a second launch adds the parts in ascending order, adds the bias
 * and writes every column of y (deterministic: no atomics).  The sums differ from the one-part call's in rounding order only.
 *
 * srigl_structured_split_plan: the library's choice of parts for these sizes (1 = do not split) and the workspace
 * bytes that choice needs (parts * B * n_active * 4; 0 for one part).  Host-only.
 * srigl_structured_linear_fwd_split: splits = 0 takes that choice (with tile = SRIGL_TILE_AUTO; a forced tile with
 * splits = 0 keeps one part), splits = 1..16 forces it; every part must hold at least one LDS stage of the tile
 * (SRIGL_ERR_INVALID_ARG otherwise).  workspace (device, 4-byte aligned, owned by the caller, contents undefined
 * afterwards) smaller than parts * B * n_active * 4 bytes: SRIGL_ERR_CAPACITY.  Calls that share a workspace must not
 * overlap. */
srigl_status srigl_structured_split_plan(int32_t B, int32_t d_in, int32_t n_active, int32_t d_out, srigl_dtype dtype, int32_t* splits,
                                         size_t* workspace_bytes);

srigl_status srigl_structured_linear_fwd_split(const void* x, srigl_dtype x_dtype, int32_t B, int32_t d_in, const void* Wd,
                                               srigl_dtype w_dtype, const int32_t* active, int32_t n_active, const float* bias,
                                               int32_t d_out, float* y, srigl_gemm_tile tile, int32_t splits, void* workspace,
                                               size_t workspace_bytes, void* stream);

/* Which of the two representations of a layer is expected to run its forward pass faster for a batch of B rows
 * (Sec. 4.4 / Fig. 4: the condensed form wins at small batch and high sparsity, the structured-only form at large batch
 * and modest sparsity).  Host-only arithmetic on the sizes, from timings of both kernels on MI355X; the two estimates
 * (microseconds) are written when the pointers are not NULL.  Layers whose rows are not a multiple of 16 bytes always
 * get SRIGL_REPR_CONDENSED. */
typedef enum srigl_representation { SRIGL_REPR_CONDENSED = 0, SRIGL_REPR_STRUCTURED = 1 } srigl_representation;

srigl_representation srigl_choose_representation(int32_t B, int32_t d_in, int32_t n_active, int32_t K, int32_t d_out,
                                                 srigl_dtype dtype, float* est_condensed_us, float* est_structured_us);

/* An empty kernel on `stream`: the dispatch floor against which microsecond-scale calls are read. */
srigl_status srigl_launch_empty(void* stream);

/* Plain device copy kernel of n_bytes (multiple of 16), the reference for bandwidth counters. */
srigl_status srigl_copy_bytes(const void* src, void* dst, size_t n_bytes, void* stream);

const char* srigl_status_str(srigl_status s);

#ifdef __cplusplus
}
#endif
#endif /* SRIGL_H_ */
