"""GPU parity, floating-point side: srigl_condensed_linear_fwd against the CPU oracle (Alg. 1).

Gate: |y_gpu - y_ref| <= tol * max(|y_ref|, S) per element, S = |bias| + sum_k |w x| from the
oracle; tol = 1e-5 for fp32 storage, 1e-2 for bf16 storage (fp32 accumulate).  Columns of ablated
neurons and integer-valued problems are compared bit for bit.
"""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from gpu_util import TOL_BF16, TOL_F32, dev, gate, host, oracle_condensed, oracle_seg
from paper_2305_02299_amd import binding as B_

pytestmark = pytest.mark.gpu

ALGOS = {"auto": None, "generic": B_.FWD_GENERIC, "klane": B_.FWD_KLANE, "rowlane": B_.FWD_ROWLANE, "rowloop": B_.FWD_ROWLOOP}
GUARD = 1024


def run_gpu(L, W_c, idx, active, bias, algo=None, tuning=None, seg=True, x=None, packed=False):
    """Runs the library on device copies; y sits between two guard zones that must stay untouched."""
    xsrc = x if x is not None else (L.x_bf16 if L.dtype == "bf16" else L.x)
    Bn, d_in, d_out = xsrc.shape[0], L.d_in, L.d_out
    n_active, K = W_c.shape
    flat = torch.full((Bn * d_out + 2 * GUARD,), 777.0, dtype=torch.float32, device="cuda")
    y = flat[GUARD:GUARD + Bn * d_out].view(Bn, d_out)
    sg = dev(oracle_seg(idx, d_in)) if (seg and n_active and K) else None
    pk = None
    if packed and n_active and K:      # the streaming copy of the same rows, written by the library from the canonical arrays
        pk = torch.empty((B_.srigl_packed_bytes(n_active, K, d_in, B_.BF16 if L.dtype == "bf16" else B_.F32),), dtype=torch.uint8,
                         device="cuda")
        B_.srigl_pack_terms(dev(W_c), dev(idx), n_active, K, d_in, pk)
    B_.srigl_condensed_linear_fwd(dev(xsrc), Bn, d_in, dev(W_c), dev(idx), dev(active), n_active, K, dev(bias), d_out, y,
                                  sg, algo=algo, tuning=tuning, packed=pk)
    torch.cuda.synchronize()
    out = flat.cpu().numpy()
    assert (out[:GUARD] == 777.0).all() and (out[GUARD + Bn * d_out:] == 777.0).all(), "write outside y"
    return out[GUARD:GUARD + Bn * d_out].reshape(Bn, d_out).copy()


def check_layer(L, algo, tuning=None, bias=True, seg=True, unsupported_ok=False, packed=False):
    W_c, idx, active = oracle_condensed(L)
    bias_v = L.bias if bias else None
    xsrc = L.x_bf16 if L.dtype == "bf16" else L.x
    y_ref, S = oracle.fwd(xsrc, W_c, idx, active, bias_v, L.d_out, want_scale=True)
    act_arg = None if len(active) == L.d_out else active
    try:
        y = run_gpu(L, W_c, idx, act_arg, bias_v, algo, tuning, seg, packed=packed)
    except B_.SriglError as e:
        if e.status == B_.ERR_UNSUPPORTED and algo is not None:
            if unsupported_ok:
                return None
            pytest.skip("algorithm does not run these sizes")
        raise
    worst = gate(y, y_ref, S, TOL_BF16 if L.dtype == "bf16" else TOL_F32)
    ablated = np.setdiff1d(np.arange(L.d_out), active)
    if len(ablated):
        exp = (L.bias if bias else np.zeros(L.d_out, np.float32))[ablated]
        assert np.array_equal(y[:, ablated].view(np.uint32), np.tile(exp, (L.B, 1)).view(np.uint32)), "ablated column != bias"
    return worst


# ----------------------------------------------------------------------------- the named configurations
@pytest.mark.parametrize("algo", list(ALGOS))
@pytest.mark.parametrize("cfg,B", [("c1", 1), ("c2", 256), ("c3", 1), ("c3", 256)])
def test_named_configs(cfg, B, algo):
    L = si.config(cfg, B=B)
    worst = check_layer(L, ALGOS[algo])
    print("%s B=%d %s: worst err/scale %.2e" % (cfg, B, algo, worst))
    assert worst < 2e-6   # fp32 accumulation of <= 307 terms stays far inside the gate


def test_c2_through_gpu_condense():
    """Config 2 end to end on the GPU: dense W + mask -> srigl_condense -> forward."""
    from paper_2305_02299_amd import condense_layer
    L = si.config("c2")
    layer = condense_layer(dev(L.W), dev(L.mask), L.K, dev(L.bias))
    W_c, idx, active = oracle_condensed(L)
    assert layer.n_active == 3072 and layer.active is None
    assert np.array_equal(host(layer.idx), idx) and np.array_equal(host(layer.W_c).view(np.uint32), W_c.view(np.uint32))
    y = host(layer.forward(dev(L.x)))
    y_ref, S = oracle.fwd(L.x, W_c, idx, active, L.bias, L.d_out, want_scale=True)
    gate(y, y_ref, S, TOL_F32)
    # same call twice: identical bits
    y2 = host(layer.forward(dev(L.x)))
    assert np.array_equal(y.view(np.uint32), y2.view(np.uint32))


# ----------------------------------------------------------------------------- ragged shapes, every algorithm
RAGGED = [
    # d_in, d_out, K, B, ablate
    (16, 8, 3, 3, 0.25),
    (50, 7, 1, 5, 0.0),
    (77, 33, 20, 70, 0.1),
    (1001, 130, 333, 65, 0.5),
    (257, 5, 257, 2, 0.0),
    (768, 100, 77, 130, 0.0),
    (768, 3072, 8, 16, 0.0),
    (3072, 200, 615, 64, 0.05),
    (640, 1000, 39, 33, 0.9),
]


@pytest.mark.parametrize("algo", list(ALGOS))
@pytest.mark.parametrize("d_in,d_out,K,B,abl", RAGGED)
def test_ragged_shapes(d_in, d_out, K, B, abl, algo):
    L = si.make_layer(d_in, d_out, K, B, ablate_frac=abl, seed=200 + d_in + B)
    check_layer(L, ALGOS[algo])


@pytest.mark.parametrize("algo", list(ALGOS))
def test_no_bias_and_no_seg(algo):
    L = si.make_layer(512, 96, 40, 67, ablate_frac=0.2, seed=31)
    check_layer(L, ALGOS[algo], bias=False)
    check_layer(L, ALGOS[algo], seg=False)


@pytest.mark.parametrize("tuning", [
    {"rows_per_lane": 1, "waves": 4, "neurons_per_wave": 1, "chunk_cols": 64},
    {"rows_per_lane": 1, "waves": 16, "neurons_per_wave": 6, "chunk_cols": 256},
    {"rows_per_lane": 2, "waves": 8, "neurons_per_wave": 3, "chunk_cols": 128},
    {"rows_per_lane": 2, "waves": 16, "neurons_per_wave": 4, "chunk_cols": 256},
    {"term_slices": 2, "waves": 16, "neurons_per_wave": 3},
    {"rows_per_lane": 2, "term_slices": 2, "waves": 16, "neurons_per_wave": 3},
    {"rows_per_lane": 2, "term_slices": 2, "waves": 4, "neurons_per_wave": 4, "chunk_cols": 128},
    {"rows_per_lane": 2, "term_slices": 4, "waves": 16, "neurons_per_wave": 3},
    {"rows_per_lane": 4, "term_slices": 4, "waves": 16, "neurons_per_wave": 3},
    {"rows_per_lane": 4, "term_slices": 4, "waves": 4, "neurons_per_wave": 1, "chunk_cols": 128},
    {"rows_per_lane": 4, "term_slices": 2, "waves": 16, "neurons_per_wave": 2},
    {"rows_per_lane": 4, "term_slices": 2, "waves": 8, "neurons_per_wave": 3, "chunk_cols": 64},
    {"rows_per_lane": 2, "term_slices": 4, "waves": 8, "neurons_per_wave": 2, "chunk_cols": 192},
    {"term_slices": 2, "waves": 8, "neurons_per_wave": 6, "chunk_cols": 192},
    {"term_slices": 4, "waves": 8, "neurons_per_wave": 6},
    {"term_slices": 4, "waves": 16, "neurons_per_wave": 2, "chunk_cols": 128},
    {"term_slices": 4, "waves": 2, "neurons_per_wave": 1, "chunk_cols": 64},
    {"rows_per_lane": 1, "term_slices": 1, "waves": 16, "neurons_per_wave": 8, "chunk_cols": 128},
    {"rows_per_lane": 1, "term_slices": 2, "waves": 3, "neurons_per_wave": 8},
    {"rows_per_lane": 1, "term_slices": 4, "waves": 16, "neurons_per_wave": 8, "chunk_cols": 256},
    {"rows_per_lane": 2, "term_slices": 1, "waves": 16, "neurons_per_wave": 8, "chunk_cols": 128},
    {"rows_per_lane": 2, "term_slices": 1, "waves": 5, "neurons_per_wave": 6, "chunk_cols": 64},
    {"rows_per_lane": 2, "term_slices": 2, "waves": 16, "neurons_per_wave": 8},
    {"rows_per_lane": 2, "term_slices": 2, "waves": 7, "neurons_per_wave": 6, "chunk_cols": 128},
    {"rows_per_lane": 2, "term_slices": 4, "waves": 16, "neurons_per_wave": 6},
    {"rows_per_lane": 2, "term_slices": 4, "waves": 12, "neurons_per_wave": 8, "chunk_cols": 192},
])
def test_rowlane_launch_shapes(tuning):
    for (d_in, d_out, K, B, abl) in ((768, 300, 77, 300, 0.1), (3072, 96, 307, 70, 0.3), (1001, 64, 100, 257, 0.0),
                                     (768, 40, 8, 17, 0.0), (1024, 50, 615, 33, 0.2)):
        L = si.make_layer(d_in, d_out, K, B, ablate_frac=abl, seed=77)
        ran = check_layer(L, B_.FWD_ROWLANE, tuning, unsupported_ok=True)
        assert ran is not None or d_in % 16 != 0     # only the ragged-width layer may be refused (slow staging: H = R = 1)


@pytest.mark.parametrize("tuning", [
    None,
    {"term_slices": 4, "waves": 16, "neurons_per_wave": 1},
    {"term_slices": 4, "waves": 3, "neurons_per_wave": 7},
    {"term_slices": 4, "waves": 16, "neurons_per_wave": 5, "xcd_order": 2},
    {"term_slices": 4, "waves": 8, "neurons_per_wave": 2, "xcd_order": 1},
    {"term_slices": 2, "waves": 16, "neurons_per_wave": 2},
    {"term_slices": 2, "waves": 5, "neurons_per_wave": 3, "xcd_order": 2},
    {"term_slices": 2, "waves": 1, "neurons_per_wave": 40},
    {"term_slices": 4, "waves": 4, "neurons_per_wave": 24},     # 96 stored rows per workgroup, 24 to a wavefront
    {"term_slices": 2, "waves": 2, "neurons_per_wave": 30},
    {"term_slices": 4, "waves": 15, "neurons_per_wave": 7},     # 105 rows: a last group that is not full on every layer below
])
def test_whole_input_batched_kernel_launch_shapes(tuning):
    """ROWLOOP: every column of x in one LDS tile, a wavefront walks its stored rows one after the other.  Rows of one block of
    terms per slice up to rows longer than the four preloaded blocks (K = 300 in four slices: 75 steps, K = 500 in two: 250),
    batches with a ragged last tile, stored columns with and without ablated ones between them, fp32 and bf16; few and many stored rows per
    wavefront, with a last group that is not full."""
    for (d_in, d_out, K, B, abl, dtype) in ((768, 300, 77, 300, 0.1, "f32"), (512, 333, 300, 70, 0.0, "f32"), (512, 90, 500, 33, 0.3, "f32"),
                                            (256, 1000, 8, 257, 0.0, "bf16"), (1024, 130, 1, 65, 0.5, "f32"), (16, 40, 16, 100, 0.2, "f32"),
                                            (640, 2100, 39, 95, 0.6, "bf16")):
        L = si.make_layer(d_in, d_out, K, B, dtype=dtype, ablate_frac=abl, seed=91)
        ran = check_layer(L, B_.FWD_ROWLOOP, tuning, unsupported_ok=True)
        # the 64-row tile of two term slices holds inputs up to 600 columns wide, the 32-row one up to 1100
        assert (ran is not None) == (d_in <= 512 or tuning is None or tuning["term_slices"] == 4), (d_in, tuning)


def test_whole_input_batched_kernel_few_stored_neurons_among_many_ablated():
    """Runs of output columns longer than the workgroup's column table: the lanes write their stored column and the ablated ones
    in front of it."""
    for (d_in, d_out, K, B, abl) in ((128, 30000, 9, 40, 0.97), (1024, 40000, 40, 33, 0.998), (64, 5000, 3, 70, 0.9)):
        L = si.make_layer(d_in, d_out, K, B, ablate_frac=abl, seed=92)
        for tuning in (None, {"waves": 2, "neurons_per_wave": 1}, {"term_slices": 2, "waves": 16, "neurons_per_wave": 1}):
            ran = check_layer(L, B_.FWD_ROWLOOP, tuning, unsupported_ok=True)
            assert ran is not None or (d_in == 1024 and tuning and tuning.get("term_slices") == 2)


def test_whole_input_batched_kernel_refuses_what_it_cannot_hold():
    for (d_in, K) in ((3072, 77), (1200, 30), (100, 7)):     # wider than the LDS tile; not a multiple of 16 columns
        L = si.make_layer(d_in, 64, K, 40, seed=93)
        assert check_layer(L, B_.FWD_ROWLOOP, None, unsupported_ok=True) is None
    L = si.make_layer(256, 64, 20, 40, seed=93)
    for tuning in ({"rows_per_lane": 1}, {"term_slices": 1}, {"waves": 17}, {"xcd_order": 3}, {"neurons_per_wave": 4096}):
        assert check_layer(L, B_.FWD_ROWLOOP, tuning, unsupported_ok=True) is None, tuning


def test_rowlane_row_of_more_chunks_than_a_wavefront_has_lanes():
    """65 chunks of 64 columns: the per-row register of chunk boundaries (one lane per chunk) is reloaded on the way."""
    L = si.make_layer(4160, 40, 130, 70, ablate_frac=0.1, seed=79)
    assert check_layer(L, B_.FWD_ROWLANE, {"rows_per_lane": 1, "term_slices": 1, "waves": 4, "neurons_per_wave": 2, "chunk_cols": 64}) is not None
    L = si.make_layer(8192, 24, 300, 33, seed=80)      # 128 chunks: two reloads
    assert check_layer(L, B_.FWD_ROWLANE, {"rows_per_lane": 1, "term_slices": 1, "waves": 2, "neurons_per_wave": 3, "chunk_cols": 64}) is not None


@pytest.mark.parametrize("tuning", [{"lanes_per_neuron": l, "rows_per_block": r} for l in (1, 4, 16, 64) for r in (1, 2, 4, 8)])
def test_klane_launch_shapes(tuning):
    for (d_in, d_out, K, B, abl) in ((768, 300, 77, 9, 0.1), (3072, 96, 307, 3, 0.3), (100, 64, 5, 1, 0.0)):
        L = si.make_layer(d_in, d_out, K, B, ablate_frac=abl, seed=78)
        check_layer(L, B_.FWD_KLANE, tuning)


# ----------------------------------------------------------------------------- the streaming copy in place of W_c / idx
@pytest.mark.parametrize("cfg,B", [("c1", 1), ("c2", 256), ("c3", 1), ("c3", 256)])
@pytest.mark.parametrize("algo", ["auto", "klane", "rowlane"])
def test_named_configs_through_the_streaming_copy(cfg, B, algo):
    L = si.config(cfg, B=B) if cfg == "c3" else si.config(cfg)
    worst = check_layer(L, ALGOS[algo], {"terms_from_copy": 1} if algo == "rowlane" else None, packed=True)
    assert worst < 2e-6


@pytest.mark.parametrize("tuning", [{"lanes_per_neuron": l, "rows_per_block": r, "direct_gather": g}
                                    for l in (1, 4, 16, 64) for r in (1, 2, 8) for g in (1, 2)])
def test_klane_launch_shapes_through_the_streaming_copy(tuning):
    for (d_in, d_out, K, B, abl, dtype) in ((768, 300, 77, 9, 0.1, "f32"), (3072, 96, 307, 3, 0.3, "f32"), (100, 64, 5, 1, 0.0, "f32"),
                                            (1300, 70, 130, 5, 0.2, "bf16"), (70000, 12, 9, 2, 0.0, "bf16"), (64, 40, 64, 11, 0.0, "f32")):
        L = si.make_layer(d_in, d_out, K, B, ablate_frac=abl, dtype=dtype, seed=78)
        # (terms_from_copy: the copy is read with several batch rows per workgroup too, which the library would not do by itself)
        check_layer(L, B_.FWD_KLANE, dict(tuning, terms_from_copy=1), packed=True,
                    unsupported_ok=(d_in > 40960 and tuning["direct_gather"] == 2))


@pytest.mark.parametrize("tuning", [
    {"rows_per_lane": 1, "waves": 4, "neurons_per_wave": 1, "chunk_cols": 64},
    {"rows_per_lane": 1, "waves": 16, "neurons_per_wave": 6, "chunk_cols": 256},
    {"rows_per_lane": 2, "waves": 16, "neurons_per_wave": 4, "chunk_cols": 256},
    {"rows_per_lane": 2, "term_slices": 2, "waves": 16, "neurons_per_wave": 3},
    {"rows_per_lane": 2, "term_slices": 4, "waves": 8, "neurons_per_wave": 2, "chunk_cols": 192},
    {"rows_per_lane": 4, "term_slices": 4, "waves": 16, "neurons_per_wave": 3},
    {"term_slices": 2, "waves": 8, "neurons_per_wave": 6, "chunk_cols": 192},
    {"term_slices": 4, "waves": 16, "neurons_per_wave": 2, "chunk_cols": 128},
    {"rows_per_lane": 1, "term_slices": 1, "waves": 16, "neurons_per_wave": 8, "chunk_cols": 128},
    {"rows_per_lane": 2, "term_slices": 1, "waves": 16, "neurons_per_wave": 8, "chunk_cols": 128},
    {"rows_per_lane": 2, "term_slices": 2, "waves": 7, "neurons_per_wave": 6, "chunk_cols": 128},
    {"rows_per_lane": 2, "term_slices": 4, "waves": 12, "neurons_per_wave": 8, "chunk_cols": 192},
])
def test_rowlane_launch_shapes_through_the_streaming_copy(tuning):
    """The batched kernel with its terms read from the streaming copy (one load per block of terms): every tile shape, fp32
    and bf16 storage, rows whose padded length differs from K, and a bf16 layer too wide for 16-bit indices (which the
    kernel reads from the arrays)."""
    for (d_in, d_out, K, B, abl, dtype) in ((768, 300, 77, 300, 0.1, "f32"), (3072, 96, 307, 70, 0.3, "f32"), (768, 40, 8, 17, 0.0, "f32"),
                                            (1024, 50, 615, 33, 0.2, "f32"), (1024, 200, 102, 130, 0.2, "bf16"),
                                            (4096, 64, 205, 70, 0.0, "bf16"), (65552, 20, 9, 40, 0.0, "bf16")):
        L = si.make_layer(d_in, d_out, K, B, ablate_frac=abl, dtype=dtype, seed=79)
        assert check_layer(L, B_.FWD_ROWLANE, dict(tuning, terms_from_copy=1), packed=True, unsupported_ok=True) is not None


def test_padded_places_of_the_streaming_copy_never_meet_an_activation():
    """A row of 77 terms fills 19 units and a quarter; the three padded places carry index 0.  A non-finite activation in
    column 0 must reach only the rows that really name column 0."""
    L = si.make_layer(768, 200, 77, 3, ablate_frac=0.2, seed=5)
    L.x[1, 0] = np.inf
    W_c, idx, active = oracle_condensed(L)
    names_col0 = idx[:, 0] == 0
    assert names_col0.any() and not names_col0.all()
    for tuning in ({"direct_gather": 1}, {"direct_gather": 2}):
        y = run_gpu(L, W_c, idx, active, L.bias, B_.FWD_KLANE, tuning, packed=True)
        assert np.isfinite(y[1, active[~names_col0]]).all() and np.isinf(y[1, active[names_col0]]).all()
        y_ref, S = oracle.fwd(L.x[[0, 2]], W_c, idx, active, L.bias, L.d_out, want_scale=True)
        gate(y[[0, 2]], y_ref, S, TOL_F32)


# ----------------------------------------------------------------------------- exact cases
@pytest.mark.parametrize("algo", list(ALGOS))
def test_integer_inputs_are_bit_exact(algo):
    """Integer operands: every partial sum is an integer below 2^24, so any summation order gives the same bits."""
    rng = np.random.default_rng(41)
    for (d_in, d_out, K, B, abl) in ((768, 256, 154, 70, 0.1), (3072, 64, 615, 3, 0.3)):
        L = si.make_layer(d_in, d_out, K, B, ablate_frac=abl, seed=41)
        L.W = rng.integers(-8, 9, size=L.W.shape).astype(np.float32)
        L.x = rng.integers(-8, 9, size=L.x.shape).astype(np.float32)
        L.bias = rng.integers(-8, 9, size=L.bias.shape).astype(np.float32)
        W_c, idx, active = oracle_condensed(L)
        y_ref = oracle.fwd(L.x, W_c, idx, active, L.bias, d_out)
        try:
            y = run_gpu(L, W_c, idx, active, L.bias, ALGOS[algo])
        except B_.SriglError as e:
            assert e.status == B_.ERR_UNSUPPORTED
            continue
        assert np.array_equal(y.view(np.uint32), y_ref.view(np.uint32))


@pytest.mark.parametrize("algo", list(ALGOS))
def test_one_hot_rows_are_bit_exact(algo):
    """x = e_j: y[n] = bias[n] + W[n][j] M[n][j], a single rounding."""
    L = si.make_layer(768, 200, 77, 64, ablate_frac=0.2, seed=42)
    cols = np.random.default_rng(42).integers(0, 768, size=64)
    L.x = np.zeros((64, 768), np.float32)
    L.x[np.arange(64), cols] = 1.0
    W_c, idx, active = oracle_condensed(L)
    y = run_gpu(L, W_c, idx, active, L.bias, ALGOS[algo])
    exp = (L.bias[None, :].astype(np.float64) + (L.W * L.mask)[:, cols].T.astype(np.float64)).astype(np.float32)
    assert np.array_equal(y.view(np.uint32), exp.view(np.uint32))


@pytest.mark.parametrize("algo", ["auto", "generic", "klane", "rowloop"])
def test_unsorted_and_duplicate_indices(algo):
    """Alg. 1 is a plain sum over k: without seg the library must accept any in-range index order."""
    L = si.make_layer(304 if algo == "rowloop" else 300, 50, 21, 40, seed=43)    # (ROWLOOP: whole 16-column units)
    W_c, idx, active = oracle_condensed(L)
    rng = np.random.default_rng(43)
    perm = np.stack([rng.permutation(21) for _ in range(50)])
    Wp, ip = np.take_along_axis(W_c, perm, 1), np.take_along_axis(idx, perm, 1)
    ip[:, 3] = ip[:, 2]
    y_ref, S = oracle.fwd(L.x, Wp, ip, None, L.bias, 50, want_scale=True)
    y = run_gpu(L, Wp, ip, None, L.bias, ALGOS[algo], seg=False)
    gate(y, y_ref, S, TOL_F32)


# ----------------------------------------------------------------------------- degenerate problems
def test_degenerate_problems():
    L = si.make_layer(64, 12, 5, 3, ablate_frac=0.25, seed=44)
    W_c, idx, active = oracle_condensed(L)
    # n_active = 0: bias broadcast
    y = run_gpu(L, W_c[:0], idx[:0], active[:0], L.bias, None)
    assert np.array_equal(y, np.tile(L.bias, (3, 1)))
    # K = 0
    y = run_gpu(L, np.zeros((9, 0), np.float32), np.zeros((9, 0), np.int32), active, L.bias, None)
    assert np.array_equal(y, np.tile(L.bias, (3, 1)))
    # no bias, nothing stored: zeros
    y = run_gpu(L, W_c[:0], idx[:0], active[:0], None, None)
    assert (y == 0).all()
    # B = 0 returns without touching anything
    y = run_gpu(L, W_c, idx, active, L.bias, None, x=L.x[:0])
    assert y.shape == (0, 12)
    # out-of-range columns in `active` are skipped, not written
    bad_active = active.copy()
    bad_active[-1] = 12
    y = run_gpu(L, W_c, idx, bad_active, L.bias, B_.FWD_GENERIC)
    assert y.shape == (3, 12)


def test_fwd_host_side_argument_errors():
    L = si.make_layer(64, 12, 5, 3, seed=45)
    W_c, idx, active = oracle_condensed(L)
    x, W, i, y = dev(L.x), dev(W_c), dev(idx), torch.empty((3, 12), device="cuda")
    with pytest.raises(B_.SriglError) as e:   # active == NULL needs n_active == d_out
        B_.srigl_condensed_linear_fwd(x, 3, 64, W, i, None, 11, 5, None, 12, y)
    assert e.value.status == B_.ERR_INVALID_ARG
    with pytest.raises(B_.SriglError) as e:   # K > d_in
        B_.srigl_condensed_linear_fwd(x, 3, 4, W, i, None, 12, 5, None, 12, y)
    assert e.value.status == B_.ERR_INVALID_ARG
    with pytest.raises(B_.SriglError) as e:   # mixed storage types
        B_.srigl_condensed_linear_fwd(x, 3, 64, W.to(torch.int16), i, None, 12, 5, None, 12, y)
    assert e.value.status == B_.ERR_UNSUPPORTED
    with pytest.raises(B_.SriglError) as e:   # a launch shape the kernels do not have
        B_.srigl_condensed_linear_fwd(x, 3, 64, W, i, None, 12, 5, None, 12, y, None, algo=B_.FWD_ROWLANE,
                                      tuning={"rows_per_lane": 3})
    assert e.value.status == B_.ERR_UNSUPPORTED
    # ROWLANE over several LDS chunks needs the seg table
    L = si.make_layer(3072, 16, 30, 3, seed=45)
    W_c, idx, active = oracle_condensed(L)
    with pytest.raises(B_.SriglError) as e:
        B_.srigl_condensed_linear_fwd(dev(L.x), 3, 3072, dev(W_c), dev(idx), None, 16, 30, None, 16,
                                      torch.empty((3, 16), device="cuda"), None, algo=B_.FWD_ROWLANE)
    assert e.value.status == B_.ERR_UNSUPPORTED


# ----------------------------------------------------------------------------- bf16 storage
@pytest.mark.parametrize("algo", list(ALGOS))
@pytest.mark.parametrize("d_in,d_out,K,B,abl", [(4096, 512, 205, 96, 0.2), (130, 9, 7, 5, 0.0), (768, 300, 77, 1, 0.1)])
def test_bf16_storage(d_in, d_out, K, B, abl, algo):
    L = si.make_layer(d_in, d_out, K, B, ablate_frac=abl, dtype="bf16", idx_dist="clustered" if d_in >= 1024 else "uniform", seed=46)
    worst = check_layer(L, ALGOS[algo])
    assert worst < 2e-6   # same bf16 inputs on both sides: only the fp32 accumulation differs


# ----------------------------------------------------------------------------- the sparsity x batch sweep
@pytest.mark.parametrize("d_in,d_out,s,K,B", si.sweep_points())
def test_sweep_points(d_in, d_out, s, K, B):
    L = si.make_layer(d_in, d_out, K, B, seed=0)
    check_layer(L, None)


# ----------------------------------------------------------------------------- full-size stress layer, sampled
def test_large_layer_sampled_rows():
    """4096 -> 16384, K = 205, bf16 storage, B = 2048, 20 % ablated, clustered indices: the GPU runs the
    whole batch; the oracle recomputes a sample of batch rows (first, last, tile edges, random)."""
    L = si.config("c5")
    W_c, idx, active = oracle_condensed(L)
    assert W_c.shape == (13108, 205)
    # tile edges, and three interior rows of every 128-row tile (the tallest batch tile of the batched kernel)
    rng = np.random.default_rng(5)
    rows = np.unique(np.concatenate([[0, 1, 63, 64, 127, 128, 255, 256, 1023, 2046, 2047]] +
                                    [128 * t + rng.choice(np.arange(2, 126), size=3, replace=False) for t in range(16)]))
    assert all(((rows // 128 == t) & (rows % 128 > 1) & (rows % 128 < 126)).sum() >= 2 for t in range(16))
    y_ref, S = oracle.fwd(L.x_bf16[rows], W_c, idx, active, L.bias, L.d_out, want_scale=True)
    for algo, packed in ((None, False), (B_.FWD_ROWLANE, False), (B_.FWD_ROWLANE, True)):
        y = run_gpu(L, W_c, idx, active, L.bias, algo, {"terms_from_copy": 1} if packed else None, packed=packed)
        gate(y[rows], y_ref, S, TOL_BF16)
        ablated = np.setdiff1d(np.arange(L.d_out), active)
        assert np.array_equal(y[:, ablated].view(np.uint32), np.tile(L.bias[ablated], (2048, 1)).view(np.uint32))
        assert np.isfinite(y).all()


# ----------------------------------------------------------------------------- non-finite activations stay local
@pytest.mark.parametrize("algo", list(ALGOS))
def test_non_finite_activation_only_reaches_its_own_terms(algo):
    """y[b][n] depends on x[b][j] only for j in idx[n]: an inf / NaN in one column must not touch neurons that do not
    index that column (padding inside the kernels must never multiply 0 by it)."""
    L = si.make_layer(768, 200, 77, 70, ablate_frac=0.1, seed=47)
    W_c, idx, active = oracle_condensed(L)
    x = L.x.copy()
    bad_cols = [0, 63, 64, 383, 384, 767]          # tile / chunk edges
    x[3, bad_cols] = np.inf
    x[40, bad_cols] = np.nan
    y = run_gpu(L, W_c, idx, active, L.bias, ALGOS[algo], x=x)
    y_ref, S = oracle.fwd(x, W_c, idx, active, L.bias, L.d_out, want_scale=True)
    touches = np.isin(idx, bad_cols).any(axis=1)                     # stored rows that index a bad column
    clean_cols = active[~touches]
    assert len(clean_cols) > 50
    assert np.isfinite(y[:, clean_cols]).all()
    fin = np.isfinite(y_ref)
    assert np.array_equal(np.isfinite(y), fin)
    assert np.max(np.abs(y[fin] - y_ref[fin]) / np.maximum(np.maximum(np.abs(y_ref[fin]), S[fin]), 1e-30)) < TOL_F32


@pytest.mark.parametrize("B", [1, 3, 40])
def test_input_wider_than_the_lds_row_of_the_small_batch_kernel(B):
    """d_in = 49152: one fp32 row of x (192 KB) does not fit the LDS.  The small-batch kernel then gathers its activations from
    global memory (its staged form refuses), the batched kernel walks chunks of columns; every path matches the oracle."""
    L = si.make_layer(49152, 48, 64, B, ablate_frac=0.1, seed=11)
    assert check_layer(L, None, None) is not None
    assert check_layer(L, B_.FWD_KLANE, None, unsupported_ok=True) is not None                          # gathers
    assert check_layer(L, B_.FWD_KLANE, dict(direct_gather=2), unsupported_ok=True) is None             # staging refuses
    assert check_layer(L, B_.FWD_ROWLANE, None, unsupported_ok=True) is not None                        # the batched kernel runs it


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("gather", [1, 2])
@pytest.mark.parametrize("B,rb", [(1, 1), (2, 2), (3, 2), (5, 4), (9, 8), (33, 4), (7, 1)])
def test_small_batch_kernel_gathered_and_staged_activations(B, rb, gather, dtype):
    """Both sources of the activations (gathered from global memory, staged in LDS), every rows-per-workgroup setting, batches
    that leave the last workgroup row ragged; K = 77 leaves the last request of a lane group partly past the row."""
    L = si.make_layer(320, 200, 77, B, ablate_frac=0.15, seed=B + 10 * rb, dtype=dtype)
    worst = check_layer(L, B_.FWD_KLANE, dict(direct_gather=gather, rows_per_block=rb))
    assert worst < (TOL_BF16 if dtype == "bf16" else 2e-6)


@pytest.mark.parametrize("gather", [1, 2])
def test_small_batch_kernel_forced_at_a_batch_beyond_its_workgroup_limit(gather):
    """More row blocks than the 2048 (staged) or 8192 (gathered) workgroups the launch is held to: one workgroup per row block
    that walks all stored rows."""
    B = 2100 if gather == 2 else 8300
    L = si.make_layer(2048, 24, 40, B, ablate_frac=0.2, seed=B)
    worst = check_layer(L, B_.FWD_KLANE, dict(direct_gather=gather, rows_per_block=1))
    assert worst < 2e-6


@pytest.mark.parametrize("xcd_order", [1, 2])
@pytest.mark.parametrize("shape", [(768, 300, 77, 300), (3072, 200, 307, 200), (320, 130, 40, 1100), (2048, 96, 64, 530)])
def test_batched_kernel_either_xcd_order(shape, xcd_order):
    """Both assignments of workgroups to XCDs (by groups of stored rows, by batch tiles), with tile and group counts that are
    not multiples of eight, so that some workgroup ids of the padded grid have nothing to do."""
    d_in, d_out, K, B = shape
    L = si.make_layer(d_in, d_out, K, B, ablate_frac=0.2, seed=d_in + B)
    worst = check_layer(L, B_.FWD_ROWLANE, dict(xcd_order=xcd_order))
    assert worst < 2e-6


@pytest.mark.parametrize("dist", ["uniform", "clustered"])
@pytest.mark.parametrize("shape", [(768, 300, 77, 300, dict(neurons_per_wave=3)), (2048, 1000, 205, 200, dict(rows_per_lane=2, term_slices=1, neurons_per_wave=6)),
                                   (4096, 530, 64, 130, dict(rows_per_lane=1, term_slices=2, waves=12, neurons_per_wave=2)),
                                   (1024, 96, 64, 530, dict(chunk_cols=256, neurons_per_wave=2)),
                                   (320, 130, 40, 70, dict(rows_per_lane=4, term_slices=4, neurons_per_wave=2, chunk_cols=64))])
@pytest.mark.parametrize("mode", [2, 3])
def test_batched_kernel_rows_dealt_out_by_median_column(shape, dist, mode):
    """A workgroup's stored rows shared out among its wavefronts in the order of their median column instead of in runs of
    consecutive rows: same sums (a row's terms are added in the same order), with a last workgroup that holds fewer rows
    than places, ablated columns between the stored ones, one to six rows per wavefront and several chunks per row."""
    d_in, d_out, K, B, tn = shape
    L = si.make_layer(d_in, d_out, K, B, ablate_frac=0.2, seed=d_in + B, idx_dist=dist)
    tuning = dict(tn or {}, spread_rows=mode)
    assert B_.srigl_fwd_plan_query(B, d_in, int(L.mask.any(1).sum()), K, d_out, B_.F32, True, True, algo=B_.FWD_ROWLANE, tuning=tuning)["spread_rows"] == mode
    worst = check_layer(L, B_.FWD_ROWLANE, tuning)
    assert worst < 2e-6


@pytest.mark.parametrize("tuning", [dict(rows_per_lane=2, term_slices=1, neurons_per_wave=8), dict(rows_per_lane=2, term_slices=2, neurons_per_wave=8),
                                    dict(rows_per_lane=1, term_slices=1, neurons_per_wave=8), dict(rows_per_lane=2, term_slices=4, neurons_per_wave=6)])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_six_and_eight_rows_per_wavefront_with_and_without_dealing(tuning, dtype):
    """Clustered rows in several chunks, a last workgroup that holds fewer rows than places, both storage types."""
    L = si.make_layer(2048, 700, 102, 150, ablate_frac=0.25, seed=12, dtype=dtype, idx_dist="clustered")
    for mode in (1, 2, 3):
        worst = check_layer(L, B_.FWD_ROWLANE, dict(tuning, chunk_cols=256, spread_rows=mode))
        assert worst < (TOL_BF16 if dtype == "bf16" else 2e-6)


def test_rows_are_not_dealt_out_one_to_a_wavefront_or_from_the_copy():
    """One stored row per wavefront leaves nothing to deal out, and the kernel that reads the streaming copy keeps consecutive
    rows: both refuse the forced setting; the library's own choice deals rows out from four chunks per row on where a workgroup
    runs long enough for the test of the medians not to show."""
    L = si.make_layer(320, 130, 40, 70, ablate_frac=0.2, seed=1)
    assert check_layer(L, B_.FWD_ROWLANE, dict(neurons_per_wave=1, spread_rows=2), unsupported_ok=True) is None
    assert check_layer(L, B_.FWD_ROWLANE, dict(terms_from_copy=1, spread_rows=2), unsupported_ok=True, packed=True) is None
    q = lambda B, d_in, n, K, **kw: B_.srigl_fwd_plan_query(B, d_in, n, K, n, kw.pop("dtype", B_.F32), False, True, algo=B_.FWD_ROWLANE, **kw)
    assert q(2048, 4096, 16384, 205, dtype=B_.BF16)["spread_rows"] == 3      # 16 chunks of 256 columns
    assert q(1024, 4096, 4096, 205)["spread_rows"] == 3                      # 16 chunks, ~65 us per workgroup
    assert q(256, 4096, 4096, 205)["spread_rows"] == 1                       # 8 chunks of 512, but ~35 us per workgroup
    assert q(256, 768, 3072, 77)["spread_rows"] == 1                         # 2 chunks
    assert q(1024, 768, 3072, 77)["spread_rows"] == 1                        # 3 chunks


@pytest.mark.parametrize("abl,B", [(0.3, 70), (0.7, 200), (0.9, 64), (0.97, 300), (0.995, 33)])
def test_batched_kernel_writes_ablated_columns_between_stored_ones(abl, B):
    """Runs of output columns per workgroup from a few dozen (30 % ablated) to beyond the column table (99.5 %: the per-lane
    loop), every ablated column bit-equal to its bias (checked by check_layer)."""
    L = si.make_layer(512, 4000, 40, B, ablate_frac=abl, seed=int(abl * 1000))
    for shape in (dict(), dict(term_slices=4), dict(rows_per_lane=2), dict(rows_per_lane=2, term_slices=2)):
        worst = check_layer(L, B_.FWD_ROWLANE, shape)
        assert worst < 2e-6
