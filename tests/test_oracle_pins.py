"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests compares the oracle with itself: the expected values come
from a hand-worked fixture (App. E's definition applied with pencil and paper),
from numpy's float64 matmul on the dense masked matrix (App. E: the condensed and
the ordinary product are equal for any matrix), from closed forms (one-hot
inputs, integer-exact inputs), and from the sampler's own ground truth.
"""
import json
import os

import numpy as np
import pytest

import oracle
import synth_inputs as si


def _dense_ref(x, W, mask, bias):
    """Library routine: float64 matmul of the dense masked matrix (App. E, first equation)."""
    Wm = W.astype(np.float64) * (mask != 0)
    y = x.astype(np.float64) @ Wm.T
    if bias is not None:
        y = y + bias.astype(np.float64)
    return y


# ----------------------------------------------------------------------------- hand-worked fixture
def test_handworked_fixture(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "appE_handworked.json")))
    W = np.array(g["W"], np.float32)
    mask = np.array(g["mask"], np.uint8)
    bias = np.array(g["bias"], np.float32)
    x = np.array(g["x"], np.float32)
    rep = oracle.check_fanin_mask(mask)
    assert rep == {"K": 2, "n_active": 3, "n_bad_rows": 0, "first_bad_row": -1, "status": 0}
    W_c, idx, active = oracle.condense(W, mask, g["K"])
    assert W_c.tolist() == g["W_c"] and idx.tolist() == g["idx"] and active.tolist() == g["active"]
    y = oracle.fwd(x, W_c, idx, active, bias, g["d_out"])
    assert y.tolist() == g["y"]
    assert oracle.fwd(x, W_c, idx, active, None, g["d_out"]).tolist() == g["y_no_bias"]
    assert oracle.dense_masked_fwd(x, W, mask, bias).tolist() == g["y"]
    # compact output (no scatter): the s-th stored neuron is column s
    yc = oracle.fwd(x, W_c, idx, None, bias[active], 3)
    assert yc.tolist() == [[r[c] for c in g["active"]] for r in g["y"]]


# ----------------------------------------------------------------------------- condense
@pytest.mark.parametrize("d_in,d_out,K,abl,seed", [(16, 8, 3, 0.25, 1), (768, 96, 77, 0.0, 2), (3072, 40, 307, 0.3, 3),
                                                   (64, 33, 64, 0.1, 4), (50, 7, 1, 0.0, 5)])
def test_condense_matches_sampler_ground_truth(d_in, d_out, K, abl, seed):
    L = si.make_layer(d_in, d_out, K, 2, ablate_frac=abl, seed=seed)
    W_c, idx, active = oracle.condense(L.W, L.mask, K)
    assert np.array_equal(idx, L.true_idx)
    assert np.array_equal(active, L.true_active)
    assert np.array_equal(W_c.view(np.uint32), si.gather_condensed(L).view(np.uint32))
    # invariant: exactly K strictly ascending in-range columns per stored neuron
    assert idx.shape == (L.n_active, K)
    assert (idx >= 0).all() and (idx < d_in).all()
    if K > 1:
        assert (np.diff(idx, axis=1) > 0).all()
    # round trip: scattering back gives W (.) M bit for bit
    back = np.zeros_like(L.W)
    back[active[:, None], idx] = W_c
    assert np.array_equal(back.view(np.uint32), np.where(L.mask != 0, L.W, np.float32(0)).view(np.uint32))


def test_condense_is_mask_driven_and_bit_exact():
    """A kept weight that is -0.0, +0.0, NaN or inf is copied bit for bit and counts toward K."""
    L = si.make_layer(32, 6, 4, 1, seed=7)
    W = L.W.copy()
    specials = np.array([0x80000000, 0x00000000, 0x7FC00123, 0xFF800000], np.uint32).view(np.float32)
    W[0, L.true_idx[0]] = specials
    W_c, idx, active = oracle.condense(W, L.mask, 4)
    assert np.array_equal(W_c[0].view(np.uint32), specials.view(np.uint32))
    assert np.array_equal(idx, L.true_idx)
    # an unmasked non-zero value is ignored
    assert (L.mask[1] == 0).sum() > 0


def test_condense_bf16_bit_copy():
    L = si.make_layer(64, 10, 9, 1, dtype="bf16", ablate_frac=0.2, seed=8)
    W_c, idx, active = oracle.condense(L.W_bf16, L.mask, 9)
    assert W_c.dtype == np.uint16
    assert np.array_equal(W_c, L.W_bf16[L.true_active[:, None], L.true_idx])
    assert np.array_equal(idx, L.true_idx) and np.array_equal(active, L.true_active)


def test_condense_rejects_wrong_fanin():
    L = si.make_layer(32, 6, 4, 1, seed=9)
    m = L.mask.copy()
    j = int(np.flatnonzero(m[3] == 0)[0])
    m[3, j] = 1
    with pytest.raises(ValueError, match="row 3"):
        oracle.condense(L.W, m, 4)


# ----------------------------------------------------------------------------- check_fanin
def test_check_fanin_accepts_generated_and_flags_single_flip():
    L = si.make_layer(96, 20, 10, 1, ablate_frac=0.25, seed=11)
    rep = oracle.check_fanin_mask(L.mask)
    assert rep == {"K": 10, "n_active": 15, "n_bad_rows": 0, "first_bad_row": -1, "status": 0}
    assert oracle.check_fanin_mask(L.mask, 10)["status"] == 0
    for r in (int(L.true_active[2]), int(L.true_active[-1])):
        for newval, col in ((1, int(np.flatnonzero(L.mask[r] == 0)[0])), (0, int(np.flatnonzero(L.mask[r])[0]))):
            m = L.mask.copy()
            m[r, col] = newval
            rep = oracle.check_fanin_mask(m, 10)
            assert rep["n_bad_rows"] == 1 and rep["first_bad_row"] == r and rep["status"] == 2
            assert rep["n_active"] == 14
    # any non-zero byte counts as kept
    m = L.mask.copy() * 200
    assert oracle.check_fanin_mask(m, 10)["status"] == 0
    # wrong expectation: every stored row is bad
    rep = oracle.check_fanin_mask(L.mask, 9)
    assert rep["n_bad_rows"] == 15 and rep["first_bad_row"] == int(L.true_active[0])
    # all rows ablated
    z = np.zeros((4, 8), np.uint8)
    assert oracle.check_fanin_mask(z) == {"K": 0, "n_active": 0, "n_bad_rows": 0, "first_bad_row": -1, "status": 0}


def test_check_fanin_idx_mode():
    L = si.make_layer(96, 20, 10, 1, seed=12)
    assert oracle.check_fanin_idx(L.true_idx, 96)["status"] == 0
    bad = L.true_idx.copy()
    bad[5, 3] = bad[5, 2]                    # duplicate -> not strictly ascending
    rep = oracle.check_fanin_idx(bad, 96)
    assert rep["n_bad_rows"] == 1 and rep["first_bad_row"] == 5
    bad = L.true_idx.copy()
    bad[7, -1] = 96                          # out of range
    assert oracle.check_fanin_idx(bad, 96)["first_bad_row"] == 7
    bad = L.true_idx.copy()
    bad[0, 0] = -1
    assert oracle.check_fanin_idx(bad, 96)["first_bad_row"] == 0
    bad = L.true_idx.copy()
    bad[9, [1, 2]] = bad[9, [2, 1]]          # swapped -> descending pair
    assert oracle.check_fanin_idx(bad, 96)["first_bad_row"] == 9


# ----------------------------------------------------------------------------- forward
@pytest.mark.parametrize("d_in,d_out,K,B,abl,seed", [(16, 8, 3, 3, 0.25, 21), (768, 64, 77, 4, 0.0, 22),
                                                     (3072, 24, 307, 2, 0.3, 23), (40, 9, 40, 5, 0.0, 24)])
def test_fwd_equals_dense_masked_product(d_in, d_out, K, B, abl, seed):
    """App. E: the condensed product equals the ordinary product for any matrix."""
    L = si.make_layer(d_in, d_out, K, B, ablate_frac=abl, seed=seed)
    W_c, idx, active = oracle.condense(L.W, L.mask, K)
    y = oracle.fwd(L.x, W_c, idx, active, L.bias, d_out)
    ref = _dense_ref(L.x, L.W, L.mask, L.bias)
    # float64 sums of <= 3072 terms rounded once to fp32: at most one fp32 ulp apart
    assert np.array_equal(y, ref.astype(np.float32)) or np.max(np.abs(y - ref) / np.maximum(np.abs(ref), 1e-30)) < 2.0 ** -23
    yd = oracle.dense_masked_fwd(L.x, L.W, L.mask, L.bias)
    assert np.max(np.abs(yd.astype(np.float64) - ref)) <= np.max(np.abs(ref)) * 2.0 ** -23
    # asymmetric in every operand: a transposed or mis-indexed operand cannot pass
    assert not np.allclose(y, _dense_ref(L.x, L.W, L.mask, None).astype(np.float32))


def test_fwd_dense_special_case_K_equals_d_in():
    """K = d_in with identity indices is an ordinary dense linear layer."""
    rng = np.random.default_rng(31)
    B, d_in, d_out = 5, 24, 7
    W = rng.standard_normal((d_out, d_in)).astype(np.float32)
    x = rng.standard_normal((B, d_in)).astype(np.float32)
    bias = rng.standard_normal(d_out).astype(np.float32)
    idx = np.tile(np.arange(d_in, dtype=np.int32), (d_out, 1))
    y = oracle.fwd(x, W, idx, None, bias, d_out)
    ref = x.astype(np.float64) @ W.astype(np.float64).T + bias
    assert np.max(np.abs(y - ref)) <= np.max(np.abs(ref)) * 2.0 ** -23


def test_fwd_ablated_columns_hold_bias_bits():
    L = si.make_layer(64, 20, 6, 3, ablate_frac=0.4, seed=33)
    W_c, idx, active = oracle.condense(L.W, L.mask, 6)
    y = oracle.fwd(L.x, W_c, idx, active, L.bias, 20)
    ablated = np.setdiff1d(np.arange(20), active)
    assert len(ablated) == 8
    for b in range(3):
        assert np.array_equal(y[b, ablated].view(np.uint32), L.bias[ablated].view(np.uint32))
    y0 = oracle.fwd(L.x, W_c, idx, active, None, 20)
    assert (y0[:, ablated] == 0).all()


def test_fwd_one_hot_input_reads_single_weight():
    """x = e_j: y[n] = bias[n] + W[n][j] M[n][j], one rounding."""
    L = si.make_layer(48, 12, 5, 1, ablate_frac=0.25, seed=34)
    W_c, idx, active = oracle.condense(L.W, L.mask, 5)
    for j in (0, 17, 47):
        x = np.zeros((1, 48), np.float32)
        x[0, j] = 1.0
        y = oracle.fwd(x, W_c, idx, active, L.bias, 12)
        exp = (L.bias.astype(np.float64) + L.W[:, j].astype(np.float64) * (L.mask[:, j] != 0)).astype(np.float32)
        assert np.array_equal(y[0].view(np.uint32), exp.view(np.uint32))


def test_fwd_small_integers_exact():
    """Integer operands: every partial sum is an integer below 2^24, so the result is exact."""
    rng = np.random.default_rng(35)
    B, d_in, d_out, K = 4, 100, 10, 30
    L = si.make_layer(d_in, d_out, K, B, ablate_frac=0.2, seed=35)
    W = rng.integers(-8, 9, size=(d_out, d_in)).astype(np.float32)
    x = rng.integers(-8, 9, size=(B, d_in)).astype(np.float32)
    bias = rng.integers(-8, 9, size=d_out).astype(np.float32)
    W_c, idx, active = oracle.condense(W, L.mask, K)
    y = oracle.fwd(x, W_c, idx, active, bias, d_out)
    exp = x.astype(np.int64) @ (W.astype(np.int64) * L.mask).T + bias.astype(np.int64)
    assert np.array_equal(y.astype(np.int64), exp) and np.array_equal(y, exp.astype(np.float32))


def test_fwd_any_index_order_and_duplicates():
    """Alg. 1 is a plain sum over k: permuting (w, idx) pairs within a row changes nothing
    beyond rounding, and a repeated index contributes twice."""
    L = si.make_layer(64, 8, 7, 3, seed=36)
    W_c, idx, active = oracle.condense(L.W, L.mask, 7)
    rng = np.random.default_rng(36)
    perm = np.stack([rng.permutation(7) for _ in range(8)])
    Wp = np.take_along_axis(W_c, perm, 1)
    ip = np.take_along_axis(idx, perm, 1)
    y = oracle.fwd(L.x, W_c, idx, active, L.bias, 8)
    yp = oracle.fwd(L.x, Wp, ip, active, L.bias, 8)
    assert np.max(np.abs(y - yp)) < 1e-6
    dup_idx = idx.copy()
    dup_idx[:, 1] = dup_idx[:, 0]
    yd = oracle.fwd(L.x, W_c, dup_idx, active, None, 8)
    exp = np.einsum("nk,bnk->bn", W_c.astype(np.float64), L.x.astype(np.float64)[:, dup_idx])
    assert np.max(np.abs(yd - exp)) < 1e-5


def test_fwd_bf16_widens_exactly():
    L = si.make_layer(128, 16, 13, 3, dtype="bf16", ablate_frac=0.25, seed=37)
    W_c, idx, active = oracle.condense(L.W_bf16, L.mask, 13)
    y = oracle.fwd(L.x_bf16, W_c, idx, active, L.bias, 16)
    ref = _dense_ref(L.x, L.W, L.mask, L.bias)          # L.W / L.x are the exactly widened values
    assert np.max(np.abs(y - ref)) <= np.max(np.abs(ref)) * 2.0 ** -23
    # and identical to the fp32 entry point on the widened values
    y32 = oracle.fwd(L.x, si.bf16_bits_to_f32(W_c), idx, active, L.bias, 16)
    assert np.array_equal(y, y32)


def test_fwd_scale_is_sum_of_term_magnitudes():
    L = si.make_layer(40, 6, 5, 2, ablate_frac=0.34, seed=38)
    W_c, idx, active = oracle.condense(L.W, L.mask, 5)
    y, S = oracle.fwd(L.x, W_c, idx, active, L.bias, 6, want_scale=True)
    exp = np.abs(L.x.astype(np.float64)) @ (np.abs(L.W.astype(np.float64)) * L.mask).T + np.abs(L.bias.astype(np.float64))
    assert np.allclose(S, exp, rtol=1e-12, atol=0)
    assert (S >= np.abs(y) * (1 - 1e-6)).all()


def test_fwd_degenerate_shapes():
    # B = 0
    L = si.make_layer(16, 4, 3, 0, seed=39)
    W_c, idx, active = oracle.condense(L.W, L.mask, 3)
    assert oracle.fwd(L.x, W_c, idx, active, L.bias, 4).shape == (0, 4)
    # n_active = 0: bias broadcast
    L = si.make_layer(16, 4, 3, 2, ablate_frac=1.0, seed=40)
    W_c, idx, active = oracle.condense(L.W, L.mask, 3)
    assert W_c.shape == (0, 3)
    y = oracle.fwd(L.x, W_c, idx, active, L.bias, 4)
    assert np.array_equal(y, np.tile(L.bias, (2, 1)))
    # K = 0
    y = oracle.fwd(L.x, np.zeros((4, 0), np.float32), np.zeros((4, 0), np.int32), None, L.bias, 4)
    assert np.array_equal(y, np.tile(L.bias, (2, 1)))


def test_allcores_timing_companion_agrees_with_the_oracle():
    L = si.make_layer(256, 40, 30, 9, ablate_frac=0.2, seed=50)
    W_c, idx, active = oracle.condense(L.W, L.mask, 30)
    y, S = oracle.fwd(L.x, W_c, idx, active, L.bias, 40, want_scale=True)
    y2, threads = oracle.fwd_allcores(L.x, W_c, idx, active, L.bias, 40)
    assert threads >= 1
    assert (np.abs(y2.astype(np.float64) - y) <= 1e-5 * np.maximum(np.abs(y), S)).all()
    ablated = np.setdiff1d(np.arange(40), active)
    assert np.array_equal(y2[:, ablated], y[:, ablated])


# ----------------------------------------------------------------------------- structured-only representation
@pytest.mark.parametrize("d_in,d_out,K,B,abl,dtype", [(64, 12, 5, 3, 0.25, "f32"), (768, 40, 77, 4, 0.3, "f32"), (128, 9, 128, 2, 0.0, "f32"),
                                                      (96, 10, 7, 3, 0.2, "bf16")])
def test_structured_only_representation(d_in, d_out, K, B, abl, dtype):
    """Ablated neurons removed, remaining rows dense (Sec. 4.4 / Fig. 4): same result as the dense masked product."""
    L = si.make_layer(d_in, d_out, K, B, ablate_frac=abl, dtype=dtype, seed=60)
    Wsrc, xsrc = (L.W_bf16, L.x_bf16) if dtype == "bf16" else (L.W, L.x)
    W_c, idx, active = oracle.condense(Wsrc, L.mask, K)
    Wd = oracle.densify(W_c, idx, d_in)
    # densify against plain indexing of the masked dense matrix (bit for bit)
    exp = np.where(L.mask[active] != 0, Wsrc[active], np.zeros((), Wsrc.dtype))
    assert Wd.dtype == Wsrc.dtype and np.array_equal(Wd.view(np.uint8), exp.view(np.uint8))
    y = oracle.structured_fwd(xsrc, Wd, active, L.bias, d_out)
    ref = _dense_ref(L.x, L.W, L.mask, L.bias)      # numpy float64 matmul; L.W / L.x hold the widened values for bf16
    assert np.max(np.abs(y - ref)) <= np.max(np.abs(ref)) * 2.0 ** -23
    ablated = np.setdiff1d(np.arange(d_out), active)
    assert np.array_equal(y[:, ablated], np.tile(L.bias[ablated], (B, 1)))
    # and the condensed oracle agrees (both are sums of the same non-zero terms in ascending column order)
    yc = oracle.fwd(xsrc, W_c, idx, active, L.bias, d_out)
    assert np.max(np.abs(y - yc)) <= np.max(np.abs(ref)) * 2.0 ** -23


# ---- MLP block: activation and width reduction (Sec. 3.1, App. H) -----------------------------------------

def test_activation_closed_forms():
    v = np.array([0.0, 1.0, -1.0, 2.5, -2.5, 30.0, -30.0], dtype=np.float32)
    assert np.array_equal(oracle.activate(v, oracle.ACT_NONE), v)
    assert np.array_equal(oracle.activate(v, oracle.ACT_RELU), np.maximum(v, 0))
    g = oracle.activate(v, oracle.ACT_GELU).astype(np.float64)
    assert g[0] == 0.0
    assert abs(g[1] - 0.8413447460685429) < 1e-7          # Phi(1), a tabulated constant
    assert np.allclose(g[1] - g[2], 1.0, atol=1e-7)        # v Phi(v) - (-v) Phi(-v) = v
    assert np.allclose(g[3] - g[4], 2.5, atol=1e-6)
    assert g[5] == 30.0 and g[6] == 0.0                    # the tails
    # against scipy's normal distribution function on a grid
    from scipy.stats import norm
    grid = np.linspace(-6, 6, 241).astype(np.float32)
    assert np.allclose(oracle.activate(grid, oracle.ACT_GELU), grid.astype(np.float64) * norm.cdf(grid.astype(np.float64)),
                       rtol=1.5e-7, atol=1e-30)     # the result is rounded to fp32 once


def test_fold_handworked_fixture():
    import json
    import os
    fx = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "fold_handworked.json")))
    idx, W, bias = oracle.fold_ablated_inputs(np.array(fx["idx2"], np.int32), np.array(fx["W_c2"], np.float32),
                                              np.array(fx["bias2"], np.float32), np.array(fx["active2"], np.int32), fx["d_out2"],
                                              np.array(fx["active1"], np.int32), fx["d_hidden"], np.array(fx["bias1"], np.float32),
                                              fx["act"])
    assert idx.tolist() == fx["expect_idx"]
    assert W.tolist() == fx["expect_W_c"]
    assert bias.tolist() == fx["expect_bias"]


@pytest.mark.parametrize("act", [0, 1, 2])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_folded_pair_equals_the_unfolded_pair(act, dtype):
    """linear -> activation -> linear computed two ways with the pinned forward: full-width hidden vector and the original
    second layer, or compact hidden vector (stored neurons only) and the folded second layer."""
    L1 = si.make_layer(48, 96, 7, 9, ablate_frac=0.4, dtype=dtype, seed=21)
    L2 = si.make_layer(96, 40, 13, 9, ablate_frac=0.2, dtype=dtype, seed=22)
    W1, x = (L1.W_bf16, L1.x_bf16) if dtype == "bf16" else (L1.W, L1.x)
    W2 = L2.W_bf16 if dtype == "bf16" else L2.W
    Wc1, idx1, act1 = oracle.condense(W1, L1.mask, L1.K)
    Wc2, idx2, act2 = oracle.condense(W2, L2.mask, L2.K)
    conv = (lambda h: si.f32_to_bf16_bits(h)) if dtype == "bf16" else (lambda h: h)
    # unfolded: hidden at full width, ablated neurons hold act(bias)
    h_full = oracle.activate(oracle.fwd(x, Wc1, idx1, act1, L1.bias, L1.d_out), act)
    y_ref, S = oracle.fwd(conv(h_full), Wc2, idx2, act2, L2.bias, L2.d_out, want_scale=True)
    # folded: hidden holds the stored neurons only
    h_compact = oracle.activate(oracle.fwd(x, Wc1, idx1, None, L1.bias[act1], len(act1)), act)
    assert np.array_equal(h_compact, h_full[:, act1])
    idx_f, W_f, bias_f = oracle.fold_ablated_inputs(idx2, Wc2, L2.bias, act2, L2.d_out, act1, L1.d_out, L1.bias, act)
    y = oracle.fwd(conv(h_compact), W_f, idx_f, act2, bias_f, L2.d_out)
    # in bf16 storage the constant act(bias) is rounded to bf16 on the unfolded side only: allow that rounding
    tol = 1e-6 if dtype == "f32" else 8e-3
    assert np.all(np.abs(y.astype(np.float64) - y_ref) <= tol * np.maximum(S, 1e-30))
    # shape of the folded rows
    assert np.all(np.diff(idx_f, axis=1) > 0) and idx_f.min() >= 0 and idx_f.max() < len(act1)
    pos = {int(c): p for p, c in enumerate(act1)}
    for n in range(idx2.shape[0]):
        kept = [(pos[int(j)], Wc2[n, k]) for k, j in enumerate(idx2[n]) if int(j) in pos]
        got = {int(i): W_f[n, k] for k, i in enumerate(idx_f[n])}
        for p_, w in kept:
            assert got[p_].tobytes() == w.tobytes()
        fillers = [i for i in got if i not in dict(kept)]
        assert all(got[i].tobytes() == b"\x00" * W_f.dtype.itemsize for i in fillers)
        unused_smaller = [g for g in range(max(fillers, default=-1)) if g not in got]
        assert not unused_smaller                     # fillers are the smallest unused positions


def test_packed_copy_handworked_fixture():
    """The streaming copy of the two App. E arrays against bytes written out by hand (fp32 and bf16 storage)."""
    fx = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "packed_handworked.json")))
    idx = np.array(fx["idx"], np.int32)
    for W, key in ((np.array(fx["W_c_f32"], np.float32), "packed_f32_hex"), (np.array(fx["W_c_bf16_bits"], np.uint16), "packed_bf16_hex")):
        got = oracle.pack_terms(W, idx, fx["d_in"])
        assert [row.tobytes().hex() for row in got] == [h.replace(" ", "") for h in fx[key]]


def test_packed_copy_holds_every_term_once_and_wide_indices_when_needed():
    """Reading the bytes back with plain struct unpacking returns the canonical arrays; a bf16 layer wider than 65536
    columns keeps 32-bit indices behind the weight's half-word and 16 zero bits."""
    import struct
    rng = np.random.default_rng(3)
    for (n, K, d_in, bf16) in ((5, 77, 768, False), (3, 9, 70000, True), (4, 12, 4096, True)):
        idx = np.sort(np.stack([rng.choice(d_in, K, replace=False) for _ in range(n)]), axis=1).astype(np.int32)
        W = rng.integers(1, 65535, size=(n, K)).astype(np.uint16) if bf16 else rng.normal(size=(n, K)).astype(np.float32)
        raw = oracle.pack_terms(W, idx, d_in)
        tb = 4 if (bf16 and d_in <= 65536) else 8
        terms = (K + 3) // 4 * 4
        assert raw.shape == (n, terms * tb)
        for s in range(n):
            b = raw[s].tobytes()
            for t in range(terms):
                if tb == 4:
                    w, col = struct.unpack_from("<HH", b, 4 * t)
                elif bf16:
                    w, zero, col = struct.unpack_from("<HHi", b, 8 * t)
                    assert zero == 0
                else:
                    w, col = struct.unpack_from("<fi", b, 8 * t)
                assert (w, col) == ((W[s, t], idx[s, t]) if t < K else (0, 0))


def test_compact_hidden_layer_is_the_first_layer_without_its_ablated_columns():
    """Pin: the full-width first layer's output restricted to the stored columns equals the compact layer's output when
    the compact layer uses bias_compact and writes position p for stored neuron p (Alg. 1 on both sides)."""
    L = si.make_layer(48, 40, 7, 5, ablate_frac=0.4, seed=12)
    W_c, idx, active = oracle.condense(L.W, L.mask, L.K)
    width = (len(active) + 15) // 16 * 16
    bias_c, active_c = oracle.compact_hidden_layer(L.bias, active, L.d_out, width)
    full = oracle.fwd(L.x, W_c, idx, active, L.bias, L.d_out)
    compact = oracle.fwd(L.x, W_c, idx, active_c, bias_c, width)
    assert np.array_equal(compact[:, :len(active)].view(np.uint32), full[:, active].view(np.uint32))
    assert (compact[:, len(active):] == 0).all() and active_c.tolist() == list(range(len(active)))
    b0, a0 = oracle.compact_hidden_layer(None, None, 4, 6)
    assert b0.tolist() == [0.0] * 6 and a0.tolist() == [0, 1, 2, 3]


def test_a_filler_of_a_folded_row_meets_a_non_finite_hidden_value():
    """What the header of srigl_compact_hidden_layer warns of: a folded row is refilled with zero-weight entries at real
    hidden positions, and Alg. 1 multiplies every stored term, so an infinite hidden value there gives 0 * inf = NaN in a
    row that never named that neuron; the unfolded layer has no such term."""
    d_hidden = 6
    active1 = np.array([0, 2, 3, 5], np.int32)                  # neurons 1 and 4 of layer 1 are ablated
    idx2 = np.array([[1, 5]], np.int32)                         # the row reads ablated neuron 1 and stored neuron 5
    W2 = np.array([[0.5, 2.0]], np.float32)
    bias1 = np.zeros(d_hidden, np.float32)
    idx_f, W_f, bias_f = oracle.fold_ablated_inputs(idx2, W2, None, None, 1, active1, d_hidden, bias1, 0)
    assert idx_f.tolist() == [[0, 3]] and W_f.tolist() == [[0.0, 2.0]]          # filler at compact position 0 = neuron 0
    hidden_full = np.array([[np.inf, 0.0, 1.0, 1.0, 0.0, 3.0]], np.float32)     # neuron 0 overflowed; the row never named it
    y_unfolded = oracle.fwd(hidden_full, W2, idx2, None, None, 1)
    y_folded = oracle.fwd(hidden_full[:, active1], W_f, idx_f, None, bias_f, 1)
    assert y_unfolded[0, 0] == 6.0 and np.isnan(y_folded[0, 0])


def test_fold_refuses_a_fan_in_wider_than_the_compact_layer():
    idx2 = np.arange(5, dtype=np.int32)[None, :]
    with pytest.raises(ValueError):
        oracle.fold_ablated_inputs(idx2, np.ones((1, 5), np.float32), None, None, 1, np.array([0, 2, 4], np.int32), 5, None, 0)


# ---- SRigL connectivity update (Sec. 3.1 steps 1-7) ---------------------------------------------------------

def _mask_update_by_lexsort(W, mask, grad, k, K_upd, gamma_percent, budget):
    """The same reading of Sec. 3.1 written with whole-array numpy primitives (lexsort rankings), for tiny inputs."""
    d_out, d_in = mask.shape
    mag = np.abs(W).view(np.uint32).astype(np.int64).ravel()
    gmag = np.abs(grad).view(np.uint32).astype(np.int64).ravel()
    pos = np.arange(d_out * d_in)
    kept = mask.ravel() != 0
    kp, pp = pos[kept], pos[~kept]
    kp = kp[np.lexsort((kp, mag[kp]))]                       # ascending magnitude, then position
    pp = pp[np.lexsort((pp, -gmag[pp]))]                     # descending gradient, then position
    salient = np.bincount(kp[K_upd:] // d_in, minlength=d_out) + np.bincount(pp[:K_upd] // d_in, minlength=d_out)
    held = mask.sum(axis=1)
    remains = (held > 0) & ~((salient < 1) | (salient * 100 < gamma_percent * k))
    n_rem = int(remains.sum())
    k_new = min(d_in, budget // n_rem) if n_rem else 0
    cand = kp[remains[kp // d_in]]
    keep = np.zeros(d_out * d_in, bool)
    keep[cand[K_upd:]] = True
    m2 = np.zeros_like(mask)
    W2 = np.zeros_like(W)
    for r in np.flatnonzero(remains):
        cols = np.arange(d_in)
        kr = keep[r * d_in:(r + 1) * d_in]
        mine = cols[kr][np.lexsort((cols[kr], -mag[r * d_in + cols[kr]]))][:k_new]
        free = cols[~kr][np.lexsort((cols[~kr], -gmag[r * d_in + cols[~kr]]))][:max(k_new - len(mine), 0)]
        m2[r, mine] = 1
        m2[r, free] = 1
        W2[r, mine] = W[r, mine]
    return m2, W2, {"k_new": k_new, "n_remaining": n_rem, "n_ablated_now": int(((held > 0) & ~remains).sum()),
                    "n_pruned": int(min(K_upd, len(cand)))}


def test_mask_update_handworked_fixture():
    import json
    import os
    fx = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "mask_update_handworked.json")))
    m, w, info = oracle.mask_update(np.array(fx["W"], np.float32), np.array(fx["mask"], np.uint8), np.array(fx["grad"], np.float32),
                                    fx["k"], fx["K_upd"], fx["gamma_percent"], fx["budget"])
    assert m.tolist() == fx["expect_mask"]
    assert w.tolist() == np.array(fx["expect_W"], np.float32).tolist()
    assert info == fx["expect_info"]


def test_mask_update_without_pruning_or_ablation_changes_nothing():
    L = si.make_layer(40, 30, 6, 1, ablate_frac=0.2, seed=4)
    g = np.random.default_rng(1).normal(size=L.W.shape).astype(np.float32)
    Wm = np.where(L.mask != 0, L.W, 0).astype(np.float32)
    m, w, info = oracle.mask_update(Wm, L.mask, g, L.K, 0, 0)
    assert np.array_equal(m, L.mask) and w.tobytes() == Wm.tobytes()
    assert info == {"k_new": L.K, "n_remaining": int((L.mask.sum(axis=1) > 0).sum()), "n_ablated_now": 0, "n_pruned": 0}


@pytest.mark.parametrize("seed", range(6))
def test_mask_update_invariants_and_lexsort_crosscheck(seed):
    rng = np.random.default_rng(100 + seed)
    d_in, d_out, k = int(rng.integers(8, 40)), int(rng.integers(6, 30)), 0
    k = int(rng.integers(1, d_in // 2 + 1))
    L = si.make_layer(d_in, d_out, k, 1, ablate_frac=float(rng.choice([0.0, 0.3])), seed=seed)
    Wm = np.where(L.mask != 0, L.W, 0).astype(np.float32)
    g = rng.normal(size=L.W.shape).astype(np.float32)
    if seed % 2:                      # coarse values: many equal magnitudes, so the position order decides
        Wm = (np.round(Wm * 4) / 4).astype(np.float32)
        g = (np.round(g * 2) / 2).astype(np.float32)
    n_kept = int(L.mask.sum())
    K_upd = int(rng.integers(0, n_kept // 2 + 1))
    gamma = int(rng.choice([0, 30, 60, 95]))
    m, w, info = oracle.mask_update(Wm, L.mask, g, k, K_upd, gamma)
    m2, w2, info2 = _mask_update_by_lexsort(Wm, L.mask, g, k, K_upd, gamma, n_kept)
    assert np.array_equal(m, m2) and w.tobytes() == w2.tobytes() and info == info2
    rows = m.sum(axis=1)
    assert set(np.unique(rows)) <= {0, info["k_new"]}                       # constant fan-in k' or ablated
    assert int((rows > 0).sum()) == info["n_remaining"] or info["k_new"] == 0
    assert np.all(rows[L.mask.sum(axis=1) == 0] == 0)                          # an ablated neuron stays ablated
    assert info["k_new"] * info["n_remaining"] <= n_kept                       # the layer's weight budget is not exceeded
    assert info["k_new"] >= k or info["n_remaining"] == 0                      # fewer neurons share the same budget
    assert np.all(w[m == 0] == 0)
    same = (m != 0) & (L.mask != 0) & (w != 0)
    assert np.array_equal(w[same], Wm[same])                                   # kept weights are copied, grown ones are zero
    assert np.all(w[(m != 0) & (L.mask == 0)] == 0)


def test_narrow_idx_is_the_same_numbers_in_two_bytes():
    """App. E's index array in 16-bit words: read back byte by byte (low byte first) the words give the same column
    numbers, at both ends of the range; a layer wider than 65536 columns, or an entry that names no column, has no
    such form."""
    rng = np.random.default_rng(5)
    idx = rng.integers(0, 65536, (37, 11)).astype(np.int32)
    idx[0, 0], idx[0, 1], idx[1, 0] = 0, 65535, 32768
    out = oracle.narrow_idx(idx, 65536)
    assert out.dtype == np.uint16 and out.shape == idx.shape
    b = out.reshape(-1).view(np.uint8).astype(np.int64)
    assert np.array_equal(b[0::2] + 256 * b[1::2], idx.reshape(-1))
    with pytest.raises(ValueError):
        oracle.narrow_idx(idx, 65537)
    with pytest.raises(ValueError):
        oracle.narrow_idx(np.array([3, 100], dtype=np.int32), 100)
    with pytest.raises(ValueError):
        oracle.narrow_idx(np.array([-1], dtype=np.int32), 100)
    assert oracle.narrow_idx(np.empty((0, 4), np.int32), 8).shape == (0, 4)


def _csr_of(W, mask):
    """Compressed sparse row form of the kept weights, built here with plain loops (test-side helper)."""
    vals, cols, ptr = [], [], [0]
    for r in range(mask.shape[0]):
        for j in range(mask.shape[1]):
            if mask[r, j]:
                vals.append(W[r, j])
                cols.append(j)
        ptr.append(len(vals))
    return np.array(vals, np.float32), np.array(cols, np.int32), np.array(ptr, np.int32)


@pytest.mark.parametrize("seed", range(3))
def test_csr_forward_equals_the_masked_matmul_and_the_library_product(seed):
    """The unstructured comparison (Sec. 4.4 / Fig. 4) computes the same function as the masked dense layer: against the
    all-terms definition, against scipy's own CSR product in fp64, and - on a constant fan-in mask - against Alg. 1 on the
    condensed form of the same weights.  Rows without entries output their bias."""
    import scipy.sparse as sp
    rng = np.random.default_rng(40 + seed)
    d_in, d_out, B = 37, 23, 5
    W = rng.normal(size=(d_out, d_in)).astype(np.float32)
    mask = (rng.random((d_out, d_in)) < 0.2).astype(np.uint8)     # unstructured: row lengths differ
    mask[3] = 0
    mask[d_out - 1] = 0
    x = rng.normal(size=(B, d_in)).astype(np.float32)
    bias = rng.normal(size=d_out).astype(np.float32)
    vals, cols, ptr = _csr_of(W, mask)
    y = oracle.csr_fwd(x, vals, cols, ptr, bias)
    assert np.array_equal(y, oracle.dense_masked_fwd(x, W, mask, bias))
    lib = sp.csr_matrix((vals.astype(np.float64), cols, ptr), shape=(d_out, d_in))
    assert np.allclose(y, (lib @ x.astype(np.float64).T).T + bias, rtol=1e-6, atol=1e-6)
    assert np.array_equal(y[:, 3], np.broadcast_to(bias[3], (B,)))
    # constant fan-in: the condensed form of the same weights gives the same numbers
    L = si.make_layer(48, 20, 7, 4, ablate_frac=0.2, seed=seed)
    W_c, idx, active = oracle.condense(L.W, L.mask, L.K)
    v2, c2, p2 = _csr_of(L.W, L.mask)
    assert np.array_equal(oracle.csr_fwd(L.x, v2, c2, p2, L.bias), oracle.fwd(L.x, W_c, idx, active, L.bias, L.d_out))
