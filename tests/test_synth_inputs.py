"""The input generator: shapes, fan-in structure and determinism (no method arithmetic)."""
import numpy as np

import synth_inputs as si


def test_fan_in_formula_integer():
    assert [si.fan_in_for_sparsity(768, s) for s in (80, 90, 95, 99)] == [154, 77, 39, 8]
    assert [si.fan_in_for_sparsity(3072, s) for s in (80, 90, 95, 99)] == [615, 308, 154, 31]


def test_named_configs_shapes():
    c1 = si.config("c1")
    assert (c1.d_in, c1.d_out, c1.K, c1.B, c1.n_active) == (768, 3072, 77, 1, 3072)
    assert c1.mask.sum(1).tolist() == [77] * 3072
    c3 = si.config("c3", B=1)
    assert (c3.d_in, c3.d_out, c3.K, c3.n_active) == (3072, 768, 307, 538)
    counts = c3.mask.sum(1)
    assert set(counts.tolist()) == {0, 307} and (counts == 0).sum() == 230


def test_determinism_and_seed_dependence():
    a = si.make_layer(64, 16, 5, 2, seed=3)
    b = si.make_layer(64, 16, 5, 2, seed=3)
    c = si.make_layer(64, 16, 5, 2, seed=4)
    assert np.array_equal(a.W, b.W) and np.array_equal(a.mask, b.mask) and np.array_equal(a.x, b.x)
    assert not np.array_equal(a.mask, c.mask)


def test_clustered_rows_structure():
    L = si.make_layer(4096, 64, 205, 1, idx_dist="clustered", dtype="bf16", ablate_frac=0.2, seed=5)
    assert L.n_active == 64 - 12
    idx = L.true_idx
    assert idx.shape == (52, 205) and (np.diff(idx, axis=1) > 0).all() and idx.min() >= 0 and idx.max() < 4096
    # at least floor(K/2) entries of each row sit in one 512-wide window
    for row in idx:
        best = max(np.searchsorted(row, row[i] + 512) - i for i in range(len(row)))
        assert best >= 102
    assert L.W_bf16.dtype == np.uint16 and np.array_equal(si.f32_to_bf16_bits(L.W), L.W_bf16)


def test_bf16_rounding_is_nearest_even():
    v = np.array([1.0, 1.00390625, 1.01171875, -2.5, 0.0], np.float32)  # 1+2^-8 ties to even (down), 1+3*2^-8 ties up
    bits = si.f32_to_bf16_bits(v)
    assert bits.tolist() == [0x3F80, 0x3F80, 0x3F82, 0xC020, 0x0000]
    assert si.bf16_bits_to_f32(bits).tolist() == [1.0, 1.0, 1.015625, -2.5, 0.0]
