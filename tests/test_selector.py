"""Host-side choice between the condensed and the structured-only representation (Sec. 4.4 / Fig. 4): properties that
hold whatever the calibration, plus the two ends of the paper's comparison.  No GPU work: the function is arithmetic on sizes."""
import pytest

import synth_inputs as si


@pytest.fixture(scope="module")
def B_():
    from paper_2305_02299_amd import binding
    return binding


def test_small_batches_stay_condensed(B_):
    """Online inference (one row) in either storage type, and batches up to 16 in fp32 (where the matrix pipe is slow)."""
    for (d_in, d_out, sp, K, B) in si.sweep_points():
        for dt in (B_.F32, B_.BF16):
            if B == 1 or (B <= 16 and dt == B_.F32):
                r, c, s = B_.srigl_choose_representation(B, d_in, d_out, K, d_out, dt)
                assert r == B_.REPR_CONDENSED, (d_in, d_out, K, B, dt, c, s)


def test_large_bf16_batch_at_modest_sparsity_goes_structured(B_):
    L = si.config("c5")
    r, c, s = B_.srigl_choose_representation(L.B, L.d_in, L.d_out, L.K, L.d_out, B_.BF16)
    assert r == B_.REPR_STRUCTURED and s < c


def test_online_inference_config_stays_condensed(B_):
    L = si.config("c1")
    r, c, s = B_.srigl_choose_representation(1, L.d_in, L.d_out, L.K, L.d_out, B_.F32)
    assert r == B_.REPR_CONDENSED and c < s


@pytest.mark.parametrize("dt", [0, 1])
def test_denser_rows_never_move_the_choice_towards_condensed(B_, dt):
    """The structured estimate does not depend on K, the condensed one grows with it."""
    for B in (64, 256, 1024, 4096):
        seen_structured = False
        prev_c = None
        for K in (1, 8, 39, 77, 154, 307, 768):
            r, c, s = B_.srigl_choose_representation(B, 768, 3072, K, 3072, dt)
            if prev_c is not None:
                assert c >= prev_c
            prev_c = c
            if seen_structured:
                assert r == B_.REPR_STRUCTURED
            seen_structured = seen_structured or r == B_.REPR_STRUCTURED


def test_rows_that_are_not_whole_16_byte_pieces_stay_condensed(B_):
    r, c, s = B_.srigl_choose_representation(4096, 770, 3072, 385, 3072, B_.F32)
    assert r == B_.REPR_CONDENSED
    r, c, s = B_.srigl_choose_representation(4096, 772, 3072, 385, 3072, B_.BF16)
    assert r == B_.REPR_CONDENSED


def test_parts_of_d_in_for_the_structured_only_product(B_):
    """Host-only plan: a wide fp32 layer with few stored neurons at a modest batch is cut into parts (its tiles alone reach a
    fraction of the compute units); a product with thousands of tiles is not; the workspace is parts x B x n_active floats."""
    L = si.config("c3", B=256)
    n = 538
    parts, need = B_.srigl_structured_split_plan(256, L.d_in, n, L.d_out, B_.F32)
    assert 2 <= parts <= 16 and need == parts * 256 * n * 4
    L5 = si.config("c5")
    assert B_.srigl_structured_split_plan(L5.B, L5.d_in, 13108, L5.d_out, B_.BF16) == (1, 0)
    # every part keeps at least four stages of 128 bytes: 64 fp32 columns are two stages, so one part
    assert B_.srigl_structured_split_plan(16, 64, 64, 64, B_.F32) == (1, 0)
    for (B, d_in, n_active) in [(1, 768, 3072), (64, 3072, 538), (300, 1024, 96), (2048, 4096, 100)]:
        for dt in (B_.F32, B_.BF16):
            parts, need = B_.srigl_structured_split_plan(B, d_in, n_active, n_active, dt)
            stages = (d_in * (4 if dt == B_.F32 else 2) + 127) // 128
            assert 1 <= parts <= max(1, min(16, stages // 4))
            assert need == (parts * B * n_active * 4 if parts > 1 else 0)
    assert B_.srigl_structured_split_plan(0, 768, 0, 3072, B_.F32) == (1, 0)
