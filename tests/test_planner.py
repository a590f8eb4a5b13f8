"""Host logic of the forward pass: which kernel and launch shape the library's own choice takes (srigl_fwd_plan_query is host
arithmetic only, so these run without a GPU).  The expectations are the shapes that measured best on MI355X for the
named configurations and for the corner cases the planner's rules exist for."""
import pytest

from paper_2305_02299_amd import binding as B_


def plan(B, d_in, d_out, K, n_active=None, **kw):
    n = d_out if n_active is None else n_active
    return B_.srigl_fwd_plan_query(B, d_in, n, K, d_out, has_active=(n != d_out), **kw)


def test_single_row_takes_the_small_batch_kernel():
    for (d_in, d_out, K) in ((768, 3072, 77), (3072, 768, 308), (4096, 16384, 205), (64, 8, 3)):
        p = plan(1, d_in, d_out, K)
        assert p["algo"] == B_.FWD_KLANE and p["rows_per_block"] == 1 and p["rows_per_lane"] == 0
    assert plan(1, 768, 3072, 77)["lanes_per_neuron"] == 32      # 77 terms: at most 4 per lane
    assert plan(1, 768, 3072, 8)["lanes_per_neuron"] == 4


def test_headline_batch_is_one_workgroup_per_compute_unit():
    # the whole 768-wide input fits one 32-row tile in LDS: wavefronts walk six stored rows each, 11.6 / 10.1 us cold / cached
    p = plan(256, 768, 3072, 77)
    assert p["algo"] == B_.FWD_ROWLOOP
    assert (p["rows_per_lane"], p["term_slices"], p["waves"], p["neurons_per_wave"]) == (2, 4, 16, 6)
    assert p["workgroups"] == 256 and p["chunk_cols"] == 768
    # the chunked batched kernel on the same layer (12.8 / 11.9 us):
    p = plan(256, 768, 3072, 77, algo=B_.FWD_ROWLANE)
    # 64-row tiles (two rows per lane in two term slices), 16 wavefronts of three stored rows: 12.9 / 11.8 us cold / cached
    # against 14.2 / 12.9 with one row per lane
    assert (p["rows_per_lane"], p["term_slices"], p["waves"], p["neurons_per_wave"]) == (2, 2, 16, 3)
    assert p["workgroups"] == 256 and p["chunk_cols"] == 384


def test_wide_inputs_get_16_row_tiles_and_one_row_per_workgroup():
    p = plan(256, 3072, 768, 307, n_active=538)
    assert p["algo"] == B_.FWD_ROWLANE and p["term_slices"] == 4 and p["neurons_per_wave"] == 3
    # staged activations: one row per workgroup for wide inputs, two for narrow ones from batch 5
    assert plan(256, 3072, 768, 31, algo=B_.FWD_KLANE, tuning=dict(direct_gather=2))["rows_per_block"] == 1
    assert plan(8, 768, 3072, 77, algo=B_.FWD_KLANE, tuning=dict(direct_gather=2))["rows_per_block"] == 2


def test_small_batches_gather_their_activations():
    """Measured: up to a few million gathered terms the small-batch kernel is faster reading x through the caches than staging
    rows of it in LDS (3072 -> 768 at B = 1: 3.7 vs 6.4 us cold), with one, two or four batch rows per workgroup."""
    for (B, d_in, d_out, K, rb) in ((1, 768, 3072, 77, 1), (1, 3072, 768, 308, 1), (4, 3072, 768, 308, 1), (8, 3072, 768, 308, 2),
                                    (4, 768, 3072, 77, 1), (8, 4096, 1024, 410, 2), (2, 4096, 16384, 205, 2)):
        p = plan(B, d_in, d_out, K)
        assert (p["algo"], p["direct_gather"], p["rows_per_block"]) == (B_.FWD_KLANE, 1, rb), (B, d_in, d_out, K, p)
    # 8 to 32 rows on inputs up to 1024 wide with moderate fan-in and 2048 stored rows or more: rows of x staged, few lanes per
    # stored row (measured ahead of the gathering form and of the batched kernel: 768 -> 3072 at B = 8 / 16 / 32 5.1 / 5.8 / 6.6 us
    # cold against 5.6 / 6.1 / 7.7)
    for (B, d_in, d_out, K, lanes, rb) in ((8, 768, 3072, 77, 16, 2), (16, 768, 3072, 77, 8, 2), (32, 768, 3072, 77, 8, 2),
                                           (32, 768, 3072, 39, 8, 2), (8, 1024, 4096, 102, 16, 2), (8, 768, 3072, 154, 16, 2)):
        p = plan(B, d_in, d_out, K, **(dict(algo=B_.FWD_KLANE) if B == 32 else {}))   # (at 32 rows the whole-input kernel is compared too)
        assert (p["algo"], p["direct_gather"], p["lanes_per_neuron"], p["rows_per_block"]) == (B_.FWD_KLANE, 0, lanes, rb), (B, d_in, K, p)
    # not beyond B x K of about 2500, nor on wide inputs, few stored rows, long rows from 16 batch rows on, or very short rows
    assert plan(8, 2048, 2048, 204)["direct_gather"] == 1
    assert plan(8, 1024, 1024, 102)["direct_gather"] == 1
    assert plan(16, 768, 3072, 154)["algo"] == B_.FWD_ROWLANE
    assert plan(32, 768, 3072, 154)["algo"] == B_.FWD_ROWLANE
    assert plan(8, 3072, 768, 308)["direct_gather"] == 1
    assert plan(16, 768, 3072, 8)["direct_gather"] == 1
    # very sparse layers at larger batches: many distinct lines per gather, the staged rows win
    p = plan(256, 768, 3072, 8, algo=B_.FWD_KLANE)                     # 8.9 / 7.3 us staged, 10.9 / 9.4 gathered, 9.4 / 8.4 batched
    assert (p["algo"], p["direct_gather"], p["rows_per_block"]) == (B_.FWD_KLANE, 0, 2)
    # 4096 -> 4096 at 99 % and 64 rows: the batched kernel (16.0 / 11.8 us) is ahead of staged (17.9 / 14.4) and gathered
    assert plan(64, 4096, 4096, 41)["algo"] == B_.FWD_ROWLANE
    # a row of x that does not fit the LDS can only be gathered
    p = plan(1, 49152, 48, 64)
    assert (p["algo"], p["direct_gather"]) == (B_.FWD_KLANE, 1)
    # large layers from a few rows on: the batched kernel (every further pass re-reads W_c / idx from beyond the L2)
    assert plan(8, 4096, 16384, 205)["algo"] == B_.FWD_ROWLANE            # 23.5 / 20.7 us vs 39.3 / 34.8 gathered


def test_rounds_are_counted_per_xcd():
    """3072 -> 768 at B = 320: four stored rows per wavefront would be 12 groups, two of them on four of the eight XCDs (40
    workgroups on 32 compute units); two or six rows per wavefront fit in one round per XCD or split evenly."""
    p = plan(320, 3072, 768, 308)
    assert p["algo"] == B_.FWD_ROWLANE and p["neurons_per_wave"] in (2, 6)
    # 768 -> 3072 at B = 384: 128-row tiles with three rows per wavefront are one round of 192 workgroups
    p = plan(384, 768, 3072, 77, algo=B_.FWD_ROWLANE)
    assert (p["rows_per_lane"], p["neurons_per_wave"], p["workgroups"]) == (2, 3, 192)
    p = plan(640, 768, 3072, 77, algo=B_.FWD_ROWLANE)
    assert (p["rows_per_lane"], p["neurons_per_wave"]) == (2, 4)


def test_long_rows_take_two_rows_per_lane_in_two_slices():
    """64-row tiles whose lanes hold two batch rows and work on two terms at once: one 8-byte LDS read per two rows and term.
    Measured against one row per lane: 768 -> 3072 K = 154 at B = 256 19.9 -> 17.1 us, 1024 -> 4096 K = 102 19.9 -> 16.5,
    2048 -> 2048 K = 205 at B = 384 35.0 -> 27.6, 4096 -> 1024 K = 410 at B = 1024 69.2 -> 52.4; at K = 77 (B = 256:
    13.6 -> 12.4 with two blocks of 32 terms preloaded per stored row and chunk instead of three); at a fan-in of 39 the fitted
    ranking takes the 32-row tile of two rows per lane with six stored rows per wavefront (12.6 / 10.7 -> 11.2 / 9.9 us cold /
    cached against the plain 64-row tile, which the estimate alone would keep)."""
    for (B, d_in, d_out, K) in ((256, 768, 3072, 154), (256, 1024, 4096, 102), (384, 2048, 2048, 205), (1024, 4096, 1024, 410),
                                (256, 768, 3072, 77)):
        p = plan(B, d_in, d_out, K, algo=B_.FWD_ROWLANE)
        assert (p["algo"], p["rows_per_lane"], p["term_slices"]) == (B_.FWD_ROWLANE, 2, 2), (B, d_in, d_out, K, p)
    for (B, d_in, d_out, K) in ((256, 768, 3072, 39),):
        p = plan(B, d_in, d_out, K, algo=B_.FWD_ROWLANE)
        assert (p["rows_per_lane"], p["term_slices"], p["neurons_per_wave"]) == (2, 4, 6), (B, d_in, d_out, K, p)
    # wide inputs, long rows: 32-row tiles the same way (four slices of 16 lanes); 4096 -> 1024 K = 410 at B = 512: 39.6 -> 31.4 us
    p = plan(512, 4096, 1024, 410)
    assert (p["rows_per_lane"], p["term_slices"]) == (2, 4)


def test_which_workgroups_share_an_xcd():
    """Each of the 8 XCDs has its own L2: either every XCD fetches all of x (and one group's W_c / idx), or its own batch tiles
    of x and all of W_c / idx; the batched kernel takes the order that fetches fewer bytes once an XCD has two tiles."""
    assert plan(256, 768, 3072, 77, algo=B_.FWD_ROWLANE)["xcd_order"] == 1          # x 0.8 MB < W_c + idx 1.9 MB; only four batch tiles
    assert plan(2048, 768, 3072, 77, algo=B_.FWD_ROWLANE)["xcd_order"] == 2         # x 6.3 MB; 65.9 -> 62.0 us
    assert plan(256, 3072, 768, 307, n_active=538)["xcd_order"] == 2   # 16 tiles of 16 rows; x 3.1 MB > 1.3 MB
    assert plan(128, 2048, 512, 205, algo=B_.FWD_ROWLANE)["xcd_order"] == 1   # one tile per XCD: 9.6 vs 10.4 us


def test_very_sparse_layers_stay_on_the_small_batch_kernel_at_larger_batches():
    assert plan(96, 3072, 768, 31)["algo"] == B_.FWD_KLANE            # 5.9 / 4.8 us (cold / cached) vs 11.9 / 10.7
    assert plan(96, 768, 3072, 8)["algo"] == B_.FWD_KLANE             # 6.0 / 5.0 vs 8.1 / 7.4
    assert plan(256, 768, 3072, 8)["algo"] in (B_.FWD_KLANE, B_.FWD_ROWLOOP)   # 8.8 / 8.1 us against 9.1 / 7.1
    assert plan(256, 768, 3072, 39)["algo"] == B_.FWD_ROWLOOP
    assert plan(4096, 3072, 768, 31)["algo"] == B_.FWD_ROWLANE      # above 2048 rows always the batched kernel


def test_mid_batches_follow_the_estimates():
    assert plan(8, 768, 3072, 77)["algo"] == B_.FWD_KLANE
    assert plan(16, 768, 3072, 77)["algo"] == B_.FWD_KLANE            # staged, 8 lanes per stored row: 6.2 / 5.0 us vs 7.4 / 5.3 chunked
    assert plan(32, 768, 3072, 77)["algo"] == B_.FWD_ROWLOOP          # 6.1 / 5.4 us against 7.5 / 6.4 staged
    assert plan(64, 768, 3072, 77)["algo"] == B_.FWD_ROWLOOP          # 7.0 / 6.6 us against 7.4 / 6.9 chunked
    assert plan(64, 768, 3072, 77, algo=B_.FWD_ROWLANE)["workgroups"] == 256
    assert plan(32, 2048, 512, 205)["algo"] == B_.FWD_KLANE         # few stored rows: the batched kernel cannot fill the GPU
    assert plan(96, 2048, 512, 205)["algo"] == B_.FWD_ROWLANE
    assert plan(16, 2560, 2560, 256)["algo"] == B_.FWD_ROWLANE        # wide input, many stored rows: 9.6 vs 13.7 us measured
    assert plan(16, 3072, 768, 615)["algo"] == B_.FWD_KLANE           # wide input, few stored rows: 8.1 vs 11.9 us


def test_fallbacks():
    # a row of x that does not fit the LDS of the small-batch kernel: gathered, or the batched kernel
    assert plan(2, 49152, 48, 64)["algo"] in (B_.FWD_KLANE, B_.FWD_ROWLANE)
    # d_in not a multiple of 16 and no seg table: the batched kernel needs the whole row in one LDS tile
    p = plan(64, 100, 40, 7, has_seg=False)
    assert p["algo"] in (B_.FWD_ROWLANE, B_.FWD_KLANE)
    # nothing stored: no forward kernel at all
    assert plan(4, 64, 8, 0)["algo"] == 0 and plan(0, 64, 8, 3)["workgroups"] == 0
    with pytest.raises(B_.SriglError):
        B_.srigl_fwd_plan_query(4, 8, 9, 3, 8)                      # more stored neurons than neurons


def test_forced_small_batch_kernel_at_batches_beyond_its_workgroup_limit():
    """The small-batch kernel gives a workgroup more stored rows until the launch has at most 2048 (staged) or 8192 (gathered)
    workgroups; a batch with more row blocks than that takes one workgroup per row block, every stored row in it."""
    for B, d_in, rb in ((2049, 2048, 1), (4096, 2048, 1), (65535, 2048, 1), (4100, 768, 2), (20000, 768, 2)):
        p = plan(B, d_in, 300, 40, algo=B_.FWD_KLANE, tuning=dict(direct_gather=2))
        assert p["rows_per_block"] == rb and p["workgroups"] == -(-B // rb), (B, d_in, p)
    p = plan(9000, 2048, 300, 40, algo=B_.FWD_KLANE, tuning=dict(direct_gather=1, rows_per_block=1))
    assert p["workgroups"] == 9000
    with pytest.raises(B_.SriglError):
        plan(65536, 2048, 300, 40, algo=B_.FWD_KLANE, tuning=dict(rows_per_block=1))   # the batch is the grid's second dimension


def test_fitted_ranking_moves_the_shape_only_when_it_is_well_ahead():
    """The shape of smallest estimate stays unless the ranking fitted to measured shapes has another one more than 5 % ahead:
    the headline layer keeps its shape (the ranking has a 32-row tile 4 % ahead, measured level), the changes below measured
    10-22 % faster; rows of fewer than 16 terms keep the estimate's shape."""
    p = plan(256, 768, 3072, 77, algo=B_.FWD_ROWLANE)
    assert (p["rows_per_lane"], p["term_slices"], p["neurons_per_wave"], p["chunk_cols"]) == (2, 2, 3, 384)
    p = plan(256, 3072, 768, 307, n_active=538)
    assert (p["rows_per_lane"], p["term_slices"], p["neurons_per_wave"], p["waves"]) == (1, 4, 3, 12)
    p = plan(2048, 4096, 16384, 205, n_active=13108, dtype_code=B_.BF16)
    assert (p["rows_per_lane"], p["term_slices"], p["neurons_per_wave"]) == (2, 1, 8)
    for (B, d_in, d_out, K, shape) in ((1024, 3072, 768, 154, (2, 4, 6)),      # 36.9 / 28.2 -> 28.8 / 22.7 us
                                       (512, 768, 3072, 39, (2, 2, 6)),        # 18.6 / 16.5 -> 16.5 / 14.6
                                       (128, 4096, 4096, 41, (1, 4, 8)),       # 22.7 / 16.6 -> 17.8 / 13.4
                                       (1024, 2048, 2048, 102, (2, 2, 8))):    # 45.1 / 38.6 -> 39.0 / 32.1
        p = plan(B, d_in, d_out, K, algo=B_.FWD_ROWLANE)
        assert (p["rows_per_lane"], p["term_slices"], p["neurons_per_wave"]) == shape, (B, d_in, d_out, K, p)
    legacy = plan(1024, 768, 3072, 8, algo=B_.FWD_ROWLANE)
    assert (legacy["rows_per_lane"], legacy["term_slices"], legacy["neurons_per_wave"]) == (2, 1, 6)


def test_every_plan_is_one_the_kernels_accept():
    """Seeded random sizes: whatever the estimates choose is a launch shape inside the kernels' documented limits, and asking
    for the plan of that algorithm with that shape forced gives the same plan back."""
    import random
    rng = random.Random(20230502)
    for _ in range(400):
        d_in = rng.choice([16, 48, 64, 100, 256, 768, 1000, 1024, 1536, 2048, 3072, 4096, 8192, 49152])
        d_out = rng.choice([1, 7, 64, 300, 768, 1024, 3072, 4096, 16384])
        n_active = max(1, int(d_out * rng.choice([1.0, 1.0, 0.9, 0.7, 0.25])))
        K = max(1, min(d_in, int(d_in * rng.choice([0.01, 0.05, 0.1, 0.2, 0.5, 1.0]))))
        B = rng.choice([1, 2, 3, 5, 8, 16, 31, 64, 100, 256, 777, 2048, 5000])
        dtype = rng.choice([B_.F32, B_.BF16])
        if B * d_in >= 2 ** 31 or n_active * K >= 2 ** 30:
            continue
        p = B_.srigl_fwd_plan_query(B, d_in, n_active, K, d_out, dtype_code=dtype, has_active=(n_active != d_out))
        assert p["algo"] in (B_.FWD_GENERIC, B_.FWD_KLANE, B_.FWD_ROWLANE, B_.FWD_ROWLOOP), (B, d_in, d_out, n_active, K, p)
        assert p["workgroups"] >= 1
        if p["algo"] == B_.FWD_ROWLANE:
            assert p["rows_per_lane"] in (1, 2) and p["term_slices"] in (1, 2, 4) and 1 <= p["waves"] <= 16
            assert p["neurons_per_wave"] in (1, 2, 3, 4, 6, 8) and p["chunk_cols"] % 64 == 0 and p["chunk_cols"] >= 64
            assert p["xcd_order"] in (1, 2)
            forced = dict(rows_per_lane=p["rows_per_lane"], term_slices=p["term_slices"], waves=p["waves"],
                          neurons_per_wave=p["neurons_per_wave"], chunk_cols=p["chunk_cols"], xcd_order=p["xcd_order"])
        elif p["algo"] == B_.FWD_ROWLOOP:
            assert p["rows_per_lane"] == 2 and p["term_slices"] in (2, 4) and p["waves"] == 16 and p["neurons_per_wave"] >= 1
            tile_rows = 128 // p["term_slices"]
            assert d_in % 16 == 0 and p["chunk_cols"] == d_in and p["xcd_order"] in (1, 2)
            # the tile of x, the all-zero column and the result tile fit the LDS
            assert ((d_in + 1) * (tile_rows + 4) + tile_rows * (p["neurons_per_wave"] * 16 + 1)) * 4 <= 160 * 1024
            forced = dict(term_slices=p["term_slices"], waves=p["waves"], neurons_per_wave=p["neurons_per_wave"], xcd_order=p["xcd_order"])
        elif p["algo"] == B_.FWD_KLANE:
            L = p["lanes_per_neuron"]
            assert 4 <= L <= 64 and L & (L - 1) == 0 and p["rows_per_block"] in (1, 2, 4) and p["direct_gather"] in (0, 1)
            if p["direct_gather"] == 0:
                assert p["rows_per_block"] * d_in * 4 <= 160 * 1024      # the staged rows fit the LDS
            forced = dict(lanes_per_neuron=L, rows_per_block=p["rows_per_block"], direct_gather=1 if p["direct_gather"] else 2)
        else:
            continue
        q = B_.srigl_fwd_plan_query(B, d_in, n_active, K, d_out, dtype_code=dtype, has_active=(n_active != d_out), algo=p["algo"],
                                    tuning=forced)
        assert q == p, (B, d_in, d_out, n_active, K, p, q)
