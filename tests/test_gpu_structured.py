"""GPU parity of the structured-only representation (Sec. 4.4 / Fig. 4 / App. H): dense rows of the stored
neurons, product on the matrix cores, against the oracle's plain loops."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from gpu_util import TOL_BF16, TOL_F32, dev, gate, host, oracle_condensed

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B_():
    from paper_2305_02299_amd import binding
    return binding


def run_case(B_, L, tol, tile=None, splits=None):
    W_c, idx, active = oracle_condensed(L)
    n, K = W_c.shape
    x = L.x_bf16 if L.dtype == "bf16" else L.x
    Wd_ref = oracle.densify(W_c, idx, L.d_in)
    Wd = torch.full((max(n, 1), L.d_in), 0x7fc1 if L.dtype == "bf16" else 0, dtype=torch.int16 if L.dtype == "bf16" else torch.float32,
                    device="cuda")
    if L.dtype != "bf16":
        Wd.fill_(float("nan"))
    B_.srigl_densify(dev(W_c), dev(idx), n, K, L.d_in, Wd)
    got_Wd = host(Wd)[:n]
    assert np.array_equal(got_Wd.view(np.uint16 if L.dtype == "bf16" else np.uint32),
                          Wd_ref.view(np.uint16 if L.dtype == "bf16" else np.uint32))
    y = torch.full((L.B, L.d_out), float("nan"), device="cuda")
    if splits is None:
        B_.srigl_structured_linear_fwd(dev(x), L.B, L.d_in, Wd, dev(active), n, dev(L.bias), L.d_out, y, tile=tile)
    else:   # d_in cut into parts (0: as many as the library would take); the partial sums start as NaN
        parts = splits or B_.srigl_structured_split_plan(L.B, L.d_in, n, L.d_out, B_.BF16 if L.dtype == "bf16" else B_.F32)[0]
        ws = torch.full((max(parts * L.B * n, 1),), float("nan"), device="cuda") if parts > 1 else None
        B_.srigl_structured_linear_fwd_split(dev(x), L.B, L.d_in, Wd, dev(active), n, dev(L.bias), L.d_out, y, ws, splits=splits, tile=tile)
    torch.cuda.synchronize()
    y_ref = oracle.structured_fwd(x, Wd_ref, active, L.bias, L.d_out)
    _, S = oracle.fwd(x, W_c, idx, active, L.bias, L.d_out, want_scale=True)
    return gate(host(y), y_ref, S, tol)


@pytest.mark.parametrize("name,B", [("c1", 1), ("c1", 16), ("c1", 256), ("c2", 1), ("c2", 64), ("c2", 256), ("c3", 256)])
def test_named_configs_f32(B_, name, B):
    L = si.config(name, B=B)
    worst = run_case(B_, L, TOL_F32)
    print("structured %s B=%d worst err/scale %.2e" % (name, B, worst))


@pytest.mark.parametrize("d_in,d_out,K,B,abl", [
    (64, 64, 8, 64, 0.0), (68, 33, 5, 7, 0.3), (132, 257, 13, 130, 0.2), (200, 129, 200, 65, 0.0),
    (36, 300, 1, 129, 0.5), (1024, 96, 100, 300, 0.1), (4, 5, 2, 3, 0.0), (260, 640, 26, 513, 0.25),
])
def test_ragged_shapes_f32(B_, d_in, d_out, K, B, abl):
    L = si.make_layer(d_in, d_out, K, B, ablate_frac=abl, seed=d_in * 7 + B)
    run_case(B_, L, TOL_F32)


@pytest.mark.parametrize("d_in,d_out,K,B,abl", [
    (64, 64, 8, 64, 0.0), (72, 33, 5, 7, 0.3), (136, 257, 13, 130, 0.2), (1024, 1024, 102, 512, 0.1), (8, 5, 2, 3, 0.0),
])
def test_shapes_bf16(B_, d_in, d_out, K, B, abl):
    L = si.make_layer(d_in, d_out, K, B, ablate_frac=abl, dtype="bf16", seed=d_in + B)
    run_case(B_, L, TOL_BF16)


TILE_NAMES = ["256x256", "256x256_h", "256x128_w4", "256x128", "128x128", "64x64"]


@pytest.mark.parametrize("tile", TILE_NAMES)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_every_tile_shape(B_, tile, dtype):
    """Each workgroup tile on shapes with ragged edges in all three dimensions, one and several slabs, and fewer
    slabs than LDS stages."""
    tol = TOL_BF16 if dtype == "bf16" else TOL_F32
    for (d_in, d_out, K, B, abl) in [(520, 700, 52, 300, 0.2), (40, 97, 4, 33, 0.0), (136, 513, 14, 257, 0.4)]:
        L = si.make_layer(d_in, d_out, K, B, ablate_frac=abl, dtype=dtype, seed=d_in + 3 * B)
        run_case(B_, L, tol, tile=B_.TILES[tile])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("splits", [2, 3, 7, 16])
def test_d_in_cut_into_parts(B_, dtype, splits):
    """Forced numbers of parts on the smallest and one larger tile: ragged edges in all three dimensions, parts of unequal
    numbers of stages, a last stage that is cut short by the row end, with and without ablated neurons."""
    tol = TOL_BF16 if dtype == "bf16" else TOL_F32
    for (d_in, d_out, K, B, abl) in [(1040, 300, 52, 130, 0.2), (2048, 97, 64, 33, 0.0), (1096, 513, 14, 70, 0.4)]:
        L = si.make_layer(d_in, d_out, K, B, ablate_frac=abl, dtype=dtype, seed=d_in + 3 * B + splits)
        run_case(B_, L, tol, tile=B_.TILES["64x64"], splits=splits)
        run_case(B_, L, tol, tile=B_.TILES["128x128"], splits=splits)


@pytest.mark.parametrize("name,B", [("c3", 256), ("c3", 64), ("c2", 16), ("c1", 1)])
def test_library_choice_of_parts(B_, name, B):
    """The plan's own number of parts on the named layers (the wide layer with few stored neurons is the case it exists for)."""
    L = si.config(name, B=B)
    W_c, _, _ = oracle_condensed(L)
    parts, need = B_.srigl_structured_split_plan(B, L.d_in, W_c.shape[0], L.d_out, B_.F32)
    assert (parts > 1) == (need > 0) and need == (parts * B * W_c.shape[0] * 4 if parts > 1 else 0)
    if name == "c3":
        assert parts > 1
    run_case(B_, L, TOL_F32, splits=0)


def test_parts_argument_errors(B_):
    from paper_2305_02299_amd.binding import SriglError
    L = si.make_layer(256, 64, 8, 16, seed=3)
    W_c, idx, active = oracle.condense(L.W, L.mask, L.K)
    n = len(active)
    Wd = dev(oracle.densify(W_c, idx, L.d_in))
    y = torch.empty((L.B, L.d_out), device="cuda")
    args = (dev(L.x), L.B, L.d_in, Wd, dev(active), n, dev(L.bias), L.d_out, y)
    ws = torch.empty((4 * L.B * n,), device="cuda")
    with pytest.raises(SriglError) as e:     # workspace of 4 parts offered for 8
        B_.srigl_structured_linear_fwd_split(*args, ws, splits=8, tile=B_.TILES["64x64"])
    assert e.value.status == B_.ERR_CAPACITY
    with pytest.raises(SriglError) as e:     # no workspace at all
        B_.srigl_structured_linear_fwd_split(*args, None, splits=2, tile=B_.TILES["64x64"])
    assert e.value.status == B_.ERR_CAPACITY
    with pytest.raises(SriglError) as e:     # 256 fp32 columns are 8 stages of 128 bytes: 16 parts would leave empty ones
        B_.srigl_structured_linear_fwd_split(*args, torch.empty((16 * L.B * n,), device="cuda"), splits=16, tile=B_.TILES["64x64"])
    assert e.value.status == B_.ERR_INVALID_ARG
    with pytest.raises(SriglError):
        B_.srigl_structured_linear_fwd_split(*args, ws, splits=17)
    B_.srigl_structured_linear_fwd_split(*args, ws, splits=4, tile=B_.TILES["64x64"])   # the same call with a workspace that fits


def test_integer_inputs_bit_exact(B_):
    """Small integers: every product and partial sum is exact in fp32, so any summation order gives the same bits."""
    L = si.make_layer(256, 200, 20, 96, ablate_frac=0.2, seed=5)
    rng = np.random.default_rng(9)
    L.W[...] = rng.integers(-8, 9, L.W.shape).astype(np.float32)
    L.x[...] = rng.integers(-8, 9, L.x.shape).astype(np.float32)
    L.bias[...] = rng.integers(-8, 9, L.bias.shape).astype(np.float32)
    W_c, idx, active = oracle.condense(L.W, L.mask, L.K)
    n = W_c.shape[0]
    Wd = torch.empty((n, L.d_in), device="cuda")
    B_.srigl_densify(dev(W_c), dev(idx), n, L.K, L.d_in, Wd)
    y = torch.empty((L.B, L.d_out), device="cuda")
    B_.srigl_structured_linear_fwd(dev(L.x), L.B, L.d_in, Wd, dev(active), n, dev(L.bias), L.d_out, y)
    y_ref = oracle.fwd(L.x, W_c, idx, active, L.bias, L.d_out)
    assert np.array_equal(host(y), y_ref)


def test_all_ablated_and_no_active_list(B_):
    L = si.make_layer(64, 40, 8, 9, ablate_frac=0.0, seed=3)
    y = torch.full((L.B, L.d_out), float("nan"), device="cuda")
    B_.srigl_structured_linear_fwd(dev(L.x), L.B, L.d_in, None, None, 0, dev(L.bias), L.d_out, y)
    assert np.array_equal(host(y), np.broadcast_to(L.bias, (L.B, L.d_out)))
    # every neuron stored, no active list, no bias
    W_c, idx, active = oracle.condense(L.W, L.mask, L.K)
    Wd_ref = oracle.densify(W_c, idx, L.d_in)
    y = torch.full((L.B, L.d_out), float("nan"), device="cuda")
    B_.srigl_structured_linear_fwd(dev(L.x), L.B, L.d_in, dev(Wd_ref), None, L.d_out, None, L.d_out, y)
    y_ref, S = oracle.fwd(L.x, W_c, idx, None, None, L.d_out, want_scale=True)
    gate(host(y), y_ref, S, TOL_F32)


def test_argument_errors(B_):
    from paper_2305_02299_amd.binding import SriglError
    L = si.make_layer(66, 40, 8, 9, seed=3)      # 66 fp32 columns: rows are not multiples of 16 bytes
    W_c, idx, active = oracle.condense(L.W, L.mask, L.K)
    Wd = dev(oracle.densify(W_c, idx, L.d_in))
    y = torch.empty((L.B, L.d_out), device="cuda")
    with pytest.raises(SriglError) as e:
        B_.srigl_structured_linear_fwd(dev(L.x), L.B, L.d_in, Wd, dev(active), len(active), dev(L.bias), L.d_out, y)
    assert e.value.status == B_.ERR_UNSUPPORTED
    with pytest.raises(SriglError):
        B_.srigl_structured_linear_fwd(dev(L.x), L.B, L.d_in, Wd, dev(active), L.d_out + 1, dev(L.bias), L.d_out, y)
    with pytest.raises(SriglError):
        B_.srigl_densify(dev(W_c), dev(idx), len(active), L.d_in + 1, L.d_in, Wd)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_layer_object_runs_either_representation(dtype):
    """The device-buffer holder: "structured" and "auto" give the oracle's result like "condensed" does."""
    from paper_2305_02299_amd import condense_layer
    L = si.make_layer(256, 384, 26, 192, ablate_frac=0.25, dtype=dtype, seed=11)
    Wsrc, xsrc = (L.W_bf16, L.x_bf16) if dtype == "bf16" else (L.W, L.x)
    layer = condense_layer(dev(Wsrc), dev(L.mask), L.K, dev(L.bias))
    W_c, idx, active = oracle_condensed(L)
    y_ref, S = oracle.fwd(xsrc, W_c, idx, active, L.bias, L.d_out, want_scale=True)
    tol = TOL_BF16 if dtype == "bf16" else TOL_F32
    for rep in ("condensed", "structured", "auto"):
        y = layer.forward(dev(xsrc), representation=rep)
        torch.cuda.synchronize()
        gate(host(y), y_ref, S, tol)


def test_large_layer_sampled_rows_in_the_timed_configuration(B_):
    """4096 -> 16384, bf16 storage, B = 2048, 20 % of the neurons ablated: the configuration `bench.py --structured` times,
    through the library's own tile choice.  The GPU runs the whole batch; the oracle recomputes a sample of batch rows
    (first, last, tile edges, random) from the condensed arrays; ablated columns must equal the bias bit for bit."""
    L = si.config("c5")
    W_c, idx, active = oracle_condensed(L)
    n = W_c.shape[0]
    Wd = torch.empty((n, L.d_in), dtype=torch.int16, device="cuda")
    B_.srigl_densify(dev(W_c), dev(idx), n, L.K, L.d_in, Wd)
    y = torch.full((L.B, L.d_out), float("nan"), device="cuda")
    B_.srigl_structured_linear_fwd(dev(L.x_bf16), L.B, L.d_in, Wd, dev(active), n, dev(L.bias), L.d_out, y)
    torch.cuda.synchronize()
    y = host(y)
    rows = np.unique(np.concatenate([[0, 1, 127, 128, 255, 256, 257, 1023, 1024, 2046, 2047],
                                     np.random.default_rng(6).integers(0, 2048, size=5)]))
    y_ref, S = oracle.fwd(L.x_bf16[rows], W_c, idx, active, L.bias, L.d_out, want_scale=True)
    gate(y[rows], y_ref, S, TOL_BF16)
    ablated = np.setdiff1d(np.arange(L.d_out), active)
    assert np.array_equal(y[:, ablated].view(np.uint32), np.tile(L.bias[ablated], (L.B, 1)).view(np.uint32))
    assert np.isfinite(y).all()
    # densify at full size: a sample of rows against the definition
    got = host(Wd)
    for s in (0, 1, n // 2, n - 1):
        ref = np.zeros(L.d_in, np.uint16)
        ref[idx[s]] = W_c[s]
        assert np.array_equal(got[s], ref)
