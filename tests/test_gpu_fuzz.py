"""Seeded random shapes through every forward algorithm and through condense, against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from gpu_util import TOL_BF16, TOL_F32, dev, gate, host, oracle_condensed, oracle_seg
from paper_2305_02299_amd import binding as B_
from paper_2305_02299_amd import condense_layer

pytestmark = pytest.mark.gpu


def _cases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        d_in = int(rng.choice([16 * int(rng.integers(1, 80)), int(rng.integers(1, 1300))]))
        d_out = int(rng.integers(1, 400))
        K = int(rng.integers(1, min(d_in, 400) + 1))
        B = int(rng.choice([1, 2, 3, 5, 8, 15, 16, 17, 31, 33, 64, 65, 100, 129, 200]))
        abl = float(rng.choice([0.0, 0.0, 0.1, 0.5, 0.9]))
        dtype = "bf16" if rng.random() < 0.3 else "f32"
        out.append((d_in, d_out, K, B, abl, dtype, 1000 + i))
    return out


@pytest.mark.parametrize("d_in,d_out,K,B,abl,dtype,seed", _cases(40, 2024))
def test_random_layer_every_algorithm(d_in, d_out, K, B, abl, dtype, seed):
    L = si.make_layer(d_in, d_out, K, B, ablate_frac=abl, dtype=dtype, seed=seed)
    Wsrc, xsrc = (L.W_bf16, L.x_bf16) if dtype == "bf16" else (L.W, L.x)
    W_c, idx, active = oracle.condense(Wsrc, L.mask, K)
    # condense on the GPU: bit-exact, then forward from the GPU's own arrays
    layer = condense_layer(dev(Wsrc), dev(L.mask), K, dev(L.bias))
    n = len(active)
    assert layer.n_active == n
    assert np.array_equal(host(layer.idx), idx) and np.array_equal(host(layer.W_c), W_c)
    if n < d_out:
        assert np.array_equal(host(layer.active), active)
    if n:
        assert np.array_equal(host(layer.seg), oracle_seg(idx, d_in))
    y_ref, S = oracle.fwd(xsrc, W_c, idx, active, L.bias, d_out, want_scale=True)
    ablated = np.setdiff1d(np.arange(d_out), active)
    ran = 0
    for algo in (None, B_.FWD_GENERIC, B_.FWD_KLANE, B_.FWD_ROWLANE, B_.FWD_ROWLOOP):
        y = torch.full((B, d_out), 3.0e38, dtype=torch.float32, device="cuda")
        try:
            B_.srigl_condensed_linear_fwd(dev(xsrc), B, d_in, layer.W_c, layer.idx, layer.active, n, K, layer.bias, d_out, y,
                                          layer.seg, algo=algo)
        except B_.SriglError as e:
            assert e.status == B_.ERR_UNSUPPORTED and algo is not None
            continue
        yh = host(y)
        gate(yh, y_ref, S, TOL_BF16 if dtype == "bf16" else TOL_F32)
        if len(ablated):
            assert np.array_equal(yh[:, ablated].view(np.uint32), np.tile(L.bias[ablated], (B, 1)).view(np.uint32))
        ran += 1
    assert ran >= 3
    # the batched kernel in every tile shape and either XCD order (whichever the sizes allow)
    shapes = 0
    for rows_per_lane, term_slices in ((1, 1), (1, 2), (1, 4), (2, 1), (2, 2), (2, 4)):
        for xcd_order in (1, 2):
            y = torch.full((B, d_out), 3.0e38, dtype=torch.float32, device="cuda")
            try:
                B_.srigl_condensed_linear_fwd(dev(xsrc), B, d_in, layer.W_c, layer.idx, layer.active, n, K, layer.bias, d_out, y,
                                              layer.seg, algo=B_.FWD_ROWLANE,
                                              tuning=dict(rows_per_lane=rows_per_lane, term_slices=term_slices, xcd_order=xcd_order))
            except B_.SriglError as e:
                assert e.status == B_.ERR_UNSUPPORTED
                continue
            gate(host(y), y_ref, S, TOL_BF16 if dtype == "bf16" else TOL_F32)
            shapes += 1
        # the same tile with a workgroup's stored rows dealt out among its wavefronts (always; where their medians lie apart)
        for spread_rows in (2, 3):
            y = torch.full((B, d_out), 3.0e38, dtype=torch.float32, device="cuda")
            try:
                B_.srigl_condensed_linear_fwd(dev(xsrc), B, d_in, layer.W_c, layer.idx, layer.active, n, K, layer.bias, d_out, y,
                                              layer.seg, algo=B_.FWD_ROWLANE,
                                              tuning=dict(rows_per_lane=rows_per_lane, term_slices=term_slices, neurons_per_wave=2 + seed % 2,
                                                          waves=(4, 7, 16)[seed % 3], spread_rows=spread_rows))
            except B_.SriglError as e:
                assert e.status == B_.ERR_UNSUPPORTED
                continue
            yh = host(y)
            gate(yh, y_ref, S, TOL_BF16 if dtype == "bf16" else TOL_F32)
            if len(ablated):
                assert np.array_equal(yh[:, ablated].view(np.uint32), np.tile(L.bias[ablated], (B, 1)).view(np.uint32))
    assert shapes >= 2 or d_in % 16 != 0


@pytest.mark.parametrize("seed", range(24))
def test_structured_random_shapes(seed):
    """Seeded random shapes through the structured-only path: densify bit-exact, forward within tolerance, every tile choice
    the library makes on its own plus one forced tile per case."""
    import oracle
    from paper_2305_02299_amd import binding as B_
    from gpu_util import TOL_BF16, TOL_F32, dev, gate, host, oracle_condensed
    rng = np.random.default_rng(9000 + seed)
    dtype = "bf16" if seed % 2 else "f32"
    unit = 8 if dtype == "bf16" else 4
    d_in = int(rng.integers(1, 200)) * unit
    d_out = int(rng.integers(1, 900))
    K = int(rng.integers(1, min(d_in, 64) + 1))
    B = int(rng.choice([1, 3, 17, 64, 100, 257, 600]))
    abl = float(rng.choice([0.0, 0.0, 0.3, 0.8]))
    L = si.make_layer(d_in, d_out, K, B, ablate_frac=abl, dtype=dtype, seed=seed)
    W_c, idx, active = oracle_condensed(L)
    n = W_c.shape[0]
    x = L.x_bf16 if dtype == "bf16" else L.x
    Wd_ref = oracle.densify(W_c, idx, d_in)
    Wd = torch.empty((max(n, 1), d_in), dtype=torch.int16 if dtype == "bf16" else torch.float32, device="cuda")
    B_.srigl_densify(dev(W_c), dev(idx), n, K, d_in, Wd)
    assert host(Wd)[:n].tobytes() == Wd_ref.tobytes()
    y_ref, S = oracle.fwd(x, W_c, idx, active, L.bias, d_out, want_scale=True)
    for tile in (None, int(rng.integers(1, 7))):
        y = torch.full((B, d_out), float("nan"), device="cuda")
        B_.srigl_structured_linear_fwd(dev(x), B, d_in, Wd, dev(active), n, dev(L.bias), d_out, y, tile=tile)
        torch.cuda.synchronize()
        gate(host(y), y_ref, S, TOL_BF16 if dtype == "bf16" else TOL_F32)
    # the same product with d_in cut into parts: the library's own choice, and a forced number that the rows allow
    stages = (d_in * (2 if dtype == "bf16" else 4) + 127) // 128
    for splits in (0, int(rng.integers(1, min(stages, 16) + 1))):
        parts = splits or B_.srigl_structured_split_plan(B, d_in, n, d_out, B_.BF16 if dtype == "bf16" else B_.F32)[0]
        ws = torch.full((max(parts * B * n, 1),), float("nan"), device="cuda") if parts > 1 else None
        y = torch.full((B, d_out), float("nan"), device="cuda")
        B_.srigl_structured_linear_fwd_split(dev(x), B, d_in, Wd, dev(active), n, dev(L.bias), d_out, y, ws, splits=splits,
                                             tile=B_.TILES["64x64"] if splits else None)
        torch.cuda.synchronize()
        gate(host(y), y_ref, S, TOL_BF16 if dtype == "bf16" else TOL_F32)
