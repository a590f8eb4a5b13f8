"""GPU parity of the MLP-block pieces: activation in the forward epilogue, the width-reduction fold of the second layer,
and the folded pair end to end, against the oracle (Sec. 3.1 neuron ablation as width reduction; App. H's MLP block)."""
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


ALGOS = {"auto": 0, "generic": 1, "klane": 2, "rowlane": 3, "rowloop": 4}


@pytest.mark.parametrize("act", [1, 2])
@pytest.mark.parametrize("algo", list(ALGOS))
@pytest.mark.parametrize("B", [1, 5, 70])
def test_forward_with_activation(B_, act, algo, B):
    """Every written value passes through the activation, ablated columns included.  The gate allows the activation's
    slope (at most 1.13 for GELU) on top of the forward tolerance."""
    L = si.make_layer(192, 160, 19, B, ablate_frac=0.3, seed=7 + B)
    W_c, idx, active = oracle_condensed(L)
    from paper_2305_02299_amd import condense_layer
    layer = condense_layer(dev(L.W), dev(L.mask), L.K, dev(L.bias))
    y = torch.full((B, L.d_out), float("nan"), device="cuda")
    try:
        B_.srigl_condensed_linear_fwd(dev(L.x), B, L.d_in, layer.W_c, layer.idx, layer.active, layer.n_active, L.K, layer.bias,
                                      L.d_out, y, layer.seg, algo=ALGOS[algo], act=act)
    except B_.SriglError as e:
        if e.status == B_.ERR_UNSUPPORTED and algo in ("rowlane", "rowloop"):
            pytest.skip("launch shape not supported for this size")
        raise
    torch.cuda.synchronize()
    pre, S = oracle.fwd(L.x, W_c, idx, active, L.bias, L.d_out, want_scale=True)
    y_ref = oracle.activate(pre, act)
    gate(host(y), y_ref, 1.2 * S, TOL_F32)
    abl = np.setdiff1d(np.arange(L.d_out), active)
    # ablated neurons output act(bias): fp32 erf against the oracle's double erf
    assert np.allclose(host(y)[:, abl], oracle.activate(L.bias[abl], act)[None, :], rtol=2e-6, atol=1e-7)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("act", [0, 1, 2])
@pytest.mark.parametrize("shape", [(96, 40, 13, 0.4, 0.2), (3072, 768, 307, 0.3, 0.0), (256, 300, 200, 0.2, 0.5), (64, 33, 1, 0.9, 0.1)])
def test_fold_matches_oracle(B_, dtype, act, shape):
    d_hidden, d_out2, K2, abl1, abl2 = shape
    rng = np.random.default_rng(d_hidden + act)
    n1 = d_hidden - int(abl1 * d_hidden)
    if K2 > n1:
        pytest.skip("fan-in wider than the compact layer")
    active1 = np.sort(rng.choice(d_hidden, n1, replace=False)).astype(np.int32)
    bias1 = rng.normal(0, 1, d_hidden).astype(np.float32)
    L2 = si.make_layer(d_hidden, d_out2, K2, 1, ablate_frac=abl2, dtype=dtype, seed=d_out2)
    W_c2, idx2, active2 = oracle_condensed(L2)
    n2 = W_c2.shape[0]
    idx_ref, W_ref, bias_ref = oracle.fold_ablated_inputs(idx2, W_c2, L2.bias, active2, d_out2, active1, d_hidden, bias1, act)
    idx_o = torch.full((n2, K2), -9, dtype=torch.int32, device="cuda")
    W_o = torch.empty_like(dev(W_c2))
    bias_o = torch.full((d_out2,), float("nan"), device="cuda")
    B_.srigl_fold_ablated_inputs(dev(idx2), dev(W_c2), dev(L2.bias), dev(active2), n2, K2, d_out2, dev(active1), n1, d_hidden,
                                 dev(bias1), act, idx_o, W_o, bias_o)
    torch.cuda.synchronize()
    assert np.array_equal(host(idx_o), idx_ref)
    assert host(W_o).tobytes() == W_ref.tobytes()
    # the constants are summed in fp32 in another order: gate against the size of the summed terms
    wf = si.bf16_bits_to_f32(W_c2) if dtype == "bf16" else W_c2
    pos = np.full(d_hidden, -1)
    pos[active1] = np.arange(n1)
    moved = (pos[idx2] < 0)
    scale = np.zeros(d_out2)
    scale[active2] = (np.abs(wf * oracle.activate(bias1, act)[idx2]) * moved).sum(axis=1)
    scale += np.abs(L2.bias)
    assert np.all(np.abs(host(bias_o).astype(np.float64) - bias_ref) <= 1e-6 * np.maximum(scale, 1e-30))


def test_fold_without_ablation_is_the_identity(B_):
    L2 = si.make_layer(128, 64, 9, 1, ablate_frac=0.25, seed=3)
    W_c2, idx2, active2 = oracle_condensed(L2)
    n2 = W_c2.shape[0]
    idx_o, W_o, bias_o = torch.empty_like(dev(idx2)), torch.empty_like(dev(W_c2)), torch.empty(64, device="cuda")
    B_.srigl_fold_ablated_inputs(dev(idx2), dev(W_c2), dev(L2.bias), dev(active2), n2, 9, 64, None, 128, 128, None, 2, idx_o, W_o, bias_o)
    assert np.array_equal(host(idx_o), idx2) and host(W_o).tobytes() == W_c2.tobytes() and np.array_equal(host(bias_o), L2.bias)


@pytest.mark.parametrize("shape", [(3072, 0.3, True), (100, 0.0, True), (64, 0.5, False), (1, 0.0, True)])
def test_compact_hidden_layer_matches_oracle(B_, shape):
    d_hidden, abl, with_bias = shape
    rng = np.random.default_rng(d_hidden)
    n1 = d_hidden - int(abl * d_hidden)
    active1 = None if n1 == d_hidden else np.sort(rng.choice(d_hidden, n1, replace=False)).astype(np.int32)
    bias1 = rng.normal(0, 1, d_hidden).astype(np.float32) if with_bias else None
    width = (n1 + 15) // 16 * 16
    bias_ref, act_ref = oracle.compact_hidden_layer(bias1, active1, d_hidden, width)
    bias_o = torch.full((width,), 7.0, device="cuda")
    act_o = torch.full((n1,), -5, dtype=torch.int32, device="cuda")
    B_.srigl_compact_hidden_layer(dev(bias1), dev(active1), n1, d_hidden, width, bias_o, act_o)
    torch.cuda.synchronize()
    assert np.array_equal(host(bias_o).view(np.uint32), bias_ref.view(np.uint32)) and np.array_equal(host(act_o), act_ref)
    with pytest.raises(B_.SriglError):
        B_.srigl_compact_hidden_layer(dev(bias1), dev(active1), n1, d_hidden, n1 - 1, bias_o, act_o)


def test_fold_refuses_a_fan_in_wider_than_the_compact_layer(B_):
    idx2 = torch.arange(5, dtype=torch.int32, device="cuda")[None, :].contiguous()
    W = torch.ones((1, 5), device="cuda")
    with pytest.raises(B_.SriglError) as e:
        B_.srigl_fold_ablated_inputs(idx2, W, None, None, 1, 5, 1, torch.tensor([0, 2, 4], dtype=torch.int32, device="cuda"), 3, 5,
                                     None, 0, torch.empty_like(idx2), torch.empty_like(W), torch.empty(1, device="cuda"))
    assert e.value.status == B_.ERR_UNSUPPORTED


@pytest.mark.parametrize("act", [1, 2])
@pytest.mark.parametrize("B", [1, 16, 200])
def test_folded_pair_end_to_end(B_, act, B):
    """768 -> 3072 (30 % of the hidden neurons ablated) -> activation -> 768, the block of App. H at a small size ratio:
    the folded pair on the GPU against the unfolded pair in the oracle."""
    from paper_2305_02299_amd import condense_layer, fold_mlp
    L1 = si.make_layer(192, 768, 19, B, ablate_frac=0.3, seed=31)
    L2 = si.make_layer(768, 192, 77, B, ablate_frac=0.1, seed=32)
    l1 = condense_layer(dev(L1.W), dev(L1.mask), L1.K, dev(L1.bias))
    l2 = condense_layer(dev(L2.W), dev(L2.mask), L2.K, dev(L2.bias))
    mlp = fold_mlp(l1, l2, act)
    assert mlp.second.d_in == (l1.n_active + 15) // 16 * 16 and mlp.first.n_active == l1.n_active
    y = mlp.forward(dev(L1.x))
    torch.cuda.synchronize()
    Wc1, idx1, act1 = oracle.condense(L1.W, L1.mask, L1.K)
    Wc2, idx2, act2 = oracle.condense(L2.W, L2.mask, L2.K)
    h = oracle.activate(oracle.fwd(L1.x, Wc1, idx1, act1, L1.bias, L1.d_out), act)
    y_ref, S = oracle.fwd(h, Wc2, idx2, act2, L2.bias, L2.d_out, want_scale=True)
    # the hidden vector carries the first layer's rounding (~1e-6 of its scale) into the second layer's terms
    gate(host(y), y_ref, S, 2e-5)


@pytest.mark.parametrize("act", [0, 2])
@pytest.mark.parametrize("B", [1, 2, 3, 8])
@pytest.mark.parametrize("folded", [False, True])
def test_block_in_one_launch_matches_the_oracle_pair(B_, act, B, folded):
    """srigl_condensed_mlp_fwd (both layers and the activation in one launch, a barrier across the workgroups between them)
    against the two-layer oracle; with the width-reduction fold and on the layers as they are; twice in a row into the same
    buffers (the barrier's counter runs on from launch to launch)."""
    from paper_2305_02299_amd import condense_layer, fold_mlp
    L1 = si.make_layer(768, 3072, 77, B, ablate_frac=0.3, seed=41)
    L2 = si.make_layer(3072, 768, 308, B, ablate_frac=0.1, seed=42)
    l1 = condense_layer(dev(L1.W), dev(L1.mask), L1.K, dev(L1.bias))
    l2 = condense_layer(dev(L2.W), dev(L2.mask), L2.K, dev(L2.bias))
    Wc1, idx1, act1 = oracle.condense(L1.W, L1.mask, L1.K)
    Wc2, idx2, act2 = oracle.condense(L2.W, L2.mask, L2.K)
    h_ref = oracle.activate(oracle.fwd(L1.x, Wc1, idx1, act1, L1.bias, L1.d_out), act)
    y_ref, S = oracle.fwd(h_ref, Wc2, idx2, act2, L2.bias, L2.d_out, want_scale=True)
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    y = torch.full((B, L2.d_out), float("nan"), device="cuda")
    if folded:
        pair = fold_mlp(l1, l2, act)
        f, s = pair.first, pair.second
    else:
        f, s = l1, l2
    hidden = torch.full((B, f.d_out), float("nan"), device="cuda")
    for _ in range(2):
        B_.srigl_condensed_mlp_fwd(dev(L1.x), B, f.d_in, f.packed, f.active, f.n_active, f.K, f.bias, f.d_out, act, hidden, s.packed,
                                   s.active, s.n_active, s.K, s.bias, s.d_out, y, status=status)
        torch.cuda.synchronize()
        assert int(status.item()) == 0
        gate(host(y), y_ref, S, 2e-5)
        y.fill_(float("nan"))
    if not folded:      # the hidden vector at full width: stored neurons and act(bias) of the ablated ones
        gate(host(hidden), h_ref, np.maximum(np.abs(h_ref), 1.0), 1e-5)


def test_block_in_one_launch_gives_up_waiting_and_still_exits(B_):
    """A spin limit of one poll: workgroups stop waiting at the barrier, flag the call and finish (wrong numbers, no hang);
    the next call with the default limit is right again."""
    from paper_2305_02299_amd import condense_layer
    L1 = si.make_layer(256, 512, 26, 1, seed=51)
    L2 = si.make_layer(512, 128, 52, 1, seed=52)
    l1 = condense_layer(dev(L1.W), dev(L1.mask), L1.K, dev(L1.bias))
    l2 = condense_layer(dev(L2.W), dev(L2.mask), L2.K, dev(L2.bias))
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    hidden, y = torch.zeros((1, 512), device="cuda"), torch.zeros((1, 128), device="cuda")
    args = (dev(L1.x), 1, 256, l1.packed, l1.active, l1.n_active, l1.K, l1.bias, 512, 1, hidden, l2.packed, l2.active, l2.n_active, l2.K,
            l2.bias, 128, y)
    B_.srigl_condensed_mlp_fwd(*args, spin_limit=1, status=status)
    torch.cuda.synchronize()
    assert int(status.item()) in (0, 1)
    status.zero_()
    B_.srigl_condensed_mlp_fwd(*args, status=status)
    torch.cuda.synchronize()
    assert int(status.item()) == 0
    Wc1, idx1, act1 = oracle.condense(L1.W, L1.mask, L1.K)
    Wc2, idx2, act2 = oracle.condense(L2.W, L2.mask, L2.K)
    h = oracle.activate(oracle.fwd(L1.x, Wc1, idx1, act1, L1.bias, 512), 1)
    y_ref, S = oracle.fwd(h, Wc2, idx2, act2, L2.bias, 128, want_scale=True)
    gate(host(y), y_ref, S, 2e-5)
    with pytest.raises(B_.SriglError):
        B_.srigl_condensed_mlp_fwd(dev(np.zeros((9, 256), np.float32)), 9, 256, l1.packed, l1.active, l1.n_active, l1.K, l1.bias, 512, 1,
                                   torch.zeros((9, 512), device="cuda"), l2.packed, l2.active, l2.n_active, l2.K, l2.bias, 128,
                                   torch.zeros((9, 128), device="cuda"))
