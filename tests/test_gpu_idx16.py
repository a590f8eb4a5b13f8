"""GPU parity of the 16-bit index storage (App. E: one column index per kept weight): the narrowing copy is bit-exact,
the forward pass with 16-bit indices matches the oracle on the layer's own (32-bit) indices and is bit-identical to the
32-bit call of the same kernel."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from gpu_util import TOL_BF16, TOL_F32, dev, gate, host, oracle_condensed

pytestmark = pytest.mark.gpu

ALGOS = {"auto": 0, "generic": 1, "klane": 2, "rowlane": 3, "rowloop": 4}


@pytest.fixture(scope="module")
def B_():
    from paper_2305_02299_amd import binding
    return binding


@pytest.mark.parametrize("n", [0, 1, 7, 8, 9, 4099, 1000003])
@pytest.mark.parametrize("shift", [0, 1, 3])
def test_narrow_is_a_bit_exact_copy(B_, n, shift):
    """Aligned and unaligned starts, lengths around the 8-entry vector width, both ends of the 16-bit range."""
    d_in = 65536
    rng = np.random.default_rng(n + shift)
    idx = rng.integers(0, d_in, n + shift, dtype=np.int32)
    if n >= 2:
        idx[shift], idx[-1] = 65535, 0
    src = dev(idx)[shift:]
    dst = torch.full((n + shift + 8,), -1, dtype=torch.int16, device="cuda")
    B_.srigl_narrow_idx(src, d_in, dst[shift:shift + n])
    torch.cuda.synchronize()
    got = host(dst)
    assert np.array_equal(got[shift:shift + n], oracle.narrow_idx(idx[shift:], d_in))
    assert (got[:shift] == 0xffff).all() and (got[shift + n:] == 0xffff).all()   # nothing written outside


def test_narrow_limits(B_):
    idx = dev(np.array([5, -3, 70000, 99], dtype=np.int32))
    out = torch.empty(4, dtype=torch.int16, device="cuda")
    with pytest.raises(B_.SriglError) as e:
        B_.srigl_narrow_idx(idx, 65537, out)
    assert e.value.status == B_.ERR_UNSUPPORTED
    B_.srigl_narrow_idx(idx, 100, out)   # entries that name no column are clamped into the layer
    torch.cuda.synchronize()
    assert host(out).tolist() == [5, 0, 99, 99]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("algo", list(ALGOS))
@pytest.mark.parametrize("shape", [(768, 320, 77, 1, 0.0), (768, 320, 77, 37, 0.2), (3072, 192, 307, 5, 0.3), (200, 70, 9, 130, 0.1),
                                   (4096, 512, 205, 300, 0.2)])
def test_forward_with_narrow_indices(B_, dtype, algo, shape):
    d_in, d_out, K, B, abl = shape
    L = si.make_layer(d_in, d_out, K, B, ablate_frac=abl, dtype=dtype, seed=d_in + B)
    W_c, idx, active = oracle_condensed(L)
    from paper_2305_02299_amd import condense_layer
    layer = condense_layer(dev(L.W_bf16 if dtype == "bf16" else L.W), dev(L.mask), L.K, dev(L.bias))
    nar = layer.narrow()
    torch.cuda.synchronize()
    assert np.array_equal(host(nar.idx), oracle.narrow_idx(idx, d_in))
    x = dev(L.x_bf16 if dtype == "bf16" else L.x)
    y16 = torch.full((B, d_out), float("nan"), device="cuda")
    y32 = torch.full((B, d_out), float("nan"), device="cuda")
    try:
        import dataclasses
        nar.forward(x, y16, algo=ALGOS[algo])
        dataclasses.replace(layer, packed=None).forward(x, y32, algo=ALGOS[algo])   # the 32-bit arrays, not their streaming copy
    except B_.SriglError as e:
        if e.status == B_.ERR_UNSUPPORTED and algo in ("rowlane", "klane", "rowloop"):
            pytest.skip("launch shape not supported for this size")
        raise
    torch.cuda.synchronize()
    y_ref, S = oracle.fwd(L.x_bf16 if dtype == "bf16" else L.x, W_c, idx, active, L.bias, d_out, want_scale=True)
    gate(host(y16), y_ref, S, TOL_BF16 if dtype == "bf16" else TOL_F32)
    assert np.array_equal(host(y16), host(y32))   # same kernel, same order of additions


@pytest.mark.parametrize("B", [2, 70])
def test_widest_layer_that_fits_16_bits(B_, B):
    """d_in = 65536: column numbers use all 16 bits (a signed reading of the word would go wrong from 32768 on)."""
    d_in, d_out, K = 65536, 24, 40
    rng = np.random.default_rng(B)
    idx = np.stack([np.concatenate([np.sort(rng.choice(d_in - 2, K - 2, replace=False)), [65534, 65535]]) for _ in range(d_out)]).astype(np.int32)
    W_c = rng.normal(0, 0.2, (d_out, K)).astype(np.float32)
    x = rng.normal(0, 1, (B, d_in)).astype(np.float32)
    bias = rng.normal(0, 0.1, d_out).astype(np.float32)
    idx16 = torch.empty((d_out, K), dtype=torch.int16, device="cuda")
    B_.srigl_narrow_idx(dev(idx), d_in, idx16)
    seg = torch.empty((d_out, B_.srigl_seg_stride(d_in)), dtype=torch.int16, device="cuda")
    ws, rep = B_.new_workspace(d_out), B_.new_report()
    B_.srigl_check_fanin(None, dev(idx), d_out, d_in, K, seg, ws, rep)
    y = torch.full((B, d_out), float("nan"), device="cuda")
    B_.srigl_condensed_linear_fwd(dev(x), B, d_in, dev(W_c), idx16, None, d_out, K, dev(bias), d_out, y, seg)
    torch.cuda.synchronize()
    y_ref, S = oracle.fwd(x, W_c, idx, None, bias, d_out, want_scale=True)
    gate(host(y), y_ref, S, TOL_F32)


def test_wider_layers_are_refused(B_):
    d_in = 65552
    z = torch.zeros((2, d_in), device="cuda")
    with pytest.raises(B_.SriglError) as e:
        B_.srigl_condensed_linear_fwd(z, 2, d_in, torch.zeros((4, 3), device="cuda"), torch.zeros((4, 3), dtype=torch.int16, device="cuda"),
                                      None, 4, 3, None, 4, torch.empty((2, 4), device="cuda"), None)
    assert e.value.status == B_.ERR_UNSUPPORTED
