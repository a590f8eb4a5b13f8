"""GPU parity of the compressed-sparse-row forward (the unstructured comparison of Sec. 4.4 / Fig. 4) against the oracle,
on unstructured masks (rows of different length, empty rows) and on a constant fan-in mask, where it must also agree with
the condensed forward of the same weights."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from gpu_util import TOL_F32, dev, gate, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B_():
    from paper_2305_02299_amd import binding
    return binding


def csr_of(W, mask):
    rows, cols = np.nonzero(mask)                      # row-major order: ascending rows, ascending columns within a row
    ptr = np.zeros(mask.shape[0] + 1, np.int32)
    np.cumsum(np.bincount(rows, minlength=mask.shape[0]), out=ptr[1:])
    return W[rows, cols].astype(np.float32), cols.astype(np.int32), ptr


@pytest.mark.parametrize("act", [0, 2])
@pytest.mark.parametrize("shape", [(37, 23, 1, 0.2), (768, 300, 1, 0.1), (768, 300, 7, 0.1), (3072, 200, 3, 0.1), (3072, 200, 33, 0.02),
                                   (200, 1000, 70, 0.5), (64, 5, 2, 1.0), (512, 2048, 400, 0.02), (49152, 40, 3, 0.002)])
def test_unstructured_masks(B_, shape, act):
    """Small cases gather their activations from global memory; 512 -> 2048 at 2 % and 400 rows stages rows of x in LDS; the
    49152-wide input does not fit the LDS and can only be gathered."""
    d_in, d_out, B, density = shape
    rng = np.random.default_rng(d_in + d_out + B)
    W = rng.normal(0, 1 / np.sqrt(max(density * d_in, 1)), (d_out, d_in)).astype(np.float32)
    mask = (rng.random((d_out, d_in)) < density).astype(np.uint8)
    mask[d_out // 2] = 0                                # a row without entries outputs its bias
    if d_out > 3:
        mask[d_out - 1] = 0
    x = rng.normal(size=(B, d_in)).astype(np.float32)
    bias = rng.normal(0, 0.1, d_out).astype(np.float32)
    vals, cols, ptr = csr_of(W, mask)
    y = torch.full((B, d_out), float("nan"), device="cuda")
    B_.srigl_csr_linear_fwd(dev(x), B, d_in, dev(vals) if vals.size else torch.empty(0, device="cuda"),
                            dev(cols) if cols.size else torch.empty(0, dtype=torch.int32, device="cuda"), dev(ptr), dev(bias), d_out, y,
                            act=act)
    torch.cuda.synchronize()
    pre, S = oracle.csr_fwd(x, vals, cols, ptr, bias, want_scale=True)
    gate(host(y), oracle.activate(pre, act), 1.2 * S, TOL_F32)


def test_batch_of_more_row_blocks_than_the_workgroup_limit(B_):
    """2100 rows of a 2048-wide input are staged one row per workgroup: more row blocks than the 2048 workgroups the launch
    is held to, so every workgroup walks all rows of the matrix."""
    d_in, d_out, B = 2048, 24, 2100
    rng = np.random.default_rng(9)
    W = rng.normal(0, 0.1, (d_out, d_in)).astype(np.float32)
    mask = (rng.random((d_out, d_in)) < 0.02).astype(np.uint8)
    x = rng.normal(size=(B, d_in)).astype(np.float32)
    bias = rng.normal(0, 0.1, d_out).astype(np.float32)
    vals, cols, ptr = csr_of(W, mask)
    y = torch.full((B, d_out), float("nan"), device="cuda")
    B_.srigl_csr_linear_fwd(dev(x), B, d_in, dev(vals), dev(cols), dev(ptr), dev(bias), d_out, y)
    torch.cuda.synchronize()
    ref, S = oracle.csr_fwd(x, vals, cols, ptr, bias, want_scale=True)
    gate(host(y), ref, 1.2 * S, TOL_F32)


@pytest.mark.parametrize("B", [1, 16, 256])
def test_constant_fan_in_mask_agrees_with_the_condensed_forward(B_, B):
    L = si.make_layer(768, 512, 77, B, ablate_frac=0.1, seed=3)
    vals, cols, ptr = csr_of(L.W, L.mask)
    y = torch.full((B, L.d_out), float("nan"), device="cuda")
    B_.srigl_csr_linear_fwd(dev(L.x), B, L.d_in, dev(vals), dev(cols), dev(ptr), dev(L.bias), L.d_out, y)
    torch.cuda.synchronize()
    W_c, idx, active = oracle.condense(L.W, L.mask, L.K)
    y_ref, S = oracle.fwd(L.x, W_c, idx, active, L.bias, L.d_out, want_scale=True)
    gate(host(y), y_ref, S, TOL_F32)


def test_argument_errors(B_):
    z = torch.zeros((2, 8), device="cuda")
    ptr = torch.zeros(5, dtype=torch.int32, device="cuda")
    e = torch.empty(0, device="cuda")
    ei = torch.empty(0, dtype=torch.int32, device="cuda")
    y = torch.full((2, 4), float("nan"), device="cuda")
    B_.srigl_csr_linear_fwd(z, 2, 8, e, ei, ptr, None, 4, y)       # no entries at all: every output is zero
    torch.cuda.synchronize()
    assert (host(y) == 0).all()
    with pytest.raises(B_.SriglError) as err:
        B_.srigl_csr_linear_fwd(z.to(torch.bfloat16), 2, 8, e.to(torch.bfloat16), ei, ptr, None, 4, y)
    assert err.value.status == B_.ERR_UNSUPPORTED
