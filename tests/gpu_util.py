"""Shared helpers of the GPU parity tests: host<->device moves, the oracle side, the error gate."""
import numpy as np
import torch

import oracle
import synth_inputs as si

TOL_F32 = 1e-5    # max error relative to the size of the summed terms, fp32 storage
TOL_BF16 = 1e-2   # bf16 storage, fp32 accumulate


def dev(a):
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(a).cuda()


def host(t):
    a = t.cpu().numpy()
    return a.view(np.uint16) if a.dtype == np.int16 else a


def gate(y_gpu, y_ref, S, tol):
    """|y_gpu - y_ref| <= tol * max(|y_ref|, S), S = |bias| + sum_k |w x| from the oracle (fp64).
    Returns the worst ratio err / (tol * bound) so that a test can also print it."""
    y_gpu = y_gpu.astype(np.float64)
    y_ref = y_ref.astype(np.float64)
    assert y_gpu.shape == y_ref.shape
    assert np.isfinite(y_gpu).all()
    bound = np.maximum(np.abs(y_ref), S)
    err = np.abs(y_gpu - y_ref)
    ok = err <= tol * bound
    worst = float(np.max(err / np.maximum(bound, 1e-300))) if err.size else 0.0
    assert ok.all(), "max err/scale %.3e > tol %.1e at %s" % (worst, tol, np.argwhere(~ok)[:4].tolist())
    return worst


def oracle_condensed(L: si.Layer):
    """Oracle-side condensed form of a synthetic layer (W_c in the layer's storage type)."""
    Wsrc = L.W_bf16 if L.dtype == "bf16" else L.W
    return oracle.condense(Wsrc, L.mask, L.K)


def oracle_seg(idx, d_in, seg_cols=64):
    """seg[s][c] = number of entries of row s below seg_cols*c (definition of the table)."""
    n, K = idx.shape
    stride = (d_in + seg_cols - 1) // seg_cols + 1
    bounds = np.arange(stride) * seg_cols
    out = np.empty((n, stride), dtype=np.uint16)
    for s in range(n):
        out[s] = np.searchsorted(idx[s], bounds, side="left")
    return out
