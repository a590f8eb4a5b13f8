"""srigl_condense_static (the condense call with the library's built-in scratch, for callers that cannot allocate) against
srigl_condense on the same inputs, through the C ABI: every output bit for bit, on two calls in a row, the second one
smaller than the first (what the first call left in the scratch must not show)."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from gpu_util import dev, host

pytestmark = pytest.mark.gpu


def _both(B_, L):
    Wsrc = L.W_bf16 if L.dtype == "bf16" else L.W
    d_out, d_in, K = L.d_out, L.d_in, L.K
    W, m = dev(Wsrc), dev(L.mask)
    code = B_.BF16 if L.dtype == "bf16" else B_.F32
    outs = []
    for static in (False, True):
        W_c = torch.full((d_out, K), 0x5A5A if L.dtype == "bf16" else 1234.5, dtype=W.dtype, device="cuda")
        idx = torch.full((d_out, K), -99, dtype=torch.int32, device="cuda")
        active = torch.full((d_out,), -99, dtype=torch.int32, device="cuda")
        seg = torch.full((d_out, B_.srigl_seg_stride(d_in)), -1, dtype=torch.int16, device="cuda")
        packed = torch.full((B_.srigl_packed_bytes(d_out, K, d_in, code),), 0xA5, dtype=torch.uint8, device="cuda")
        rep = B_.new_report()
        if static:
            B_.srigl_condense_static(W, m, d_out, d_in, K, d_out, W_c, idx, active, seg, rep, packed=packed)
        else:
            B_.srigl_condense(W, m, d_out, d_in, K, d_out, W_c, idx, active, seg, B_.new_workspace(d_out), rep, packed=packed)
        torch.cuda.synchronize()
        outs.append((B_.read_report(rep), host(W_c), host(idx), host(active), host(seg), host(packed)))
    return outs


def test_static_scratch_condense_matches_condense_twice_in_a_row():
    from paper_2305_02299_amd import binding as B_
    first = si.make_layer(768, 3072, 77, 1, ablate_frac=0.3, seed=41)               # 3072 rows
    second = si.make_layer(1001, 130, 333, 1, ablate_frac=0.5, seed=42)            # fewer rows, ragged width
    third = si.make_layer(4096, 512, 205, 1, ablate_frac=0.2, dtype="bf16", seed=43)
    for L in (first, second, third):
        plain, static = _both(B_, L)
        assert static[0] == plain[0] and plain[0]["status"] == 0 and 0 < plain[0]["n_active"] < L.d_out
        for a, b in zip(plain[1:], static[1:]):
            assert a.dtype == b.dtype and np.array_equal(a.view(np.uint8), b.view(np.uint8))
    # a bad row is reported the same way, and sizes beyond the built-in scratch are refused before anything is launched
    bad = second.mask.copy()
    r = int(second.true_active[2])
    bad[r, int(np.flatnonzero(bad[r] == 0)[0])] = 1
    second.mask = bad
    plain, static = _both(B_, second)
    assert static[0] == plain[0] and plain[0]["status"] == B_.ERR_FANIN and plain[0]["first_bad_row"] == r
    with pytest.raises(B_.SriglError) as e:
        B_.srigl_condense_static(dev(first.W), dev(first.mask), 65537, 768, 77, 1, None, None, None, None, B_.new_report())
    assert e.value.status == B_.ERR_CAPACITY
