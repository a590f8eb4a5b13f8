"""GPU parity, integer side: srigl_check_fanin and srigl_condense against the CPU oracle (bit-exact)."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from gpu_util import dev, host, oracle_seg

pytestmark = pytest.mark.gpu

from paper_2305_02299_amd import binding as B_


def _gpu_check_mask(mask, K_expected=-1):
    n_rows, d_in = mask.shape
    m = dev(mask)
    ws, rep = B_.new_workspace(n_rows), B_.new_report()
    B_.srigl_check_fanin(m, None, n_rows, d_in, K_expected, None, ws, rep)
    return B_.read_report(rep)


def _gpu_condense(L, cap_rows=None, want_seg=True, mask=None):
    Wsrc = L.W_bf16 if L.dtype == "bf16" else L.W
    mask = L.mask if mask is None else mask
    d_out, d_in, K = L.d_out, L.d_in, L.K
    cap = d_out if cap_rows is None else cap_rows
    W, m = dev(Wsrc), dev(mask)
    W_c = torch.full((cap, K), 0x5A5A if L.dtype == "bf16" else 1234.5, dtype=W.dtype, device="cuda")
    idx = torch.full((cap, K), -99, dtype=torch.int32, device="cuda")
    active = torch.full((cap,), -99, dtype=torch.int32, device="cuda")
    ss = B_.srigl_seg_stride(d_in)
    seg = torch.full((cap, ss), -1, dtype=torch.int16, device="cuda") if want_seg else None
    ws, rep = B_.new_workspace(d_out), B_.new_report()
    B_.srigl_condense(W, m, d_out, d_in, K, cap, W_c, idx, active, seg, ws, rep)
    torch.cuda.synchronize()
    return B_.read_report(rep), host(W_c), host(idx), host(active), (host(seg) if want_seg else None)


SHAPES = [
    # d_in, d_out, K, ablate, dtype
    (768, 3072, 77, 0.0, "f32"),      # the 90 % sparse up-projection
    (3072, 768, 307, 0.30, "f32"),    # down-projection with 30 % of the neurons ablated
    (16, 8, 3, 0.25, "f32"),
    (50, 7, 1, 0.0, "f32"),           # d_in not a multiple of 4: unaligned mask rows
    (77, 33, 20, 0.1, "f32"),
    (1001, 130, 333, 0.5, "f32"),     # ragged tail in the last 256-column pass
    (257, 5, 257, 0.0, "f32"),        # K == d_in
    (4096, 512, 205, 0.2, "bf16"),
    (130, 9, 7, 0.0, "bf16"),
]


@pytest.mark.parametrize("d_in,d_out,K,abl,dtype", SHAPES)
def test_condense_bit_exact(d_in, d_out, K, abl, dtype):
    L = si.make_layer(d_in, d_out, K, 1, ablate_frac=abl, dtype=dtype, seed=100 + d_in)
    W_c_o, idx_o, act_o = oracle.condense(L.W_bf16 if dtype == "bf16" else L.W, L.mask, K)
    rep, W_c, idx, active, seg = _gpu_condense(L)
    n = len(act_o)
    assert rep == {"K": K, "n_active": n, "n_bad_rows": 0, "first_bad_row": -1, "status": 0}
    assert np.array_equal(idx[:n], idx_o)
    assert np.array_equal(active[:n], act_o)
    bits = np.uint16 if dtype == "bf16" else np.uint32
    assert np.array_equal(W_c[:n].view(bits), W_c_o.view(bits))
    assert np.array_equal(seg[:n], oracle_seg(idx_o, d_in))
    # rows past n_active are left untouched
    assert (idx[n:] == -99).all() and (active[n:] == -99).all() and (seg[n:].view(np.int16) == -1).all()
    # the mask check agrees with the oracle's
    assert _gpu_check_mask(L.mask) == oracle.check_fanin_mask(L.mask)


@pytest.mark.parametrize("d_in,d_out,K,abl,dtype", SHAPES + [(70000, 6, 9, 0.0, "bf16")])
def test_packed_copy_bit_exact(d_in, d_out, K, abl, dtype):
    """The streaming copy written by srigl_condense, and by srigl_pack_terms from the canonical arrays, against the oracle's
    bytes; rows past n_active stay untouched."""
    L = si.make_layer(d_in, d_out, K, 1, ablate_frac=abl, dtype=dtype, seed=100 + d_in)
    Wsrc = L.W_bf16 if dtype == "bf16" else L.W
    W_c_o, idx_o, act_o = oracle.condense(Wsrc, L.mask, K)
    n = len(act_o)
    ref = oracle.pack_terms(W_c_o, idx_o, d_in)
    code = B_.BF16 if dtype == "bf16" else B_.F32
    nbytes = B_.srigl_packed_bytes(d_out, K, d_in, code)
    assert nbytes == d_out * ref.shape[1] and B_.srigl_packed_bytes(n, K, d_in, code) == ref.size
    W, m = dev(Wsrc), dev(L.mask)
    W_c = torch.empty((d_out, K), dtype=W.dtype, device="cuda")
    idx = torch.empty((d_out, K), dtype=torch.int32, device="cuda")
    active = torch.empty((d_out,), dtype=torch.int32, device="cuda")
    packed = torch.full((nbytes,), 0xA5, dtype=torch.uint8, device="cuda")
    ws, rep = B_.new_workspace(d_out), B_.new_report()
    B_.srigl_condense(W, m, d_out, d_in, K, d_out, W_c, idx, active, None, ws, rep, packed=packed)
    torch.cuda.synchronize()
    assert B_.read_report(rep)["status"] == 0
    got = host(packed).reshape(d_out, -1)
    assert np.array_equal(got[:n], ref) and (got[n:] == 0xA5).all()
    assert np.array_equal(host(idx)[:n], idx_o)
    packed2 = torch.full((ref.size,), 0x5A, dtype=torch.uint8, device="cuda")
    B_.srigl_pack_terms(dev(W_c_o), dev(idx_o), n, K, d_in, packed2)
    torch.cuda.synchronize()
    assert np.array_equal(host(packed2).reshape(n, -1), ref)
    # too small a buffer is refused on the host
    with pytest.raises(B_.SriglError) as e:
        B_.srigl_condense(W, m, d_out, d_in, K, d_out, W_c, idx, active, None, ws, rep, packed=packed[:nbytes - 16])
    assert e.value.status == B_.ERR_CAPACITY


def test_condense_special_values_are_bit_copied():
    L = si.make_layer(64, 6, 4, 1, seed=7)
    specials = np.array([0x80000000, 0x00000000, 0x7FC00123, 0xFF800000], np.uint32).view(np.float32)
    L.W[0, L.true_idx[0]] = specials
    rep, W_c, idx, active, _ = _gpu_condense(L)
    assert rep["status"] == 0
    assert np.array_equal(W_c[0].view(np.uint32), specials.view(np.uint32))
    W_c_o, idx_o, _ = oracle.condense(L.W, L.mask, 4)
    assert np.array_equal(W_c.view(np.uint32), W_c_o.view(np.uint32)) and np.array_equal(idx, idx_o)


def test_condense_reports_bad_fanin_row():
    L = si.make_layer(96, 40, 10, 1, ablate_frac=0.25, seed=11)
    for r in (int(L.true_active[3]), int(L.true_active[-1])):
        m = L.mask.copy()
        m[r, int(np.flatnonzero(m[r] == 0)[0])] = 1
        rep, *_ = _gpu_condense(L, mask=m)
        o = oracle.check_fanin_mask(m, 10)
        assert rep["status"] == B_.ERR_FANIN and rep["n_bad_rows"] == 1 and rep["first_bad_row"] == r == o["first_bad_row"]
        assert rep["n_active"] == o["n_active"]
        with pytest.raises(ValueError):
            oracle.condense(L.W, m, 10)


def test_condense_capacity_is_reported_and_respected():
    L = si.make_layer(64, 20, 6, 1, seed=12)
    W_c_o, idx_o, act_o = oracle.condense(L.W, L.mask, 6)
    rep, W_c, idx, active, _ = _gpu_condense(L, cap_rows=12)
    assert rep["status"] == B_.ERR_CAPACITY and rep["n_active"] == 20
    assert np.array_equal(idx, idx_o[:12]) and np.array_equal(active, act_o[:12])


@pytest.mark.parametrize("d_in,n_rows,K,abl", [(768, 3072, 77, 0.0), (3072, 768, 307, 0.3), (50, 9, 4, 0.3), (4096, 2500, 205, 0.2)])
def test_check_fanin_mask_mode(d_in, n_rows, K, abl):
    L = si.make_layer(d_in, n_rows, K, 1, ablate_frac=abl, seed=13)
    assert _gpu_check_mask(L.mask) == oracle.check_fanin_mask(L.mask)
    assert _gpu_check_mask(L.mask, K) == oracle.check_fanin_mask(L.mask, K)
    assert _gpu_check_mask(L.mask * 255, K) == oracle.check_fanin_mask(L.mask, K)       # any non-zero byte is "kept"
    assert _gpu_check_mask(L.mask, K - 1) == oracle.check_fanin_mask(L.mask, K - 1)     # every stored row is bad
    rng = np.random.default_rng(14)
    for _ in range(3):                                                                   # one flipped byte
        m = L.mask.copy()
        r, c = int(rng.integers(n_rows)), int(rng.integers(d_in))
        m[r, c] ^= 1
        assert _gpu_check_mask(m, K) == oracle.check_fanin_mask(m, K)
    z = np.zeros((5, d_in), np.uint8)
    assert _gpu_check_mask(z) == oracle.check_fanin_mask(z)
    # first non-empty row decides the inferred K
    m = L.mask.copy()
    first = int(L.true_active[0])
    m[first, int(np.flatnonzero(m[first])[0])] = 0
    assert _gpu_check_mask(m) == oracle.check_fanin_mask(m)


def _gpu_check_idx(idx, d_in, want_seg=True):
    n, K = idx.shape
    ws, rep = B_.new_workspace(n), B_.new_report()
    ss = B_.srigl_seg_stride(d_in)
    seg = torch.full((n, ss), -1, dtype=torch.int16, device="cuda") if want_seg else None
    B_.srigl_check_fanin(None, dev(idx), n, d_in, K, seg, ws, rep)
    return B_.read_report(rep), (host(seg) if want_seg else None)


def test_check_fanin_index_mode_and_seg():
    for d_in, n, K in ((768, 300, 77), (3072, 100, 307), (100, 17, 100), (70, 5, 1)):
        L = si.make_layer(d_in, n, K, 1, seed=15)
        rep, seg = _gpu_check_idx(L.true_idx, d_in)
        assert rep == oracle.check_fanin_idx(L.true_idx, d_in)
        assert np.array_equal(seg, oracle_seg(L.true_idx, d_in))
    L = si.make_layer(768, 64, 77, 1, seed=16)
    cases = []
    bad = L.true_idx.copy(); bad[5, 3] = bad[5, 2]; cases.append(bad)                 # duplicate
    bad = L.true_idx.copy(); bad[7, -1] = 768; cases.append(bad)                      # too large
    bad = L.true_idx.copy(); bad[0, 0] = -1; cases.append(bad)                        # negative
    bad = L.true_idx.copy(); bad[63, [10, 11]] = bad[63, [11, 10]]; cases.append(bad)  # descending pair
    bad = L.true_idx.copy(); bad[9, 0] = 5000; bad[40, 76] = -3; cases.append(bad)     # two bad rows
    for bad in cases:
        rep, seg = _gpu_check_idx(bad, 768)
        o = oracle.check_fanin_idx(bad, 768)
        assert rep["n_bad_rows"] == o["n_bad_rows"] and rep["first_bad_row"] == o["first_bad_row"]
        assert rep["n_active"] == o["n_active"] and rep["status"] == B_.ERR_INDEX_RANGE
        bad_rows = [r for r in range(64) if oracle.check_fanin_idx(bad[r:r + 1], 768)["n_bad_rows"]]
        assert (seg[bad_rows] == 0).all()


def test_host_side_argument_errors():
    rep, ws = B_.new_report(), B_.new_workspace(4)
    m = torch.zeros((4, 8), dtype=torch.uint8, device="cuda")
    i = torch.zeros((4, 2), dtype=torch.int32, device="cuda")
    with pytest.raises(B_.SriglError) as e:
        B_.srigl_check_fanin(m, i, 4, 8, 2, None, ws, rep)          # both mask and idx
    assert e.value.status == B_.ERR_INVALID_ARG
    with pytest.raises(B_.SriglError) as e:
        B_.srigl_check_fanin(None, None, 4, 8, 2, None, ws, rep)    # neither
    assert e.value.status == B_.ERR_INVALID_ARG
    with pytest.raises(B_.SriglError) as e:
        B_.srigl_check_fanin(m, None, 4, 8, -1, None, torch.empty(8, dtype=torch.uint8, device="cuda"), rep)
    assert e.value.status == B_.ERR_CAPACITY
    with pytest.raises(B_.SriglError) as e:
        B_.srigl_check_fanin(m, None, 4, 8, 9, None, ws, rep)       # K > d_in
    assert e.value.status == B_.ERR_INVALID_ARG
    W = torch.zeros((4, 8), dtype=torch.float32, device="cuda")
    with pytest.raises(B_.SriglError) as e:
        B_.srigl_condense(W, m, 4, 8, 9, 4, W, i, i, None, ws, rep)
    assert e.value.status == B_.ERR_INVALID_ARG
