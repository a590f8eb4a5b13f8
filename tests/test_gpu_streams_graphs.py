"""The library's calls are asynchronous on the caller's stream, allocate nothing and clear nothing with memset nodes: they
can run on a side stream and be captured in a HIP graph.  Every replay is checked against the eager result, with eager work
and synchronisations between the replays."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from gpu_util import TOL_F32, dev, gate, host, oracle_condensed

pytestmark = pytest.mark.gpu


def test_forward_pair_and_structured_in_a_graph():
    from paper_2305_02299_amd import binding as B_
    from paper_2305_02299_amd import condense_layer, fold_mlp
    L1 = si.make_layer(192, 512, 19, 48, ablate_frac=0.3, seed=41)
    L2 = si.make_layer(512, 160, 51, 48, ablate_frac=0.1, seed=42)
    l1 = condense_layer(dev(L1.W), dev(L1.mask), L1.K, dev(L1.bias))
    l2 = condense_layer(dev(L2.W), dev(L2.mask), L2.K, dev(L2.bias))
    pair = fold_mlp(l1, l2, B_.ACT_GELU)
    Wd = l1.dense_rows()
    x = dev(L1.x)
    hidden = torch.empty((48, pair.first.d_out), device="cuda")
    y_pair = torch.empty((48, 160), device="cuda")
    y_struct = torch.empty((48, 512), device="cuda")
    y_cond = torch.empty((48, 512), device="cuda")

    y_parts = torch.empty((48, 512), device="cuda")
    parts_ws = torch.empty((3 * 48 * l1.n_active,), device="cuda")

    def work():
        pair.forward(x, y_pair, hidden)
        B_.srigl_structured_linear_fwd(x, 48, 192, Wd, l1.active, l1.n_active, l1.bias, 512, y_struct)
        B_.srigl_structured_linear_fwd_split(x, 48, 192, Wd, l1.active, l1.n_active, l1.bias, 512, y_parts, parts_ws, splits=3,
                                             tile=B_.TILES["64x64"])
        B_.srigl_condensed_linear_fwd(x, 48, 192, l1.W_c, l1.idx, l1.active, l1.n_active, l1.K, l1.bias, 512, y_cond, l1.seg)

    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        work()                                    # eager, on a side stream
    side.synchronize()
    eager = [t.clone() for t in (y_pair, y_struct, y_cond, y_parts)]
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        work()
    for rep in range(4):
        for t in (y_pair, y_struct, y_cond, y_parts, parts_ws, hidden):
            t.fill_(float("nan"))                 # eager work between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for got, want in zip((y_pair, y_struct, y_cond, y_parts), eager):
            assert torch.equal(got, want), "replay %d differs from the eager run" % rep
    # and the eager result is the oracle's
    W_c, idx, active = oracle_condensed(L1)
    y_ref, S = oracle.fwd(L1.x, W_c, idx, active, L1.bias, 512, want_scale=True)
    gate(host(y_cond), y_ref, S, TOL_F32)
    gate(host(y_struct), y_ref, S, TOL_F32)
    gate(host(y_parts), y_ref, S, TOL_F32)


def test_condense_and_update_in_a_graph():
    from paper_2305_02299_amd import binding as B_
    L = si.make_layer(200, 150, 20, 1, ablate_frac=0.2, seed=43)
    Wm = np.where(L.mask != 0, L.W, 0).astype(np.float32)
    g_np = np.random.default_rng(3).normal(size=Wm.shape).astype(np.float32)
    W_d, m_d, g_d = dev(Wm), dev(L.mask), dev(g_np)
    mask_o, W_o = torch.empty_like(m_d), torch.empty_like(W_d)
    ws_u = torch.empty(B_.srigl_mask_update_workspace_bytes(150, 200), dtype=torch.uint8, device="cuda")
    rep_u = torch.zeros(4, dtype=torch.int64, device="cuda")
    W_c = torch.empty((150, 20), device="cuda")
    idx = torch.empty((150, 20), dtype=torch.int32, device="cuda")
    active = torch.empty(150, dtype=torch.int32, device="cuda")
    seg = torch.empty((150, B_.srigl_seg_stride(200)), dtype=torch.int16, device="cuda")
    ws_c, rep_c = B_.new_workspace(150), B_.new_report()
    K_upd = int(0.3 * L.mask.sum())

    def work():
        B_.srigl_mask_update(W_d, m_d, g_d, 150, 200, 20, K_upd, 30, int(L.mask.sum()), mask_o, W_o, ws_u, rep_u)
        B_.srigl_condense(W_d, m_d, 150, 200, 20, 150, W_c, idx, active, seg, ws_c, rep_c)

    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        work()
    side.synchronize()
    eager = [t.clone() for t in (mask_o, W_o, rep_u, W_c, idx, active)]
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        work()
    for rep in range(3):
        mask_o.fill_(9); W_o.fill_(-1.0); rep_u.fill_(-5); idx.fill_(-3)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        n = B_.read_report(rep_c)["n_active"]
        for got, want in zip((mask_o, W_o, rep_u, idx[:n], active[:n]), (eager[0], eager[1], eager[2], eager[4][:n], eager[5][:n])):
            assert torch.equal(got, want), "replay %d differs from the eager run" % rep
    m_ref, w_ref, info = oracle.mask_update(Wm, L.mask, g_np, 20, K_upd, 30)
    assert np.array_equal(host(mask_o), m_ref) and host(W_o).tobytes() == w_ref.tobytes()
