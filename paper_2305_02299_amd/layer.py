"""Device-buffer holder around the three library calls (no arithmetic here)."""
from __future__ import annotations

from dataclasses import dataclass

import torch

from . import binding as B_


@dataclass
class CondensedLinear:
    """The condensed form of one layer on the GPU: W_c / idx [n_active, K], active [n_active],
    bias [d_out], seg [n_active, seg_stride] (chunk offsets used by the batched kernel)."""

    d_in: int
    d_out: int
    K: int
    n_active: int
    W_c: torch.Tensor
    idx: torch.Tensor
    active: torch.Tensor | None
    bias: torch.Tensor | None
    seg: torch.Tensor | None

    def forward(self, x: torch.Tensor, y: torch.Tensor | None = None, algo=None, tuning=None) -> torch.Tensor:
        assert x.dim() == 2 and x.shape[1] == self.d_in
        Bn = x.shape[0]
        if y is None:
            y = torch.empty((Bn, self.d_out), dtype=torch.float32, device=x.device)
        B_.srigl_condensed_linear_fwd(x, Bn, self.d_in, self.W_c, self.idx, self.active, self.n_active, self.K, self.bias,
                                      self.d_out, y, self.seg, algo=algo, tuning=tuning)
        return y


def condense_layer(W: torch.Tensor, mask: torch.Tensor, K: int, bias: torch.Tensor | None = None,
                   want_seg: bool = True) -> CondensedLinear:
    """srigl_condense on device tensors; reads the report back (one synchronisation) to size the result."""
    d_out, d_in = mask.shape
    dev = W.device
    W_c = torch.empty((d_out, K), dtype=W.dtype, device=dev)
    idx = torch.empty((d_out, K), dtype=torch.int32, device=dev)
    active = torch.empty((d_out,), dtype=torch.int32, device=dev)
    ss = B_.srigl_seg_stride(d_in)
    seg = torch.empty((d_out, ss), dtype=torch.int16, device=dev) if want_seg else None
    ws = B_.new_workspace(d_out, dev)
    rep = B_.new_report(dev)
    B_.srigl_condense(W, mask, d_out, d_in, K, d_out, W_c, idx, active, seg, ws, rep)
    r = B_.read_report(rep)
    if r["status"] != B_.OK:
        raise B_.SriglError(r["status"], "srigl_condense (first bad row %d)" % r["first_bad_row"])
    n = r["n_active"]
    return CondensedLinear(d_in, d_out, K, n, W_c[:n].contiguous(), idx[:n].contiguous(),
                           None if n == d_out else active[:n].contiguous(), bias,
                           seg[:n].contiguous() if want_seg else None)
