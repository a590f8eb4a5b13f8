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
    Wd: torch.Tensor | None = None   # dense rows of the stored neurons (structured-only form), built on first use

    def dense_rows(self) -> torch.Tensor:
        if self.Wd is None:
            self.Wd = torch.empty((max(self.n_active, 1), self.d_in), dtype=self.W_c.dtype, device=self.W_c.device)
            B_.srigl_densify(self.W_c, self.idx, self.n_active, self.K, self.d_in, self.Wd)
        return self.Wd

    def choose(self, batch: int) -> int:
        return B_.srigl_choose_representation(batch, self.d_in, self.n_active, self.K, self.d_out, B_._dtype_code(self.W_c))[0]

    def forward(self, x: torch.Tensor, y: torch.Tensor | None = None, algo=None, tuning=None,
                representation: str = "condensed") -> torch.Tensor:
        """representation: "condensed", "structured", or "auto" (the library's estimate for this batch size)."""
        assert x.dim() == 2 and x.shape[1] == self.d_in
        Bn = x.shape[0]
        if y is None:
            y = torch.empty((Bn, self.d_out), dtype=torch.float32, device=x.device)
        if representation == "auto":
            representation = "structured" if self.choose(Bn) == B_.REPR_STRUCTURED else "condensed"
        if representation == "structured":
            B_.srigl_structured_linear_fwd(x, Bn, self.d_in, self.dense_rows(), self.active, self.n_active, self.bias, self.d_out, y)
            return y
        assert representation == "condensed"
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
