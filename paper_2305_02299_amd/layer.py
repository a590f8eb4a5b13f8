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
    idx_wide: torch.Tensor | None = None   # the int32 indices when idx holds the 16-bit copy
    packed: torch.Tensor | None = None     # the streaming copy of W_c / idx (bytes), read by the kernels that can stream it
    split_ws: torch.Tensor | None = None   # partial sums of the structured-only product when it cuts d_in into parts (grown on demand)

    def narrow(self) -> "CondensedLinear":
        """The same layer with 16-bit column indices (d_in <= 65536); weights, active, bias and seg are shared."""
        if self.idx.dtype != torch.int32:
            return self
        idx16 = torch.empty(self.idx.shape, dtype=torch.int16, device=self.idx.device)
        B_.srigl_narrow_idx(self.idx, self.d_in, idx16)
        return CondensedLinear(self.d_in, self.d_out, self.K, self.n_active, self.W_c, idx16, self.active, self.bias, self.seg,
                               self.Wd, self.idx)

    def dense_rows(self) -> torch.Tensor:
        if self.Wd is None:
            self.Wd = torch.empty((max(self.n_active, 1), self.d_in), dtype=self.W_c.dtype, device=self.W_c.device)
            B_.srigl_densify(self.W_c, self.idx if self.idx_wide is None else self.idx_wide, self.n_active, self.K, self.d_in, self.Wd)
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
            _, need = B_.srigl_structured_split_plan(Bn, self.d_in, self.n_active, self.d_out, B_._dtype_code(self.W_c))
            if need and (self.split_ws is None or self.split_ws.numel() < need):
                self.split_ws = torch.empty((need,), dtype=torch.uint8, device=x.device)
            B_.srigl_structured_linear_fwd_split(x, Bn, self.d_in, self.dense_rows(), self.active, self.n_active, self.bias, self.d_out, y,
                                                 self.split_ws if need else None)
            return y
        assert representation == "condensed"
        B_.srigl_condensed_linear_fwd(x, Bn, self.d_in, self.W_c, self.idx, self.active, self.n_active, self.K, self.bias,
                                      self.d_out, y, self.seg, algo=algo, tuning=tuning,
                                      packed=self.packed if self.idx.dtype == torch.int32 else None)
        return y


def condense_layer(W: torch.Tensor, mask: torch.Tensor, K: int, bias: torch.Tensor | None = None,
                   want_seg: bool = True, want_packed: bool = True) -> CondensedLinear:
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
    code = B_._dtype_code(W)
    packed = torch.empty((max(B_.srigl_packed_bytes(d_out, K, d_in, code), 16),), dtype=torch.uint8, device=dev) if want_packed else None
    B_.srigl_condense(W, mask, d_out, d_in, K, d_out, W_c, idx, active, seg, ws, rep, packed=packed)
    r = B_.read_report(rep)
    if r["status"] != B_.OK:
        raise B_.SriglError(r["status"], "srigl_condense (first bad row %d)" % r["first_bad_row"])
    n = r["n_active"]
    return CondensedLinear(d_in, d_out, K, n, W_c[:n].contiguous(), idx[:n].contiguous(),
                           None if n == d_out else active[:n].contiguous(), bias,
                           seg[:n].contiguous() if want_seg else None,
                           packed=packed[:B_.srigl_packed_bytes(n, K, d_in, code)] if want_packed and n and K else None)


@dataclass
class CondensedMLP:
    """linear -> activation -> linear with the first layer's ablation used as width reduction: the hidden vector holds the
    stored neurons of layer 1 only (activation applied in layer 1's epilogue) and layer 2 has been rewritten by
    srigl_fold_ablated_inputs to read it.  Holds device buffers and calls the library; no arithmetic here."""

    first: CondensedLinear          # compact output: column p is stored neuron p; width padded to a multiple of 16
    second: CondensedLinear         # d_in == first.d_out
    act: int

    def forward(self, x: torch.Tensor, y: torch.Tensor | None = None, hidden: torch.Tensor | None = None,
                fused: bool | None = None) -> torch.Tensor:
        Bn = x.shape[0]
        f, s = self.first, self.second
        if hidden is None:
            hidden = torch.empty((Bn, f.d_out), dtype=torch.float32, device=x.device)
        if y is None:
            y = torch.empty((Bn, s.d_out), dtype=torch.float32, device=x.device)
        if fused:      # both layers in one launch (batches up to 8; measured slower than two launches on MI355X: not the default)
            B_.srigl_condensed_mlp_fwd(x, Bn, f.d_in, f.packed, f.active, f.n_active, f.K, f.bias, f.d_out, self.act, hidden, s.packed,
                                       s.active, s.n_active, s.K, s.bias, s.d_out, y)
            return y
        B_.srigl_condensed_linear_fwd(x, Bn, f.d_in, f.W_c, f.idx, f.active, f.n_active, f.K, f.bias, f.d_out, hidden, f.seg, act=self.act,
                                      packed=f.packed)
        B_.srigl_condensed_linear_fwd(hidden, Bn, s.d_in, s.W_c, s.idx, s.active, s.n_active, s.K, s.bias, s.d_out, y, s.seg,
                                      packed=s.packed)
        return y


def fold_mlp(layer1: CondensedLinear, layer2: CondensedLinear, act: int) -> CondensedMLP:
    """Both layers in fp32 storage (the hidden vector is fp32).  layer2.d_in must equal layer1.d_out."""
    assert layer2.d_in == layer1.d_out
    assert layer1.W_c.dtype == torch.float32 and layer2.W_c.dtype == torch.float32
    dev = layer1.W_c.device
    n1 = layer1.n_active
    # The hidden vector's width is padded to a multiple of 16 columns (the batched kernel stages rows of whole 64-byte
    # pieces); the padding columns are "ablated neurons" with zero bias, which no row of the second layer reads.
    n1p = (n1 + 15) // 16 * 16
    bias1_compact = torch.empty((n1p,), dtype=torch.float32, device=dev)
    active_first = None if n1p == n1 else torch.empty((n1,), dtype=torch.int32, device=dev)
    B_.srigl_compact_hidden_layer(layer1.bias, layer1.active, n1, layer1.d_out, n1p, bias1_compact, active_first)
    first = CondensedLinear(layer1.d_in, n1p, layer1.K, n1, layer1.W_c, layer1.idx, active_first, bias1_compact, layer1.seg,
                            packed=layer1.packed)
    idx_f = torch.empty_like(layer2.idx)
    W_f = torch.empty_like(layer2.W_c)
    bias_f = torch.empty((layer2.d_out,), dtype=torch.float32, device=dev)
    B_.srigl_fold_ablated_inputs(layer2.idx, layer2.W_c, layer2.bias, layer2.active, layer2.n_active, layer2.K, layer2.d_out,
                                 layer1.active, n1, layer1.d_out, layer1.bias, act, idx_f, W_f, bias_f)
    # the chunk table of the rewritten rows (and a check that they are ascending and in range)
    seg = torch.empty((max(layer2.n_active, 1), B_.srigl_seg_stride(n1p)), dtype=torch.int16, device=dev)
    ws, rep = B_.new_workspace(layer2.n_active, dev), B_.new_report(dev)
    B_.srigl_check_fanin(None, idx_f, layer2.n_active, n1p, layer2.K, seg, ws, rep)
    r = B_.read_report(rep)
    if r["status"] != B_.OK:
        raise B_.SriglError(r["status"], "srigl_fold_ablated_inputs produced a bad row (%d)" % r["first_bad_row"])
    packed2 = None
    if layer2.n_active and layer2.K:
        packed2 = torch.empty((B_.srigl_packed_bytes(layer2.n_active, layer2.K, n1p, B_.F32),), dtype=torch.uint8, device=dev)
        B_.srigl_pack_terms(W_f, idx_f, layer2.n_active, layer2.K, n1p, packed2)
    second = CondensedLinear(n1p, layer2.d_out, layer2.K, layer2.n_active, W_f, idx_f, layer2.active, bias_f, seg, packed=packed2)
    return CondensedMLP(first, second, act)
