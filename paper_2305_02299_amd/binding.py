"""Thin ctypes binding of libsrigl.so: argument marshalling only.

Function names and argument order follow include/srigl.h.  Every array argument is a
torch tensor on the GPU (PyTorch is used for device memory and streams, nothing else);
the binding passes its data pointer and the current HIP stream.  All arithmetic runs
in the library's HIP kernels.  If the library is missing the import of this module
fails: there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libsrigl.so")

OK, ERR_INVALID_ARG, ERR_FANIN, ERR_CAPACITY, ERR_INDEX_RANGE, ERR_UNSUPPORTED, ERR_HIP = range(7)
F32, BF16 = 0, 1
REPR_CONDENSED, REPR_STRUCTURED = 0, 1
ACT_NONE, ACT_RELU, ACT_GELU = 0, 1, 2
FWD_AUTO, FWD_GENERIC, FWD_KLANE, FWD_ROWLANE, FWD_ROWLOOP = range(5)
TILE_AUTO, TILE_256x256, TILE_256x256_H, TILE_256x128_W4, TILE_256x128, TILE_128x128, TILE_64x64 = range(7)
TILES = {"256x256": TILE_256x256, "256x256_h": TILE_256x256_H, "256x128_w4": TILE_256x128_W4, "256x128": TILE_256x128,
         "128x128": TILE_128x128, "64x64": TILE_64x64}

EXPORTS = (
    "srigl_workspace_bytes", "srigl_seg_stride", "srigl_check_fanin", "srigl_condense", "srigl_condense_static",
    "srigl_packed_bytes", "srigl_pack_terms",
    "srigl_condensed_linear_fwd", "srigl_condensed_linear_fwd_algo", "srigl_launch_empty",
    "srigl_copy_bytes", "srigl_status_str", "srigl_densify", "srigl_structured_linear_fwd",
    "srigl_structured_linear_fwd_tile", "srigl_structured_split_plan", "srigl_structured_linear_fwd_split", "srigl_choose_representation",
    "srigl_condensed_linear_fwd_act", "srigl_fold_ablated_inputs", "srigl_mask_update_workspace_bytes", "srigl_mask_update",
    "srigl_compact_hidden_layer", "srigl_condensed_mlp_fwd", "srigl_narrow_idx", "srigl_condensed_linear_fwd_idx16", "srigl_csr_linear_fwd", "srigl_fwd_plan_query", "srigl_fwd_plan_query_algo",
)


class SriglError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = int(status)
        super().__init__("%s: %s (status %d)" % (where, status_str(status), status))


class FwdTuning(ctypes.Structure):
    _fields_ = [("rows_per_lane", ctypes.c_int32), ("waves", ctypes.c_int32), ("neurons_per_wave", ctypes.c_int32),
                ("chunk_cols", ctypes.c_int32), ("lanes_per_neuron", ctypes.c_int32), ("rows_per_block", ctypes.c_int32),
                ("term_slices", ctypes.c_int32), ("direct_gather", ctypes.c_int32), ("xcd_order", ctypes.c_int32),
                ("terms_from_copy", ctypes.c_int32), ("spread_rows", ctypes.c_int32)]


class FwdPlan(ctypes.Structure):
    _fields_ = [("algo", ctypes.c_int32), ("rows_per_lane", ctypes.c_int32), ("term_slices", ctypes.c_int32), ("waves", ctypes.c_int32),
                ("neurons_per_wave", ctypes.c_int32), ("chunk_cols", ctypes.c_int32), ("lanes_per_neuron", ctypes.c_int32),
                ("rows_per_block", ctypes.c_int32), ("workgroups", ctypes.c_int64), ("direct_gather", ctypes.c_int32),
                ("xcd_order", ctypes.c_int32), ("spread_rows", ctypes.c_int32)]


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError("libsrigl.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(hipcc --offload-arch=gfx950) first; there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    lib.srigl_workspace_bytes.restype = sz
    lib.srigl_workspace_bytes.argtypes = [i32]
    lib.srigl_seg_stride.restype = i32
    lib.srigl_seg_stride.argtypes = [i32]
    lib.srigl_check_fanin.restype = ctypes.c_int
    lib.srigl_check_fanin.argtypes = [vp, vp, i32, i32, i32, vp, vp, sz, vp, vp]
    lib.srigl_condense.restype = ctypes.c_int
    lib.srigl_condense.argtypes = [vp, ctypes.c_int, vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, sz, vp, sz, vp, vp]
    lib.srigl_condense_static.restype = ctypes.c_int
    lib.srigl_condense_static.argtypes = [vp, ctypes.c_int, vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, sz, vp, vp]
    lib.srigl_packed_bytes.restype = sz
    lib.srigl_packed_bytes.argtypes = [i32, i32, i32, ctypes.c_int]
    lib.srigl_pack_terms.restype = ctypes.c_int
    lib.srigl_pack_terms.argtypes = [vp, ctypes.c_int, vp, i32, i32, i32, vp, sz, vp]
    lib.srigl_condensed_linear_fwd.restype = ctypes.c_int
    lib.srigl_condensed_linear_fwd.argtypes = [vp, ctypes.c_int, i32, i32, vp, ctypes.c_int, vp, vp, i32, i32, vp, i32, vp, vp, vp, vp]
    lib.srigl_condensed_linear_fwd_algo.restype = ctypes.c_int
    lib.srigl_condensed_linear_fwd_algo.argtypes = [vp, ctypes.c_int, i32, i32, vp, ctypes.c_int, vp, vp, i32, i32, vp, i32,
                                                    vp, vp, vp, ctypes.c_int, ctypes.POINTER(FwdTuning), vp]
    lib.srigl_densify.restype = ctypes.c_int
    lib.srigl_densify.argtypes = [vp, ctypes.c_int, vp, i32, i32, i32, vp, vp]
    lib.srigl_structured_linear_fwd.restype = ctypes.c_int
    lib.srigl_structured_linear_fwd.argtypes = [vp, ctypes.c_int, i32, i32, vp, ctypes.c_int, vp, i32, vp, i32, vp, vp]
    lib.srigl_structured_linear_fwd_tile.restype = ctypes.c_int
    lib.srigl_structured_linear_fwd_tile.argtypes = [vp, ctypes.c_int, i32, i32, vp, ctypes.c_int, vp, i32, vp, i32, vp, ctypes.c_int, vp]
    lib.srigl_structured_split_plan.restype = ctypes.c_int
    lib.srigl_structured_split_plan.argtypes = [i32, i32, i32, i32, ctypes.c_int, ctypes.POINTER(i32), ctypes.POINTER(ctypes.c_size_t)]
    lib.srigl_structured_linear_fwd_split.restype = ctypes.c_int
    lib.srigl_structured_linear_fwd_split.argtypes = [vp, ctypes.c_int, i32, i32, vp, ctypes.c_int, vp, i32, vp, i32, vp, ctypes.c_int, i32,
                                                      vp, ctypes.c_size_t, vp]
    lib.srigl_choose_representation.restype = ctypes.c_int
    lib.srigl_choose_representation.argtypes = [i32, i32, i32, i32, i32, ctypes.c_int, ctypes.POINTER(ctypes.c_float),
                                                ctypes.POINTER(ctypes.c_float)]
    lib.srigl_condensed_linear_fwd_act.restype = ctypes.c_int
    lib.srigl_condensed_linear_fwd_act.argtypes = [vp, ctypes.c_int, i32, i32, vp, ctypes.c_int, vp, vp, i32, i32, vp, i32,
                                                   vp, vp, vp, ctypes.c_int, ctypes.c_int, ctypes.POINTER(FwdTuning), vp]
    lib.srigl_fold_ablated_inputs.restype = ctypes.c_int
    lib.srigl_fold_ablated_inputs.argtypes = [vp, vp, ctypes.c_int, vp, vp, i32, i32, i32, vp, i32, i32, vp, ctypes.c_int, vp, vp, vp, vp]
    lib.srigl_compact_hidden_layer.restype = ctypes.c_int
    lib.srigl_compact_hidden_layer.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp]
    lib.srigl_condensed_mlp_fwd.restype = ctypes.c_int
    lib.srigl_condensed_mlp_fwd.argtypes = [vp, i32, i32, vp, vp, i32, i32, vp, i32, ctypes.c_int, vp, vp, vp, i32, i32, vp, i32, vp, i32, vp, vp]
    lib.srigl_mask_update_workspace_bytes.restype = sz
    lib.srigl_mask_update_workspace_bytes.argtypes = [i32, i32]
    lib.srigl_mask_update.restype = ctypes.c_int
    lib.srigl_mask_update.argtypes = [vp, vp, vp, i32, i32, i32, ctypes.c_int64, i32, ctypes.c_int64, vp, vp, vp, sz, vp, vp]
    lib.srigl_narrow_idx.restype = ctypes.c_int
    lib.srigl_narrow_idx.argtypes = [vp, ctypes.c_int64, i32, vp, vp]
    lib.srigl_condensed_linear_fwd_idx16.restype = ctypes.c_int
    lib.srigl_condensed_linear_fwd_idx16.argtypes = [vp, ctypes.c_int, i32, i32, vp, ctypes.c_int, vp, vp, i32, i32, vp, i32,
                                                     vp, vp, ctypes.c_int, ctypes.c_int, ctypes.POINTER(FwdTuning), vp]
    lib.srigl_csr_linear_fwd.restype = ctypes.c_int
    lib.srigl_csr_linear_fwd.argtypes = [vp, ctypes.c_int, i32, i32, vp, ctypes.c_int, vp, vp, ctypes.c_int64, vp, i32, vp, ctypes.c_int, vp]
    lib.srigl_fwd_plan_query.restype = ctypes.c_int
    lib.srigl_fwd_plan_query.argtypes = [i32, i32, i32, i32, i32, ctypes.c_int, i32, i32, ctypes.POINTER(FwdPlan)]
    lib.srigl_fwd_plan_query_algo.restype = ctypes.c_int
    lib.srigl_fwd_plan_query_algo.argtypes = [i32, i32, i32, i32, i32, ctypes.c_int, i32, i32, ctypes.c_int, ctypes.POINTER(FwdTuning),
                                              ctypes.POINTER(FwdPlan)]
    lib.srigl_launch_empty.restype = ctypes.c_int
    lib.srigl_launch_empty.argtypes = [vp]
    lib.srigl_copy_bytes.restype = ctypes.c_int
    lib.srigl_copy_bytes.argtypes = [vp, vp, sz, vp]
    lib.srigl_status_str.restype = ctypes.c_char_p
    lib.srigl_status_str.argtypes = [ctypes.c_int]
    return lib


lib = _load()


def status_str(status: int) -> str:
    return lib.srigl_status_str(int(status)).decode()


def _ptr(t):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensors only"
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dtype_code(t) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype in (torch.bfloat16, torch.uint16, torch.int16):
        return BF16   # 16-bit containers carry bf16 bit patterns
    raise TypeError("unsupported element type %s" % t.dtype)


def _check(status: int, where: str):
    if status != OK:
        raise SriglError(status, where)


def srigl_workspace_bytes(n_rows: int) -> int:
    return int(lib.srigl_workspace_bytes(int(n_rows)))


def srigl_seg_stride(d_in: int) -> int:
    return int(lib.srigl_seg_stride(int(d_in)))


def new_workspace(n_rows: int, device="cuda"):
    return torch.empty(srigl_workspace_bytes(n_rows), dtype=torch.uint8, device=device)


def new_report(device="cuda"):
    return torch.full((8,), -7, dtype=torch.int32, device=device)


def read_report(report) -> dict:
    """Synchronising read of the 32-byte device report."""
    r = report.cpu().tolist()
    return {"K": r[0], "n_active": r[1], "n_bad_rows": r[2], "first_bad_row": r[3], "status": r[4]}


def srigl_check_fanin(mask, idx, n_rows, d_in, K_expected, seg, workspace, report):
    st = lib.srigl_check_fanin(_ptr(mask), _ptr(idx), int(n_rows), int(d_in), int(K_expected), _ptr(seg), _ptr(workspace),
                               0 if workspace is None else workspace.numel() * workspace.element_size(), _ptr(report), _stream())
    _check(st, "srigl_check_fanin")


def _nbytes(t) -> int:
    return 0 if t is None else t.numel() * t.element_size()


def srigl_condense(W, mask, d_out, d_in, K, cap_rows, W_c, idx, active, seg, workspace, report, packed=None):
    st = lib.srigl_condense(_ptr(W), _dtype_code(W), _ptr(mask), int(d_out), int(d_in), int(K), int(cap_rows), _ptr(W_c),
                            _ptr(idx), _ptr(active), _ptr(seg), _ptr(packed), _nbytes(packed), _ptr(workspace), _nbytes(workspace),
                            _ptr(report), _stream())
    _check(st, "srigl_condense")


def srigl_condense_static(W, mask, d_out, d_in, K, cap_rows, W_c, idx, active, seg, report, packed=None):
    """srigl_condense with the library's built-in scratch in place of a workspace (no allocation on either side)."""
    st = lib.srigl_condense_static(_ptr(W), _dtype_code(W), _ptr(mask), int(d_out), int(d_in), int(K), int(cap_rows), _ptr(W_c),
                                   _ptr(idx), _ptr(active), _ptr(seg), _ptr(packed), _nbytes(packed), _ptr(report), _stream())
    _check(st, "srigl_condense_static")


def srigl_packed_bytes(n_rows: int, K: int, d_in: int, dtype_code: int) -> int:
    return int(lib.srigl_packed_bytes(int(n_rows), int(K), int(d_in), int(dtype_code)))


def srigl_pack_terms(W_c, idx, n_rows, K, d_in, packed):
    _check(lib.srigl_pack_terms(_ptr(W_c), _dtype_code(W_c), _ptr(idx), int(n_rows), int(K), int(d_in), _ptr(packed), _nbytes(packed),
                                _stream()), "srigl_pack_terms")


def _tuning(tuning):
    if tuning is None:
        return None
    tn = FwdTuning()
    for k, v in tuning.items():
        setattr(tn, k, int(v))
    return tn


def srigl_condensed_linear_fwd(x, B, d_in, W_c, idx, active, n_active, K, bias, d_out, y, seg=None, algo=None, tuning=None, act=None,
                               packed=None):
    """algo None: the library's own entry point; otherwise the forced-algorithm entry point; act: the entry point with an
    activation in the epilogue (ACT_* codes); idx in a 16-bit container: the narrow-index entry point (no streaming copy);
    packed: the streaming copy of W_c / idx."""
    tn = _tuning(tuning)
    tn_ref = ctypes.byref(tn) if tn is not None else None
    head = (_ptr(x), _dtype_code(x), int(B), int(d_in), _ptr(W_c), _dtype_code(W_c), _ptr(idx), _ptr(active), int(n_active), int(K),
            _ptr(bias), int(d_out), _ptr(y), _ptr(seg))
    if idx.dtype != torch.int32:       # a 16-bit container carries unsigned 16-bit column indices
        assert packed is None
        _check(lib.srigl_condensed_linear_fwd_idx16(*head, int(act or ACT_NONE), int(algo or FWD_AUTO), tn_ref, _stream()),
               "srigl_condensed_linear_fwd_idx16")
    elif act is not None:
        _check(lib.srigl_condensed_linear_fwd_act(*head, _ptr(packed), int(act), int(algo or FWD_AUTO), tn_ref, _stream()),
               "srigl_condensed_linear_fwd_act")
    elif algo is None and tuning is None:
        _check(lib.srigl_condensed_linear_fwd(*head, _ptr(packed), _stream()), "srigl_condensed_linear_fwd")
    else:
        _check(lib.srigl_condensed_linear_fwd_algo(*head, _ptr(packed), int(algo or FWD_AUTO), tn_ref, _stream()),
               "srigl_condensed_linear_fwd_algo")


def srigl_narrow_idx(idx, d_in, idx16):
    """idx int32 (any shape, contiguous) -> idx16, a 16-bit container of the same number of elements."""
    assert idx.dtype == torch.int32 and idx16.dtype in (torch.int16, torch.uint16) and idx16.numel() == idx.numel()
    _check(lib.srigl_narrow_idx(_ptr(idx), int(idx.numel()), int(d_in), _ptr(idx16), _stream()), "srigl_narrow_idx")


def srigl_csr_linear_fwd(x, B, d_in, values, col_idx, row_ptr, bias, d_out, y, act=None):
    """The layer's kept weights in compressed sparse row form (the unstructured comparison)."""
    nnz = int(values.numel())
    _check(lib.srigl_csr_linear_fwd(_ptr(x), _dtype_code(x), int(B), int(d_in), _ptr(values), _dtype_code(values), _ptr(col_idx),
                                    _ptr(row_ptr), nnz, _ptr(bias), int(d_out), _ptr(y), int(act or ACT_NONE), _stream()),
           "srigl_csr_linear_fwd")


def srigl_fwd_plan_query(B, d_in, n_active, K, d_out, dtype_code=F32, has_active=False, has_seg=True, algo=None, tuning=None) -> dict:
    """The kernel and launch shape the library's own choice (or the forced algo / tuning dict) takes for these sizes (host
    arithmetic, no GPU call)."""
    p = FwdPlan()
    tn = None
    if tuning is not None:
        tn = FwdTuning()
        for k, v in tuning.items():
            setattr(tn, k, int(v))
    _check(lib.srigl_fwd_plan_query_algo(int(B), int(d_in), int(n_active), int(K), int(d_out), int(dtype_code), int(bool(has_active)),
                                         int(bool(has_seg)), int(algo or FWD_AUTO), ctypes.byref(tn) if tn is not None else None,
                                         ctypes.byref(p)), "srigl_fwd_plan_query_algo")
    return {name: int(getattr(p, name)) for name, _ in FwdPlan._fields_}


def srigl_densify(W_c, idx, n_active, K, d_in, Wd):
    _check(lib.srigl_densify(_ptr(W_c), _dtype_code(W_c), _ptr(idx), int(n_active), int(K), int(d_in), _ptr(Wd), _stream()),
           "srigl_densify")


def srigl_structured_linear_fwd(x, B, d_in, Wd, active, n_active, bias, d_out, y, tile=None):
    """tile None: the library's own entry point; otherwise the forced-tile entry point (TILE_* codes)."""
    wcode = _dtype_code(Wd if Wd is not None else x)
    if tile is None:
        st = lib.srigl_structured_linear_fwd(_ptr(x), _dtype_code(x), int(B), int(d_in), _ptr(Wd), wcode, _ptr(active),
                                             int(n_active), _ptr(bias), int(d_out), _ptr(y), _stream())
    else:
        st = lib.srigl_structured_linear_fwd_tile(_ptr(x), _dtype_code(x), int(B), int(d_in), _ptr(Wd), wcode, _ptr(active),
                                                  int(n_active), _ptr(bias), int(d_out), _ptr(y), int(tile), _stream())
    _check(st, "srigl_structured_linear_fwd")


def srigl_structured_split_plan(B, d_in, n_active, d_out, dtype_code):
    """Returns (parts of d_in the library would take, workspace bytes that needs)."""
    n, b = ctypes.c_int32(0), ctypes.c_size_t(0)
    _check(lib.srigl_structured_split_plan(int(B), int(d_in), int(n_active), int(d_out), int(dtype_code), ctypes.byref(n), ctypes.byref(b)),
           "srigl_structured_split_plan")
    return int(n.value), int(b.value)


def srigl_structured_linear_fwd_split(x, B, d_in, Wd, active, n_active, bias, d_out, y, workspace, splits=0, tile=None):
    """splits 0: the library's choice (srigl_structured_split_plan); workspace: a device byte tensor (or None for one part)."""
    wcode = _dtype_code(Wd if Wd is not None else x)
    st = lib.srigl_structured_linear_fwd_split(_ptr(x), _dtype_code(x), int(B), int(d_in), _ptr(Wd), wcode, _ptr(active), int(n_active),
                                               _ptr(bias), int(d_out), _ptr(y), int(tile or 0), int(splits), _ptr(workspace),
                                               _nbytes(workspace), _stream())
    _check(st, "srigl_structured_linear_fwd_split")


def srigl_choose_representation(B, d_in, n_active, K, d_out, dtype_code):
    """Returns (REPR_CONDENSED | REPR_STRUCTURED, estimated condensed us, estimated structured us)."""
    c, s = ctypes.c_float(0), ctypes.c_float(0)
    r = lib.srigl_choose_representation(int(B), int(d_in), int(n_active), int(K), int(d_out), int(dtype_code),
                                        ctypes.byref(c), ctypes.byref(s))
    return int(r), c.value, s.value


def srigl_fold_ablated_inputs(idx2, W_c2, bias2, active2, n2, K2, d_out2, active1, n_active1, d_hidden, bias1, act,
                              idx_out, W_out, bias_out):
    st = lib.srigl_fold_ablated_inputs(_ptr(idx2), _ptr(W_c2), _dtype_code(W_c2), _ptr(bias2), _ptr(active2), int(n2), int(K2),
                                       int(d_out2), _ptr(active1), int(n_active1), int(d_hidden), _ptr(bias1), int(act),
                                       _ptr(idx_out), _ptr(W_out), _ptr(bias_out), _stream())
    _check(st, "srigl_fold_ablated_inputs")


def srigl_compact_hidden_layer(bias1, active1, n_active1, d_hidden, width, bias_compact, active_compact):
    _check(lib.srigl_compact_hidden_layer(_ptr(bias1), _ptr(active1), int(n_active1), int(d_hidden), int(width), _ptr(bias_compact),
                                          _ptr(active_compact), _stream()), "srigl_compact_hidden_layer")


def srigl_condensed_mlp_fwd(x, B, d_in, packed1, active1, n_active1, K1, bias1, d_hidden, act, hidden, packed2, active2, n_active2, K2,
                            bias2, d_out, y, spin_limit=0, status=None):
    _check(lib.srigl_condensed_mlp_fwd(_ptr(x), int(B), int(d_in), _ptr(packed1), _ptr(active1), int(n_active1), int(K1), _ptr(bias1),
                                       int(d_hidden), int(act), _ptr(hidden), _ptr(packed2), _ptr(active2), int(n_active2), int(K2),
                                       _ptr(bias2), int(d_out), _ptr(y), int(spin_limit), _ptr(status), _stream()),
           "srigl_condensed_mlp_fwd")


def srigl_mask_update_workspace_bytes(d_out: int, d_in: int) -> int:
    return int(lib.srigl_mask_update_workspace_bytes(int(d_out), int(d_in)))


def srigl_mask_update(W, mask, grad, d_out, d_in, k, K_upd, gamma_percent, budget, mask_out, W_out, workspace, report):
    """report: int64[4] device tensor -> {k', remaining neurons, ablated by this update, pruned in step 6}."""
    st = lib.srigl_mask_update(_ptr(W), _ptr(mask), _ptr(grad), int(d_out), int(d_in), int(k), int(K_upd), int(gamma_percent),
                               int(budget), _ptr(mask_out), _ptr(W_out), _ptr(workspace),
                               0 if workspace is None else workspace.numel() * workspace.element_size(), _ptr(report), _stream())
    _check(st, "srigl_mask_update")


def srigl_launch_empty():
    _check(lib.srigl_launch_empty(_stream()), "srigl_launch_empty")


def srigl_copy_bytes(src, dst, n_bytes):
    _check(lib.srigl_copy_bytes(_ptr(src), _ptr(dst), int(n_bytes), _stream()), "srigl_copy_bytes")
