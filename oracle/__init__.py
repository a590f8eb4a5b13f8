"""ctypes front end of the CPU oracle (oracle/srigl_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports this module and
this module never imports the product package.

Every wrapper takes and returns plain numpy arrays; the arithmetic is in the C++
file, which states, per function, the passage of the paper it follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "srigl_oracle.cpp")
_LIB = os.path.join(_HERE, "libsrigl_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (plain -O2; -fopenmp only serves the all-cores timing companion)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-fopenmp", "-fPIC", "-shared", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dt):
    return None if a is None else np.ascontiguousarray(a, dtype=dt)


def check_fanin_mask(mask: np.ndarray, K_expected: int = -1) -> dict:
    mask = _c(mask, np.uint8)
    n_rows, d_in = mask.shape
    rep = np.zeros(4, dtype=np.int32)
    rc = _load().oracle_check_fanin_mask(_p(mask), n_rows, d_in, int(K_expected), _p(rep))
    return {"K": int(rep[0]), "n_active": int(rep[1]), "n_bad_rows": int(rep[2]),
            "first_bad_row": int(rep[3]), "status": int(rc)}


def check_fanin_idx(idx: np.ndarray, d_in: int) -> dict:
    idx = _c(idx, np.int32)
    n_rows, K = idx.shape
    rep = np.zeros(4, dtype=np.int32)
    rc = _load().oracle_check_fanin_idx(_p(idx), n_rows, K, int(d_in), _p(rep))
    return {"K": int(rep[0]), "n_active": int(rep[1]), "n_bad_rows": int(rep[2]),
            "first_bad_row": int(rep[3]), "status": int(rc)}


def condense(W: np.ndarray, mask: np.ndarray, K: int):
    """W: float32 [d_out, d_in] or uint16 (bf16 bits).  Returns (W_c, idx, active);
    raises ValueError naming the first row whose count is neither 0 nor K."""
    assert W.dtype in (np.float32, np.uint16)
    W = np.ascontiguousarray(W)
    mask = _c(mask, np.uint8)
    d_out, d_in = mask.shape
    assert W.shape == (d_out, d_in)
    W_c = np.zeros((d_out, K), dtype=W.dtype)
    idx = np.zeros((d_out, K), dtype=np.int32)
    active = np.zeros(d_out, dtype=np.int32)
    n_active = ctypes.c_int32(0)
    bad = ctypes.c_int32(-1)
    rc = _load().oracle_condense(_p(W), W.dtype.itemsize, _p(mask), d_out, d_in, int(K), _p(W_c), _p(idx),
                                 _p(active), ctypes.byref(n_active), ctypes.byref(bad))
    if rc != 0:
        raise ValueError("row %d does not hold 0 or %d kept weights" % (bad.value, K))
    n = n_active.value
    return W_c[:n].copy(), idx[:n].copy(), active[:n].copy()


def fwd(x: np.ndarray, W_c: np.ndarray, idx: np.ndarray, active, bias, d_out: int, want_scale: bool = False):
    """Alg. 1 + bias + scatter.  x / W_c both float32, or both uint16 (bf16 bits)."""
    bf16 = x.dtype == np.uint16
    assert (W_c.dtype == np.uint16) == bf16
    x = np.ascontiguousarray(x)
    W_c = np.ascontiguousarray(W_c)
    idx = _c(idx, np.int32)
    active = _c(active, np.int32)
    bias = _c(bias, np.float32)
    B, d_in = x.shape
    n_active, K = W_c.shape
    assert idx.shape == (n_active, K)
    if active is None:
        assert n_active == d_out
    y = np.empty((B, d_out), dtype=np.float32)
    scale = np.empty((B, d_out), dtype=np.float64) if want_scale else None
    fn = _load().oracle_fwd_bf16 if bf16 else _load().oracle_fwd_f32
    fn(_p(x), B, d_in, _p(W_c), _p(idx), _p(active), n_active, K, _p(bias), int(d_out), _p(y), _p(scale))
    return (y, scale) if want_scale else y


def csr_fwd(x: np.ndarray, values: np.ndarray, col_idx: np.ndarray, row_ptr: np.ndarray, bias, want_scale: bool = False):
    """The same weights in compressed sparse row form (the unstructured comparison of Sec. 4.4 / Fig. 4), fp32."""
    x = _c(x, np.float32)
    values = _c(values, np.float32)
    col_idx = _c(col_idx, np.int32)
    row_ptr = _c(row_ptr, np.int32)
    bias = _c(bias, np.float32)
    B, d_in = x.shape
    d_out = row_ptr.shape[0] - 1
    assert row_ptr[0] == 0 and row_ptr[-1] == values.shape[0] == col_idx.shape[0]
    assert col_idx.size == 0 or (col_idx.min() >= 0 and col_idx.max() < d_in)
    y = np.empty((B, d_out), dtype=np.float32)
    scale = np.empty((B, d_out), dtype=np.float64) if want_scale else None
    _load().oracle_csr_fwd_f32(_p(x), B, d_in, _p(values), _p(col_idx), _p(row_ptr), _p(bias), d_out, _p(y), _p(scale))
    return (y, scale) if want_scale else y


def dense_masked_fwd(x: np.ndarray, W: np.ndarray, mask: np.ndarray, bias) -> np.ndarray:
    x = _c(x, np.float32)
    W = _c(W, np.float32)
    mask = _c(mask, np.uint8)
    bias = _c(bias, np.float32)
    B, d_in = x.shape
    d_out = W.shape[0]
    y = np.empty((B, d_out), dtype=np.float32)
    _load().oracle_dense_masked_fwd_f32(_p(x), B, d_in, _p(W), _p(mask), _p(bias), d_out, _p(y))
    return y


def densify(W_c: np.ndarray, idx: np.ndarray, d_in: int) -> np.ndarray:
    """Dense rows of the stored neurons (structured-only representation): [n_active, d_in], same element type."""
    assert W_c.dtype in (np.float32, np.uint16)
    W_c = np.ascontiguousarray(W_c)
    idx = _c(idx, np.int32)
    n, K = W_c.shape
    Wd = np.empty((n, d_in), dtype=W_c.dtype)
    _load().oracle_densify(_p(W_c), W_c.dtype.itemsize, _p(idx), n, K, int(d_in), _p(Wd))
    return Wd


def structured_fwd(x: np.ndarray, Wd: np.ndarray, active, bias, d_out: int) -> np.ndarray:
    bf16 = x.dtype == np.uint16
    assert (Wd.dtype == np.uint16) == bf16
    x = np.ascontiguousarray(x)
    Wd = np.ascontiguousarray(Wd)
    active = _c(active, np.int32)
    bias = _c(bias, np.float32)
    B, d_in = x.shape
    n = Wd.shape[0]
    if active is None:
        assert n == d_out
    y = np.empty((B, d_out), dtype=np.float32)
    fn = _load().oracle_structured_fwd_bf16 if bf16 else _load().oracle_structured_fwd_f32
    fn(_p(x), B, d_in, _p(Wd), _p(active), n, _p(bias), int(d_out), _p(y))
    return y


ACT_NONE, ACT_RELU, ACT_GELU = 0, 1, 2


def activate(y: np.ndarray, act: int) -> np.ndarray:
    """Activation of an MLP block applied to fp32 values (evaluated in double): identity, ReLU, erf-form GELU."""
    out = np.ascontiguousarray(y, dtype=np.float32).copy()
    _load().oracle_activate(_p(out), ctypes.c_longlong(out.size), int(act))
    return out


def fold_ablated_inputs(idx2, W_c2, bias2, active2, d_out2, active1, d_hidden, bias1, act):
    """Layer 2 rewritten to read the compact outputs of layer 1's stored neurons; returns (idx, W_c, bias[d_out2]).
    Raises ValueError if layer 2's fan-in exceeds the number of stored neurons of layer 1."""
    assert W_c2.dtype in (np.float32, np.uint16)
    idx2 = _c(idx2, np.int32)
    W_c2 = np.ascontiguousarray(W_c2)
    bias2 = _c(bias2, np.float32)
    active2 = _c(active2, np.int32)
    active1 = _c(active1, np.int32)
    bias1 = _c(bias1, np.float32)
    n2, K2 = idx2.shape
    idx_out = np.empty_like(idx2)
    W_out = np.empty_like(W_c2)
    bias_out = np.empty(d_out2, dtype=np.float32)
    rc = _load().oracle_fold_ablated_inputs(_p(idx2), _p(W_c2), W_c2.dtype.itemsize, _p(bias2), _p(active2), n2, K2, int(d_out2),
                                            _p(active1), len(active1), int(d_hidden), _p(bias1), int(act),
                                            _p(idx_out), _p(W_out), _p(bias_out))
    if rc != 0:
        raise ValueError("fan-in %d exceeds the %d stored neurons of the first layer" % (K2, len(active1)))
    return idx_out, W_out, bias_out


def pack_terms(W_c: np.ndarray, idx: np.ndarray, d_in: int) -> np.ndarray:
    """The streaming copy of App. E's two n x k arrays as bytes, [n][row_bytes]: the terms of a row in order, each weight next
    to its column index, rows padded to a multiple of four terms with weight bits 0 and index 0.  A term is 8 bytes (fp32
    weight, 32-bit index), 4 bytes for bf16 weights when d_in <= 65536 (weight in the low half-word, 16-bit index in the high
    one), else 8 bytes (bf16 weight, 16 zero bits, 32-bit index).  Little-endian words."""
    assert W_c.dtype in (np.float32, np.uint16) and W_c.shape == idx.shape
    n, K = idx.shape
    bf16 = W_c.dtype == np.uint16
    term_bytes = 4 if (bf16 and d_in <= 65536) else 8
    terms = (K + 3) // 4 * 4
    out = np.zeros((n, terms * term_bytes), dtype=np.uint8)
    wbits = W_c.view(np.uint16 if bf16 else np.uint32)
    for s in range(n):
        for t in range(K):
            w, col = int(wbits[s, t]), int(idx[s, t])
            word = (w | (col << 16)) if term_bytes == 4 else (w | (col << 32))
            out[s, t * term_bytes:(t + 1) * term_bytes] = [(word >> (8 * b)) & 0xFF for b in range(term_bytes)]
    return out


def compact_hidden_layer(bias1, active1, d_hidden, width):
    """The first layer of a folded pair writes its stored neurons next to each other (Sec. 3.1: ablation reduces the layer's
    width): position p of the compact hidden vector is neuron active1[p].  Returns (bias_compact[width], active_compact):
    the stored neurons' biases in that order, zero at the padding positions, and the positions themselves."""
    active1 = np.arange(d_hidden, dtype=np.int32) if active1 is None else np.asarray(active1, np.int32)
    n1 = len(active1)
    assert n1 <= width
    out = np.zeros(width, dtype=np.float32)
    for p in range(n1):
        out[p] = 0.0 if bias1 is None else bias1[active1[p]]
    return out, np.arange(n1, dtype=np.int32)


def mask_update(W, mask, grad, k, K_upd, gamma_percent, budget=None):
    """One SRigL connectivity update of a layer (Sec. 3.1 steps 1-7).  Returns (mask', W', info) with info =
    {k_new, n_remaining, n_ablated_now, n_pruned}."""
    W = _c(W, np.float32)
    mask = _c(mask, np.uint8)
    grad = _c(grad, np.float32)
    d_out, d_in = mask.shape
    if budget is None:
        budget = int(np.count_nonzero(mask))
    mask_out = np.empty_like(mask)
    W_out = np.empty_like(W)
    out4 = np.zeros(4, dtype=np.int64)
    _load().oracle_mask_update(_p(W), _p(mask), _p(grad), d_out, d_in, int(k), ctypes.c_longlong(int(K_upd)), int(gamma_percent),
                               ctypes.c_longlong(int(budget)), _p(mask_out), _p(W_out), _p(out4))
    return mask_out, W_out, {"k_new": int(out4[0]), "n_remaining": int(out4[1]), "n_ablated_now": int(out4[2]),
                             "n_pruned": int(out4[3])}


def fwd_allcores(x, W_c, idx, active, bias, d_out):
    """Timing companion (fp32 accumulate, OpenMP over batch x neurons): returns (y, threads used)."""
    x = _c(x, np.float32)
    W_c = _c(W_c, np.float32)
    idx = _c(idx, np.int32)
    active = _c(active, np.int32)
    bias = _c(bias, np.float32)
    B, d_in = x.shape
    n_active, K = W_c.shape
    y = np.empty((B, d_out), dtype=np.float32)
    lib = _load()
    lib.oracle_fwd_f32_allcores(_p(x), B, d_in, _p(W_c), _p(idx), _p(active), n_active, K, _p(bias), int(d_out), _p(y))
    return y, int(lib.oracle_num_threads())


def narrow_idx(idx: np.ndarray, d_in: int) -> np.ndarray:
    """App. E's index array held in 16 bits: the same column numbers, one 16-bit word each.  Defined only when every
    column number fits (d_in <= 65536) and every entry names a column of the layer."""
    idx = np.asarray(idx)
    if d_in > 65536:
        raise ValueError("column numbers of a layer this wide do not fit 16 bits")
    if idx.size and (idx.min() < 0 or idx.max() >= d_in):
        raise ValueError("an entry names no column of the layer")
    out = np.empty(idx.shape, dtype=np.uint16)
    flat_in, flat_out = idx.reshape(-1), out.reshape(-1)
    for i in range(flat_in.size):
        flat_out[i] = int(flat_in[i])
    return out
