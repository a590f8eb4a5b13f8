"""Seeded synthetic layers for the condensed constant fan-in linear layer.

This module only draws random inputs (dense weights, constant fan-in masks,
activations, biases) with the shapes of the paper's benchmark layer (Sec. 4.4,
App. H: the 768 <-> 3072 ViT-B/16 MLP projections, fp32).  It holds none of the
method's arithmetic: no condensing, no forward product.  Both the CPU oracle's
tests and the GPU path's tests draw their inputs from here so that the two are
compared on identical bits.

The paper's trained ViT-B/16 masks are not available; random constant fan-in
topologies of the same shape stand in for them.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


# --------------------------------------------------------------------------- #
# helpers
# --------------------------------------------------------------------------- #
def fan_in_for_sparsity(d_in: int, sparsity_percent: int) -> int:
    """K = ceil((1 - s) * d_in) evaluated in integers (no floating ceil)."""
    return (d_in * (100 - sparsity_percent) + 99) // 100


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _uniform_rows(rng: np.random.Generator, n_rows: int, d_in: int, K: int) -> np.ndarray:
    """Per row: K distinct columns, uniform without replacement, ascending."""
    out = np.empty((n_rows, K), dtype=np.int32)
    step = max(1, (1 << 22) // max(d_in, 1))
    for r0 in range(0, n_rows, step):
        r1 = min(n_rows, r0 + step)
        keys = rng.random((r1 - r0, d_in), dtype=np.float32)
        if K < d_in:
            sel = np.argpartition(keys, K - 1, axis=1)[:, :K]
        else:
            sel = np.tile(np.arange(d_in), (r1 - r0, 1))
        out[r0:r1] = np.sort(sel, axis=1).astype(np.int32)
    return out


def _clustered_rows(rng: np.random.Generator, n_rows: int, d_in: int, K: int, window: int) -> np.ndarray:
    """Per row: floor(K/2) distinct columns from one random contiguous window of
    `window` columns, the rest uniform over [0, d_in) rejecting duplicates; ascending."""
    out = np.empty((n_rows, K), dtype=np.int32)
    window = min(window, d_in)
    k_in = min(K // 2, window)
    for r in range(n_rows):
        start = int(rng.integers(0, d_in - window + 1))
        inside = start + rng.choice(window, size=k_in, replace=False)
        chosen = np.zeros(d_in, dtype=bool)
        chosen[inside] = True
        need = K - k_in
        rest = np.flatnonzero(~chosen)
        extra = rng.choice(rest, size=need, replace=False)
        chosen[extra] = True
        out[r] = np.flatnonzero(chosen).astype(np.int32)
    return out


# --------------------------------------------------------------------------- #
# layer
# --------------------------------------------------------------------------- #
@dataclass
class Layer:
    """One synthetic sparse layer plus one activation batch (all host arrays).

    W      [d_out, d_in] float32   dense weights (values everywhere, mask decides)
    mask   [d_out, d_in] uint8     1 = kept; every row holds 0 (ablated) or K ones
    bias   [d_out]       float32
    x      [B, d_in]     float32
    true_idx    [n_active, K] int32   the column sets the sampler drew (ascending)
    true_active [n_active]    int32   rows that were not ablated (ascending)
    W_bf16 / x_bf16: uint16 bit patterns (only when dtype == "bf16"); in that case
    W and x hold the exactly-widened values of those bit patterns.
    """

    d_in: int
    d_out: int
    K: int
    B: int
    dtype: str
    seed: int
    W: np.ndarray
    mask: np.ndarray
    bias: np.ndarray
    x: np.ndarray
    true_idx: np.ndarray
    true_active: np.ndarray
    W_bf16: np.ndarray | None = None
    x_bf16: np.ndarray | None = None
    name: str = ""
    meta: dict = field(default_factory=dict)

    @property
    def n_active(self) -> int:
        return int(self.true_active.shape[0])


def make_layer(
    d_in: int,
    d_out: int,
    K: int,
    B: int,
    *,
    ablate_frac: float = 0.0,
    dtype: str = "f32",
    idx_dist: str = "uniform",
    window: int = 512,
    seed: int = 0,
    name: str = "",
) -> Layer:
    """Draw a layer: W ~ N(0, 1/K), bias ~ N(0, 0.01) (variance), x ~ N(0, 1).

    n_ablated = floor(ablate_frac * d_out) rows, chosen uniformly without
    replacement, get an all-zero mask row.
    """
    assert 0 <= K <= d_in and d_out >= 0 and B >= 0
    rng = np.random.default_rng(np.random.PCG64(seed))
    n_abl = int(np.floor(ablate_frac * d_out + 1e-9))
    ablated = np.sort(rng.choice(d_out, size=n_abl, replace=False)) if n_abl else np.empty(0, np.int64)
    keep = np.ones(d_out, dtype=bool)
    keep[ablated] = False
    active = np.flatnonzero(keep).astype(np.int32)
    if K == 0:
        active = np.empty(0, dtype=np.int32)

    if idx_dist == "uniform":
        idx = _uniform_rows(rng, active.shape[0], d_in, K)
    elif idx_dist == "clustered":
        idx = _clustered_rows(rng, active.shape[0], d_in, K, window)
    else:
        raise ValueError(idx_dist)

    mask = np.zeros((d_out, d_in), dtype=np.uint8)
    if active.shape[0] and K:
        mask[np.repeat(active, K), idx.reshape(-1)] = 1

    std_w = 1.0 / np.sqrt(max(K, 1))
    W = (rng.standard_normal((d_out, d_in), dtype=np.float32) * np.float32(std_w)).astype(np.float32)
    bias = (rng.standard_normal(d_out, dtype=np.float32) * np.float32(0.1)).astype(np.float32)
    x = rng.standard_normal((B, d_in), dtype=np.float32)

    W_b = x_b = None
    if dtype == "bf16":
        W_b = f32_to_bf16_bits(W)
        x_b = f32_to_bf16_bits(x)
        W = bf16_bits_to_f32(W_b)
        x = bf16_bits_to_f32(x_b)
    elif dtype != "f32":
        raise ValueError(dtype)

    return Layer(d_in, d_out, K, B, dtype, seed, W, mask, bias, x, idx, active, W_b, x_b, name,
                 {"ablate_frac": ablate_frac, "idx_dist": idx_dist})


def gather_condensed(layer: Layer) -> np.ndarray:
    """W_c implied by the sampler's own index sets (pure indexing, used only to
    cross-check a condense implementation against the generator's ground truth)."""
    if layer.n_active == 0 or layer.K == 0:
        return np.empty((layer.n_active, layer.K), dtype=np.float32)
    return layer.W[layer.true_active[:, None], layer.true_idx]


# --------------------------------------------------------------------------- #
# the benchmark's named configurations
# --------------------------------------------------------------------------- #
def config(name: str, *, B: int | None = None, seed: int = 0) -> Layer:
    """c1: 768->3072, K=77, B=1.   c2: same layer, B=256.
    c3: 3072->768, K=307, 30% of neurons ablated (n_active=538), B in {1,256}.
    c5: 4096->16384, K=205, bf16, 20% ablated, clustered indices, B=2048."""
    if name == "c1":
        return make_layer(768, 3072, 77, 1 if B is None else B, seed=seed, name="c1")
    if name == "c2":
        return make_layer(768, 3072, 77, 256 if B is None else B, seed=seed, name="c2")
    if name == "c3":
        return make_layer(3072, 768, 307, 256 if B is None else B, ablate_frac=0.30, seed=seed, name="c3")
    if name == "c5":
        return make_layer(4096, 16384, 205, 2048 if B is None else B, ablate_frac=0.20, dtype="bf16",
                          idx_dist="clustered", seed=seed, name="c5")
    raise ValueError(name)


def sweep_points():
    """(d_in, d_out, sparsity%, K, B) of the sparsity x batch sweep."""
    pts = []
    for d_in, d_out in ((768, 3072), (3072, 768)):
        for s in (80, 90, 95, 99):
            for B in (1, 16, 64, 256, 1024):
                pts.append((d_in, d_out, s, fan_in_for_sparsity(d_in, s), B))
    return pts
