"""Plain CPU oracle of the column-tiled fully-connected layer (numpy, float64).

THIS IS TEST INFRASTRUCTURE.  Only tests, the smoke check and the CPU-baseline leg of the benchmark may
import it; the HIP library never does, and nothing in here touches the HIP library.

The paper's GPU Inference Kernel section tiles a fully-connected weight along its second dimension: an
``out x in`` matrix is stored as one ``out x q`` block, ``q = in / k``, and the same block is used again for
every one of the k column blocks.  With the per-copy scalars of Eq. 7-8 the layer's weight is

    W_hat[o, c*q + j] = alpha[c] * t[o, j],      c = 0..k-1,  j = 0..q-1,  t in {-1, +1}

and the layer computes ``Y = X W_hat^T`` (the layer operation stated after Eq. 8).  The tile is built as in
Eq. 1-3 with the k column blocks as the k summands, and alpha[c] is the mean magnitude of column block c
(Eq. 7-8), or one mean over the whole matrix (Eq. 6).

Tiles are ``uint32`` arrays: entry (o, j) is bit ``(o*q + j) % 32`` of word ``(o*q + j) // 32``.
Every function is the definition written out; nothing is blocked, fused or reordered.
"""
from __future__ import annotations

import numpy as np


def _check(out: int, cin: int, k: int):
    if out <= 0 or cin <= 0 or k <= 0 or cin % k:
        raise ValueError("in must be a positive multiple of k")
    return cin // k


def tile_words(out: int, cin: int, k: int) -> int:
    q = _check(out, cin, k)
    return (out * q + 31) // 32


def pack_coltile(w_real, out: int, cin: int, k: int, n_alpha: int = 1, a_real=None):
    """Eq. 1-3 with column blocks as summands; Eq. 6 (n_alpha = 1) or Eq. 7-8 (n_alpha = k).

    Returns (tile uint32[], alpha float32[]).  A sum that is zero (or not a number) gives bit 0, i.e. -1.
    """
    q = _check(out, cin, k)
    if n_alpha not in (1, k):
        raise ValueError("n_alpha must be 1 or k")
    w = np.asarray(w_real, dtype=np.float32).reshape(out, cin).astype(np.float64)
    a = w if a_real is None else np.asarray(a_real, dtype=np.float32).reshape(out, cin).astype(np.float64)
    s = np.zeros((out, q), dtype=np.float64)
    for c in range(k):                       # Eq. 2: the k blocks are added one after the other
        s = s + w[:, c * q:(c + 1) * q]
    bits = (s > 0.0).reshape(-1)             # Eq. 3
    padded = np.zeros(tile_words(out, cin, k) * 32, dtype=np.uint8)
    padded[:bits.size] = bits
    weights = (np.uint64(1) << np.arange(32, dtype=np.uint64))
    tile = (padded.reshape(-1, 32).astype(np.uint64) * weights).sum(axis=1).astype(np.uint32)
    if n_alpha == 1:
        alpha = np.array([np.abs(a).sum() / (out * cin)], dtype=np.float64)
    else:
        alpha = np.array([np.abs(a[:, c * q:(c + 1) * q]).sum() / (out * q) for c in range(k)], dtype=np.float64)
    return tile, alpha.astype(np.float32)


def tile_signs(tile, out: int, q: int) -> np.ndarray:
    """The +-1 block t of shape (out, q), float64."""
    tile = np.asarray(tile, dtype=np.uint32)
    idx = np.arange(out * q, dtype=np.int64)
    bit = (tile[idx // 32] >> (idx % 32).astype(np.uint32)) & np.uint32(1)
    return (2.0 * bit.astype(np.float64) - 1.0).reshape(out, q)


def materialise_coltile(tile, alpha, out: int, cin: int, k: int) -> np.ndarray:
    """W_hat of shape (out, in), float64."""
    q = _check(out, cin, k)
    alpha = np.asarray(alpha, dtype=np.float32).astype(np.float64)
    if alpha.size not in (1, k):
        raise ValueError("alpha must hold 1 or k scalars")
    t = tile_signs(tile, out, q)
    w_hat = np.empty((out, cin), dtype=np.float64)
    for c in range(k):
        w_hat[:, c * q:(c + 1) * q] = (alpha[c] if alpha.size == k else alpha[0]) * t
    return w_hat


def linear_coltiled_forward(x, tile, alpha, out: int, k: int, relu: bool = False) -> np.ndarray:
    """Y = X W_hat^T for X of shape (M, in); float64 (M, out)."""
    x = np.asarray(x, dtype=np.float64)
    if x.ndim != 2:
        raise ValueError("x must be (M, in)")
    w_hat = materialise_coltile(tile, alpha, out, x.shape[1], k)
    y = x @ w_hat.T
    return np.maximum(y, 0.0) if relu else y
