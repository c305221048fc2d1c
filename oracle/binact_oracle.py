"""Plain CPU oracle of the fully-connected tiled-bit layer with binary activations (numpy, float64).

THIS IS TEST INFRASTRUCTURE.  Only tests, the smoke check and the CPU-baseline leg of the benchmark may
import it; the HIP library never does, and nothing in here touches the HIP library.

The paper's Conclusion names, as its first direction of future work, tiled-bit layers in models whose
activations are binary as well; it gives no formula.  The reading taken here is the one the paper's own
binarisation implies: an activation becomes +1 or -1 by the rule that Eq. 3 applies to a weight sum
(+1 where the value is greater than zero, -1 otherwise, so zero and not-a-number give -1), and the layer
operation stated after Eq. 8 is applied to those signs unchanged:

    s[m, j] = +1 if x[m, j] > 0 else -1
    y[m, o] = sum_{j < in} s[m, j] * alpha[(o*in + j) // p  (or 0)] * t[(o*in + j) % p],      p = in*out/k

No scalar is attached to the activations (the paper defines none).

Sign rows are ``uint32`` arrays of shape (M, ceil(in / 32)): activation j of row m is bit ``j % 32`` of word
``j // 32`` of that row (1 for +1); the unused high bits of a row's last word are zero.
Every function is the definition written out; nothing is blocked, fused or reordered.
"""
from __future__ import annotations

import numpy as np

from . import tbn_oracle


def row_words(cin: int) -> int:
    """32-bit words per row of sign bits."""
    if cin <= 0:
        raise ValueError("in must be positive")
    return (cin + 31) // 32


def sign_pack(x) -> np.ndarray:
    """Sign bits of an (M, in) array by the rule of Eq. 3: bit 1 where x > 0.  uint32 (M, ceil(in/32))."""
    x = np.asarray(x, dtype=np.float64)
    if x.ndim != 2 or x.shape[1] == 0:
        raise ValueError("x must be (M, in) with in > 0")
    M, cin = x.shape
    bits = np.zeros((M, row_words(cin) * 32), dtype=np.uint64)
    with np.errstate(invalid="ignore"):
        bits[:, :cin] = x > 0.0
    weights = np.uint64(1) << np.arange(32, dtype=np.uint64)
    return (bits.reshape(M, -1, 32) * weights).sum(axis=2).astype(np.uint32)


def signs(xbits, cin: int) -> np.ndarray:
    """The +-1 matrix (M, in), float64, that rows of sign bits stand for."""
    xbits = np.asarray(xbits, dtype=np.uint32)
    if xbits.ndim != 2 or xbits.shape[1] != row_words(cin):
        raise ValueError("xbits must be (M, ceil(in/32))")
    j = np.arange(cin)
    b = (xbits[:, j // 32] >> (j % 32).astype(np.uint32)) & np.uint32(1)
    return b.astype(np.float64) * 2.0 - 1.0


def linear_forward(xbits, cin: int, tile, alpha, out: int, k: int) -> np.ndarray:
    """Y = S * B_hat^T with S the +-1 matrix of the sign rows and B_hat the dense weight of Eq. 4-5 scaled by
    alpha (the layer operation stated after Eq. 8); float64 (M, out)."""
    s = signs(xbits, cin)
    w_hat = tbn_oracle.materialise(tile, alpha, out * cin, k).reshape(out, cin)
    return s @ w_hat.T


def linear_forward_signs(xbits, cin: int, tile, alpha, out: int, k: int) -> np.ndarray:
    """The layer followed by the binarisation of its outputs (what the next binary-activation layer consumes):
    rows of sign bits of Y, bit 1 where y > 0 (the rule of Eq. 3 once more); uint32 (M, ceil(out/32))."""
    return sign_pack(linear_forward(xbits, cin, tile, alpha, out, k))
