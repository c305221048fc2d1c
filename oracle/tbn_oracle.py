"""ctypes front end of the plain CPU oracle in ``tbn_oracle.c``.

THIS IS TEST INFRASTRUCTURE.  Only tests, the smoke check and the CPU-baseline
leg of the benchmark may import it; the HIP library never does, and nothing in
here touches the HIP library.

The arithmetic lives in the C file (one function per definition of the paper's
Method section and Algorithm 1).  This module only converts numpy arrays to the
C calling convention:

* real weights are float32 arrays of any shape, flattened row-major;
* tiles are ``uint32`` arrays, entry ``i`` in word ``i // 32`` at bit ``i % 32``;
* activations are converted to float64 before the call (float32 and bfloat16
  values are exactly representable, so this adds no rounding);
* all results of the layer operations are float64.

Notation: ``n`` weights, ``k`` tile repeats, ``p = n // k`` tile bits (the paper
writes N, p and q for these).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tbn_oracle.c")
_LIB = os.path.join(_HERE, "libtbn_oracle.so")
_lib = None

_i64 = ctypes.c_int64
_i32 = ctypes.c_int32
_vp = ctypes.c_void_p


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc into ``oracle/libtbn_oracle.so``."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-ffp-contract=off", _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.tbn_oracle_threads.restype = ctypes.c_int
        for name in ("tbn_oracle_pack_tile", "tbn_oracle_materialise", "tbn_oracle_linear",
                     "tbn_oracle_linear_at", "tbn_oracle_conv2d", "tbn_oracle_conv2d_at",
                     "tbn_oracle_linear_alg1"):
            getattr(_lib, name).restype = ctypes.c_int
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(_vp)


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"{what}: oracle rejected the arguments (code {rc})")


def threads() -> int:
    """Number of OpenMP threads the layer loops will use."""
    return int(_load().tbn_oracle_threads())


def tile_words(n: int, k: int) -> int:
    """Number of 32-bit words that hold a tile of n // k bits."""
    if n <= 0 or k <= 0 or n % k:
        raise ValueError("n must be a positive multiple of k")
    return (n // k + 31) // 32


def pack_tile(w_real, k: int, n_alpha: int = 1, a_real=None):
    """Eq. 1-3 (tile) and Eq. 6 or Eq. 7-8 (alpha).  Returns (tile uint32[], alpha float32[])."""
    w = np.ascontiguousarray(w_real, dtype=np.float32).reshape(-1)
    a = None if a_real is None else np.ascontiguousarray(a_real, dtype=np.float32).reshape(-1)
    n = w.size
    if a is not None and a.size != n:
        raise ValueError("a_real must have as many elements as w_real")
    if k <= 0 or n == 0 or n % k:
        raise ValueError("n must be a positive multiple of k")
    tile = np.zeros(tile_words(n, k), dtype=np.uint32)
    alpha = np.zeros(n_alpha if n_alpha > 0 else 1, dtype=np.float32)
    rc = _load().tbn_oracle_pack_tile(_ptr(w), None if a is None else _ptr(a), _i64(n), _i32(k),
                                      _i32(n_alpha), _ptr(tile), _ptr(alpha))
    _check(rc, "pack_tile")
    return tile, alpha


def materialise(tile, alpha, n: int, k: int) -> np.ndarray:
    """Eq. 4-5 and the alpha scaling: the dense weight, flat float64 of n entries."""
    tile = np.ascontiguousarray(tile, dtype=np.uint32)
    alpha = np.ascontiguousarray(alpha, dtype=np.float32)
    if n <= 0 or k <= 0 or n % k or tile.size != tile_words(n, k):
        raise ValueError("tile size does not match n and k")
    w_hat = np.empty(n, dtype=np.float64)
    rc = _load().tbn_oracle_materialise(_ptr(tile), _ptr(alpha), _i32(alpha.size), _i64(n), _i32(k),
                                        _ptr(w_hat))
    _check(rc, "materialise")
    return w_hat


def linear_forward(x, tile, alpha, out: int, k: int) -> np.ndarray:
    """Y = X * B_hat^T for X of shape (M, in); float64 (M, out)."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    M, cin = x.shape
    w_hat = materialise(tile, alpha, out * cin, k)
    y = np.empty((M, out), dtype=np.float64)
    rc = _load().tbn_oracle_linear(_ptr(x), _i64(M), _i64(cin), _i64(out), _ptr(w_hat), _ptr(y))
    _check(rc, "linear_forward")
    return y


def linear_forward_at(x, tile, alpha, out: int, k: int, rows, cols) -> np.ndarray:
    """Entries Y[rows[q], cols[q]] of the fully-connected layer, float64."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    M, cin = x.shape
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    cols = np.ascontiguousarray(cols, dtype=np.int64)
    if rows.shape != cols.shape or rows.ndim != 1:
        raise ValueError("rows and cols must be 1-D and of equal length")
    w_hat = materialise(tile, alpha, out * cin, k)
    y = np.empty(rows.size, dtype=np.float64)
    rc = _load().tbn_oracle_linear_at(_ptr(x), _i64(M), _i64(cin), _i64(out), _ptr(w_hat),
                                      _ptr(rows), _ptr(cols), _i64(rows.size), _ptr(y))
    _check(rc, "linear_forward_at")
    return y


def conv_out_hw(H, W, kh, kw, stride, pad):
    return (H + 2 * pad[0] - kh) // stride[0] + 1, (W + 2 * pad[1] - kw) // stride[1] + 1


def conv2d_forward(x, tile, alpha, O: int, kh: int, kw: int, k: int, stride=(1, 1), pad=(0, 0)) -> np.ndarray:
    """Convolution layer for NCHW x with the implicit (O, C, kh, kw) weight; float64 (N, O, Ho, Wo)."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    N, C, H, W = x.shape
    w_hat = materialise(tile, alpha, O * C * kh * kw, k)
    Ho, Wo = conv_out_hw(H, W, kh, kw, stride, pad)
    if Ho <= 0 or Wo <= 0:
        raise ValueError("kernel larger than padded input")
    y = np.empty((N, O, Ho, Wo), dtype=np.float64)
    rc = _load().tbn_oracle_conv2d(_ptr(x), _i64(N), _i64(C), _i64(H), _i64(W), _i64(O), _i32(kh), _i32(kw),
                                   _i32(stride[0]), _i32(stride[1]), _i32(pad[0]), _i32(pad[1]),
                                   _ptr(w_hat), _ptr(y))
    _check(rc, "conv2d_forward")
    return y


def conv2d_forward_at(x, tile, alpha, O: int, kh: int, kw: int, k: int, flat_idx, stride=(1, 1), pad=(0, 0)):
    """Entries of the convolution output at flat indices into (N, O, Ho, Wo), float64."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    N, C, H, W = x.shape
    idx = np.ascontiguousarray(flat_idx, dtype=np.int64)
    w_hat = materialise(tile, alpha, O * C * kh * kw, k)
    y = np.empty(idx.size, dtype=np.float64)
    rc = _load().tbn_oracle_conv2d_at(_ptr(x), _i64(N), _i64(C), _i64(H), _i64(W), _i64(O), _i32(kh), _i32(kw),
                                      _i32(stride[0]), _i32(stride[1]), _i32(pad[0]), _i32(pad[1]),
                                      _ptr(w_hat), _ptr(idx), _i64(idx.size), _ptr(y))
    _check(rc, "conv2d_forward_at")
    return y


def linear_forward_alg1(x, tile, alpha, out: int, k: int, relu: bool = False) -> np.ndarray:
    """Algorithm 1 (running tile and alpha index over the flattened weight), float64 (M, out)."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    M, cin = x.shape
    tile = np.ascontiguousarray(tile, dtype=np.uint32)
    alpha = np.ascontiguousarray(alpha, dtype=np.float32)
    n = out * cin
    if k <= 0 or n % k or tile.size != tile_words(n, k):
        raise ValueError("tile size does not match n and k")
    y = np.empty((M, out), dtype=np.float64)
    rc = _load().tbn_oracle_linear_alg1(_ptr(x), _i64(M), _i64(cin), _i64(out), _ptr(tile), _i64(n // k),
                                        _ptr(alpha), _i32(alpha.size), _i32(1 if relu else 0), _ptr(y))
    _check(rc, "linear_forward_alg1")
    return y
