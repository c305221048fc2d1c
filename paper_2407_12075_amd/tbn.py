"""Thin ctypes binding of libtbn (include/tbn.h).  Argument marshalling only: every step of the
computation runs in the HIP kernels of the library.  PyTorch supplies device memory and the
stream; tensors must live on the current CUDA (HIP) device and be contiguous.

There is no CPU fallback: if ``libtbn.so`` is missing the import of a symbol raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

TBN_OK = 0
TBN_F32 = 0
TBN_BF16 = 1
TBN_FLAG_RELU = 0x1
TBN_FLAG_FORCE_GENERIC = 0x100
TBN_FLAG_LARGE_BATCH = 0x200
TBN_FLAG_BLOCK_KERNEL = 0x400
TBN_FLAG_STREAM_KERNEL = 0x800
TBN_FLAG_SPLIT_K = 0x1000
TBN_FLAG_TILE_KERNEL = 0x2000
TBN_FLAG_SIGN_OUT = 0x4000

_STATUS = {1: "TBN_ERR_NULL", 2: "TBN_ERR_SHAPE", 3: "TBN_ERR_UNSUPPORTED", 4: "TBN_ERR_DEVICE",
           5: "TBN_ERR_WORKSPACE"}

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libtbn.so")
_lib = None

_c_i64, _c_i32, _c_u32, _c_vp, _c_sz = ctypes.c_int64, ctypes.c_int32, ctypes.c_uint32, ctypes.c_void_p, ctypes.c_size_t


class TbnError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{_STATUS.get(status, status)}: {message}")
        self.status = status


def lib() -> ctypes.CDLL:
    """Load libtbn.so (built by ``python -m paper_2407_12075_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} not found: build it with `python -m paper_2407_12075_amd.build`")
        L = ctypes.CDLL(_LIB_PATH)
        L.tbn_tile_words.restype = _c_sz
        L.tbn_tile_words.argtypes = [_c_i64, _c_i32]
        L.tbn_last_error.restype = ctypes.c_char_p
        L.tbn_last_error.argtypes = []
        L.tbn_version.restype = ctypes.c_char_p
        L.tbn_version.argtypes = []
        L.tbn_pack_workspace_bytes.restype = _c_sz
        L.tbn_pack_workspace_bytes.argtypes = [_c_i64, _c_i32, _c_i32]
        L.tbn_pack_tile.restype = ctypes.c_int
        L.tbn_pack_tile.argtypes = [_c_vp, _c_vp, _c_i64, _c_i32, _c_i32, _c_vp, _c_vp, _c_vp, _c_sz, _c_vp]
        L.tbn_pack_tile_noalloc.restype = ctypes.c_int
        L.tbn_pack_tile_noalloc.argtypes = [_c_vp, _c_vp, _c_i64, _c_i32, _c_i32, _c_vp, _c_vp, _c_vp]
        L.tbn_linear_forward.restype = ctypes.c_int
        L.tbn_linear_forward.argtypes = [_c_vp, _c_vp, ctypes.c_int, _c_i64, _c_i64, _c_i64, _c_vp, _c_i32, _c_vp,
                                         _c_i32, _c_u32, _c_vp]
        L.tbn_linear_forward_kernel.restype = ctypes.c_char_p
        L.tbn_linear_forward_kernel.argtypes = [_c_vp, _c_vp, ctypes.c_int, _c_i64, _c_i64, _c_i64, _c_i32, _c_i32, _c_u32]
        L.tbn_linear_forward_workspace_bytes.restype = _c_sz
        L.tbn_linear_forward_workspace_bytes.argtypes = [ctypes.c_int, _c_i64, _c_i64, _c_i64, _c_i32, ctypes.c_uint32]
        L.tbn_linear_forward_ws.restype = ctypes.c_int
        L.tbn_linear_forward_ws.argtypes = [_c_vp, _c_vp, ctypes.c_int, _c_i64, _c_i64, _c_i64, _c_vp, _c_i32, _c_vp,
                                            _c_i32, ctypes.c_uint32, _c_vp, _c_sz, _c_vp]
        L.tbn_conv2d_forward.restype = ctypes.c_int
        L.tbn_conv2d_forward.argtypes = [_c_vp, _c_vp, ctypes.c_int, _c_i64, _c_i64, _c_i64, _c_i64, _c_i64, _c_i32,
                                         _c_i32, _c_i32, _c_i32, _c_i32, _c_i32, _c_vp, _c_i32, _c_vp, _c_i32, _c_u32,
                                         _c_vp]
        L.tbn_pack_coltile_workspace_bytes.restype = _c_sz
        L.tbn_pack_coltile_workspace_bytes.argtypes = [_c_i64, _c_i64, _c_i32, _c_i32]
        L.tbn_pack_coltile.restype = ctypes.c_int
        L.tbn_pack_coltile.argtypes = [_c_vp, _c_vp, _c_i64, _c_i64, _c_i32, _c_i32, _c_vp, _c_vp, _c_vp, _c_sz, _c_vp]
        L.tbn_linear_coltiled_workspace_bytes.restype = _c_sz
        L.tbn_linear_coltiled_workspace_bytes.argtypes = [ctypes.c_int, _c_i64, _c_i64, _c_i32]
        L.tbn_linear_coltiled_forward.restype = ctypes.c_int
        L.tbn_linear_coltiled_forward.argtypes = [_c_vp, _c_vp, ctypes.c_int, _c_i64, _c_i64, _c_i64, _c_vp, _c_i32,
                                                  _c_vp, _c_i32, _c_u32, _c_vp, _c_sz, _c_vp]
        L.tbn_sign_row_words.restype = _c_sz
        L.tbn_sign_row_words.argtypes = [_c_i64]
        L.tbn_sign_pack.restype = ctypes.c_int
        L.tbn_sign_pack.argtypes = [_c_vp, ctypes.c_int, _c_i64, _c_i64, _c_vp, _c_vp]
        L.tbn_linear_forward_binact.restype = ctypes.c_int
        L.tbn_linear_forward_binact.argtypes = [_c_vp, _c_vp, ctypes.c_int, _c_i64, _c_i64, _c_i64, _c_vp, _c_i32, _c_vp,
                                                _c_i32, ctypes.c_uint32, _c_vp]
        L.tbn_diag_empty_launch.restype = ctypes.c_int
        L.tbn_diag_empty_launch.argtypes = [_c_vp]
        L.tbn_diag_stream.restype = ctypes.c_int
        L.tbn_diag_stream.argtypes = [_c_vp, _c_vp, _c_sz, _c_vp, _c_vp]
        L.tbn_diag_mfma.restype = ctypes.c_int
        L.tbn_diag_mfma.argtypes = [_c_i32, _c_i32, _c_vp, _c_vp]
        L.tbn_diag_mfma_fp4.restype = ctypes.c_int
        L.tbn_diag_mfma_fp4.argtypes = [_c_i32, _c_i32, _c_vp, _c_vp]
        _lib = L
    return _lib


def _raise(status: int):
    raise TbnError(status, lib().tbn_last_error().decode())


_recording = None   # list of (C function, marshalled arguments) while tbn_bind runs a wrapper
_owned = None       # buffers a wrapper allocated for itself while tbn_bind runs it: the bound call keeps them alive


def _call(name: str, *cargs) -> int:
    f = getattr(lib(), name)
    if _recording is not None:
        _recording.append((f, cargs))
        return TBN_OK
    return f(*cargs)


def _own(t: torch.Tensor) -> torch.Tensor:
    if _owned is not None:
        _owned.append(t)
    return t


def tbn_bind(fn, *args, **kwargs):
    """Marshal once, launch many times: runs the wrapper `fn(*args, **kwargs)` (any of the layer, packing and sign-packing
    wrappers of this module) with all its checks and allocations but without launching, and returns a callable that
    makes exactly that library call every time it is invoked and returns what the wrapper would have returned.  For
    loops that repeat a call on the same buffers (a serving loop refilling x in place): the Python side of a call
    drops from about 5 us to under 1 us.  The tensors, sizes, flags and the stream are those of the time of binding
    and are kept alive by the callable.  Not thread-safe while binding."""
    global _recording, _owned
    if _recording is not None:
        raise RuntimeError("tbn_bind: already binding")
    _recording, _owned = [], []
    try:
        result = fn(*args, **kwargs)
    finally:
        calls, _recording = _recording, None
        owned, _owned = _owned, None
    if not calls:
        raise ValueError("tbn_bind: the wrapper made no library call that can be bound")

    def replay(_calls=tuple(calls), _keep=(args, kwargs, owned), _result=result):
        for f, cargs in _calls:
            st = f(*cargs)
            if st != TBN_OK:
                _raise(st)
        return _result

    return replay


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _dev(t: torch.Tensor, name: str, dtype=None) -> int:
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must have dtype {dtype}, got {t.dtype}")
    return t.data_ptr()


def _check_layer_tensors(fn: str, x: torch.Tensor, tile: torch.Tensor, alpha: torch.Tensor, n: int, k: int, *others):
    """Sizes and devices the C side cannot see behind raw pointers: an undersized tile or alpha would be an
    out-of-bounds device read.  (Illegal n, k, n_alpha are left to the C side, which reports them.)"""
    words = tbn_tile_words(n, k) if k > 0 else 0
    if words and tile.numel() < words:
        raise ValueError(f"{fn}: tile has {tile.numel()} words, {words} needed")
    if alpha.numel() < 1:
        raise ValueError(f"{fn}: alpha is empty")
    for t in (tile, alpha, *others):
        if t is not None and t.device != x.device:
            raise ValueError(f"{fn}: all tensors must live on {x.device}")


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return TBN_F32
    if t.dtype == torch.bfloat16:
        return TBN_BF16
    raise ValueError(f"activations must be float32 or bfloat16, got {t.dtype}")


def tbn_version() -> str:
    return lib().tbn_version().decode()


def tbn_tile_words(n: int, k: int) -> int:
    return int(lib().tbn_tile_words(n, k))


def tbn_pack_workspace_bytes(n: int, k: int, n_alpha: int) -> int:
    return int(lib().tbn_pack_workspace_bytes(n, k, n_alpha))


def tbn_pack_tile(w_real: torch.Tensor, k: int, n_alpha: int = 1, a_real: Optional[torch.Tensor] = None,
                  tile_out: Optional[torch.Tensor] = None, alpha_out: Optional[torch.Tensor] = None,
                  workspace: Optional[torch.Tensor] = None, stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Tile (int32 tensor holding the 32-bit words) and alpha (float32) from real weights."""
    n = w_real.numel()
    words = tbn_tile_words(n, k)
    dev = w_real.device
    if tile_out is None:
        tile_out = torch.empty(max(words, 1), dtype=torch.int32, device=dev)
    if alpha_out is None:
        alpha_out = torch.empty(max(n_alpha, 1), dtype=torch.float32, device=dev)
    need = tbn_pack_workspace_bytes(n, k, n_alpha)
    if workspace is None:
        if _recording is not None:
            raise ValueError("tbn_bind(tbn_pack_tile, ...): pass the workspace (the bound call does not own one)")
        workspace = torch.empty(max(need, 8), dtype=torch.uint8, device=dev)
    if tile_out.numel() < words or alpha_out.numel() < n_alpha or any(t.device != dev for t in (tile_out, alpha_out, workspace)) \
            or (a_real is not None and (a_real.numel() != n or a_real.device != dev)):
        raise ValueError("tbn_pack_tile: tile_out, alpha_out, a_real or workspace too small or on another device")
    st = _call("tbn_pack_tile", _dev(w_real, "w_real", torch.float32),
                             None if a_real is None else _dev(a_real, "a_real", torch.float32),
                             n, k, n_alpha, _dev(tile_out, "tile_out", torch.int32),
                             _dev(alpha_out, "alpha_out", torch.float32), _dev(workspace, "workspace"),
                             workspace.numel() * workspace.element_size(), _stream(stream))
    if st != TBN_OK:
        _raise(st)
    return tile_out, alpha_out


def tbn_pack_tile_noalloc(w_real: torch.Tensor, k: int, n_alpha: int, tile_out: torch.Tensor, alpha_out: torch.Tensor,
                          a_real: Optional[torch.Tensor] = None, stream=None) -> None:
    """tbn_pack_tile without a workspace; the outputs are the caller's (this wrapper allocates nothing either)."""
    if tile_out.numel() < tbn_tile_words(w_real.numel(), k) or alpha_out.numel() < n_alpha or tile_out.device != w_real.device \
            or alpha_out.device != w_real.device or (a_real is not None and (a_real.numel() != w_real.numel() or a_real.device != w_real.device)):
        raise ValueError("tbn_pack_tile_noalloc: tile_out, alpha_out or a_real too small or on another device")
    st = _call("tbn_pack_tile_noalloc", _dev(w_real, "w_real", torch.float32),
                                     None if a_real is None else _dev(a_real, "a_real", torch.float32),
                                     w_real.numel(), k, n_alpha, _dev(tile_out, "tile_out", torch.int32),
                                     _dev(alpha_out, "alpha_out", torch.float32), _stream(stream))
    if st != TBN_OK:
        _raise(st)


def tbn_linear_forward(x: torch.Tensor, tile: torch.Tensor, alpha: torch.Tensor, out_features: int, k: int,
                       y: Optional[torch.Tensor] = None, flags: int = 0, stream=None) -> torch.Tensor:
    """Y = X * B_hat^T for x of shape (M, in); y has shape (M, out_features) and x's dtype."""
    if x.dim() != 2:
        raise ValueError("x must be (M, in)")
    M, cin = x.shape
    if y is None:
        y = torch.empty((M, out_features), dtype=x.dtype, device=x.device)
    elif tuple(y.shape) != (M, out_features) or y.dtype != x.dtype:
        raise ValueError("y must be (M, out) with x's dtype")
    _check_layer_tensors("tbn_linear_forward", x, tile, alpha, cin * out_features, k, y)
    st = _call("tbn_linear_forward", _dev(x, "x"), _dev(y, "y"), _dt(x), M, cin, out_features,
               _dev(tile, "tile", torch.int32), k, _dev(alpha, "alpha", torch.float32), alpha.numel(), flags, _stream(stream))
    if st != TBN_OK:
        _raise(st)
    return y


def tbn_linear_forward_kernel(dtype: torch.dtype, M: int, cin: int, out_features: int, k: int, n_alpha: int = 1,
                              flags: int = 0, x_ptr: int = 0, y_ptr: int = 0) -> str:
    """Name of the kernel family tbn_linear_forward would launch for these sizes ("" on sizes it rejects); x_ptr and
    y_ptr are the addresses the call would get (only their alignment matters; 0 counts as aligned)."""
    dt = TBN_F32 if dtype == torch.float32 else TBN_BF16
    return lib().tbn_linear_forward_kernel(x_ptr or None, y_ptr or None, dt, M, cin, out_features, k, n_alpha, flags).decode()


def tbn_linear_forward_workspace_bytes(dtype: torch.dtype, M: int, cin: int, out_features: int, k: int, flags: int = 0) -> int:
    """Bytes of workspace with which tbn_linear_forward_ws takes its fastest path for these sizes (0: none needed)."""
    dt = TBN_F32 if dtype == torch.float32 else TBN_BF16
    return int(lib().tbn_linear_forward_workspace_bytes(dt, M, cin, out_features, k, flags))


def tbn_linear_forward_ws(x: torch.Tensor, tile: torch.Tensor, alpha: torch.Tensor, out_features: int, k: int,
                          workspace: Optional[torch.Tensor], y: Optional[torch.Tensor] = None, flags: int = 0,
                          stream=None) -> torch.Tensor:
    """tbn_linear_forward with a caller-supplied device workspace (None or too small: the same as tbn_linear_forward)."""
    if x.dim() != 2:
        raise ValueError("x must be (M, in)")
    M, cin = x.shape
    if y is None:
        y = torch.empty((M, out_features), dtype=x.dtype, device=x.device)
    elif tuple(y.shape) != (M, out_features) or y.dtype != x.dtype:
        raise ValueError("y must be (M, out) with x's dtype")
    _check_layer_tensors("tbn_linear_forward_ws", x, tile, alpha, cin * out_features, k, y, workspace)
    ws_ptr = None if workspace is None else _dev(workspace, "workspace")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = _call("tbn_linear_forward_ws", _dev(x, "x"), _dev(y, "y"), _dt(x), M, cin, out_features,
               _dev(tile, "tile", torch.int32), k, _dev(alpha, "alpha", torch.float32), alpha.numel(), flags, ws_ptr, ws_bytes,
               _stream(stream))
    if st != TBN_OK:
        _raise(st)
    return y


def conv_out_hw(H: int, W: int, kh: int, kw: int, stride, pad) -> Tuple[int, int]:
    return (H + 2 * pad[0] - kh) // stride[0] + 1, (W + 2 * pad[1] - kw) // stride[1] + 1


def tbn_pack_coltile(w_real: torch.Tensor, k: int, n_alpha: int = 1, a_real: Optional[torch.Tensor] = None,
                     workspace: Optional[torch.Tensor] = None, stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Tile and alpha of the column-tiled layout from a real (out, in) weight; k column blocks."""
    if w_real.dim() != 2:
        raise ValueError("w_real must be (out, in)")
    out, cin = w_real.shape
    dev = w_real.device
    tile_out = torch.empty(max(tbn_tile_words(out * cin, k), 1), dtype=torch.int32, device=dev)
    alpha_out = torch.empty(max(n_alpha, 1), dtype=torch.float32, device=dev)
    need = int(lib().tbn_pack_coltile_workspace_bytes(out, cin, k, n_alpha))
    if workspace is None:
        workspace = _own(torch.empty(max(need, 8), dtype=torch.uint8, device=dev))
    st = _call("tbn_pack_coltile", _dev(w_real, "w_real", torch.float32),
                                None if a_real is None else _dev(a_real, "a_real", torch.float32),
                                out, cin, k, n_alpha, _dev(tile_out, "tile_out", torch.int32),
                                _dev(alpha_out, "alpha_out", torch.float32), _dev(workspace, "workspace"),
                                workspace.numel() * workspace.element_size(), _stream(stream))
    if st != TBN_OK:
        _raise(st)
    return tile_out, alpha_out


def tbn_linear_coltiled_workspace_bytes(x: torch.Tensor, k: int) -> int:
    return int(lib().tbn_linear_coltiled_workspace_bytes(_dt(x), x.shape[0], x.shape[1], k))


def tbn_linear_coltiled_forward(x: torch.Tensor, tile: torch.Tensor, alpha: torch.Tensor, out_features: int, k: int,
                                y: Optional[torch.Tensor] = None, flags: int = 0,
                                workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Column-tiled layer: W_hat[o, c*q + j] = alpha[c] * t[o, j]; y has shape (M, out_features) and x's dtype."""
    if x.dim() != 2:
        raise ValueError("x must be (M, in)")
    M, cin = x.shape
    if y is None:
        y = torch.empty((M, out_features), dtype=x.dtype, device=x.device)
    elif tuple(y.shape) != (M, out_features) or y.dtype != x.dtype:
        raise ValueError("y must be (M, out) with x's dtype")
    if workspace is None:
        workspace = _own(torch.empty(max(tbn_linear_coltiled_workspace_bytes(x, k), 16), dtype=torch.uint8, device=x.device))
    _check_layer_tensors("tbn_linear_coltiled_forward", x, tile, alpha, cin * out_features, k, y, workspace)
    st = _call("tbn_linear_coltiled_forward", _dev(x, "x"), _dev(y, "y"), _dt(x), M, cin, out_features,
                                           _dev(tile, "tile", torch.int32), k, _dev(alpha, "alpha", torch.float32),
                                           alpha.numel(), flags, _dev(workspace, "workspace"),
                                           workspace.numel() * workspace.element_size(), _stream(stream))
    if st != TBN_OK:
        _raise(st)
    return y


def tbn_conv2d_forward(x: torch.Tensor, tile: torch.Tensor, alpha: torch.Tensor, out_channels: int, kh: int,
                       kw: int, k: int, stride=(1, 1), pad=(0, 0), y: Optional[torch.Tensor] = None,
                       flags: int = 0, stream=None) -> torch.Tensor:
    """NCHW convolution with the implicit (O, C, kh, kw) tiled-bit weight."""
    if x.dim() != 4:
        raise ValueError("x must be (N, C, H, W)")
    N, C, H, W = x.shape
    Ho, Wo = conv_out_hw(H, W, kh, kw, stride, pad)
    if y is None:
        y = torch.empty((N, out_channels, max(Ho, 0), max(Wo, 0)), dtype=x.dtype, device=x.device)
    elif tuple(y.shape) != (N, out_channels, Ho, Wo) or y.dtype != x.dtype:
        raise ValueError("y must be (N, O, Ho, Wo) with x's dtype")
    _check_layer_tensors("tbn_conv2d_forward", x, tile, alpha, out_channels * C * kh * kw, k, y)
    st = _call("tbn_conv2d_forward", _dev(x, "x"), _dev(y, "y"), _dt(x), N, C, H, W, out_channels, kh, kw,
                                  stride[0], stride[1], pad[0], pad[1], _dev(tile, "tile", torch.int32), k,
                                  _dev(alpha, "alpha", torch.float32), alpha.numel(), flags, _stream(stream))
    if st != TBN_OK:
        _raise(st)
    return y


def tbn_sign_row_words(cin: int) -> int:
    return int(lib().tbn_sign_row_words(cin))


def tbn_sign_pack(x: torch.Tensor, xbits: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Rows of sign bits of x (M, in): int32 (M, ceil(in / 32)), bit j % 32 of word j // 32 set where x[m, j] > 0."""
    if x.dim() != 2:
        raise ValueError("x must be (M, in)")
    M, cin = x.shape
    words = tbn_sign_row_words(cin)
    if xbits is None:
        xbits = torch.empty((M, words), dtype=torch.int32, device=x.device)
    elif tuple(xbits.shape) != (M, words) or xbits.device != x.device:
        raise ValueError(f"xbits must be ({M}, {words}) on {x.device}")
    st = _call("tbn_sign_pack", _dev(x, "x"), _dt(x), M, cin, _dev(xbits, "xbits", torch.int32), _stream(stream))
    if st != TBN_OK:
        _raise(st)
    return xbits


def tbn_linear_forward_binact(xbits: torch.Tensor, cin: int, tile: torch.Tensor, alpha: torch.Tensor, out_features: int,
                              k: int, dtype: torch.dtype = torch.float32, y: Optional[torch.Tensor] = None, flags: int = 0,
                              stream=None) -> torch.Tensor:
    """The layer on rows of sign bits (M, ceil(in / 32)); y has shape (M, out_features) and the given dtype."""
    if xbits.dim() != 2 or xbits.shape[1] != tbn_sign_row_words(cin):
        raise ValueError("xbits must be (M, ceil(in / 32))")
    M = xbits.shape[0]
    if flags & TBN_FLAG_SIGN_OUT:   # rows of sign bits of the outputs
        shape, ydt = (M, tbn_sign_row_words(out_features)), torch.int32
    else:
        shape, ydt = (M, out_features), dtype
    if y is None:
        y = torch.empty(shape, dtype=ydt, device=xbits.device)
    elif tuple(y.shape) != shape or (flags & TBN_FLAG_SIGN_OUT and y.dtype != torch.int32):
        raise ValueError(f"y must be {shape}" + (" int32" if flags & TBN_FLAG_SIGN_OUT else ""))
    _check_layer_tensors("tbn_linear_forward_binact", xbits, tile, alpha, cin * out_features, k, y)
    st = _call("tbn_linear_forward_binact", _dev(xbits, "xbits", torch.int32), _dev(y, "y"),
                                         TBN_F32 if flags & TBN_FLAG_SIGN_OUT else _dt(y), M, cin, out_features,
                                         _dev(tile, "tile", torch.int32), k, _dev(alpha, "alpha", torch.float32),
                                         alpha.numel(), flags, _stream(stream))
    if st != TBN_OK:
        _raise(st)
    return y


def tbn_diag_empty_launch(stream=None) -> None:
    st = lib().tbn_diag_empty_launch(_stream(stream))
    if st != TBN_OK:
        _raise(st)


def tbn_diag_stream(src: torch.Tensor, dst: Optional[torch.Tensor] = None, stream=None) -> None:
    """Streaming read of src (copy into dst if given); measurement aid."""
    nbytes = src.numel() * src.element_size()
    st = lib().tbn_diag_stream(_dev(src, "src"), None if dst is None else _dev(dst, "dst"), nbytes, None, _stream(stream))
    if st != TBN_OK:
        _raise(st)


def tbn_diag_mfma(blocks: int, iters: int, stream=None) -> None:
    st = lib().tbn_diag_mfma(blocks, iters, None, _stream(stream))
    if st != TBN_OK:
        _raise(st)


def tbn_diag_mfma_fp4(blocks: int, iters: int, stream=None) -> None:
    st = lib().tbn_diag_mfma_fp4(blocks, iters, None, _stream(stream))
    if st != TBN_OK:
        _raise(st)
