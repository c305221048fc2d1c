"""CPU-side checks of the C ABI: the library loads, exports what include/tbn.h declares, and its
argument validation (which runs before any device call) reports the documented status codes."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "tbn.h")
LIB = os.path.join(ROOT, "paper_2407_12075_amd", "libtbn.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2407_12075_amd import build
        build.build(verbose=False)
    from paper_2407_12075_amd import tbn
    return tbn.lib()


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tbn_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_three_entry_points():
    syms = declared_symbols()
    for name in ("tbn_pack_tile", "tbn_linear_forward", "tbn_conv2d_forward", "tbn_tile_words", "tbn_last_error"):
        assert name in syms


def test_library_exports_every_declared_symbol(lib):
    for name in declared_symbols():
        assert hasattr(lib, name), f"libtbn.so does not export {name}"


def test_tile_words(lib):
    assert lib.tbn_tile_words(65536, 4) == 512
    assert lib.tbn_tile_words(784 * 128, 4) == 784          # 25,088 bits: the microcontroller MLP's first layer
    assert lib.tbn_tile_words(33, 1) == 2
    assert lib.tbn_tile_words(32, 1) == 1
    assert lib.tbn_tile_words(10, 3) == 0                    # k must divide n
    assert lib.tbn_tile_words(0, 1) == 0
    assert lib.tbn_tile_words(8, 0) == 0
    assert lib.tbn_tile_words(4096 * 4096, 8) == 65536


def test_pack_workspace_bytes(lib):
    assert lib.tbn_pack_workspace_bytes(10, 3, 1) == 0
    assert lib.tbn_pack_workspace_bytes(16, 4, 2) == 0
    need = lib.tbn_pack_workspace_bytes(4096 * 4096, 8, 8)
    assert need > 0 and need % 8 == 0


def _err(lib):
    return lib.tbn_last_error().decode()


def test_validation_status_codes(lib):
    p = ctypes.c_void_p
    fake = p(256)  # never dereferenced: validation fails first
    # NULL pointers
    assert lib.tbn_pack_tile(None, None, 16, 2, 1, fake, fake, fake, 1 << 20, None) == 1
    assert "NULL" in _err(lib)
    assert lib.tbn_linear_forward(None, fake, 0, 1, 4, 4, fake, 2, fake, 1, 0, None) == 1
    assert lib.tbn_conv2d_forward(fake, None, 0, 1, 1, 4, 4, 2, 3, 3, 1, 1, 0, 0, fake, 2, fake, 1, 0, None) == 1
    # n not divisible by k, n_alpha not in {1, k}
    assert lib.tbn_pack_tile(fake, None, 10, 3, 1, fake, fake, fake, 1 << 20, None) == 2
    assert "divisible" in _err(lib)
    assert lib.tbn_pack_tile(fake, None, 16, 4, 2, fake, fake, fake, 1 << 20, None) == 2
    assert lib.tbn_linear_forward(fake, fake, 0, 1, 5, 3, fake, 2, fake, 1, 0, None) == 2
    assert lib.tbn_linear_forward(fake, fake, 0, -1, 4, 4, fake, 2, fake, 1, 0, None) == 2
    assert lib.tbn_linear_forward(fake, fake, 0, 1, 0, 4, fake, 2, fake, 1, 0, None) == 2
    # kernel larger than the padded input
    assert lib.tbn_conv2d_forward(fake, fake, 0, 1, 1, 2, 2, 2, 5, 5, 1, 1, 0, 0, fake, 2, fake, 1, 0, None) == 2
    assert lib.tbn_conv2d_forward(fake, fake, 0, 1, 1, 4, 4, 2, 3, 3, 0, 1, 0, 0, fake, 2, fake, 1, 0, None) == 2
    # unknown dtype / flag
    assert lib.tbn_linear_forward(fake, fake, 7, 1, 4, 4, fake, 2, fake, 1, 0, None) == 3
    assert lib.tbn_linear_forward(fake, fake, 0, 1, 4, 4, fake, 2, fake, 1, 0x8000, None) == 3
    assert lib.tbn_conv2d_forward(fake, fake, 9, 1, 1, 4, 4, 2, 3, 3, 1, 1, 0, 0, fake, 2, fake, 1, 0, None) == 3
    # workspace too small / missing / misaligned
    assert lib.tbn_pack_tile(fake, None, 1 << 20, 2, 1, fake, fake, fake, 8, None) == 5
    assert lib.tbn_pack_tile(fake, None, 1 << 20, 2, 1, fake, fake, None, 1 << 30, None) == 5
    assert lib.tbn_pack_tile(fake, None, 1 << 20, 2, 1, fake, fake, p(260), 1 << 30, None) == 5
    # empty batch is legal and touches nothing
    assert lib.tbn_linear_forward(fake, fake, 0, 0, 4, 4, fake, 2, fake, 1, 0, None) == 0
    assert lib.tbn_conv2d_forward(fake, fake, 0, 0, 1, 4, 4, 2, 3, 3, 1, 1, 0, 0, fake, 2, fake, 1, 0, None) == 0


def test_column_tiled_entry_points_validate(lib):
    p = ctypes.c_void_p
    fake = p(256)
    assert lib.tbn_pack_coltile_workspace_bytes(16, 10, 4, 4) == 0       # k must divide in, not just out * in
    assert lib.tbn_pack_coltile_workspace_bytes(16, 12, 4, 4) > 0
    assert lib.tbn_linear_coltiled_workspace_bytes(1, 8, 64, 4) == 8 * 16 * 2 + 256
    assert lib.tbn_linear_coltiled_workspace_bytes(0, 3, 10, 5) == 256 + 256
    assert lib.tbn_linear_coltiled_workspace_bytes(0, 3, 10, 4) == 0
    assert lib.tbn_pack_coltile(None, None, 4, 8, 2, 1, fake, fake, fake, 1 << 20, None) == 1
    assert lib.tbn_pack_coltile(fake, None, 16, 10, 4, 4, fake, fake, fake, 1 << 20, None) == 2
    assert "column blocks" in _err(lib)
    assert lib.tbn_pack_coltile(fake, None, 16, 12, 4, 2, fake, fake, fake, 1 << 20, None) == 2
    assert lib.tbn_pack_coltile(fake, None, 1024, 1024, 2, 1, fake, fake, fake, 8, None) == 5
    assert lib.tbn_linear_coltiled_forward(None, fake, 0, 1, 8, 4, fake, 2, fake, 1, 0, fake, 1 << 20, None) == 1
    assert lib.tbn_linear_coltiled_forward(fake, fake, 0, 1, 10, 4, fake, 4, fake, 1, 0, fake, 1 << 20, None) == 2
    assert lib.tbn_linear_coltiled_forward(fake, fake, 0, 1, 8, 4, fake, 2, fake, 3, 0, fake, 1 << 20, None) == 2
    assert lib.tbn_linear_coltiled_forward(fake, fake, 5, 1, 8, 4, fake, 2, fake, 1, 0, fake, 1 << 20, None) == 3
    assert lib.tbn_linear_coltiled_forward(fake, fake, 0, 1, 8, 4, fake, 2, fake, 1, 0, fake, 16, None) == 5
    assert lib.tbn_linear_coltiled_forward(fake, fake, 0, 1, 8, 4, fake, 2, fake, 1, 0, p(264), 1 << 20, None) == 5
    assert lib.tbn_linear_coltiled_forward(fake, fake, 0, 1, 8, 4, fake, 2, fake, 1, 0, None, 1 << 20, None) == 5
    assert lib.tbn_linear_coltiled_forward(fake, fake, 0, 0, 8, 4, fake, 2, fake, 1, 0, fake, 1 << 20, None) == 0


def test_binding_refuses_host_tensors():
    import torch
    from paper_2407_12075_amd import tbn
    w = torch.zeros(16)
    with pytest.raises(ValueError):
        tbn.tbn_pack_tile(w, 2)


# Which kernel family serves which shape is host arithmetic (shapes, alignment, 256 CUs where there is no device):
# the table the design states, pinned here so that a change of a dispatch rule shows up without a GPU.
KERNEL_CHOICE = [
    # dtype, M, in, out, k, flags, x address, expected family
    ("bf16", 8192, 4096, 4096, 8, 0, 0, "block"),          # the metric shape
    ("bf16", 8192, 4096, 16384, 2, 0, 0, "block"),         # more blocks than CUs: the persistent form of the same kernel
    ("bf16", 4096, 4096, 4096, 8, 0, 0, "stream"),         # at most 128 blocks: 64-row half tiles
    ("bf16", 1024, 4096, 4096, 8, 0, 0, "tile"),           # mid batches: a wave per 32 rows
    ("bf16", 64, 4096, 4096, 8, 0, 0, "small-batch"),
    ("bf16", 16, 4096, 4096, 8, 0, 0, "decode"),
    ("bf16", 1, 4096, 4096, 8, 0, 0, "decode"),
    ("bf16", 16, 4096, 4096, 8, "TBN_FLAG_LARGE_BATCH", 0, "small-batch"),   # the flag keeps the decode kernel out
    ("bf16", 8192, 256, 16384, 4, 0, 0, "general"),        # rows of 256 on a large grid
    ("f32", 12608, 384, 1536, 4, 0, 0, "tile"),            # ViT MLP
    ("f32", 12608, 1536, 384, 4, 0, 0, "tile"),
    ("f32", 8192, 196, 384, 4, 0, 0, "direct"),            # row length no multiple of 8
    ("bf16", 8192, 2050, 1026, 2, 0, 0, "direct"),
    ("bf16", 8192, 4096, 4096, 8, 0, 2, "direct"),         # activations not 16-byte aligned
    ("f32", 64, 24, 10, 3, 0, 0, "generic"),               # tile of no whole rows, row length no multiple of 8
    ("bf16", 8192, 4096, 4096, 8, "TBN_FLAG_FORCE_GENERIC", 0, "generic"),
]


@pytest.mark.parametrize("dtype,M,cin,out,k,flags,x_ptr,expected", KERNEL_CHOICE)
def test_kernel_choice(lib, dtype, M, cin, out, k, flags, x_ptr, expected):
    import torch
    from paper_2407_12075_amd import tbn
    dt = torch.float32 if dtype == "f32" else torch.bfloat16
    if isinstance(flags, str):
        flags = getattr(tbn, flags)
    assert tbn.tbn_linear_forward_kernel(dt, M, cin, out, k, 1, flags, x_ptr=x_ptr) == expected


def test_kernel_choice_rejects_what_the_forward_call_rejects(lib):
    import torch
    from paper_2407_12075_amd import tbn
    assert tbn.tbn_linear_forward_kernel(torch.float32, 0, 8, 8, 2) == ""     # empty batch: nothing is launched
    assert tbn.tbn_linear_forward_kernel(torch.float32, 4, 4, 4, 3) == ""     # n not divisible by k
    assert tbn.tbn_linear_forward_kernel(torch.float32, 4, 4, 4, 2, n_alpha=3) == ""
