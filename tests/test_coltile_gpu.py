"""GPU parity of the column-tiled layer (pack and forward, through the C ABI binding) against its CPU oracle:
tile words bit exact, alpha within one float32 ulp, outputs within 1e-5 (float32) / 2e-2 (bfloat16) of the
largest reference magnitude.  Shapes span the 16-byte and the element-wise fold, several fold blocks, every
kernel family behind the +-1 product (small batch, matrix cores, fallbacks) and ragged tails.
"""
import numpy as np
import pytest
import torch

from oracle import coltile_oracle as col
from paper_2407_12075_amd import workloads as wl
from tests.parity_util import assert_close, sample_linear, TOL, max_rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tbn():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2407_12075_amd import tbn as binding
    binding.lib()  # fails loudly if the HIP library is missing
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def ulp_diff(a, b):
    a = np.asarray(a, dtype=np.float32).view(np.int32).astype(np.int64)
    b = np.asarray(b, dtype=np.float32).view(np.int32).astype(np.int64)
    return int(np.abs(a - b).max())


PACK = [
    # out, in, k, n_alpha, separate A
    (2, 4, 2, 2, False),
    (256, 256, 4, 4, False),
    (256, 256, 4, 1, True),
    (37, 1000, 5, 5, True),       # blocks of 200: 16-byte loads, ragged last word
    (33, 999, 3, 3, False),       # blocks of 333: element-wise loads
    (7, 12, 12, 12, False),       # blocks of one column
    (64, 64, 1, 1, False),        # k = 1
    (1000, 4096, 8, 8, False),    # several kernel blocks
    (300, 1030, 5, 1, False),     # blocks of 206: even but not a multiple of 4
]


@pytest.mark.parametrize("out,cin,k,n_alpha,sep", PACK)
def test_pack_coltile_bit_exact(tbn, out, cin, k, n_alpha, sep):
    rng = np.random.default_rng(out + cin + k)
    w = (0.02 * rng.standard_normal((out, cin))).astype(np.float32)
    q = cin // k
    w[0, 0::q] = 0.0                  # an exact zero sum must give bit 0
    if k >= 2 and q >= 2:
        w[0, 1], w[0, 1 + q] = 0.25, -0.25
        w[0, 1 + 2 * q::q] = 0.0
    if k >= 3 and q >= 3:             # a term the float32 sum would lose
        w[0, 2], w[0, 2 + q], w[0, 2 + 2 * q] = 1.0, 2.0 ** -30, -1.0
        w[0, 2 + 3 * q::q] = 0.0
    a = (0.5 * rng.standard_normal((out, cin))).astype(np.float32) if sep else None
    tile_ref, alpha_ref = col.pack_coltile(w, out, cin, k, n_alpha, a_real=a)
    tile, alpha = tbn.tbn_pack_coltile(dev(w), k, n_alpha, a_real=None if a is None else dev(a))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(tile.cpu().numpy().view(np.uint32), tile_ref)
    assert ulp_diff(alpha.cpu().numpy(), alpha_ref) <= 1


FORWARD = [
    # M, in, out, k, n_alpha
    (1, 8, 3, 2, 2),
    (3, 12, 5, 3, 3),            # blocks of 4 columns: element-wise fold for bfloat16
    (8, 256, 256, 4, 4),
    (1, 784, 128, 4, 1),
    (16, 4096, 512, 8, 8),       # small-batch kernel behind the fold
    (200, 1536, 384, 4, 4),
    (130, 2048, 192, 16, 16),    # 128 folded columns: one stage of the matrix-core kernels
    (257, 1000, 130, 5, 5),      # blocks of 200
    (300, 999, 58, 3, 3),        # blocks of 333: element-wise fold, fallback product kernels
    (1500, 1024, 256, 2, 2),     # large batch: matrix-core kernels, 512 folded columns
    (700, 640, 1024, 10, 10),    # ten blocks: two rounds of the fold's loads
    (64, 100, 40, 100, 100),     # blocks of one column
    (5, 64, 7, 1, 1),            # k = 1
]


def _forward_case(tbn, M, cin, out, k, n_alpha, dtype, flags, seed):
    rng = np.random.default_rng(seed)
    w = (0.02 * rng.standard_normal((out, cin))).astype(np.float32)
    x = rng.standard_normal((M, cin)).astype(np.float32)
    bits = None
    if dtype == "bf16":
        bits = wl.f32_to_bf16_bits(x).reshape(M, cin)
        x = wl.bf16_bits_to_f32(bits).reshape(M, cin)
    tile_ref, alpha_ref = col.pack_coltile(w, out, cin, k, n_alpha)
    ref = col.linear_coltiled_forward(x, tile_ref, alpha_ref, out, k, relu=bool(flags & 1))
    xd = dev(x) if bits is None else dev(bits.view(np.int16)).view(torch.bfloat16)
    y = tbn.tbn_linear_coltiled_forward(xd, dev(tile_ref.view(np.int32)), dev(alpha_ref), out, k, flags=flags)
    torch.cuda.synchronize()
    return assert_close(y.float().cpu().numpy().astype(np.float64), ref, dtype,
                        f"column-tiled linear M={M} in={cin} out={out} k={k} {dtype} flags={flags:#x}")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("M,cin,out,k,n_alpha", FORWARD)
def test_coltiled_forward(tbn, M, cin, out, k, n_alpha, dtype):
    _forward_case(tbn, M, cin, out, k, n_alpha, dtype, 0, 100 + M + cin)
    _forward_case(tbn, M, cin, out, k, n_alpha, dtype, tbn.TBN_FLAG_RELU, 200 + M + cin)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("M,cin,out,k,n_alpha", [(200, 1536, 384, 4, 4), (300, 999, 58, 3, 3), (130, 2048, 192, 16, 16)])
def test_coltiled_forward_other_kernel_families(tbn, M, cin, out, k, n_alpha, dtype):
    _forward_case(tbn, M, cin, out, k, n_alpha, dtype, tbn.TBN_FLAG_FORCE_GENERIC, 300 + M)
    _forward_case(tbn, M, cin, out, k, n_alpha, dtype, tbn.TBN_FLAG_LARGE_BATCH, 400 + M)


def test_coltiled_pack_then_forward_on_device_and_workspace_reuse(tbn):
    out, cin, k, M = 512, 2048, 8, 96
    rng = np.random.default_rng(9)
    w = (0.02 * rng.standard_normal((out, cin))).astype(np.float32)
    tile, alpha = tbn.tbn_pack_coltile(dev(w), k, k)
    tile_ref, alpha_ref = col.pack_coltile(w, out, cin, k, k)
    x = rng.standard_normal((M, cin)).astype(np.float32)
    xd = dev(x)
    ws = torch.empty(tbn.tbn_linear_coltiled_workspace_bytes(xd, k), dtype=torch.uint8, device="cuda")
    ws.fill_(0xff)                                  # contents on entry are ignored
    for rows in (M, 40):                            # the second call, smaller, shares the workspace
        y = tbn.tbn_linear_coltiled_forward(xd[:rows].contiguous(), tile, alpha, out, k, workspace=ws)
        torch.cuda.synchronize()
        assert_close(y.cpu().numpy().astype(np.float64), col.linear_coltiled_forward(x[:rows], tile_ref, alpha_ref, out, k),
                     "f32", f"pack + forward on the device, {rows} rows")
    with pytest.raises(tbn.TbnError):
        tbn.tbn_linear_coltiled_forward(xd, tile, alpha, out, k, workspace=ws[: ws.numel() // 2])


def test_coltiled_empty_batch_and_k_equal_in(tbn):
    out, cin = 40, 96
    rng = np.random.default_rng(4)
    w = (0.02 * rng.standard_normal((out, cin))).astype(np.float32)
    tile, alpha = tbn.tbn_pack_coltile(dev(w), cin, cin)          # blocks of one column: the tile is one bit per row
    tile_ref, alpha_ref = col.pack_coltile(w, out, cin, cin, cin)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(tile.cpu().numpy().view(np.uint32), tile_ref)
    assert ulp_diff(alpha.cpu().numpy(), alpha_ref) <= 1
    y = tbn.tbn_linear_coltiled_forward(torch.empty((0, cin), device="cuda"), tile, alpha, out, cin)
    torch.cuda.synchronize()
    assert tuple(y.shape) == (0, out)
    x = rng.standard_normal((70, cin)).astype(np.float32)
    y = tbn.tbn_linear_coltiled_forward(dev(x), tile, alpha, out, cin)
    torch.cuda.synchronize()
    assert_close(y.cpu().numpy().astype(np.float64), col.linear_coltiled_forward(x, tile_ref, alpha_ref, out, cin), "f32",
                 "column-tiled layer with k = in")


def test_coltiled_full_size_sampled(tbn):
    # the metric layer's sizes in the column-tiled layout: sampled outputs, each from the definition
    M, cin, out, k = 8192, 4096, 4096, 8
    q = cin // k
    rng = np.random.default_rng(2407)
    w = (0.02 * rng.standard_normal((out, cin))).astype(np.float32)
    tile, alpha = tbn.tbn_pack_coltile(dev(w), k, k)
    torch.cuda.synchronize()
    tile_ref, alpha_ref = col.pack_coltile(w, out, cin, k, k)
    np.testing.assert_array_equal(tile.cpu().numpy().view(np.uint32), tile_ref)
    g = torch.Generator(device="cuda").manual_seed(12)
    x = torch.randn((M, cin), device="cuda", generator=g).bfloat16()
    y = tbn.tbn_linear_coltiled_forward(x, tile, alpha, out, k)
    torch.cuda.synchronize()
    rows, cols = sample_linear(M, out, cin, out * q, 2000, 5)
    xs = x[torch.from_numpy(rows).cuda()].float().cpu().numpy().astype(np.float64)
    w_hat = col.materialise_coltile(tile_ref, alpha_ref, out, cin, k)
    ref = np.einsum("ij,ij->i", xs, w_hat[cols])
    got = y[torch.from_numpy(rows).cuda(), torch.from_numpy(cols).cuda()].float().cpu().numpy().astype(np.float64)
    scale = np.abs(ref).max()
    assert np.abs(got - ref).max() / scale <= TOL["bf16"]
