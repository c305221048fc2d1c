"""GPU parity of the binary-activation layer (sign packing and forward, through the C ABI binding) against its CPU
oracle.  Sign bits are compared bit for bit.  The sums of +-1 products are integers, so wherever an output is one
alpha times one integer (one alpha for the layer, or weight rows inside one tile copy) the float32 output must equal
the oracle's float64 product rounded to float32 bit for bit, and a bfloat16 output that value rounded once more;
rows that cross tile ends with k alphas add a few float32 products and are held to 1e-6 of the largest magnitude.
Shapes span the matrix-core kernel (several blocks, ragged rows and columns, one to three super-steps and more, all
register-set rotations) and the shape-agnostic kernel (rows that are no whole words, tiles shorter than a row,
tiles that end inside words).
"""
import numpy as np
import pytest
import torch

from oracle import binact_oracle as ba
from oracle import tbn_oracle as flat
from paper_2407_12075_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tbn():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2407_12075_amd import tbn as binding
    binding.lib()  # fails loudly if the HIP library is missing
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def bits_dev(xbits):
    return dev(xbits.view(np.int32))


SIGN = [
    # M, in
    (1, 1), (3, 31), (5, 32), (7, 33), (4, 64), (9, 100), (2, 4096), (130, 384), (257, 1000), (64, 8192), (33, 2047),
]


@pytest.mark.parametrize("M,cin", SIGN)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_sign_pack_bit_exact(tbn, M, cin, dtype):
    rng = np.random.default_rng(M * 7 + cin)
    x = rng.standard_normal((M, cin)).astype(np.float32)
    x[rng.random((M, cin)) < 0.05] = 0.0
    x[rng.random((M, cin)) < 0.02] = -0.0
    x.reshape(-1)[:: max(1, x.size // 7)] = np.nan
    x.reshape(-1)[1:: max(1, x.size // 5)] = 1e-40        # a float32 subnormal is greater than zero
    if dtype == "bf16":
        xb = wl.f32_to_bf16_bits(x)
        xv = wl.bf16_bits_to_f32(xb).reshape(M, cin)
        xd = dev(xb.reshape(M, cin).view(np.int16)).view(torch.bfloat16)
    else:
        xv, xd = x, dev(x)
    want = ba.sign_pack(xv)
    got = tbn.tbn_sign_pack(xd)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(got.cpu().numpy().view(np.uint32), want)


def test_sign_pack_unaligned_pointer_takes_the_general_kernel(tbn):
    M, cin = 6, 64
    rng = np.random.default_rng(2)
    x = rng.standard_normal(M * cin + 1).astype(np.float32)
    xd = dev(x)[1:].view(M, cin)                       # 4 bytes off a 16-byte boundary
    got = tbn.tbn_sign_pack(xd)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(got.cpu().numpy().view(np.uint32), ba.sign_pack(x[1:].reshape(M, cin)))


def _layer(M, cin, out, k, n_alpha, seed):
    rng = np.random.default_rng(seed)
    w = (0.02 * rng.standard_normal(out * cin)).astype(np.float32)
    tile, alpha = flat.pack_tile(w, k, n_alpha)
    xbits = rng.integers(0, 2 ** 32, size=(M, (cin + 31) // 32), dtype=np.uint64).astype(np.uint32)
    if cin % 32:
        xbits[:, -1] &= np.uint32((1 << (cin % 32)) - 1)
    return xbits, tile, alpha


def _to_bf16(v32):
    return wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(np.ascontiguousarray(v32, dtype=np.float32))).reshape(v32.shape)


def _check(tbn, M, cin, out, k, n_alpha, dtype, flags=0, seed=0, dirty_padding=False):
    xbits, tile, alpha = _layer(M, cin, out, k, n_alpha, seed + M + cin + out + k)
    ref = ba.linear_forward(xbits, cin, tile, alpha, out, k)
    if flags & 1:
        ref = np.maximum(ref, 0.0)
    send = xbits.copy()
    if dirty_padding and cin % 32:
        send[:, -1] |= np.uint32(~((1 << (cin % 32)) - 1) & 0xFFFFFFFF)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    y = tbn.tbn_linear_forward_binact(bits_dev(send), cin, dev(tile.view(np.int32)), dev(alpha), out, k, dtype=tdt, flags=flags)
    torch.cuda.synchronize()
    got = y.float().cpu().numpy()
    p = cin * out // k
    single_product = n_alpha == 1 or p % cin == 0
    if single_product:
        want = ref.astype(np.float32)                  # alpha * integer is exact in float64: one rounding, as on the GPU
        if dtype == "bf16":
            want = _to_bf16(want)
        np.testing.assert_array_equal(got, want)
    else:
        scale = max(np.abs(ref).max(), 1e-30)
        tol = 1e-6 if dtype == "f32" else 8e-3        # bfloat16: half an ulp of the output is 2^-9 relative
        assert np.abs(got - ref).max() <= tol * scale


MFMA = [
    # M, in, out, k, n_alpha      (tile of whole rows, in % 256 == 0, U % 8 == 0)
    (64, 256, 64, 1, 1),          # one super-step
    (128, 512, 128, 2, 2),        # two
    (100, 768, 136, 1, 1),        # three; ragged rows, 136 columns: a second, mostly empty column block
    (257, 1024, 512, 4, 4),       # four: tail of one after a round of three; three row blocks
    (70, 1280, 80, 2, 1),         # five: tail of two; 40 distinct columns
    (300, 4096, 1024, 8, 8),      # sixteen super-steps, 128 distinct columns
    (1, 4096, 64, 8, 8),          # a single batch row, eight distinct columns
    (513, 2048, 768, 3, 3),       # 256 distinct columns: two column blocks
    (2100, 1536, 4096, 2, 2),     # 17 x 16 blocks, more than the chip has CUs, six super-steps
]


@pytest.mark.parametrize("M,cin,out,k,n_alpha", MFMA)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_forward_matrix_core_kernel_exact(tbn, M, cin, out, k, n_alpha, dtype):
    _check(tbn, M, cin, out, k, n_alpha, dtype)


@pytest.mark.parametrize("M,cin,out,k,n_alpha", [MFMA[3], MFMA[4]])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_forward_matrix_core_kernel_relu(tbn, M, cin, out, k, n_alpha, dtype):
    _check(tbn, M, cin, out, k, n_alpha, dtype, flags=1)


@pytest.mark.parametrize("M,cin,out,k,n_alpha", [MFMA[1], MFMA[3], MFMA[5]])
def test_matrix_core_and_general_kernel_agree_bit_for_bit(tbn, M, cin, out, k, n_alpha):
    xbits, tile, alpha = _layer(M, cin, out, k, n_alpha, 5)
    a = (bits_dev(xbits), cin, dev(tile.view(np.int32)), dev(alpha), out, k)
    y0 = tbn.tbn_linear_forward_binact(*a)
    y1 = tbn.tbn_linear_forward_binact(*a, flags=0x100)
    torch.cuda.synchronize()
    assert torch.equal(y0, y1)


GENERIC = [
    # M, in, out, k, n_alpha
    (3, 40, 12, 4, 4),            # rows that are no whole words
    (2, 35, 6, 15, 15),           # p = 14: several tile copies inside one row, tile ends inside words
    (5, 33, 4, 1, 1),
    (4, 64, 8, 8, 1),
    (9, 100, 30, 3, 3),           # p = 1000: rows cross tile ends
    (7, 96, 10, 960, 960),        # p = 1: every weight is the same bit
    (16, 384, 24, 4, 1),          # whole words, tile of whole rows, too few distinct columns for the other kernel
    (33, 1000, 64, 5, 5),
    (2, 4096, 6, 3, 3),           # in % 256 == 0 but two distinct columns
]


# tile of whole rows with shapes the matrix-core kernel declines: the direct kernel (a thread per batch row, 32 distinct
# columns per workgroup, tile words through LDS)
DIRECT = [
    (300, 196, 384, 4, 4),        # rows of 196 bits: six whole words and a masked one; 96 distinct columns
    (150, 1000, 250, 5, 5),       # 50 distinct columns: two column groups, the second ragged
    (131, 4128, 64, 2, 1),        # 129 words per row: two staging passes, the second with one word; ragged row block
    (40, 3000, 96, 3, 3),         # rows start at bit offsets that are no multiples of 32
    (1, 77, 33, 1, 1),            # k = 1, odd everything
    (260, 320, 128, 2, 2),        # whole words, 64 distinct columns (a multiple of 32: sign bits out take this kernel too)
]


@pytest.mark.parametrize("flags", [0, 0x100])   # default dispatch; the one-thread-per-output kernel forced
@pytest.mark.parametrize("M,cin,out,k,n_alpha", GENERIC + DIRECT)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_forward_general_kernel(tbn, M, cin, out, k, n_alpha, dtype, flags):
    _check(tbn, M, cin, out, k, n_alpha, dtype, flags=flags, dirty_padding=True)


def _random_shapes():
    rng = np.random.default_rng(20240712)
    shapes = []
    for i in range(36):
        if i % 3 == 0:   # shapes of the matrix-core kernel: in a multiple of 256, tile of whole rows, U a multiple of 8
            cin = 256 * int(rng.integers(1, 9))
            U = 8 * int(rng.integers(1, 40))
            k = int(rng.choice([1, 2, 3, 4, 5, 8]))
            shapes.append((int(rng.integers(1, 400)), cin, U * k, k, int(rng.choice([1, k]))))
        else:
            cin, out = int(rng.integers(1, 300)), int(rng.integers(1, 120))
            n = cin * out
            divs = [d for d in range(1, min(n, 64) + 1) if n % d == 0]
            k = int(rng.choice(divs))
            shapes.append((int(rng.integers(1, 40)), cin, out, k, int(rng.choice([1, k]))))
    return shapes


@pytest.mark.parametrize("M,cin,out,k,n_alpha", _random_shapes())
def test_forward_random_shapes(tbn, M, cin, out, k, n_alpha):
    _check(tbn, M, cin, out, k, n_alpha, "f32" if (M + cin) % 2 else "bf16", flags=(M % 2), dirty_padding=True)


def test_forward_relu_general_kernel(tbn):
    _check(tbn, 9, 100, 30, 3, 3, "f32", flags=1)


def _check_sign_out(tbn, M, cin, out, k, n_alpha, flags=0):
    xbits, tile, alpha = _layer(M, cin, out, k, n_alpha, 3 + M + cin + out + k)
    if n_alpha > 1:
        alpha[1] = -alpha[1]                      # a negative alpha flips the signs of its copy
    ref = ba.linear_forward(xbits, cin, tile, alpha, out, k)
    want = ba.sign_pack(ref)
    y = tbn.tbn_linear_forward_binact(bits_dev(xbits), cin, dev(tile.view(np.int32)), dev(alpha), out, k, flags=0x4000 | flags)
    torch.cuda.synchronize()
    got = y.cpu().numpy().view(np.uint32)
    assert got.shape == want.shape
    p = cin * out // k
    if n_alpha == 1 or p % cin == 0:
        np.testing.assert_array_equal(got, want)
    else:
        # rows that cross tile ends add float32 products: a bit may differ only where the output is zero to rounding
        diff = got ^ want
        j = np.arange(out)
        bad = ((diff[:, j // 32] >> (j % 32).astype(np.uint32)) & 1).astype(bool)
        assert np.all(np.abs(ref[bad]) <= 1e-6 * np.abs(ref).max())
        assert np.all((got[:, -1] >> np.uint32(out % 32 or 32)) == 0 if out % 32 else True)


@pytest.mark.parametrize("M,cin,out,k,n_alpha", [MFMA[0], MFMA[1], MFMA[3], MFMA[5], MFMA[7], MFMA[8]])
def test_sign_out_matrix_core_kernel(tbn, M, cin, out, k, n_alpha):
    _check_sign_out(tbn, M, cin, out, k, n_alpha)


@pytest.mark.parametrize("flags", [0, 0x100])
@pytest.mark.parametrize("M,cin,out,k,n_alpha", GENERIC + DIRECT + [MFMA[2], MFMA[4], MFMA[6]])
def test_sign_out_general_kernel(tbn, M, cin, out, k, n_alpha, flags):
    _check_sign_out(tbn, M, cin, out, k, n_alpha, flags=flags)


def test_sign_out_both_kernels_agree_and_relu_changes_nothing(tbn):
    M, cin, out, k, n_alpha = MFMA[3]
    xbits, tile, alpha = _layer(M, cin, out, k, n_alpha, 8)
    a = (bits_dev(xbits), cin, dev(tile.view(np.int32)), dev(alpha), out, k)
    y0 = tbn.tbn_linear_forward_binact(*a, flags=0x4000)
    y1 = tbn.tbn_linear_forward_binact(*a, flags=0x4000 | 0x100)
    y2 = tbn.tbn_linear_forward_binact(*a, flags=0x4000 | 0x1)
    torch.cuda.synchronize()
    assert torch.equal(y0, y1) and torch.equal(y0, y2)


def test_chain_of_two_layers_on_bits(tbn):
    """real activations -> sign bits -> layer (bits out) -> layer (real out), against the oracle's chain."""
    M, cin, hid, out = 200, 1024, 2048, 512
    rng = np.random.default_rng(12)
    x = rng.standard_normal((M, cin)).astype(np.float32)
    t1, a1 = flat.pack_tile((0.02 * rng.standard_normal(hid * cin)).astype(np.float32), 4, 4)
    t2, a2 = flat.pack_tile((0.02 * rng.standard_normal(out * hid)).astype(np.float32), 2, 2)
    xb = tbn.tbn_sign_pack(dev(x))
    hb = tbn.tbn_linear_forward_binact(xb, cin, dev(t1.view(np.int32)), dev(a1), hid, 4, flags=0x4000)
    y = tbn.tbn_linear_forward_binact(hb, hid, dev(t2.view(np.int32)), dev(a2), out, 2)
    torch.cuda.synchronize()
    hb_ref = ba.linear_forward_signs(ba.sign_pack(x), cin, t1, a1, hid, 4)
    np.testing.assert_array_equal(hb.cpu().numpy().view(np.uint32), hb_ref)
    ref = ba.linear_forward(hb_ref, hid, t2, a2, out, 2)
    np.testing.assert_array_equal(y.cpu().numpy(), ref.astype(np.float32))


def test_end_to_end_from_real_activations(tbn):
    """sign_pack then forward on the bits it wrote, against the oracle on the real activations."""
    w = wl.METRIC
    M, cin, out, k = 192, w.cin, w.cout, w.k
    xv, xb = wl.draw_x((M, cin), w.cfg, w.layer, "bf16")
    tile, alpha = flat.pack_tile(wl.draw_w_real(w.n, w.cfg, w.layer), k, w.n_alpha)
    xd = dev(xb.view(np.int16)).view(torch.bfloat16)
    bits = tbn.tbn_sign_pack(xd)
    y = tbn.tbn_linear_forward_binact(bits, cin, dev(tile.view(np.int32)), dev(alpha), out, k, dtype=torch.bfloat16)
    torch.cuda.synchronize()
    ref = ba.linear_forward(ba.sign_pack(xv), cin, tile, alpha, out, k)
    np.testing.assert_array_equal(y.float().cpu().numpy(), _to_bf16(ref.astype(np.float32)))


def test_metric_shape_sampled_rows(tbn):
    """The headline layer at its full batch, in the launch shape the benchmark times; 64 sampled rows against the
    oracle, and the replicated-column structure on every row."""
    w = wl.METRIC
    M, cin, out, k = w.M, w.cin, w.cout, w.k
    rng = np.random.default_rng(77)
    xbits = rng.integers(0, 2 ** 32, size=(M, cin // 32), dtype=np.uint64).astype(np.uint32)
    tile, alpha = flat.pack_tile(wl.draw_w_real(w.n, w.cfg, w.layer), k, w.n_alpha)
    y = tbn.tbn_linear_forward_binact(bits_dev(xbits), cin, dev(tile.view(np.int32)), dev(alpha), out, k, dtype=torch.bfloat16)
    torch.cuda.synchronize()
    rows = np.sort(rng.choice(M, size=64, replace=False))
    rows[0], rows[-1] = 0, M - 1
    ref = ba.linear_forward(xbits[rows], cin, tile, alpha, out, k)
    got = y[torch.from_numpy(rows).cuda()].float().cpu().numpy()
    np.testing.assert_array_equal(got, _to_bf16(ref.astype(np.float32)))
    # every replica is the first one scaled: |y[:, t*U + u]| / alpha[t] is the same integer for all t
    U = out // k
    z = y.float().view(M, k, U) / dev(alpha).view(1, k, 1)
    assert torch.all((z - z[:, :1, :]).abs() <= 2.0 ** -7 * z[:, :1, :].abs() + 1e-6)


def test_empty_batch_and_errors(tbn):
    tile = torch.zeros(8, dtype=torch.int32, device="cuda")
    alpha = torch.ones(1, device="cuda")
    y = tbn.tbn_linear_forward_binact(torch.zeros((0, 2), dtype=torch.int32, device="cuda"), 64, tile, alpha, 4, 1)
    assert y.shape == (0, 4)
    bits = torch.zeros((2, 2), dtype=torch.int32, device="cuda")
    with pytest.raises(Exception):
        tbn.tbn_linear_forward_binact(bits, 64, tile, alpha, 4, 3)          # 256 weights are not divisible by 3
    with pytest.raises(Exception):
        tbn.tbn_linear_forward_binact(bits, 64, tile, alpha, 4, 1, flags=0x400)   # a flag of another entry point
    with pytest.raises(ValueError):
        tbn.tbn_linear_forward_binact(bits, 96, tile, alpha, 4, 1)          # rows of 3 words expected
    assert tbn.tbn_sign_pack(torch.zeros((0, 5), device="cuda")).shape == (0, 1)
