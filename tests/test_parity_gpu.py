"""GPU parity: libtbn (through the C ABI binding) against the CPU oracle on identical seeded
inputs.  Tile words must be bit exact, alpha within one float32 ulp, layer outputs within the
stated tolerance (max error relative to the largest reference magnitude: 1e-5 for float32
activations, 2e-2 for bfloat16).

Small cases are compared element by element and span several kernel tiles plus ragged tails;
the full benchmark sizes are compared on sampled outputs that the oracle computes one by one
(random ones plus rows / columns at tile, alpha and kernel-tile boundaries).
"""
import numpy as np
import pytest
import torch

from oracle import tbn_oracle as orc
from paper_2407_12075_amd import workloads as wl
from tests.parity_util import TOL, assert_close, max_rel_err, sample_linear

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tbn():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2407_12075_amd import tbn as binding
    binding.lib()  # fails loudly if the HIP library is missing
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def x_to_device(x_vals, x_bits):
    """float32 values -> float32 tensor; bfloat16 bit patterns -> bfloat16 tensor."""
    if x_bits is None:
        return dev(x_vals)
    return dev(x_bits.view(np.int16)).view(torch.bfloat16)


def y_to_numpy(y):
    return y.float().cpu().numpy().astype(np.float64)


def tile_to_numpy(t):
    return t.cpu().numpy().view(np.uint32)


def ulp_diff(a, b):
    a = np.asarray(a, dtype=np.float32).view(np.int32).astype(np.int64)
    b = np.asarray(b, dtype=np.float32).view(np.int32).astype(np.int64)
    return int(np.abs(a - b).max())


# ------------------------------------------------------------------------------ pack
PACK_CASES = [
    # n, k, n_alpha, separate A
    (8, 2, 2, False),
    (65536, 4, 1, False),            # configuration 1
    (65536, 4, 4, True),
    (1000 * 37, 37, 37, False),      # p = 1000 (multiple of 4, ragged last word)
    (999 * 5, 5, 5, True),           # p = 999: scalar-load variant
    (4097 * 3, 3, 1, False),
    (12, 12, 12, False),             # p = 1
    (64, 1, 1, False),               # k = 1
    (3 * 5000 * 16, 16, 16, False),  # several blocks, ragged tail block
    (100 * 6400, 100, 100, False),   # more than 64 rows: every wave writes its own partial sums
    (65 * 4100, 65, 1, True),
    (2 * 1048580, 2, 2, True),
]


@pytest.mark.parametrize("n,k,n_alpha,sep", PACK_CASES)
def test_pack_tile_bit_exact(tbn, n, k, n_alpha, sep):
    rng = np.random.default_rng(n + k)
    w = (0.02 * rng.standard_normal(n)).astype(np.float32)
    p = n // k
    if p >= 4:   # plant exact cancellations (s = 0 must give bit 0) and a value the float32 sum would lose
        w[0:n:p] = 0.0
        if k >= 2:
            w[1] = 0.25
            w[1 + p] = -0.25
            w[1 + 2 * p:n:p] = 0.0
        if k >= 3:
            w[2], w[2 + p], w[2 + 2 * p] = 1.0, 2.0 ** -30, -1.0
            w[2 + 3 * p:n:p] = 0.0
    a = (0.5 * rng.standard_normal(n)).astype(np.float32) if sep else None
    tile_ref, alpha_ref = orc.pack_tile(w, k, n_alpha, a_real=a)
    tile, alpha = tbn.tbn_pack_tile(dev(w), k, n_alpha, a_real=None if a is None else dev(a))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(tile_to_numpy(tile), tile_ref)
    assert ulp_diff(alpha.cpu().numpy(), alpha_ref) <= 1


def test_pack_tile_is_reproducible_and_handles_offset_pointers(tbn):
    rng = np.random.default_rng(3)
    n, k = 8 * 4104, 8
    buf = dev((0.02 * rng.standard_normal(n + 3)).astype(np.float32))
    w = buf[3:]                       # 4-byte aligned only -> scalar-load variant
    tile_ref, alpha_ref = orc.pack_tile(w.cpu().numpy(), k, k)
    t1, a1 = tbn.tbn_pack_tile(w, k, k)
    t2, a2 = tbn.tbn_pack_tile(w.clone(), k, k)   # 16-byte aligned -> vector variant
    torch.cuda.synchronize()
    np.testing.assert_array_equal(tile_to_numpy(t1), tile_ref)
    np.testing.assert_array_equal(tile_to_numpy(t2), tile_ref)
    assert ulp_diff(a1.cpu().numpy(), alpha_ref) <= 1 and ulp_diff(a2.cpu().numpy(), alpha_ref) <= 1


# ------------------------------------------------------------------------------ linear, small
LINEAR_SMALL = [
    # M, in, out, k, n_alpha
    (8, 256, 256, 4, 1),       # configuration 1
    (1, 784, 128, 4, 4),       # microcontroller MLP first layer, per-tile alpha
    (3, 5, 3, 3, 3),
    (2, 10, 6, 4, 4),          # p = 15: tile ends mid-row
    (1, 12, 5, 10, 10),        # p = 6 < in
    (2, 9, 4, 36, 36),         # p = 1
    (5, 33, 31, 1, 1),         # k = 1
    (70, 100, 96, 6, 6),       # p = 1600 = 16 rows
    (130, 200, 120, 5, 5),     # p = 4800 = 24 rows, ragged M
    (33, 3000 // 8, 384, 9, 9),    # p = 16000, rows per tile 42 2/3: mid-row tile and alpha boundaries
    (257, 520, 260, 4, 1),     # aligned, in % 32 != 0
    (96, 512, 512, 4, 1),      # time-series encoder shape
    (16, 1024, 1024, 8, 8),
    (200, 384, 1536, 4, 1),    # ViT MLP shapes at small batch
    (200, 1536, 384, 4, 1),
    (150, 200, 90, 4, 4),      # p = 4500 = 22.5 rows: 45 distinct rows, tile ends mid-row, odd U
    (150, 200, 90, 4, 1),
    (4, 200, 90, 4, 4),
    (40, 3000, 96, 9, 9),      # p = 32000 = 10 2/3 rows, 32 distinct rows, in % 32 != 0
    (16, 3000, 96, 9, 9),
    (1, 3000, 96, 9, 9),
    (300, 264, 136, 3, 3),     # p = 11968 = 45 1/3 rows: no row repeats at all (U = out)
    (129, 64, 64, 64, 64),     # p = in: every row is the whole tile
    (64, 1024, 512, 4, 4),     # largest batch the small-batch kernel takes whatever the problem size
    (17, 512, 256, 8, 8),      # two batch slabs, the second almost empty
    (48, 200, 90, 4, 4),       # small batch with tile ends inside rows
    (65, 1024, 512, 4, 4),     # smallest batch the large-batch kernels can take
    (512, 1024, 1024, 4, 4),   # 16 x 32 = 512 workgroups of the small-batch kernel: its largest bf16 problem
    (513, 1024, 1024, 4, 4),   # one more batch slab: bf16 goes to the large-batch kernel, float32 stays
    (1040, 1024, 512, 4, 4),   # 8 x 65 workgroups: float32 on the small-batch kernel with many batch slabs
    (2, 4096, 40, 5, 5),       # 8 distinct rows only: a partly filled column tile
    # K-split matrix-core kernels: stage counts, tails, window wraps
    (130, 64, 256, 2, 2),      # one stage: the second K group only sees a stage past the end
    (130, 192, 128, 2, 1),     # three stages: 2 + 1
    (256, 904, 72, 3, 3),      # in % 64 = 8: a last stage with one valid piece
    (140, 1000, 130, 5, 5),    # 26 distinct rows: a partly filled column block
    (300, 1160, 58, 4, 4),     # p = 16820 = 14.5 rows: windows cross the tile end in many stages
    (129, 2048, 192, 3, 3),    # long enough for the steady-state loop, second row block one row
    (200, 1096, 220, 5, 5),    # steady-state loop, then a ragged last stage
    (70, 8192, 80, 4, 4),      # 64 stages per K group
    (257, 1544, 135, 5, 5),    # p = 41688 = 27 rows: odd number of distinct rows, p % 32 = 24
    (140, 600, 1024, 6, 6),    # tile ends inside rows with 16-byte stores: 512 distinct rows, 2 replicas, alpha steps inside a lane's 8 columns
    (150, 1024, 256, 2, 2),    # aligned, 128 distinct rows: one column block, 16-byte stores, second row block partly filled
    (4, 40, 16, 4, 1),         # p = 160: smallest tile the small-batch kernel takes
    (3, 160, 9, 9, 9),         # p = in = 160
    # row lengths that are no multiple of 8, tile of whole rows: the direct kernel (a thread per batch row, 16 distinct columns)
    (300, 196, 384, 4, 4),     # a Mixer's token-mixing layer: 96 distinct columns, rows of 196 elements
    (70, 300, 300, 4, 1),      # 75 distinct columns: five column groups, the last ragged; one alpha
    (33, 2050, 1026, 2, 2),    # five staging passes of K, the last one short
    (200, 77, 33, 3, 3),       # odd row length: one element per load (bfloat16 rows start at odd 2-byte offsets)
    (1, 196, 256, 1, 1),       # one batch row, k = 1
    (131, 1001, 26, 2, 1),     # odd row length over two staging passes; two row blocks, the second with three rows
]


# More than 256 blocks of 128 x 128 and a short K loop: the bf16 kernel runs in its form with two workgroups
# per CU (32-element stages).
LINEAR_MANY_BLOCKS = [
    (4224, 1000, 1024, 1, 1),   # 33 x 8 blocks; in % 64 = 40: the last stage of one K group is partly filled
    (8320, 200, 1024, 2, 2),    # 65 x 4 blocks, the last row block all valid; 512 distinct rows, 2 replicas
    (8300, 264, 544, 3, 3),     # tile ends inside rows: no row repeats, 5 column blocks, ragged row and column blocks
    (4230, 32, 1040, 1, 1),     # one stage: the second K group only sees a stage past the end
    (4230, 96, 1040, 2, 1),     # three stages
    (4500, 520, 1024, 1, 1),    # in % 64 = 8: a last stage with one valid piece
    (4224, 2048, 1024, 1, 1),   # 32 rounds of the steady-state loop
    (4224, 448, 1024, 1, 1),    # the shortest K with a steady-state round
]


def _linear_case(tbn, M, cin, cout, k, n_alpha, dtype, flags, seed):
    rng = np.random.default_rng(seed)
    w = (0.02 * rng.standard_normal(cin * cout)).astype(np.float32)
    x = rng.standard_normal((M, cin)).astype(np.float32)
    bits = None
    if dtype == "bf16":
        bits = wl.f32_to_bf16_bits(x)
        x = wl.bf16_bits_to_f32(bits).reshape(M, cin)
        bits = bits.reshape(M, cin)
    tile_ref, alpha_ref = orc.pack_tile(w, k, n_alpha)
    ref = orc.linear_forward(x, tile_ref, alpha_ref, cout, k)
    if flags & 1:
        ref = np.maximum(ref, 0.0)
    tile, alpha = dev(tile_ref.view(np.int32)), dev(alpha_ref)
    y = tbn.tbn_linear_forward(x_to_device(x, bits), tile, alpha, cout, k, flags=flags)
    torch.cuda.synchronize()
    return assert_close(y_to_numpy(y), ref, dtype, f"linear M={M} in={cin} out={cout} k={k} {dtype} flags={flags:#x}")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("M,cin,cout,k,n_alpha", LINEAR_SMALL)
def test_linear_small_generic_kernel(tbn, M, cin, cout, k, n_alpha, dtype):
    _linear_case(tbn, M, cin, cout, k, n_alpha, dtype, tbn.TBN_FLAG_FORCE_GENERIC, 1000 + M + cin)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("M,cin,cout,k,n_alpha", LINEAR_SMALL)
def test_linear_small_default_dispatch(tbn, M, cin, cout, k, n_alpha, dtype):
    _linear_case(tbn, M, cin, cout, k, n_alpha, dtype, 0, 2000 + M + cin)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("M,cin,cout,k,n_alpha", [s for s in LINEAR_SMALL if s[0] > 64])
def test_linear_small_large_batch_kernels(tbn, M, cin, cout, k, n_alpha, dtype):
    # small problems at batches above 64 go to the small-batch kernel by default; this keeps them on the
    # large-batch kernels, whose stage counts, tails and window wraps the shapes were chosen for
    _linear_case(tbn, M, cin, cout, k, n_alpha, dtype, tbn.TBN_FLAG_LARGE_BATCH, 2500 + M + cin)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("M,cin,cout,k,n_alpha", LINEAR_MANY_BLOCKS)
def test_linear_many_blocks_short_k(tbn, M, cin, cout, k, n_alpha, dtype):
    _linear_case(tbn, M, cin, cout, k, n_alpha, dtype, tbn.TBN_FLAG_RELU if cin == 200 else 0, 2700 + M + cin)


def _random_many_block_shapes(count, seed):
    rng = np.random.default_rng(seed)
    shapes = []
    while len(shapes) < count:
        M = int(rng.integers(4200, 8400))
        cin = int(rng.choice([32, 40, 64, 72, 128, 200, 256, 328, 456, 512, 600]))
        cout = int(rng.integers(520, 1200))
        n = cin * cout
        k = int(rng.choice([d for d in range(1, 9) if n % d == 0]))
        p = n // k
        U = min(cout, p // np.gcd(cin, p))
        if p < cin or ((M + 127) // 128) * ((U + 127) // 128) <= 256:
            continue
        shapes.append((M, cin, cout, k, k if rng.random() < 0.6 else 1))
    return shapes


@pytest.mark.parametrize("M,cin,cout,k,n_alpha", _random_many_block_shapes(10, 1207))
def test_linear_random_many_block_shapes(tbn, M, cin, cout, k, n_alpha):
    _linear_case(tbn, M, cin, cout, k, n_alpha, "bf16", 0, 7000 + M + cin)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("M,cin,cout,k,n_alpha", [(8, 256, 256, 4, 1), (130, 200, 120, 5, 5), (1, 784, 128, 4, 4)])
def test_linear_fused_relu(tbn, M, cin, cout, k, n_alpha, dtype):
    _linear_case(tbn, M, cin, cout, k, n_alpha, dtype, tbn.TBN_FLAG_RELU, 3000 + M)
    _linear_case(tbn, M, cin, cout, k, n_alpha, dtype, tbn.TBN_FLAG_RELU | tbn.TBN_FLAG_FORCE_GENERIC, 3000 + M)
    _linear_case(tbn, M, cin, cout, k, n_alpha, dtype, tbn.TBN_FLAG_RELU | tbn.TBN_FLAG_LARGE_BATCH, 3000 + M)


def test_config1_pack_then_forward_on_device(tbn):
    c = wl.CFG1
    w = wl.draw_w_real(c.n, c.cfg, c.layer)
    x, _ = wl.draw_x((c.M, c.cin), c.cfg, c.layer, c.dtype)
    tile_ref, alpha_ref = orc.pack_tile(w, c.k, c.n_alpha)
    tile, alpha = tbn.tbn_pack_tile(dev(w), c.k, c.n_alpha)
    y = tbn.tbn_linear_forward(dev(x), tile, alpha, c.cout, c.k)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(tile_to_numpy(tile), tile_ref)
    assert ulp_diff(alpha.cpu().numpy(), alpha_ref) <= 1
    assert_close(y_to_numpy(y), orc.linear_forward(x, tile_ref, alpha_ref, c.cout, c.k), "f32", c.name)


# ------------------------------------------------------------------------------ linear, full size
def _linear_full(tbn, c, samples=4096, full=False):
    w = wl.draw_w_real(c.n, c.cfg, c.layer)
    x, bits = wl.draw_x((c.M, c.cin), c.cfg, c.layer, c.dtype)
    tile_ref, alpha_ref = orc.pack_tile(w, c.k, c.n_alpha)
    tile, alpha = tbn.tbn_pack_tile(dev(w), c.k, c.n_alpha)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(tile_to_numpy(tile), tile_ref)
    assert ulp_diff(alpha.cpu().numpy(), alpha_ref) <= 1
    y = tbn.tbn_linear_forward(x_to_device(x, bits), dev(tile_ref.view(np.int32)), dev(alpha_ref), c.cout, c.k)
    torch.cuda.synchronize()
    yh = y_to_numpy(y)
    assert np.all(np.isfinite(yh))
    if full:
        ref = orc.linear_forward(x, tile_ref, alpha_ref, c.cout, c.k)
        return assert_close(yh, ref, c.dtype, c.name)
    rows, cols = sample_linear(c.M, c.cout, c.cin, c.p, samples, seed=c.cfg * 31 + c.k)
    ref = orc.linear_forward_at(x, tile_ref, alpha_ref, c.cout, c.k, rows, cols)
    # scale the error by a magnitude typical of the whole output, estimated from the samples
    return assert_close(yh[rows, cols], ref, c.dtype, f"{c.name} ({len(rows)} sampled outputs)")


@pytest.mark.parametrize("c", wl.CFG2, ids=lambda c: c.name)
def test_config2_vit_mlp(tbn, c):
    _linear_full(tbn, c, full=True)


@pytest.mark.parametrize("c", wl.CFG4, ids=lambda c: c.name)
def test_config4_decode(tbn, c):
    _linear_full(tbn, c, full=True)


def test_metric_shape_b8192(tbn):
    # every one of the 8192 x 4096 outputs against the oracle (a few seconds of CPU time)
    _linear_full(tbn, wl.METRIC, full=True)


@pytest.mark.parametrize("c", wl.CFG5 + wl.CFG5_MISALIGNED, ids=lambda c: c.name)
def test_config5_ffn(tbn, c):
    _linear_full(tbn, c)


@pytest.mark.parametrize("c", wl.EXTRA, ids=lambda c: c.name)
def test_extra_paper_shapes(tbn, c):
    _linear_full(tbn, c, full=True)


def _random_linear_shapes(count, seed):
    """Seeded random legal shapes: any M, in, out and any k that divides in*out (n_alpha 1 or k)."""
    rng = np.random.default_rng(seed)
    shapes = []
    while len(shapes) < count:
        M = int(rng.choice([1, 2, 7, 16, 33, 64, 65, 100, 129, 200, 257, 300]))
        cin = int(rng.choice([8, 24, 40, 64, 72, 96, 128, 200, 256, 328, 512, 600, 1000, 1024, 1536, 2048]))
        if rng.random() < 0.25:
            cin = int(rng.integers(1, 400))            # also inner sizes that are not multiples of 8
        cout = int(rng.integers(1, 700))
        n = cin * cout
        divisors = [d for d in range(1, 65) if n % d == 0]
        k = int(rng.choice(divisors))
        n_alpha = k if rng.random() < 0.6 else 1
        shapes.append((M, cin, cout, k, n_alpha))
    return shapes


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("M,cin,cout,k,n_alpha", _random_linear_shapes(40, 20240712))
def test_linear_random_shapes(tbn, M, cin, cout, k, n_alpha, dtype):
    _linear_case(tbn, M, cin, cout, k, n_alpha, dtype, 0, 5000 + M + cin)
    _linear_case(tbn, M, cin, cout, k, n_alpha, dtype, tbn.TBN_FLAG_RELU, 6000 + M + cin)
    if M > 64:
        _linear_case(tbn, M, cin, cout, k, n_alpha, dtype, tbn.TBN_FLAG_RELU | tbn.TBN_FLAG_LARGE_BATCH, 6000 + M + cin)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_linear_output_pointer_not_16_byte_aligned(tbn, dtype):
    # the 16-byte store form needs an aligned y; one element further on the element-wise form has to take over
    M, cin, cout, k, n_alpha = 200, 512, 512, 4, 4
    rng = np.random.default_rng(77)
    w = (0.02 * rng.standard_normal(cin * cout)).astype(np.float32)
    x = rng.standard_normal((M, cin)).astype(np.float32)
    bits = None
    if dtype == "bf16":
        bits = wl.f32_to_bf16_bits(x)
        x = wl.bf16_bits_to_f32(bits).reshape(M, cin)
        bits = bits.reshape(M, cin)
    tile_ref, alpha_ref = orc.pack_tile(w, k, n_alpha)
    ref = orc.linear_forward(x, tile_ref, alpha_ref, cout, k)
    xd = x_to_device(x, bits)
    big = torch.zeros(M * cout + 8, dtype=xd.dtype, device="cuda")
    y = big[1:1 + M * cout].view(M, cout)
    for flags in (tbn.TBN_FLAG_LARGE_BATCH, 0):
        big.zero_()
        tbn.tbn_linear_forward(xd, dev(tile_ref.view(np.int32)), dev(alpha_ref), cout, k, y=y, flags=flags)
        torch.cuda.synchronize()
        assert_close(y_to_numpy(y), ref, dtype, f"linear with y offset by one element, {dtype}, flags={flags:#x}")
        assert float(big[0]) == 0.0 and float(big[1 + M * cout:].abs().max()) == 0.0   # nothing written outside y


def test_aligned_output_blocks_are_scaled_copies_at_full_size(tbn):
    # a property that holds at any size: with tiles made of whole rows, output block c equals
    # alpha_c / alpha_0 times block 0 (computed from float32 sums, compared after bf16 rounding)
    c = wl.METRIC
    w = wl.draw_w_real(c.n, c.cfg, c.layer)
    x, bits = wl.draw_x((c.M, c.cin), c.cfg, c.layer, c.dtype)
    tile_ref, alpha_ref = orc.pack_tile(w, c.k, c.n_alpha)
    ones = np.ones_like(alpha_ref)
    y = tbn.tbn_linear_forward(x_to_device(x, bits), dev(tile_ref.view(np.int32)), dev(ones), c.cout, c.k)
    torch.cuda.synchronize()
    U = c.p // c.cin
    yb = y.view(c.M, c.k, U)
    for r in range(1, c.k):
        assert torch.equal(yb[:, 0], yb[:, r])


def test_bound_calls_repeat_the_library_call(tbn):
    """tbn_bind marshals a call once; the callable it returns makes the same library call on the same buffers."""
    g = torch.Generator(device="cuda")
    g.manual_seed(5)
    M, cin, cout, k = 300, 512, 1024, 4
    w = torch.randn(cin * cout, device="cuda", generator=g)
    x = torch.randn((M, cin), device="cuda", generator=g).to(torch.bfloat16)
    tile_ref, alpha_ref = tbn.tbn_pack_tile(w, k, k)
    y_ref = tbn.tbn_linear_forward(x, tile_ref, alpha_ref, cout, k)
    tile = torch.zeros_like(tile_ref)
    alpha = torch.zeros_like(alpha_ref)
    ws = torch.empty(tbn.tbn_pack_workspace_bytes(w.numel(), k, k) + 8, dtype=torch.uint8, device="cuda")
    y = torch.zeros_like(y_ref)
    pack = tbn.tbn_bind(tbn.tbn_pack_tile, w, k, k, tile_out=tile, alpha_out=alpha, workspace=ws)
    fwd = tbn.tbn_bind(tbn.tbn_linear_forward, x, tile, alpha, cout, k, y=y)
    torch.cuda.synchronize()
    assert int(tile.abs().max()) == 0 and float(y.float().abs().max()) == 0.0   # binding launches nothing
    t, a = pack()
    out = fwd()
    torch.cuda.synchronize()
    assert t is tile and a is alpha and out is y
    assert torch.equal(tile, tile_ref) and torch.equal(alpha, alpha_ref) and torch.equal(y.view(torch.int16), y_ref.view(torch.int16))
    x.neg_()                                   # the bound call reads the buffers as they are when it is invoked
    fwd()
    torch.cuda.synchronize()
    assert torch.equal(y.view(torch.int16), (-y_ref.float()).to(torch.bfloat16).view(torch.int16))
    with pytest.raises(ValueError):
        tbn.tbn_bind(tbn.tbn_pack_tile, w, k, k)            # no workspace: the bound call would not own one
    with pytest.raises(ValueError):
        tbn.tbn_bind(tbn.tbn_tile_words, w.numel(), k)      # nothing to bind


def test_bound_calls_of_the_other_layers(tbn):
    """The convolution, the layer on sign bits with its sign packing, and the column-tiled layer (whose wrapper allocates
    its own workspace, which the bound call must keep alive) as bound calls: each equals the direct call bit for bit,
    also when invoked again after other allocations."""
    g = torch.Generator(device="cuda")
    g.manual_seed(6)
    M, cin, cout, k = 200, 512, 256, 4
    w = torch.randn(cin * cout, device="cuda", generator=g)
    x = torch.randn((M, cin), device="cuda", generator=g)
    tile, alpha = tbn.tbn_pack_tile(w, k, k)
    # convolution
    xc = torch.randn((2, 32, 14, 14), device="cuda", generator=g)
    wc = torch.randn(64 * 32 * 9, device="cuda", generator=g)
    tile_c, alpha_c = tbn.tbn_pack_tile(wc, 4, 1)
    yc_ref = tbn.tbn_conv2d_forward(xc, tile_c, alpha_c, 64, 3, 3, 4, stride=(1, 1), pad=(1, 1))
    conv = tbn.tbn_bind(tbn.tbn_conv2d_forward, xc, tile_c, alpha_c, 64, 3, 3, 4, stride=(1, 1), pad=(1, 1))
    # sign bits and the layer on them
    bits_ref = tbn.tbn_sign_pack(x)
    yb_ref = tbn.tbn_linear_forward_binact(bits_ref, cin, tile, alpha, cout, k)
    bits = torch.zeros_like(bits_ref)
    sign = tbn.tbn_bind(tbn.tbn_sign_pack, x, xbits=bits)
    binact = tbn.tbn_bind(tbn.tbn_linear_forward_binact, bits, cin, tile, alpha, cout, k)
    # column-tiled layer, workspace allocated by the wrapper
    tile_t, alpha_t = tbn.tbn_pack_coltile(w.view(cout, cin), k, k)
    yt_ref = tbn.tbn_linear_coltiled_forward(x, tile_t, alpha_t, cout, k)
    colt = tbn.tbn_bind(tbn.tbn_linear_coltiled_forward, x, tile_t, alpha_t, cout, k)
    torch.cuda.synchronize()
    for _ in range(2):
        junk = [torch.full((1 << 20,), 7.0, device="cuda") for _ in range(8)]   # would reuse a freed workspace
        yc, _, yb, yt = conv(), sign(), binact(), colt()
        torch.cuda.synchronize()
        assert torch.equal(yc, yc_ref) and torch.equal(bits, bits_ref) and torch.equal(yb, yb_ref) and torch.equal(yt, yt_ref)
        del junk


# ------------------------------------------------------------------------------ conv
CONV_SMALL = [
    # N, C, H, W, O, kh, kw, stride, pad, k, n_alpha
    (2, 4, 9, 8, 6, 3, 3, (1, 1), (1, 1), 4, 1),
    (1, 3, 7, 7, 8, 3, 3, (2, 2), (0, 0), 2, 2),
    (2, 2, 6, 9, 4, 1, 1, (1, 1), (0, 0), 2, 1),
    (1, 5, 8, 5, 3, 2, 3, (1, 2), (1, 0), 5, 5),
    (1, 2, 5, 5, 2, 5, 5, (1, 1), (2, 2), 4, 4),
    (3, 16, 14, 14, 32, 3, 3, (1, 1), (1, 1), 8, 1),     # 4 whole filters per tile
    (2, 32, 14, 14, 64, 3, 3, (1, 1), (1, 1), 8, 8),
    (2, 64, 14, 14, 64, 3, 3, (1, 1), (1, 1), 3, 3),     # tile ends mid-filter
    (2, 32, 28, 28, 32, 3, 3, (2, 2), (1, 1), 4, 1),
    (1, 1, 8, 8, 2, 3, 3, (1, 1), (1, 1), 2, 1),         # the paper's two-identical-channels example
    (2, 64, 7, 7, 128, 1, 1, (1, 1), (0, 0), 2, 2),      # 1x1, 64 whole filters per tile (two filter blocks)
    (1, 32, 5, 20, 48, 3, 3, (1, 1), (1, 1), 3, 3),      # 16 whole filters per tile, 100 pixels in one block
    (3, 64, 14, 14, 64, 3, 3, (1, 1), (1, 1), 2, 1),     # 32 whole filters per tile, two row blocks per image
    (1, 32, 9, 9, 32, 3, 3, (1, 1), (0, 0), 4, 4),       # no padding
    (2, 32, 12, 10, 32, 3, 3, (2, 1), (1, 1), 2, 2),     # mixed stride
    (2, 32, 10, 10, 48, 3, 3, (1, 1), (1, 1), 9, 1),     # 5 1/3 filters per tile, one alpha
    (2, 32, 10, 10, 48, 3, 3, (1, 1), (1, 1), 9, 9),     # same with one alpha per tile (two-alpha channels)
    (1, 64, 6, 6, 40, 1, 1, (1, 1), (0, 0), 5, 5),       # 1x1, 8 filters per tile
    (128, 32, 4, 4, 128, 3, 3, (1, 1), (1, 1), 1, 1),    # 128 distinct filters, 128 images: 64 filters per workgroup (bf16)
    (128, 32, 4, 4, 128, 3, 3, (1, 1), (1, 1), 3, 3),    # same with tile ends inside filters
    (1, 32, 56, 56, 32, 3, 3, (1, 1), (1, 1), 4, 1),     # 56 wide: one output row per workgroup, the widest 3x3 patch the matrix-core kernel stages
    (1, 32, 20, 62, 32, 3, 3, (1, 1), (1, 1), 2, 2),     # 62 wide, 4 pixel tiles with a ragged last one
    # channel counts that are no multiple of 32 on the matrix-core kernel: the last chunk of channels is short
    (2, 3, 32, 32, 64, 3, 3, (1, 1), (1, 1), 4, 4),      # a colour image: one chunk with 3 of 32 channels
    (2, 48, 14, 14, 64, 3, 3, (1, 1), (1, 1), 8, 1),     # one whole chunk and a half one; whole filters per tile
    (1, 72, 9, 11, 40, 3, 3, (2, 2), (1, 1), 5, 5),      # 2 1/4 chunks, stride 2, tile starts inside filters (two alphas)
    (3, 80, 7, 7, 96, 1, 1, (1, 1), (0, 0), 3, 3),       # 1x1 with 2 1/2 chunks, 32 whole filters per tile
    (2, 33, 10, 10, 33, 3, 3, (1, 1), (1, 1), 11, 11),   # one channel beyond a chunk; 3 filters per tile
    (1, 17, 12, 12, 24, 3, 3, (1, 1), (1, 1), 9, 9),     # tile starts inside filters of a short chunk
    # rows too wide to stage at once: column blocks
    (1, 32, 6, 112, 32, 3, 3, (1, 1), (1, 1), 4, 4),     # 112 wide: two column blocks of 56
    (2, 64, 5, 130, 16, 1, 1, (1, 1), (0, 0), 2, 1),     # 1x1, 130 pixels per row: two blocks of 65
    (1, 32, 9, 150, 24, 3, 3, (2, 2), (1, 1), 3, 3),     # stride 2, 75 outputs per row in three blocks of 25; two alphas
    (1, 64, 4, 224, 8, 3, 3, (1, 1), (1, 1), 2, 2),      # 224 wide: four blocks of 56
    # windows the matrix-core kernel does not take, tile of whole filters: the direct kernel (16 filters per workgroup)
    (2, 3, 37, 41, 64, 7, 7, (2, 2), (3, 3), 4, 4),      # a 7x7, stride 2 first layer: 16 distinct filters, 147 weights each
    (3, 16, 18, 18, 40, 5, 5, (1, 1), (2, 2), 2, 1),     # 5x5: 20 distinct filters (two filter groups, the second ragged), one alpha
    (1, 24, 20, 30, 12, 5, 3, (1, 2), (2, 0), 3, 3),     # 5x3, mixed stride and padding, 4 distinct filters, 360 weights each
    (2, 40, 12, 12, 8, 4, 4, (2, 2), (1, 1), 1, 1),      # 4x4, k = 1: 640 weights per filter (two staging passes)
    (1, 2, 300, 5, 6, 2, 2, (1, 1), (0, 0), 6, 6),       # 2x2, one distinct filter, 1196 output pixels (five pixel blocks)
]


def _conv_case(tbn, N, C, H, W, O, kh, kw, stride, pad, k, n_alpha, dtype, flags, seed):
    rng = np.random.default_rng(seed)
    n = O * C * kh * kw
    w = (0.02 * rng.standard_normal(n)).astype(np.float32)
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    bits = None
    if dtype == "bf16":
        bits = wl.f32_to_bf16_bits(x).reshape(x.shape)
        x = wl.bf16_bits_to_f32(bits).reshape(x.shape)
    tile_ref, alpha_ref = orc.pack_tile(w, k, n_alpha)
    ref = orc.conv2d_forward(x, tile_ref, alpha_ref, O, kh, kw, k, stride=stride, pad=pad)
    if flags & 1:
        ref = np.maximum(ref, 0.0)
    y = tbn.tbn_conv2d_forward(x_to_device(x, bits), dev(tile_ref.view(np.int32)), dev(alpha_ref), O, kh, kw, k,
                               stride=stride, pad=pad, flags=flags)
    torch.cuda.synchronize()
    assert tuple(y.shape) == ref.shape
    return assert_close(y_to_numpy(y), ref, dtype, f"conv {N}x{C}x{H}x{W} O={O} {kh}x{kw} k={k} {dtype}")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("N,C,H,W,O,kh,kw,stride,pad,k,n_alpha", CONV_SMALL)
def test_conv_small_generic_kernel(tbn, N, C, H, W, O, kh, kw, stride, pad, k, n_alpha, dtype):
    _conv_case(tbn, N, C, H, W, O, kh, kw, stride, pad, k, n_alpha, dtype, tbn.TBN_FLAG_FORCE_GENERIC, 50 + C + O)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("N,C,H,W,O,kh,kw,stride,pad,k,n_alpha", CONV_SMALL)
def test_conv_small_default_dispatch(tbn, N, C, H, W, O, kh, kw, stride, pad, k, n_alpha, dtype):
    _conv_case(tbn, N, C, H, W, O, kh, kw, stride, pad, k, n_alpha, dtype, 0, 60 + C + O)
    _conv_case(tbn, N, C, H, W, O, kh, kw, stride, pad, k, n_alpha, dtype, tbn.TBN_FLAG_RELU, 70 + C + O)


def _random_conv_shapes(count, seed):
    """Seeded random legal convolutions; about two thirds of them with channel counts the matrix-core
    kernel takes (multiples of 32, 1x1 or 3x3)."""
    rng = np.random.default_rng(seed)
    shapes = []
    while len(shapes) < count:
        mfma_like = rng.random() < 0.67
        C = int(rng.choice([32, 64, 96])) if mfma_like else int(rng.integers(1, 20))
        kh, kw = (int(rng.choice([1, 3])),) * 2 if mfma_like else (int(rng.integers(1, 4)), int(rng.integers(1, 4)))
        H, W = int(rng.integers(max(kh, 3), 30)), int(rng.integers(max(kw, 3), 66))
        O = int(rng.integers(1, 100))
        N = int(rng.integers(1, 4))
        stride = (int(rng.integers(1, 3)), int(rng.integers(1, 3)))
        pad = (int(rng.integers(0, kh)), int(rng.integers(0, kw)))
        n = O * C * kh * kw
        k = int(rng.choice([d for d in range(1, 33) if n % d == 0]))
        n_alpha = k if rng.random() < 0.6 else 1
        shapes.append((N, C, H, W, O, kh, kw, stride, pad, k, n_alpha))
    return shapes


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("N,C,H,W,O,kh,kw,stride,pad,k,n_alpha", _random_conv_shapes(24, 12075))
def test_conv_random_shapes(tbn, N, C, H, W, O, kh, kw, stride, pad, k, n_alpha, dtype):
    _conv_case(tbn, N, C, H, W, O, kh, kw, stride, pad, k, n_alpha, dtype, 0, 7000 + C + O)


@pytest.mark.parametrize("c", [wl.CFG3, wl.CFG3_MISALIGNED], ids=lambda c: c.name)
def test_config3_conv_full_size(tbn, c):
    w = wl.draw_w_real(c.n, c.cfg, c.layer)
    x, _ = wl.draw_x((c.N, c.C, c.H, c.W), c.cfg, c.layer, c.dtype)
    tile_ref, alpha_ref = orc.pack_tile(w, c.k, c.n_alpha)
    tile, alpha = tbn.tbn_pack_tile(dev(w), c.k, c.n_alpha)
    y = tbn.tbn_conv2d_forward(dev(x), tile, alpha, c.O, c.kh, c.kw, c.k, stride=c.stride, pad=c.pad)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(tile_to_numpy(tile), tile_ref)
    yh = y_to_numpy(y)
    assert np.all(np.isfinite(yh))
    rng = np.random.default_rng(33 + c.k)
    idx = rng.integers(0, yh.size, size=20000)
    # add whole rows / columns of the output plane at image borders and the last image / channel
    Ho, Wo = yh.shape[2], yh.shape[3]
    border = [((c.N - 1) * c.O + (c.O - 1)) * Ho * Wo + i for i in range(Ho * Wo)]
    border += [i for i in range(Ho * Wo)]
    idx = np.concatenate([idx, np.array(border, dtype=np.int64)])
    ref = orc.conv2d_forward_at(x, tile_ref, alpha_ref, c.O, c.kh, c.kw, c.k, idx, stride=c.stride, pad=c.pad)
    err = float(np.abs(yh.reshape(-1)[idx] - ref).max() / np.abs(ref).max())
    assert err <= TOL[c.dtype], f"{c.name}: sampled max error / max|ref| = {err:.3e}"


# ------------------------------------------------------------------------------ edge cases
def test_empty_batch_and_error_paths(tbn):
    tile = torch.zeros(4, dtype=torch.int32, device="cuda")
    alpha = torch.ones(1, device="cuda")
    x = torch.zeros((0, 16), device="cuda")
    y = tbn.tbn_linear_forward(x, tile, alpha, 8, 1)
    assert tuple(y.shape) == (0, 8)
    with pytest.raises(tbn.TbnError) as e:
        tbn.tbn_linear_forward(torch.zeros((2, 5), device="cuda"), tile, alpha, 3, 2)
    assert e.value.status == 2
    with pytest.raises(tbn.TbnError) as e:
        tbn.tbn_pack_tile(torch.zeros(10, device="cuda"), 3)
    assert e.value.status == 2
    # outputs untouched on error
    ybuf = torch.full((2, 3), 7.0, device="cuda")
    with pytest.raises(tbn.TbnError):
        tbn.tbn_linear_forward(torch.zeros((2, 5), device="cuda"), tile, alpha, 3, 2, y=ybuf)
    torch.cuda.synchronize()
    assert torch.all(ybuf == 7.0)
