"""GPU parity in exact arithmetic: activations drawn from {-1, 0, +1} and alpha = 1 make every output of
the fully-connected layer an integer that float32 accumulation and (after the same rounding on both
sides) bfloat16 hold exactly, so the matrix-core kernels must agree with the CPU oracle bit for bit.
One wrong tile bit, window position, K slice or output column changes an output by at least 1: the
tolerance tests at long K cannot see that (2e-2 of max|y| is about 0.1 there), these can.

Shapes reach every large-batch bfloat16 kernel form: the two kernels for tiles of whole rows (128 x 128
blocks with load waves, K a multiple of 256; streaming half tiles, K a multiple of 512: ragged batches and
column blocks, several half tiles per workgroup, short K with more replicas than rounds, one replica), the
general one-block-per-tile kernel (other K, tiles that end inside rows) and, with float32 activations, the
float32 kernel.
"""
import numpy as np
import pytest
import torch

from oracle import tbn_oracle as orc
from paper_2407_12075_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tbn():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2407_12075_amd import tbn as binding
    binding.lib()
    return binding


def _ternary(rng, shape, p_nonzero):
    u = rng.random(shape, dtype=np.float32)
    x = np.zeros(shape, dtype=np.float32)
    x[u < p_nonzero / 2] = -1.0
    x[u > 1.0 - p_nonzero / 2] = 1.0
    return x


def _exact_case(tbn, M, cin, cout, k, dtype, flags, seed, alpha_vals=None, workspace=None):
    rng = np.random.default_rng(seed)
    n = cin * cout
    p = n // k
    tile_ref = rng.integers(0, 2 ** 32, size=(p + 31) // 32, dtype=np.uint64).astype(np.uint32)
    if p % 32:
        tile_ref[-1] &= np.uint32((1 << (p % 32)) - 1)   # unused high bits of the last word are zero
    # few enough non-zeros that every sum stays below 256 in magnitude (6 sigma)
    x = _ternary(rng, (M, cin), min(1.0, 1500.0 / cin))
    alpha_ref = np.ones(k, dtype=np.float32) if alpha_vals is None else np.asarray(alpha_vals, dtype=np.float32)
    ref = orc.linear_forward(x, tile_ref, alpha_ref, cout, k)
    if flags & 1:
        ref = np.maximum(ref, 0.0)
    assert np.abs(ref).max() < 2 ** 24
    tile = torch.from_numpy(tile_ref.view(np.int32)).cuda()
    alpha = torch.from_numpy(alpha_ref).cuda()
    if dtype == "bf16":
        bits = wl.f32_to_bf16_bits(x).reshape(M, cin)   # exact: -1, 0, 1 are bfloat16 numbers
        xd = torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
        want = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(ref.astype(np.float32))).reshape(M, cout)
    else:
        xd = torch.from_numpy(x).cuda()
        want = ref.astype(np.float32)
    if workspace:
        need = tbn.tbn_linear_forward_workspace_bytes(xd.dtype, M, cin, cout, k, flags)
        assert (need > 0) == (workspace == "used"), f"workspace query returned {need}"
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
        y = tbn.tbn_linear_forward_ws(xd, tile, alpha, cout, k, ws, flags=flags)
        y2 = tbn.tbn_linear_forward_ws(xd, tile, alpha, cout, k, ws, flags=flags)
        torch.cuda.synchronize()
        assert torch.equal(y.view(torch.int16), y2.view(torch.int16)), "two runs differ"
    else:
        y = tbn.tbn_linear_forward(xd, tile, alpha, cout, k, flags=flags)
    torch.cuda.synchronize()
    got = y.float().cpu().numpy()
    bad = np.argwhere(got != want)
    assert bad.size == 0, (f"M={M} in={cin} out={cout} k={k} {dtype} flags={flags:#x}: {len(bad)} of {got.size} outputs "
                           f"differ, first at {tuple(bad[0])}: got {got[tuple(bad[0])]}, want {want[tuple(bad[0])]}")


# M, in, out, k
EXACT_STREAM = [
    (128, 512, 1024, 8),      # one group of four rounds per half tile: more replicas than rounds
    (100, 512, 256, 2),       # two half tiles in one row block, the second ragged
    (8192, 4096, 4096, 8),    # the shape the headline metric is quoted on
    (8192 + 37, 1024, 1024, 4),   # ragged last row half
    (4100, 512, 1088, 8),     # U = 136: a ragged second column block; ragged rows
    (4096, 1024, 4096, 2),    # U = 2048: 16 column blocks, four half tiles per workgroup with changing columns
    (3 * 64 * 8 + 64, 1536, 512 * 16, 16),   # 16 replicas in 12 rounds; XCDs with different numbers of row halves
    (1000, 2048, 128 * 3, 1),   # one replica: k = 1
    (4224, 2048, 1024, 1),
    (640, 512, 64 * 64, 64),  # 64 replicas, U = 64: half a column block
    (11300, 512, 768, 2),     # three column blocks: a workgroup's half tiles change rows and columns
]


@pytest.mark.parametrize("kernel", ["default", "stream", "general"])
@pytest.mark.parametrize("M,cin,cout,k", EXACT_STREAM)
def test_exact_bf16_whole_row_tiles(tbn, M, cin, cout, k, kernel):
    # default: the block kernel with load waves, or the streaming kernel for small grids
    flags = {"default": 0, "stream": tbn.TBN_FLAG_STREAM_KERNEL, "general": tbn.TBN_FLAG_BLOCK_KERNEL}[kernel]
    _exact_case(tbn, M, cin, cout, k, "bf16", tbn.TBN_FLAG_LARGE_BATCH | flags, 11 * M + cin)


@pytest.mark.parametrize("M,cin,cout,k", [(8192, 4096, 4096, 8), (640, 512, 64 * 64, 64), (300, 1024, 1024, 4)])
def test_exact_bf16_default_dispatch(tbn, M, cin, cout, k):
    _exact_case(tbn, M, cin, cout, k, "bf16", 0, 13 * M + cin)


def test_exact_bf16_relu_and_scalars(tbn):
    # powers of two as scalars keep the arithmetic exact and show that replica t is scaled by alpha[t]
    for extra in (0, tbn.TBN_FLAG_STREAM_KERNEL):
        _exact_case(tbn, 640, 1024, 1024, 8, "bf16", tbn.TBN_FLAG_LARGE_BATCH | tbn.TBN_FLAG_RELU | extra, 5,
                    alpha_vals=[1, 2, 0.5, 4, 0.25, 8, 1, 2])
        _exact_case(tbn, 200, 512, 768, 4, "bf16", tbn.TBN_FLAG_LARGE_BATCH | tbn.TBN_FLAG_RELU | extra, 6,
                    alpha_vals=[2, 1, 0.5, 4])
    # 40 x 8 = 320 blocks of 128 x 128: more than the chip has CUs, so the block kernel streams its stores
    _exact_case(tbn, 5120, 512, 2048, 2, "bf16", tbn.TBN_FLAG_LARGE_BATCH | tbn.TBN_FLAG_RELU, 7, alpha_vals=[0.5, 2])


def test_exact_bf16_persistent_blocks_with_store_waves(tbn):
    """More blocks than CUs: a workgroup walks blocks, two of its waves load and two write the replicas of the block
    before while the next one is multiplied.  Ragged rows and columns (stores masked lane by lane), several replicas
    with their own scalars, more replica units than rounds."""
    L = tbn.TBN_FLAG_LARGE_BATCH
    # 33 x 8 blocks; rows end inside the last row block, U = 1000 ends inside the last column block; 4 rounds
    _exact_case(tbn, 4174, 512, 2000, 2, "bf16", L, 21, alpha_vals=[0.5, 2])
    # 17 x 16 blocks, 8 rounds, four replicas, fused ReLU
    _exact_case(tbn, 2100, 1024, 8192, 4, "bf16", L | tbn.TBN_FLAG_RELU, 22, alpha_vals=[1, 2, 0.5, 4])
    # 6 and 10 rounds (K = 768, 1280): consecutive blocks of a workgroup start in different ring slots
    _exact_case(tbn, 4174, 768, 2000, 2, "bf16", L, 24, alpha_vals=[0.5, 2])
    _exact_case(tbn, 2100, 1280, 8192, 4, "bf16", L | tbn.TBN_FLAG_RELU, 25, alpha_vals=[1, 2, 0.5, 4])
    # 9 x 29 blocks, 4 rounds, eight replicas: eight (replica, quarter, half) units per round and store wave
    _exact_case(tbn, 1100, 512, 29696, 8, "bf16", L, 23, alpha_vals=[1, 2, 0.5, 4, 0.25, 8, 1, 2])


def test_exact_one_wave_per_32_rows_many_distinct_columns(tbn):
    """The kernel with one wave per 32 batch rows on more than 512 distinct columns (many column groups, each reading
    its rows of X again), as the default dispatch picks it for small batches, and forced on a larger one."""
    _exact_case(tbn, 100, 1024, 16384, 4, "bf16", 0, 31, alpha_vals=[1, 2, 0.5, 4])      # 4096 distinct columns, K in four slices
    _exact_case(tbn, 257, 512, 4096, 2, "bf16", 0, 32, alpha_vals=[2, 0.5])              # 2048 distinct columns, short rows, ragged batch
    _exact_case(tbn, 100, 1024, 4096, 4, "f32", 0, 33, alpha_vals=[1, 2, 0.5, 4])        # float32, 1024 distinct columns
    _exact_case(tbn, 1000, 1536, 6144, 4, "bf16", tbn.TBN_FLAG_TILE_KERNEL, 34)          # 1536 distinct columns, forced
    _exact_case(tbn, 333, 768, 2304, 3, "f32", tbn.TBN_FLAG_TILE_KERNEL, 35, alpha_vals=[1, 0.5, 2])   # 768 distinct columns, three replicas
    _exact_case(tbn, 1500, 512, 4096, 2, "f32", 0, 36, alpha_vals=[2, 0.5])              # float32 large batch, 2048 distinct columns: default dispatch


def test_exact_at_most_16_rows_many_distinct_columns(tbn):
    """Up to 16 batch rows: the decode kernel, or the small-batch kernel where rows x distinct columns exceed 16384."""
    for dtype in ("bf16", "f32"):
        _exact_case(tbn, 16, 512, 4096, 2, dtype, 0, 41, alpha_vals=[2, 0.5])            # 2048 distinct columns: small-batch kernel
        _exact_case(tbn, 4, 512, 8192, 2, dtype, 0, 42, alpha_vals=[2, 0.5])             # 4096 distinct columns, 4 rows: decode kernel
        _exact_case(tbn, 9, 1024, 8192, 2, dtype, 0, 43, alpha_vals=[1, 4])              # 4096 distinct columns, 9 rows: small-batch kernel


@pytest.mark.parametrize("M,cin,cout,k", [(16640, 512, 8192, 32), (33000, 768, 8192, 64), (9000, 1024, 16384, 16)])
def test_persistent_blocks_many_replicas_equal_general_kernel(tbn, M, cin, cout, k):
    """Many replicas per block (more store units than rounds) on grids of more blocks than CUs, at sizes the dense
    oracle does not finish in seconds: in exact arithmetic (activations in {-1, 0, 1}, powers of two as scalars) the
    persistent block kernel must agree bit for bit with the general one-block-per-tile kernel, which the oracle tests
    above cover, whatever the order of the sums."""
    g = torch.Generator(device="cuda")
    g.manual_seed(1000 + k)
    x = (torch.randint(0, 8, (M, cin), device="cuda", generator=g) - 3).clamp_(-1, 1).to(torch.bfloat16)   # mostly zeros and ones
    tile = torch.randint(-2 ** 31, 2 ** 31 - 1, (cin * cout // k // 32,), device="cuda", dtype=torch.int32, generator=g)
    alpha = torch.tensor([2.0 ** ((i % 5) - 2) for i in range(k)], device="cuda", dtype=torch.float32)
    y_persistent = tbn.tbn_linear_forward(x, tile, alpha, cout, k, flags=tbn.TBN_FLAG_LARGE_BATCH)
    y_general = tbn.tbn_linear_forward(x, tile, alpha, cout, k, flags=tbn.TBN_FLAG_LARGE_BATCH | tbn.TBN_FLAG_BLOCK_KERNEL)
    torch.cuda.synchronize()
    assert torch.equal(y_persistent.view(torch.int16), y_general.view(torch.int16))
    assert float(y_general.float().abs().max()) > 0


# shapes that stay on the one-block-per-tile kernels: K no multiple of 512, tiles that end inside rows
EXACT_BLOCK = [
    (70, 8192, 80, 4),        # U = 20 distinct rows, long K
    (4224, 1000, 1024, 1),
    (2048, 3000, 3072, 9),    # tile and alpha boundaries inside rows
    (1024, 3000, 3072, 6),    # rows start at bit offsets that are no multiples of 32
    (4230, 96, 1040, 2),
    (1600, 768, 4096, 8),     # whole rows per tile, but K = 1.5 * 512
]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("M,cin,cout,k", EXACT_BLOCK)
def test_exact_block_kernels(tbn, M, cin, cout, k, dtype):
    _exact_case(tbn, M, cin, cout, k, dtype, tbn.TBN_FLAG_LARGE_BATCH, 17 * M + cin)


# float32, tile of whole rows: at most 512 distinct rows go to the kernel that feeds the matrix cores straight from
# global memory (one wave per 32 batch rows, one or four K slices per workgroup), the rest and everything under
# TBN_FLAG_BLOCK_KERNEL to the general float32 kernel
EXACT_F32_ROWS = [
    (1000, 2048, 384, 1),     # three groups of four column tiles, four K slices
    (4100, 512, 1088, 8),     # U = 136: two groups of three tiles, the last tile of the second outside; one K slice
    (12608, 384, 1536, 4),    # transformer MLP, first layer: 394 row tiles, K = 6 chunks
    (12608, 1536, 384, 4),    # second layer: U = 96, three tiles, four K slices of 384
    (65, 1024, 8, 2),         # U = 4: one tile, four waves add into it; ragged rows
    (300, 64, 64 * 5, 5),     # one chunk of K, two tiles
    (200, 1280, 2 * 520, 2),  # U = 520 > 512: general kernel
    (97, 4096, 160, 1),       # five tiles in two groups; K = 16 chunks per slice
]


@pytest.mark.parametrize("kernel", ["default", "general"])
@pytest.mark.parametrize("M,cin,cout,k", EXACT_F32_ROWS)
def test_exact_f32_whole_row_tiles(tbn, M, cin, cout, k, kernel):
    extra = tbn.TBN_FLAG_BLOCK_KERNEL if kernel == "general" else 0
    _exact_case(tbn, M, cin, cout, k, "f32", tbn.TBN_FLAG_LARGE_BATCH | extra, 19 * M + cin)
    _exact_case(tbn, M, cin, cout, k, "f32", tbn.TBN_FLAG_LARGE_BATCH | tbn.TBN_FLAG_RELU | extra, 19 * M + cin + 1,
                alpha_vals=[2.0 ** ((i % 5) - 2) for i in range(k)])


# at most 16 batch rows and whole rows per tile: the decode kernel (default) and, with the large-batch flag, the
# matrix-core small-batch kernel on the same data
EXACT_DECODE = [
    (1, 4096, 4096, 8),
    (16, 4096, 4096, 8),
    (3, 4096, 4096, 8),
    (5, 264, 96, 4),          # 24 distinct rows of 264 bits: rows start at byte, not word, boundaries
    (8, 256, 256, 4),
    (16, 8192, 80, 4),        # 20 distinct rows: a ragged last workgroup with four rows each
    (2, 1000, 70, 1),         # k = 1, one replica, K no multiple of 512
    (11, 512, 3 * 1024, 3),   # 1024 distinct rows
]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("M,cin,cout,k", EXACT_DECODE)
def test_exact_decode_shapes(tbn, M, cin, cout, k, dtype):
    _exact_case(tbn, M, cin, cout, k, dtype, 0, 23 * M + cin)
    _exact_case(tbn, M, cin, cout, k, dtype, tbn.TBN_FLAG_RELU, 23 * M + cin + 1,
                alpha_vals=[2.0 ** ((i % 5) - 2) for i in range(k)])
    _exact_case(tbn, M, cin, cout, k, dtype, tbn.TBN_FLAG_LARGE_BATCH, 23 * M + cin + 2)


# split K with a caller-supplied workspace: grids of at most half the chip's CUs on the block kernel's shapes.  By
# default the path is only taken for long rows (the cost model); TBN_FLAG_SPLIT_K takes it wherever the shape allows.
EXACT_SPLIT = [
    (512, 4096, 4096, 8),     # 16 blocks, 16 splits of one round pair
    (1000, 4096, 4096, 8),    # ragged rows; 32 blocks, 8 splits
    (2048, 4096, 4096, 8),    # 4 splits
    (4096, 4096, 4096, 8),    # 128 blocks, 2 splits
    (100, 1024, 1088, 8),     # U = 136: ragged second column block; 2 blocks, 4 splits of one round pair
    (300, 1536, 768, 2),      # 6 round pairs: 2 splits of three pairs
    (130, 512, 64 * 64, 64),  # 64 replicas, half a column block
    (700, 2048, 384, 1),      # one replica
]


@pytest.mark.parametrize("M,cin,cout,k", EXACT_SPLIT)
def test_exact_bf16_split_k_with_workspace(tbn, M, cin, cout, k):
    split = tbn.TBN_FLAG_SPLIT_K
    _exact_case(tbn, M, cin, cout, k, "bf16", split, 29 * M + cin, workspace="used")
    _exact_case(tbn, M, cin, cout, k, "bf16", split | tbn.TBN_FLAG_RELU, 29 * M + cin + 1,
                alpha_vals=[2.0 ** ((i % 5) - 2) for i in range(k)], workspace="used")


@pytest.mark.parametrize("M,cin,cout,k", [(512, 16384, 1024, 2), (200, 16384, 512, 2)])
def test_exact_bf16_split_k_chosen_for_long_rows(tbn, M, cin, cout, k):
    # no flag: the cost model takes the split for rows this long (also below 256 batch rows, where the call
    # without a workspace goes to the small-batch kernel)
    _exact_case(tbn, M, cin, cout, k, "bf16", 0, 37 * M + cin, workspace="used")


@pytest.mark.parametrize("M,cin,cout,k,dtype,flags", [
    (8192, 4096, 4096, 8, "bf16", 0x1000),   # the grid fills the chip
    (16, 4096, 4096, 8, "bf16", 0x1000),     # decode kernel
    (512, 4096, 4096, 8, "f32", 0x1000),     # float32 has no split path
    (512, 768, 4096, 8, "bf16", 0x1000),     # K = 3 * 256: no equal parts
    (512, 4096, 4096, 8, "bf16", 0),         # short rows: the cost model keeps the single kernel
])
def test_exact_workspace_entry_without_split(tbn, M, cin, cout, k, dtype, flags):
    assert tbn.TBN_FLAG_SPLIT_K == 0x1000
    _exact_case(tbn, M, cin, cout, k, dtype, flags, 31 * M + cin, workspace="unused")


def test_workspace_too_small_or_misaligned(tbn):
    M, cin, cout, k = 512, 4096, 4096, 8
    need = tbn.tbn_linear_forward_workspace_bytes(torch.bfloat16, M, cin, cout, k, tbn.TBN_FLAG_SPLIT_K)
    assert need == 16 * M * (cout // k) * 4
    x = torch.zeros((M, cin), dtype=torch.bfloat16, device="cuda")
    tile = torch.zeros(cin * cout // k // 32, dtype=torch.int32, device="cuda")
    alpha = torch.ones(k, dtype=torch.float32, device="cuda")
    small = torch.empty(need - 16, dtype=torch.uint8, device="cuda")
    y = tbn.tbn_linear_forward_ws(x, tile, alpha, cout, k, small, flags=tbn.TBN_FLAG_SPLIT_K)   # the plain forward
    torch.cuda.synchronize()
    assert float(y.float().abs().max()) == 0.0
    ws = torch.empty(need + 16, dtype=torch.uint8, device="cuda")
    with pytest.raises(RuntimeError):
        tbn.tbn_linear_forward_ws(x, tile, alpha, cout, k, ws[8:], flags=tbn.TBN_FLAG_SPLIT_K)


# bfloat16 on the kernel with one wave per 32 batch rows (default for small grids; the flag takes it everywhere)
EXACT_BF16_TILE = [
    (512, 4096, 4096, 8),     # 4 groups of 4 column tiles, 8 K slices of 512
    (1000, 4096, 4096, 8),    # ragged rows
    (100, 1024, 1088, 8),     # U = 136: two groups of three tiles, the last outside; 4 K slices of two chunks
    (1000, 2048, 384, 1),     # one replica, three groups
    (130, 512, 64 * 64, 64),  # 64 replicas, two tiles, 4 K slices of one chunk
    (300, 128, 256, 2),       # one chunk of K, one K slice
    (65, 1024, 16, 2),        # U = 8: one tile, eight waves add into it
    (2100, 256, 2048, 4),     # U = 512: all sixteen column tiles, two chunks
]


@pytest.mark.parametrize("M,cin,cout,k", EXACT_BF16_TILE)
def test_exact_bf16_wave_per_32_rows(tbn, M, cin, cout, k):
    flags = tbn.TBN_FLAG_LARGE_BATCH | tbn.TBN_FLAG_TILE_KERNEL
    _exact_case(tbn, M, cin, cout, k, "bf16", flags, 41 * M + cin)
    _exact_case(tbn, M, cin, cout, k, "bf16", flags | tbn.TBN_FLAG_RELU, 41 * M + cin + 1,
                alpha_vals=[2.0 ** ((i % 5) - 2) for i in range(k)])
