"""GPU parity on seeded random shapes, in exact arithmetic.

The listed parity cases name the shapes somebody thought of; this file draws shapes (batch, row length, number of
distinct columns, compression factor, one or k scalars, fused ReLU, activations at an address that is or is not 16-byte
aligned, the kernel-steering flags) from a seeded generator, so that every kernel family is reached at sizes and
raggedness nobody picked by hand.  Activations are drawn from {-1, 0, +1} and the scalars are powers of two: every
sum is an integer that float32 holds exactly in any order of summation, so

  * the library's choice of kernel must agree bit for bit with its one-thread-per-output kernel at any size, and
  * at sizes the CPU oracle finishes quickly both must equal the oracle's result (rounded to bfloat16 the same way).
"""
import collections
import random

import numpy as np
import pytest
import torch

from oracle import tbn_oracle as orc
from paper_2407_12075_amd import workloads as wl

pytestmark = pytest.mark.gpu

CASES_PER_SEED = 300
ORACLE_MACS = 1.0e8      # the dense oracle is called on cases of at most this many multiply-adds ...
ORACLE_CASES = 40        # ... and on at most this many per seed


@pytest.fixture(scope="module")
def tbn():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2407_12075_amd import tbn as binding
    binding.lib()
    return binding


def _row_length(rng):
    r = rng.random()
    if r < 0.25:
        return 8 * rng.randint(1, 64)
    if r < 0.50:
        return 64 * rng.randint(1, 64)
    if r < 0.65:
        return rng.choice([256, 512, 768, 1024, 1280, 2048, 4096, 8192])
    if r < 0.85:
        return rng.randint(1, 3000)       # mostly no multiple of 8: the vector-ALU kernels
    return 8 * rng.randint(1, 512)


def _batch(rng):
    r = rng.random()
    if r < 0.20:
        return rng.randint(1, 16)
    if r < 0.35:
        return rng.randint(17, 64)
    if r < 0.60:
        return rng.randint(65, 600)
    if r < 0.80:
        return rng.randint(600, 3000)
    return rng.randint(3000, 9000)


def _draw(rng, tbn):
    """One shape: (dtype, M, in, out, k, n_alpha, flags, element offset of x)."""
    while True:
        dtype = rng.choice(["f32", "bf16"])
        cin, M = _row_length(rng), _batch(rng)
        k = rng.choice([1, 2, 3, 4, 5, 8, 16])
        if rng.random() < 0.12:     # large batches of long aligned rows: the block kernels, one pass and persistent
            dtype, M, cin = "bf16", rng.randint(2000, 9000), 256 * rng.randint(1, 16)
        if rng.random() < 0.75:     # tile of whole rows: U distinct columns, k copies
            U = rng.choice([rng.randint(1, 64), 16 * rng.randint(1, 64), 128 * rng.randint(1, 16), rng.randint(1, 1500)])
            cout = U * k
        else:                       # tiles that end inside rows
            cout = rng.randint(1, 2048)
            if (cin * cout) % k:
                continue
        if M * cin > 24e6 or M * cout > 24e6 or M * cin * cout > 1.5e11:
            continue
        n_alpha = rng.choice([1, k])
        flags = rng.choice([0, tbn.TBN_FLAG_RELU]) | rng.choice(
            [0, 0, 0, tbn.TBN_FLAG_LARGE_BATCH, tbn.TBN_FLAG_BLOCK_KERNEL, tbn.TBN_FLAG_STREAM_KERNEL, tbn.TBN_FLAG_TILE_KERNEL])
        off = rng.choice([0, 0, 0, 0, 0, 1, 8])
        return dtype, M, cin, cout, k, n_alpha, flags, off


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_shapes_exact(tbn, seed):
    rng = random.Random(seed)
    families = collections.Counter()
    oracle_cases = 0
    for case in range(CASES_PER_SEED):
        dtype, M, cin, cout, k, n_alpha, flags, off = _draw(rng, tbn)
        what = f"seed {seed} case {case}: {dtype} M={M} in={cin} out={cout} k={k} n_alpha={n_alpha} flags={flags:#x} x offset {off}"
        print(what, flush=True)
        nrng = np.random.default_rng(seed * 1000 + case)
        p = cin * cout // k
        tile_ref = nrng.integers(0, 2 ** 32, size=(p + 31) // 32, dtype=np.uint64).astype(np.uint32)
        if p % 32:
            tile_ref[-1] &= np.uint32((1 << (p % 32)) - 1)
        x = nrng.integers(-1, 2, size=(M, cin)).astype(np.float32)
        alpha_ref = np.asarray([2.0 ** ((i % 5) - 2) for i in range(n_alpha)], dtype=np.float32)

        tdt = torch.float32 if dtype == "f32" else torch.bfloat16
        buf = torch.zeros(M * cin + 16, dtype=tdt, device="cuda")
        buf[off:off + M * cin] = torch.from_numpy(x).reshape(-1).cuda().to(tdt)     # -1, 0, 1 are exact in bfloat16
        xd = buf[off:off + M * cin].view(M, cin)
        tile = torch.from_numpy(tile_ref.view(np.int32)).cuda()
        alpha = torch.from_numpy(alpha_ref).cuda()

        families[tbn.tbn_linear_forward_kernel(tdt, M, cin, cout, k, n_alpha, flags, xd.data_ptr())] += 1
        y = tbn.tbn_linear_forward(xd, tile, alpha, cout, k, flags=flags)
        y_plain = tbn.tbn_linear_forward(xd, tile, alpha, cout, k, flags=(flags & tbn.TBN_FLAG_RELU) | tbn.TBN_FLAG_FORCE_GENERIC)
        torch.cuda.synchronize()
        got, plain = y.float().cpu().numpy(), y_plain.float().cpu().numpy()
        bad = np.argwhere(got != plain)     # as values: -0.0 equals 0.0
        assert bad.size == 0, (f"{what}: {len(bad)} of {got.size} outputs differ from the one-thread-per-output kernel, first at "
                               f"{tuple(bad[0])}: {got[tuple(bad[0])]} against {plain[tuple(bad[0])]}")

        if M * cin * cout <= ORACLE_MACS and oracle_cases < ORACLE_CASES:
            oracle_cases += 1
            ref = orc.linear_forward(x, tile_ref, alpha_ref, cout, k)
            if flags & tbn.TBN_FLAG_RELU:
                ref = np.maximum(ref, 0.0)
            want = ref.astype(np.float32)
            if dtype == "bf16":
                want = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(want)).reshape(M, cout)
            bad = np.argwhere(got != want)
            assert bad.size == 0, (f"{what}: {len(bad)} of {got.size} outputs differ from the oracle, first at {tuple(bad[0])}: "
                                   f"{got[tuple(bad[0])]} against {want[tuple(bad[0])]}")
    print(f"seed {seed}: kernel families reached {dict(families)}; {oracle_cases} cases also against the oracle", flush=True)
    assert oracle_cases >= 20
    assert len(families) >= 5, families


def _draw_conv(rng):
    """One convolution: (dtype, N, C, H, W, O, kh, kw, stride, pad, k, n_alpha, relu)."""
    while True:
        dtype = rng.choice(["f32", "bf16"])
        C = rng.choice([1, 3, 4, 8, 16, 24, 32, 48, 64, 96, 128, rng.randint(1, 80)])
        kh, kw = rng.choice([(1, 1), (3, 3), (3, 3), (3, 3), (5, 5), (7, 7), (1, 3), (3, 1), (2, 2)])
        H, W = rng.randint(kh, 40), rng.choice([7, 14, 16, 28, 32, 56, rng.randint(kw, 70)])
        N = rng.randint(1, 6)
        k = rng.choice([1, 2, 3, 4, 8])
        F = C * kh * kw
        if rng.random() < 0.75:     # tile of whole filters
            U = rng.choice([rng.randint(1, 16), 16 * rng.randint(1, 4), 32, 64])
            O = U * k
        else:
            O = rng.randint(1, 96)
            if (O * F) % k:
                continue
        stride = (rng.choice([1, 1, 2]), rng.choice([1, 1, 2]))
        pad = (rng.randint(0, kh // 2 + 1), rng.randint(0, kw // 2 + 1))
        Ho, Wo = (H + 2 * pad[0] - kh) // stride[0] + 1, (W + 2 * pad[1] - kw) // stride[1] + 1
        if Ho < 1 or Wo < 1 or N * O * Ho * Wo * F > 6e9 or N * O * Ho * Wo > 4e6:
            continue
        return dtype, N, C, H, W, O, kh, kw, stride, pad, k, rng.choice([1, k]), rng.choice([0, 1])


@pytest.mark.parametrize("seed", [21, 22])
def test_random_convolutions_exact(tbn, seed):
    """Convolutions drawn the same way (window shapes, strides, paddings, channel counts on both sides of the
    matrix-core kernel's limits): the library's choice of kernel against its one-thread-per-output kernel bit for bit,
    the small ones also against the oracle."""
    rng = random.Random(seed)
    oracle_cases = 0
    for case in range(150):
        dtype, N, C, H, W, O, kh, kw, stride, pad, k, n_alpha, relu = _draw_conv(rng)
        what = (f"seed {seed} case {case}: {dtype} N={N} C={C} {H}x{W} O={O} window {kh}x{kw} stride {stride} pad {pad} "
                f"k={k} n_alpha={n_alpha} relu={relu}")
        print(what, flush=True)
        nrng = np.random.default_rng(seed * 1000 + case)
        p = O * C * kh * kw // k
        tile_ref = nrng.integers(0, 2 ** 32, size=(p + 31) // 32, dtype=np.uint64).astype(np.uint32)
        if p % 32:
            tile_ref[-1] &= np.uint32((1 << (p % 32)) - 1)
        x = nrng.integers(-1, 2, size=(N, C, H, W)).astype(np.float32)
        alpha_ref = np.asarray([2.0 ** ((i % 5) - 2) for i in range(n_alpha)], dtype=np.float32)
        tdt = torch.float32 if dtype == "f32" else torch.bfloat16
        xd = torch.from_numpy(x).cuda().to(tdt)
        tile = torch.from_numpy(tile_ref.view(np.int32)).cuda()
        alpha = torch.from_numpy(alpha_ref).cuda()
        flags = tbn.TBN_FLAG_RELU if relu else 0
        y = tbn.tbn_conv2d_forward(xd, tile, alpha, O, kh, kw, k, stride=stride, pad=pad, flags=flags)
        y_plain = tbn.tbn_conv2d_forward(xd, tile, alpha, O, kh, kw, k, stride=stride, pad=pad, flags=flags | tbn.TBN_FLAG_FORCE_GENERIC)
        torch.cuda.synchronize()
        got, plain = y.float().cpu().numpy(), y_plain.float().cpu().numpy()
        bad = np.argwhere(got != plain)
        assert bad.size == 0, (f"{what}: {len(bad)} of {got.size} outputs differ from the one-thread-per-output kernel, first at "
                               f"{tuple(bad[0])}: {got[tuple(bad[0])]} against {plain[tuple(bad[0])]}")
        if got.size * C * kh * kw <= 3.0e7 and oracle_cases < 30:
            oracle_cases += 1
            ref = orc.conv2d_forward(x, tile_ref, alpha_ref, O, kh, kw, k, stride=stride, pad=pad)
            if relu:
                ref = np.maximum(ref, 0.0)
            want = ref.astype(np.float32)
            if dtype == "bf16":
                want = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(want)).reshape(want.shape)
            bad = np.argwhere(got != want)
            assert bad.size == 0, (f"{what}: {len(bad)} of {got.size} outputs differ from the oracle, first at {tuple(bad[0])}: "
                                   f"{got[tuple(bad[0])]} against {want[tuple(bad[0])]}")
    assert oracle_cases >= 15


@pytest.mark.parametrize("seed", [31, 32])
def test_random_shapes_binary_activations_exact(tbn, seed):
    """The layer on sign bits (every product is +-1, every sum an integer): the library's choice of kernel against its
    one-thread-per-output kernel bit for bit on drawn shapes, outputs as values and as sign bits."""
    rng = random.Random(seed)
    for case in range(150):
        while True:
            cin, M = _row_length(rng), _batch(rng)
            k = rng.choice([1, 2, 4, 8, 16])
            U = rng.choice([rng.randint(1, 64), 32 * rng.randint(1, 32), 128 * rng.randint(1, 8), rng.randint(1, 700)])
            cout = U * k
            if rng.random() < 0.2:
                cout = rng.randint(1, 1024)
                if (cin * cout) % k:
                    continue
            if M * cin <= 24e6 and M * cout <= 24e6 and M * cin * cout <= 1.0e11:
                break
        n_alpha = rng.choice([1, k])
        ydt = rng.choice([torch.float32, torch.bfloat16])
        flags = rng.choice([0, tbn.TBN_FLAG_RELU, tbn.TBN_FLAG_SIGN_OUT])
        what = f"seed {seed} case {case}: M={M} in={cin} out={cout} k={k} n_alpha={n_alpha} y {ydt} flags={flags:#x}"
        print(what, flush=True)
        g = torch.Generator(device="cuda")
        g.manual_seed(seed * 1000 + case)
        x = torch.randint(0, 2, (M, cin), device="cuda", generator=g).float() * 2 - 1
        p = cin * cout // k
        tile = torch.randint(-2 ** 31, 2 ** 31 - 1, ((p + 31) // 32,), device="cuda", dtype=torch.int32, generator=g)
        if p % 32:
            tile[-1] &= (1 << (p % 32)) - 1
        alpha = torch.tensor([2.0 ** ((i % 5) - 2) for i in range(n_alpha)], device="cuda", dtype=torch.float32)
        xbits = tbn.tbn_sign_pack(x)
        y = tbn.tbn_linear_forward_binact(xbits, cin, tile, alpha, cout, k, dtype=ydt, flags=flags)
        y_plain = tbn.tbn_linear_forward_binact(xbits, cin, tile, alpha, cout, k, dtype=ydt, flags=flags | tbn.TBN_FLAG_FORCE_GENERIC)
        torch.cuda.synchronize()
        if flags & tbn.TBN_FLAG_SIGN_OUT:
            assert torch.equal(y, y_plain), f"{what}: sign rows differ from the one-thread-per-output kernel"
        else:
            same = y.float() == y_plain.float()
            assert bool(same.all()), f"{what}: {int((~same).sum())} outputs differ from the one-thread-per-output kernel"
