"""Pins for the CPU oracle: each test checks it against something the paper or the
mathematics fixes, never against the oracle's own formula.

 P1  Eq. 4-5 (replicate + reshape) and Algorithm 1 (running index) give the same layer
 P2  k = 1 is the ordinary binary-weight layer alpha * sign(W)  (library: torch linear / conv2d)
 P3  tiles that hold whole rows / filters give identical output blocks (the paper's conv example)
 P4  hand-worked sign aggregation (tests/golden/hand_worked_pack.txt)
 P5  brute force on 2 x 4 layers against weight matrices written out by hand
 P6  sign / scale / permutation invariants
 P7  storage closed form against the numbers printed in Tables 6 and 7
 P8  convolution against torch.nn.functional.conv2d on a weight replicated with numpy.tile
"""
import itertools
import os

import numpy as np
import pytest
import torch

from oracle import tbn_oracle as orc

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.split("#", 1)[0].strip()
            if not line or "=" not in line:
                continue
            key, val = line.split("=", 1)
            out[key.strip()] = [float(v) for v in val.split()]
    return out


def bits_of(tile, p):
    return np.array([(int(tile[i >> 5]) >> (i & 31)) & 1 for i in range(p)], dtype=np.int64)


def words_from_bits(bits):
    words = np.zeros((len(bits) + 31) // 32, dtype=np.uint32)
    for i, b in enumerate(bits):
        if b:
            words[i >> 5] |= np.uint32(1 << (i & 31))
    return words


def dense_from_numpy_tile(bits, alpha, k, shape):
    """Eq. 4-5 with library routines only: numpy.tile for the replication, reshape for vec^-1."""
    t = np.where(np.asarray(bits) > 0, 1.0, -1.0)
    b = np.tile(t, k)
    a = np.asarray(alpha, dtype=np.float64)
    scale = np.repeat(a, len(t)) if a.size == k and k > 1 else np.full(b.size, a[0])
    return (b * scale).reshape(shape)


# ---------------------------------------------------------------- P1
@pytest.mark.parametrize("M,cin,cout,k,n_alpha", [
    (3, 5, 3, 3, 3),      # p = 5: one row per tile
    (2, 10, 6, 4, 4),     # p = 15: tile ends mid-row
    (4, 8, 8, 4, 1),      # aligned, single alpha
    (2, 7, 6, 2, 2),      # p = 21
    (1, 12, 5, 10, 10),   # p = 6 < in: several wraps inside one row
    (3, 64, 48, 6, 6),    # p = 512 = 8 rows
    (2, 33, 31, 1, 1),    # k = 1
    (2, 9, 4, 36, 36),    # p = 1
])
def test_p1_kronecker_and_running_index_agree(M, cin, cout, k, n_alpha):
    rng = np.random.default_rng(11 + cin * cout + k)
    w = rng.standard_normal(cin * cout).astype(np.float32)
    x = rng.standard_normal((M, cin)).astype(np.float32)
    tile, alpha = orc.pack_tile(w, k, n_alpha)
    y_def = orc.linear_forward(x, tile, alpha, cout, k)
    y_alg = orc.linear_forward_alg1(x, tile, alpha, cout, k)
    np.testing.assert_array_equal(y_def, y_alg)
    # the fused ReLU of the listing is max(0, .) of the same numbers
    y_relu = orc.linear_forward_alg1(x, tile, alpha, cout, k, relu=True)
    np.testing.assert_array_equal(y_relu, np.maximum(y_def, 0.0))


# ---------------------------------------------------------------- P2
def _sign_minus_at_zero(w):
    return torch.where(w > 0, torch.ones_like(w), -torch.ones_like(w))


def test_p2_k1_linear_is_binary_weight_layer():
    rng = np.random.default_rng(5)
    w = rng.standard_normal((24, 40)).astype(np.float32)
    w[3, 7] = 0.0  # sign(0) must come out as -1
    x = rng.standard_normal((6, 40)).astype(np.float32)
    tile, alpha = orc.pack_tile(w, 1, 1)
    y = orc.linear_forward(x, tile, alpha, 24, 1)
    wt = torch.from_numpy(w).double()
    a = torch.from_numpy(w).double().abs().mean().float().double()
    ref = torch.nn.functional.linear(torch.from_numpy(x).double(), a * _sign_minus_at_zero(wt))
    np.testing.assert_allclose(y, ref.numpy(), rtol=1e-12, atol=1e-12)
    assert abs(float(alpha[0]) - float(a)) <= np.spacing(np.float32(a))


def test_p2_k1_conv_is_binary_weight_layer():
    rng = np.random.default_rng(6)
    w = rng.standard_normal((5, 3, 3, 2)).astype(np.float32)
    x = rng.standard_normal((2, 3, 7, 6)).astype(np.float32)
    tile, alpha = orc.pack_tile(w, 1, 1)
    y = orc.conv2d_forward(x, tile, alpha, 5, 3, 2, 1, stride=(2, 1), pad=(1, 0))
    wt = torch.from_numpy(w).double()
    a = wt.abs().mean().float().double()
    ref = torch.nn.functional.conv2d(torch.from_numpy(x).double(), a * _sign_minus_at_zero(wt),
                                     stride=(2, 1), padding=(1, 0))
    np.testing.assert_allclose(y, ref.numpy(), rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------- P3
def test_p3_paper_conv_example_identical_channels():
    # Section "CNN Architectures", Results: one input channel, two output channels, 3x3 kernel,
    # compression 2, single alpha -> the two output channels are identical.
    rng = np.random.default_rng(7)
    w = rng.standard_normal((2, 1, 3, 3)).astype(np.float32)
    x = rng.standard_normal((3, 1, 8, 8)).astype(np.float32)
    tile, alpha = orc.pack_tile(w, 2, 1)
    y = orc.conv2d_forward(x, tile, alpha, 2, 3, 3, 2, pad=(1, 1))
    np.testing.assert_array_equal(y[:, 0], y[:, 1])
    assert np.abs(y).max() > 0


def test_p3_row_aligned_blocks_are_scaled_copies():
    rng = np.random.default_rng(8)
    cin, cout, k = 16, 12, 4          # p = 48 = 3 rows
    w = rng.standard_normal(cin * cout).astype(np.float32)
    x = rng.standard_normal((5, cin)).astype(np.float32)
    tile, alpha1 = orc.pack_tile(w, k, 1)
    y1 = orc.linear_forward(x, tile, alpha1, cout, k)
    for c in range(1, k):
        np.testing.assert_array_equal(y1[:, :3], y1[:, 3 * c:3 * c + 3])
    tile, alphak = orc.pack_tile(w, k, k)
    yk = orc.linear_forward(x, tile, alphak, cout, k)
    for c in range(k):
        np.testing.assert_allclose(yk[:, 3 * c:3 * c + 3] / float(alphak[c]), y1[:, :3] / float(alpha1[0]),
                                   rtol=1e-13)


# ---------------------------------------------------------------- P4
def test_p4_hand_worked_pack_and_forward():
    g = read_golden("hand_worked_pack.txt")
    w = np.array(g["w"], dtype=np.float32)
    k = int(g["k"][0])
    tile1, alpha1 = orc.pack_tile(w, k, 1)
    tilek, alphak = orc.pack_tile(w, k, k)
    assert tile1.tolist() == [int(g["tile_word"][0])]
    assert tilek.tolist() == [int(g["tile_word"][0])]
    np.testing.assert_allclose(alpha1, g["alpha_single"], rtol=0, atol=6e-8)
    np.testing.assert_allclose(alphak, g["alpha_per_tile"], rtol=0, atol=6e-8)
    x = np.array([g["x"]], dtype=np.float32)
    np.testing.assert_allclose(orc.linear_forward(x, tilek, alphak, 2, k)[0], g["y_per_tile"], atol=1e-6)
    np.testing.assert_allclose(orc.linear_forward(x, tile1, alpha1, 2, k)[0], g["y_single"], atol=1e-6)


def test_p4_alpha_comes_from_a_when_given():
    w = np.array([1, -1, 1, -1, 1, 1, -3, -3], dtype=np.float32)
    a = np.array([2, 2, 2, 2, 4, 4, 4, 8], dtype=np.float32)
    tile, alpha = orc.pack_tile(w, 2, 2, a_real=a)
    assert tile.tolist() == [0b0001]          # s = (2, 0, -2, -4)
    assert alpha.tolist() == [2.0, 5.0]
    tile, alpha = orc.pack_tile(w, 2, 1, a_real=a)
    assert alpha.tolist() == [3.5]


def test_p4_threshold_special_values():
    w = np.array([0.0, -0.0, np.nan, 1e-30, -1e-30, np.inf, -np.inf, 5.0], dtype=np.float32)
    tile, _ = orc.pack_tile(w, 1, 1)
    assert bits_of(tile, 8).tolist() == [0, 0, 0, 1, 0, 1, 0, 1]
    # double-precision sum: 1 + 2^-30 - 1 is positive although float32 addition would lose it
    w = np.array([1.0, 2.0 ** -30, -1.0], dtype=np.float32)
    tile, _ = orc.pack_tile(w, 3, 1)
    assert tile.tolist() == [1]


# ---------------------------------------------------------------- P5
# Dense 2 x 4 weights written out by hand for every k that divides 8.  Entries are
# (tile position, alpha index) at rows o = 0, 1 and columns j = 0..3, read off a drawing of the
# flattened weight  f = 0..7  cut into k pieces of length p = 8 / k.
HAND_2x4 = {
    1: [[(0, 0), (1, 0), (2, 0), (3, 0)], [(4, 0), (5, 0), (6, 0), (7, 0)]],
    2: [[(0, 0), (1, 0), (2, 0), (3, 0)], [(0, 1), (1, 1), (2, 1), (3, 1)]],
    4: [[(0, 0), (1, 0), (0, 1), (1, 1)], [(0, 2), (1, 2), (0, 3), (1, 3)]],
    8: [[(0, 0), (0, 1), (0, 2), (0, 3)], [(0, 4), (0, 5), (0, 6), (0, 7)]],
}


@pytest.mark.parametrize("k", [1, 2, 4, 8])
def test_p5_bruteforce_2x4_forward(k):
    p = 8 // k
    alphas_k = np.array([0.5, 1.25, 2.0, 0.75, 3.0, 0.125, 1.5, 4.0][:k], dtype=np.float32)
    inputs = np.array(list(itertools.product([-1.0, 1.0], repeat=4)), dtype=np.float32)
    for n_alpha, alpha in ((1, alphas_k[:1]), (k, alphas_k)):
        for tbits in itertools.product([0, 1], repeat=p):
            tile = words_from_bits(tbits)
            dense = np.array([[(1.0 if tbits[ti] else -1.0) * float(alpha[ai if n_alpha > 1 else 0])
                               for (ti, ai) in row] for row in HAND_2x4[k]])
            y = orc.linear_forward(inputs, tile, alpha, 2, k)
            np.testing.assert_array_equal(y, inputs.astype(np.float64) @ dense.T)
            np.testing.assert_array_equal(orc.materialise(tile, alpha, 8, k).reshape(2, 4), dense)


@pytest.mark.parametrize("k", [1, 2, 4, 8])
def test_p5_bruteforce_pack_all_ternary_weights(k):
    p = 8 // k
    for w in itertools.product([-1.0, 0.0, 1.0], repeat=8):
        w = np.array(w, dtype=np.float32)
        tile, alpha = orc.pack_tile(w, k, k)
        # "reshape to k x p, sum over the k dimension, threshold at > 0" with library routines
        expect_bits = (w.reshape(k, p).sum(axis=0) > 0).astype(np.int64)
        assert bits_of(tile, p).tolist() == expect_bits.tolist()
        np.testing.assert_allclose(alpha, np.abs(w).reshape(k, p).mean(axis=1), atol=1e-7)


# ---------------------------------------------------------------- P6
def test_p6_invariants():
    rng = np.random.default_rng(9)
    cin, cout, k = 10, 6, 4   # p = 15, misaligned
    w = rng.standard_normal(cin * cout).astype(np.float32)
    x = rng.standard_normal((7, cin)).astype(np.float32)
    tile, alpha = orc.pack_tile(w, k, k)
    y = orc.linear_forward(x, tile, alpha, cout, k)
    p = cin * cout // k
    flipped = (~tile) & np.uint32((1 << p) - 1)
    np.testing.assert_array_equal(orc.linear_forward(x, flipped, alpha, cout, k), -y)
    np.testing.assert_array_equal(orc.linear_forward(x, tile, alpha * np.float32(2), cout, k), 2 * y)
    perm = rng.permutation(7)
    np.testing.assert_array_equal(orc.linear_forward(x[perm], tile, alpha, cout, k), y[perm])
    # negating W flips every tile entry whose sum is non-zero and leaves alpha unchanged
    tile_neg, alpha_neg = orc.pack_tile(-w, k, k)
    np.testing.assert_array_equal(tile_neg, flipped)
    np.testing.assert_array_equal(alpha_neg, alpha)


def test_p6_rejects_bad_shapes():
    w = np.zeros(10, dtype=np.float32)
    with pytest.raises(ValueError):
        orc.pack_tile(w, 3, 1)            # n not divisible by k
    with pytest.raises(ValueError):
        orc.pack_tile(w, 2, 3)            # n_alpha must be 1 or k


# ---------------------------------------------------------------- P7
def test_p7_storage_closed_form_matches_printed_tables():
    g = read_golden("paper_storage_tables.txt")
    KB = 1000.0
    # microcontroller MLP 784 -> 128 -> 10; only the first layer is tiled (k = 4, one alpha per tile)
    first_tiled_bytes = orc.tile_words(784 * 128, 4) * 4
    first_untiled_bytes = orc.tile_words(784 * 128, 1) * 4
    classifier_bytes = orc.tile_words(128 * 10, 1) * 4
    assert (first_tiled_bytes, first_untiled_bytes, classifier_bytes) == (3136, 12544, 160)
    tbn_storage = first_tiled_bytes + classifier_bytes + 4 * (4 + 1)
    bwnn_storage = first_untiled_bytes + classifier_bytes
    assert round(tbn_storage / KB, 2) == g["mcu_tbn4_storage_kb"][0]
    assert round(bwnn_storage / KB, 2) == g["mcu_bwnn_storage_kb"][0]
    act = 784 * 4 + 128 * 4   # float32 input image and hidden activations
    assert round((act + first_tiled_bytes) / KB, 1) == g["mcu_tbn4_max_memory_kb"][0]
    assert round((act + first_untiled_bytes) / KB, 1) == g["mcu_bwnn_max_memory_kb"][0]
    saving = 100.0 * (1 - (act + first_tiled_bytes) / (act + first_untiled_bytes))
    assert round(saving) == g["mcu_memory_saving_percent"][0]
    # ViT parameter memory: 32-bit -> 1-bit divides by 32, tiling with k = 4 divides by 4
    assert round(g["vit_fp32_param_mb"][0] / 32, 1) == g["vit_bwnn_param_mb"][0]
    assert round(g["vit_fp32_param_mb"][0] / 32 / 4, 1) == g["vit_tbn4_param_mb"][0]
    assert g["vit_fp32_param_mb"][0] / 4 == g["vit_fp32_tiled4_param_mb"][0]


# ---------------------------------------------------------------- P8
@pytest.mark.parametrize("N,C,H,W,O,kh,kw,stride,pad,k,n_alpha", [
    (2, 4, 9, 8, 6, 3, 3, (1, 1), (1, 1), 4, 1),    # p = 54 = 1.5 filters
    (1, 3, 7, 7, 8, 3, 3, (2, 2), (0, 0), 2, 2),    # whole filters per tile
    (2, 2, 6, 9, 4, 1, 1, (1, 1), (0, 0), 2, 1),    # 1x1
    (1, 5, 8, 5, 3, 2, 3, (1, 2), (1, 0), 5, 5),    # non-square kernel, mixed stride / pad
    (1, 2, 5, 5, 2, 5, 5, (1, 1), (2, 2), 4, 4),    # kernel as large as the image
])
def test_p8_conv_matches_torch_on_numpy_tiled_weight(N, C, H, W, O, kh, kw, stride, pad, k, n_alpha):
    rng = np.random.default_rng(100 + C * O + k)
    n = O * C * kh * kw
    w = rng.standard_normal(n).astype(np.float32)
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    tile, alpha = orc.pack_tile(w, k, n_alpha)
    y = orc.conv2d_forward(x, tile, alpha, O, kh, kw, k, stride=stride, pad=pad)
    dense = dense_from_numpy_tile(bits_of(tile, n // k), alpha, k, (O, C, kh, kw))
    ref = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(dense),
                                     stride=stride, padding=pad).numpy()
    assert y.shape == ref.shape
    np.testing.assert_allclose(y, ref, rtol=1e-12, atol=1e-12)
    # sampled entry point agrees with the full one
    idx = rng.integers(0, y.size, size=17)
    ys = orc.conv2d_forward_at(x, tile, alpha, O, kh, kw, k, idx, stride=stride, pad=pad)
    np.testing.assert_array_equal(ys, y.reshape(-1)[idx])


@pytest.mark.parametrize("M,cin,cout,k,n_alpha", [(5, 24, 10, 6, 6), (3, 30, 32, 6, 1), (4, 16, 16, 16, 16)])
def test_p8_linear_matches_numpy_matmul_on_numpy_tiled_weight(M, cin, cout, k, n_alpha):
    rng = np.random.default_rng(200 + cin + k)
    w = rng.standard_normal(cin * cout).astype(np.float32)
    x = rng.standard_normal((M, cin)).astype(np.float32)
    tile, alpha = orc.pack_tile(w, k, n_alpha)
    dense = dense_from_numpy_tile(bits_of(tile, cin * cout // k), alpha, k, (cout, cin))
    y = orc.linear_forward(x, tile, alpha, cout, k)
    np.testing.assert_allclose(y, x.astype(np.float64) @ dense.T, rtol=1e-12, atol=1e-12)
    rows = rng.integers(0, M, size=9)
    cols = rng.integers(0, cout, size=9)
    np.testing.assert_array_equal(orc.linear_forward_at(x, tile, alpha, cout, k, rows, cols), y[rows, cols])
