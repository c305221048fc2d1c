"""Pins of the column-tiled oracle (CPU only): brute force on tiny inputs, a hand-worked example, the special
cases in which the layer reduces to the flat-tiled oracle (itself pinned elsewhere) or to a library routine,
and invariants.  Each would fail on a plausible mistake: a transposed tile, a block index taken from the wrong
dimension, alpha attached to rows instead of column blocks, a wrong bit order.
"""
import itertools

import numpy as np
import pytest
import torch

from oracle import coltile_oracle as col
from oracle import tbn_oracle as flat


def _bit(tile, i):
    return (int(tile[i // 32]) >> (i % 32)) & 1


def _case(M, cin, out, k, n_alpha, seed):
    rng = np.random.default_rng(seed)
    w = rng.standard_normal((out, cin)).astype(np.float32)
    x = rng.standard_normal((M, cin)).astype(np.float32)
    tile, alpha = col.pack_coltile(w, out, cin, k, n_alpha)
    return w, x, tile, alpha


@pytest.mark.parametrize("M,cin,out,k,n_alpha", [(2, 6, 3, 3, 3), (1, 8, 5, 2, 1), (3, 12, 7, 4, 4), (2, 40, 9, 5, 5)])
def test_c1_bruteforce_loops(M, cin, out, k, n_alpha):
    w, x, tile, alpha = _case(M, cin, out, k, n_alpha, 11 + cin)
    q = cin // k
    want = np.zeros((M, out))
    for m, o, j in itertools.product(range(M), range(out), range(cin)):
        sign = 1.0 if _bit(tile, o * q + (j % q)) else -1.0
        want[m, o] += float(x[m, j]) * float(alpha[(j // q) if n_alpha == k else 0]) * sign
    got = col.linear_coltiled_forward(x, tile, alpha, out, k)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


def test_c2_hand_worked_pack_and_forward():
    # two column blocks of width 2: sums [[4, -1], [-1.5, 0]] -> bits 1, 0, 0, 0 (a zero sum gives -1)
    w = np.array([[1.0, -2.0, 3.0, 1.0], [-1.0, 0.5, -0.5, -0.5]], dtype=np.float32)
    tile, alpha = col.pack_coltile(w, 2, 4, 2, 2)
    assert tile.tolist() == [0b0001]
    assert alpha.tolist() == [1.125, 1.25]
    _, alpha1 = col.pack_coltile(w, 2, 4, 2, 1)
    assert alpha1.tolist() == [1.1875]
    # W_hat = [[1.125, -1.125, 1.25, -1.25], [-1.125, -1.125, -1.25, -1.25]]
    x = np.array([[1.0, 2.0, 4.0, 8.0]])
    y = col.linear_coltiled_forward(x, tile, alpha, 2, 2)
    assert y.tolist() == [[1.125 - 2.25 + 5.0 - 10.0, -1.125 - 2.25 - 5.0 - 10.0]]
    assert col.linear_coltiled_forward(x, tile, alpha, 2, 2, relu=True).tolist() == [[0.0, 0.0]]


def test_c3_k1_is_the_binary_weight_layer():
    w, x, tile, alpha = _case(4, 24, 10, 1, 1, 5)
    want = torch.nn.functional.linear(torch.from_numpy(x).double(),
                                      torch.from_numpy(np.where(w > 0, 1.0, -1.0) * np.abs(w.astype(np.float64)).mean()))
    got = col.linear_coltiled_forward(x, tile, alpha, 10, 1)
    np.testing.assert_allclose(got, want.numpy(), rtol=1e-6)   # alpha is rounded to float32 by the pack
    # same tile, same layer in the flat oracle (k = 1: the two layouts coincide)
    tile_f, alpha_f = flat.pack_tile(w, 1, 1)
    np.testing.assert_array_equal(tile, tile_f)
    np.testing.assert_array_equal(alpha, alpha_f)
    np.testing.assert_allclose(got, flat.linear_forward(x, tile_f, alpha_f, 10, 1), rtol=1e-13)


@pytest.mark.parametrize("k,n_alpha", [(2, 2), (4, 1), (8, 8)])
def test_c4_single_output_row_coincides_with_flat_tiling(k, n_alpha):
    # out = 1: the flat tile of in / k entries is the column tile
    w, x, tile, alpha = _case(5, 64, 1, k, n_alpha, 21 + k)
    tile_f, alpha_f = flat.pack_tile(w, k, n_alpha)
    np.testing.assert_array_equal(tile, tile_f)
    np.testing.assert_array_equal(alpha, alpha_f)
    np.testing.assert_allclose(col.linear_coltiled_forward(x, tile, alpha, 1, k),
                               flat.linear_forward(x, tile_f, alpha_f, 1, k), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("M,cin,out,k", [(3, 48, 17, 4), (2, 30, 8, 5)])
def test_c5_sum_of_binary_layers_over_the_column_blocks(M, cin, out, k):
    # Y = sum_c alpha_c * (X_c t^T): k calls of the flat oracle's k = 1 layer on the blocks of X
    w, x, tile, alpha = _case(M, cin, out, k, k, 31 + out)
    q = cin // k
    want = sum(float(alpha[c]) * flat.linear_forward(x[:, c * q:(c + 1) * q], tile, np.ones(1, np.float32), out, 1)
               for c in range(k))
    np.testing.assert_allclose(col.linear_coltiled_forward(x, tile, alpha, out, k), want, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("out,cin,k,n_alpha", [(6, 20, 4, 4), (3, 12, 3, 1), (16, 64, 8, 8)])
def test_c6_pack_equals_flat_pack_of_the_block_major_weight(out, cin, k, n_alpha):
    # moving column block c in front (k, out, q) turns the blocks into the rows of Eq. 1
    rng = np.random.default_rng(out * cin)
    w = rng.standard_normal((out, cin)).astype(np.float32)
    a = rng.standard_normal((out, cin)).astype(np.float32)
    q = cin // k
    wb = np.ascontiguousarray(w.reshape(out, k, q).transpose(1, 0, 2))
    ab = np.ascontiguousarray(a.reshape(out, k, q).transpose(1, 0, 2))
    for sep in (False, True):
        tile, alpha = col.pack_coltile(w, out, cin, k, n_alpha, a_real=a if sep else None)
        tile_f, alpha_f = flat.pack_tile(wb, k, n_alpha, a_real=ab if sep else None)
        np.testing.assert_array_equal(tile, tile_f)
        np.testing.assert_array_equal(alpha, alpha_f)


def test_c7_invariants():
    w, x, tile, alpha = _case(4, 40, 12, 5, 5, 77)
    q, k = 8, 5
    y = col.linear_coltiled_forward(x, tile, alpha, 12, k)
    # permuting the column blocks of X together with the alphas changes nothing
    perm = np.array([3, 0, 4, 2, 1])
    xp = x.reshape(4, k, q)[:, perm, :].reshape(4, 40)
    np.testing.assert_allclose(col.linear_coltiled_forward(xp, tile, alpha[perm], 12, k), y, rtol=1e-12, atol=1e-12)
    # equal alphas: the layer sees only the sum of the blocks of X
    a1 = np.full(k, 0.5, np.float32)
    xs = x.reshape(4, k, q).astype(np.float64).sum(axis=1)
    np.testing.assert_allclose(col.linear_coltiled_forward(x, tile, a1, 12, k),
                               0.5 * (xs @ col.tile_signs(tile, 12, q).T), rtol=1e-12, atol=1e-12)
    # flipping every tile bit negates the output; complementing keeps the padding bits out of it
    np.testing.assert_allclose(col.linear_coltiled_forward(x, ~tile, alpha, 12, k), -y, rtol=1e-12, atol=1e-12)
    # materialised weight: every column block is alpha_c times the first one divided by alpha_0
    w_hat = col.materialise_coltile(tile, alpha, 12, 40, k)
    for c in range(k):
        np.testing.assert_allclose(w_hat[:, c * q:(c + 1) * q] * float(alpha[0]), w_hat[:, :q] * float(alpha[c]), rtol=1e-12)
    assert set(np.unique(np.abs(w_hat[:, :q]))) == {float(alpha[0])}


def test_c8_rejects_bad_shapes():
    with pytest.raises(ValueError):
        col.pack_coltile(np.zeros((3, 10), np.float32), 3, 10, 4)
    with pytest.raises(ValueError):
        col.pack_coltile(np.zeros((3, 12), np.float32), 3, 12, 4, n_alpha=2)
    with pytest.raises(ValueError):
        col.materialise_coltile(np.zeros(2, np.uint32), np.ones(3, np.float32), 3, 12, 4)
