"""Pins of the binary-activation oracle (CPU only): brute force over bits on tiny inputs, the XNOR / popcount
identity computed with an independent unpacking of the bits, the k = 1 special case against a library matrix
product on the real weights (the binary layer of the cited XNOR-Net work: alpha * sign(X) sign(W)^T), the
agreement with the real-valued C oracle on inputs that are already +-1, closed forms and invariants.  Each
would fail on a plausible mistake: a reversed bit order, zero mapped to +1, alpha taken from the wrong index,
a transposed operand, padding bits that count.
"""
import itertools

import numpy as np
import pytest

from oracle import binact_oracle as ba
from oracle import tbn_oracle as flat


def _bit(words, i):
    return (int(words[i // 32]) >> (i % 32)) & 1


def _case(M, cin, out, k, n_alpha, seed):
    rng = np.random.default_rng(seed)
    w = rng.standard_normal(out * cin).astype(np.float32)
    x = rng.standard_normal((M, cin)).astype(np.float32)
    tile, alpha = flat.pack_tile(w, k, n_alpha)
    return w, x, tile, alpha


# ---- sign bits ----------------------------------------------------------------------------------

def test_b1_sign_rule_of_eq3_and_padding():
    x = np.array([[0.0, -0.0, 1e-38, -1e-38, np.nan, np.inf, -np.inf, 3.0, -2.0, 1e-45]], dtype=np.float32)
    bits = ba.sign_pack(x)
    assert bits.shape == (1, 1) and bits.dtype == np.uint32
    want = [0, 0, 1, 0, 0, 1, 0, 1, 0, 1]          # greater than zero, nothing else
    assert [(int(bits[0, 0]) >> j) & 1 for j in range(10)] == want
    assert int(bits[0, 0]) >> 10 == 0             # unused high bits stay zero


@pytest.mark.parametrize("M,cin", [(1, 1), (3, 31), (2, 32), (4, 33), (2, 95), (1, 130)])
def test_b2_sign_bits_by_loops(M, cin):
    rng = np.random.default_rng(5 + cin)
    x = rng.standard_normal((M, cin)).astype(np.float32)
    x[rng.random((M, cin)) < 0.1] = 0.0
    bits = ba.sign_pack(x)
    assert bits.shape == (M, (cin + 31) // 32)
    for m in range(M):
        for j in range(bits.shape[1] * 32):
            want = 1 if (j < cin and x[m, j] > 0) else 0
            assert _bit(bits[m], j) == want
    s = ba.signs(bits, cin)
    np.testing.assert_array_equal(s, np.where(x > 0, 1.0, -1.0))


# ---- the layer ----------------------------------------------------------------------------------

@pytest.mark.parametrize("M,cin,out,k,n_alpha", [(2, 6, 4, 3, 3), (1, 8, 5, 2, 1), (3, 12, 7, 4, 4), (2, 40, 9, 5, 5),
                                                 (2, 35, 6, 15, 15), (1, 33, 4, 1, 1)])
def test_b3_bruteforce_loops(M, cin, out, k, n_alpha):
    _, x, tile, alpha = _case(M, cin, out, k, n_alpha, 17 + cin)
    xbits = ba.sign_pack(x)
    p = out * cin // k
    want = np.zeros((M, out))
    for m, o, j in itertools.product(range(M), range(out), range(cin)):
        f = o * cin + j
        t = 1.0 if _bit(tile, f % p) else -1.0
        s = 1.0 if _bit(xbits[m], j) else -1.0
        want[m, o] += s * float(alpha[f // p if n_alpha == k else 0]) * t
    got = ba.linear_forward(xbits, cin, tile, alpha, out, k)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("M,cin,out,k", [(5, 64, 8, 4), (3, 96, 12, 2), (4, 50, 6, 3), (2, 256, 16, 8)])
def test_b4_xnor_popcount_identity(M, cin, out, k):
    """With one alpha, y / alpha = in - 2 * (number of positions where activation bit and weight bit differ)."""
    _, x, tile, alpha = _case(M, cin, out, k, 1, 23 + cin)
    xbits = ba.sign_pack(x)
    p = out * cin // k
    tbits = np.unpackbits(tile.view(np.uint8), bitorder="little")[:p]     # independent unpacking
    wbits = np.tile(tbits, k).reshape(out, cin)
    abits = np.unpackbits(xbits.view(np.uint8).reshape(M, -1), axis=1, bitorder="little")[:, :cin]
    hamming = (abits[:, None, :] ^ wbits[None, :, :]).sum(axis=2)
    want = float(alpha[0]) * (cin - 2.0 * hamming)
    got = ba.linear_forward(xbits, cin, tile, alpha, out, k)
    np.testing.assert_allclose(got, want, rtol=1e-13, atol=0)


@pytest.mark.parametrize("M,cin,out", [(4, 48, 10), (3, 77, 5)])
def test_b5_k1_is_the_binary_layer_of_real_weights(M, cin, out):
    """k = 1: alpha = mean |W| and the tile is sign(W), so Y = mean|W| * sign(X) sign(W)^T by a library product."""
    w, x, tile, alpha = _case(M, cin, out, 1, 1, 31 + cin)
    want = np.abs(w.astype(np.float64)).mean() * (np.where(x > 0, 1.0, -1.0) @ np.where(w.reshape(out, cin) > 0, 1.0, -1.0).T)
    got = ba.linear_forward(ba.sign_pack(x), cin, tile, alpha, out, 1)
    np.testing.assert_allclose(got, want, rtol=1e-6)     # alpha itself is a float32


@pytest.mark.parametrize("M,cin,out,k,n_alpha", [(3, 40, 12, 4, 4), (2, 36, 10, 3, 3), (4, 64, 8, 8, 1)])
def test_b6_equals_real_valued_oracle_on_sign_inputs(M, cin, out, k, n_alpha):
    """The real-valued layer (C oracle, pinned on its own) fed with the +-1 values themselves."""
    _, x, tile, alpha = _case(M, cin, out, k, n_alpha, 41 + cin)
    xbits = ba.sign_pack(x)
    s = np.where(x > 0, 1.0, -1.0)
    want = flat.linear_forward_alg1(s, tile, alpha, out, k)
    got = ba.linear_forward(xbits, cin, tile, alpha, out, k)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


def test_b7_closed_forms_and_invariants():
    cin, out, k = 64, 8, 4
    p = cin * out // k
    tile = np.full(p // 32, 0xFFFFFFFF, dtype=np.uint32)                # every weight +1
    alpha = np.array([0.5, 1.0, 2.0, 4.0], dtype=np.float32)
    ones = np.full((1, cin // 32), 0xFFFFFFFF, dtype=np.uint32)         # every activation +1
    y = ba.linear_forward(ones, cin, tile, alpha, out, k)
    # p = 128 = two rows of 64: rows 2c and 2c + 1 belong to copy c
    np.testing.assert_array_equal(y[0], np.repeat(alpha.astype(np.float64), 2) * cin)
    zeros = np.zeros_like(ones)                                         # every activation -1
    np.testing.assert_array_equal(ba.linear_forward(zeros, cin, tile, alpha, out, k), -y)
    # one activation flipped changes every output by exactly 2 * alpha of its row
    one_off = ones.copy()
    one_off[0, 0] ^= np.uint32(1 << 5)
    np.testing.assert_array_equal(y - ba.linear_forward(one_off, cin, tile, alpha, out, k),
                                  (2.0 * np.repeat(alpha.astype(np.float64), 2))[None, :])
    # complementing every activation bit negates the output
    rng = np.random.default_rng(3)
    xb = rng.integers(0, 2 ** 32, size=(3, cin // 32), dtype=np.uint64).astype(np.uint32)
    tl = rng.integers(0, 2 ** 32, size=p // 32, dtype=np.uint64).astype(np.uint32)
    np.testing.assert_array_equal(ba.linear_forward(~xb, cin, tl, alpha, out, k), -ba.linear_forward(xb, cin, tl, alpha, out, k))


def test_b8_padding_bits_do_not_count():
    cin, out, k = 40, 4, 2
    rng = np.random.default_rng(9)
    tile = rng.integers(0, 2 ** 32, size=(cin * out // k + 31) // 32, dtype=np.uint64).astype(np.uint32)
    alpha = np.array([0.25], dtype=np.float32)
    xb = rng.integers(0, 2 ** 32, size=(2, 2), dtype=np.uint64).astype(np.uint32)
    dirty = xb.copy()
    dirty[:, 1] |= np.uint32(0xFFFFFF00)       # bits 40 .. 63 of a row are not activations
    np.testing.assert_array_equal(ba.linear_forward(xb, cin, tile, alpha, out, k), ba.linear_forward(dirty, cin, tile, alpha, out, k))


def test_b9_planted_mistakes_fail_the_pins():
    """The pins above can see the mistakes they are meant for: plant each in a copy of the oracle's steps."""
    _, x, tile, alpha = _case(3, 40, 12, 4, 4, 77)
    xbits = ba.sign_pack(x)
    good = ba.linear_forward(xbits, 40, tile, alpha, 12, 4)
    s = np.where(x > 0, 1.0, -1.0)
    want = flat.linear_forward_alg1(s, tile, alpha, 12, 4)
    np.testing.assert_allclose(good, want, rtol=1e-12)
    # reversed bit order inside a word
    rev = np.array([[int(f"{int(w):032b}"[::-1], 2) for w in row] for row in xbits], dtype=np.uint32)
    assert not np.allclose(ba.linear_forward(rev, 40, tile, alpha, 12, 4), want)
    # zero mapped to +1
    xz = x.copy()
    xz[0, :5] = 0.0
    assert not np.array_equal(ba.sign_pack(xz), ba.sign_pack(np.where(xz == 0, 1.0, xz)))
    # one alpha where there are k
    assert not np.allclose(ba.linear_forward(xbits, 40, tile, alpha[:1].repeat(4), 12, 4), want)


def test_b10_sign_outputs_by_loops_and_two_layer_chain():
    """Bits out: the sign of every output by loops over the definition; a chain of two layers on bits equals the
    real-valued C oracle fed with the +-1 values between the layers."""
    M, cin, hid, out, k = 3, 40, 24, 10, 4
    _, x, t1, a1 = _case(M, cin, hid, k, k, 91)
    a1[1] = -a1[1]                                  # a negative alpha flips the signs of its copy
    _, _, t2, a2 = _case(M, hid, out, 2, 1, 92)
    xb = ba.sign_pack(x)
    hb = ba.linear_forward_signs(xb, cin, t1, a1, hid, k)
    assert hb.shape == (M, 1) and hb.dtype == np.uint32
    y1 = flat.linear_forward_alg1(np.where(x > 0, 1.0, -1.0), t1, a1, hid, k)
    for m in range(M):
        for o in range(32):
            assert _bit(hb[m], o) == (1 if (o < hid and y1[m, o] > 0) else 0)
    want = flat.linear_forward_alg1(np.where(y1 > 0, 1.0, -1.0), t2, a2, out, 2)
    got = ba.linear_forward(hb, hid, t2, a2, out, 2)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)
    # an output that is exactly zero gives bit 0: all weights +1, half of the activations +1
    tile = np.full(2, 0xFFFFFFFF, dtype=np.uint32)
    half = np.array([[0x0000FFFF]], dtype=np.uint32)
    assert int(ba.linear_forward_signs(half, 32, tile, np.array([1.0], dtype=np.float32), 2, 1)[0, 0]) == 0
