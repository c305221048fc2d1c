"""tbn_pack_tile_noalloc (the entry point for callers that cannot allocate) against tbn_pack_tile, through the
C ABI: two calls in a row on the same GPU, the second with a smaller input, must give the tile words bit for bit
and the same alpha (the bar of the packing tests: bits exact, alpha within one float32 ulp of the oracle -- here
against the existing entry point, whose kernels it shares, so equality is required)."""
import ctypes

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tbn():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2407_12075_amd import tbn as binding
    binding.lib()
    return binding


def _both(tbn, n, k, n_alpha, seed, separate_a):
    L = tbn.lib()
    rng = np.random.default_rng(seed)
    w = torch.from_numpy((0.02 * rng.standard_normal(n)).astype(np.float32)).cuda()
    a = torch.from_numpy((0.02 * rng.standard_normal(n)).astype(np.float32)).cuda() if separate_a else None
    words = tbn.tbn_tile_words(n, k)
    stream = torch.cuda.current_stream().cuda_stream
    # the existing entry point, with a caller-provided workspace
    need = tbn.tbn_pack_workspace_bytes(n, k, n_alpha)
    ws = torch.empty(need + 8, dtype=torch.uint8, device="cuda")
    tile_a = torch.full((words,), -1, dtype=torch.int32, device="cuda")
    alpha_a = torch.full((n_alpha,), -1.0, dtype=torch.float32, device="cuda")
    st = L.tbn_pack_tile(w.data_ptr(), None if a is None else a.data_ptr(), n, k, n_alpha, tile_a.data_ptr(),
                         alpha_a.data_ptr(), ws.data_ptr(), ws.numel(), stream)
    assert st == 0, L.tbn_last_error().decode()
    # the entry point that allocates nothing: inputs and outputs only
    tile_b = torch.full((words,), -1, dtype=torch.int32, device="cuda")
    alpha_b = torch.full((n_alpha,), -1.0, dtype=torch.float32, device="cuda")
    st = L.tbn_pack_tile_noalloc(w.data_ptr(), None if a is None else a.data_ptr(), n, k, n_alpha,
                                 tile_b.data_ptr(), alpha_b.data_ptr(), stream)
    assert st == 0, L.tbn_last_error().decode()
    torch.cuda.synchronize()
    np.testing.assert_array_equal(tile_b.cpu().numpy(), tile_a.cpu().numpy())
    np.testing.assert_array_equal(alpha_b.cpu().numpy().view(np.int32), alpha_a.cpu().numpy().view(np.int32))


def test_noalloc_pack_matches_pack_twice_in_a_row(tbn):
    _both(tbn, 4096 * 4096, 8, 8, 1, False)      # the metric layer: half of the scratch array
    _both(tbn, 1000 * 37, 37, 37, 2, True)       # smaller, ragged last word, separate tensor for the scalars
    _both(tbn, 999 * 5, 5, 1, 3, False)          # scalar-load variant, one alpha


def test_noalloc_pack_rejects_sizes_beyond_the_scratch_array(tbn):
    L = tbn.lib()
    n, k = 4096 * 16384, 2    # needs more than the built-in array holds
    assert tbn.tbn_pack_workspace_bytes(n, k, k) > (1 << 20)
    w = torch.zeros(16, dtype=torch.float32, device="cuda")   # never read: the call must fail before any launch
    out = torch.zeros(16, dtype=torch.int32, device="cuda")
    al = torch.zeros(2, dtype=torch.float32, device="cuda")
    st = L.tbn_pack_tile_noalloc(w.data_ptr(), None, n, k, k, out.data_ptr(), al.data_ptr(), None)
    assert st == 3, "TBN_ERR_UNSUPPORTED expected"
    assert b"scratch" in L.tbn_last_error()
    st = L.tbn_pack_tile_noalloc(None, None, 64, 2, 2, out.data_ptr(), al.data_ptr(), None)
    assert st == 1
