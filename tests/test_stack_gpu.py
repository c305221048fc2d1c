"""GPU tests of the layer chains: a chain of tiled-bit layers against the oracle applied layer by
layer, one HIP graph per chain against the eager launches (several replays, eager work in between),
and the parameter-memory closed form of the paper's GPU memory experiment.
"""
import numpy as np
import pytest
import torch

from oracle import tbn_oracle as orc
from paper_2407_12075_amd import workloads as wl
from tests.parity_util import assert_close

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def stack():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2407_12075_amd import tbn as binding
    binding.lib()  # fails loudly if the HIP library is missing
    from paper_2407_12075_amd import stack as mod
    return mod


def _oracle_chain(x, specs, k, seed, dtype):
    """Reference: the oracle layer by layer; bf16 chains round every layer's output to bf16 as the
    library does (outputs have the activations' dtype)."""
    h = x.astype(np.float64)
    for i, s in enumerate(specs):
        w = wl.draw_w_real(s.cin * s.cout, 90 + seed, i) * np.float32(50.0 / np.sqrt(s.cin))
        tile, alpha = orc.pack_tile(w.astype(np.float32), k, k)
        h = orc.linear_forward(h.astype(np.float32), tile, alpha, s.cout, k)
        if s.relu:
            h = np.maximum(h, 0.0)
        if dtype == "bf16":
            h = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(h.astype(np.float32))).reshape(h.shape).astype(np.float64)
    return h


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("M", [5, 150])
def test_chain_matches_oracle_layer_by_layer(stack, M, dtype):
    specs = [stack.LayerSpec(96, 160, relu=True), stack.LayerSpec(160, 64), stack.LayerSpec(64, 96, relu=True)]
    k, seed = 4, 3
    model = stack.TiledStack(specs, k, seed=seed)
    xv, bits = wl.draw_x((M, 96), 93, 0, dtype)
    x = torch.from_numpy(xv).cuda()
    if dtype == "bf16":
        x = torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    y = model.forward(x)
    torch.cuda.synchronize()
    ref = _oracle_chain(xv, specs, k, seed, dtype)
    assert_close(y.float().cpu().numpy().astype(np.float64), ref, dtype, f"chain of three layers, M={M}, {dtype}")


def test_parameter_bytes_closed_form(stack):
    specs = stack.vit_stack_specs(blocks=1)
    for k in (1, 4, 8):
        model = stack.TiledStack(specs, k)
        want = sum(((s.cin * s.cout // k + 31) // 32) * 4 + 4 * k for s in specs)
        assert model.param_bytes() == want
        del model
    # the paper's fourfold parameter saving at k = 4 (alphas aside)
    n = sum(s.cin * s.cout for s in specs)
    assert abs(stack.TiledStack(specs, 4).param_bytes() - n / 8 / 4) <= 4 * 4 * len(specs)


@pytest.mark.parametrize("M", [1, 16, 64])
def test_graph_replays_equal_eager(stack, M):
    specs = [stack.LayerSpec(1024, 1024, relu=True)] * 3 + [stack.LayerSpec(1024, 512)]
    model = stack.TiledStack(specs, 8)
    x = torch.randn((M, 1024), device="cuda", generator=torch.Generator(device="cuda").manual_seed(5)).bfloat16()
    graph, y = model.capture(x)
    for rep in range(4):
        # new contents in the static input, eager work and a synchronisation between the replays
        x.copy_(torch.randn((M, 1024), device="cuda", generator=torch.Generator(device="cuda").manual_seed(10 + rep)))
        ref = model.forward(x).clone()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, ref), f"replay {rep} differs from the eager chain"
