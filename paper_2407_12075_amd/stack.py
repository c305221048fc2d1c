"""Chains of tiled-bit fully-connected layers on top of the C ABI: whole-block execution without host
work between the layers (one HIP graph replay per chain) and the peak-memory accounting of the paper's
GPU experiment (Section "GPU Inference Kernel", Table 7 / Figure 5) on a synthetic stack of the same
layer sizes.

Nothing here computes: every layer is one ``tbn_linear_forward`` call (ReLU fused where asked for);
PyTorch supplies device memory, the stream and the graph capture.  Only the packed tile and the alphas
of a layer are ever resident, which is what the paper's memory figures are about.

    python -m paper_2407_12075_amd.stack            # memory table + eager / graph timings on cuda:0
"""
from __future__ import annotations

import json
import sys
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np
import torch

from . import tbn
from . import workloads as wl


@dataclass
class LayerSpec:
    cin: int
    cout: int
    relu: bool = False


# The ImageNet ViT of the paper's memory experiment: six attention layers of about 8.4 M parameters each
# (Q, K, V, output projection and a feed-forward pair) and activations of 65,536 values per layer, i.e.
# 64 tokens of width 1024 with a hidden width of 2048.  The attention product itself has no weights; the
# stack keeps the weight and activation sizes and chains the projections.
VIT_DIM, VIT_HIDDEN, VIT_TOKENS, VIT_BLOCKS = 1024, 2048, 64, 6


def vit_stack_specs(blocks: int = VIT_BLOCKS, dim: int = VIT_DIM, hidden: int = VIT_HIDDEN) -> List[LayerSpec]:
    specs: List[LayerSpec] = []
    for _ in range(blocks):
        specs += [LayerSpec(dim, dim), LayerSpec(dim, dim), LayerSpec(dim, dim), LayerSpec(dim, dim),
                  LayerSpec(dim, hidden, relu=True), LayerSpec(hidden, dim)]
    return specs


class TiledStack:
    """Packed tiles and alphas of a chain of layers, and its forward pass."""

    def __init__(self, specs: Sequence[LayerSpec], k: int, per_tile_alpha: bool = True, seed: int = 0,
                 device: str = "cuda"):
        self.specs = list(specs)
        self.k = k
        self.tiles: List[torch.Tensor] = []
        self.alphas: List[torch.Tensor] = []
        for i, s in enumerate(self.specs):
            n = s.cin * s.cout
            if n % k:
                raise ValueError(f"layer {i}: {n} weights are not divisible by k = {k}")
            # synthetic real weights (the recipe of the workload module), scaled so that activations keep
            # their magnitude through the chain; they are dropped as soon as the tile is packed
            w = torch.from_numpy(wl.draw_w_real(n, 90 + seed, i)).to(device) * float(50.0 / np.sqrt(s.cin))
            tile, alpha = tbn.tbn_pack_tile(w, k, k if per_tile_alpha else 1)
            self.tiles.append(tile)
            self.alphas.append(alpha)
            del w
        torch.cuda.synchronize()

    def param_bytes(self) -> int:
        return sum(t.numel() * 4 for t in self.tiles) + sum(a.numel() * 4 for a in self.alphas)

    def forward(self, x: torch.Tensor, buffers: Optional[List[torch.Tensor]] = None) -> torch.Tensor:
        """Layer after layer on the current stream; a new output tensor per layer unless buffers are given."""
        h = x
        for i, s in enumerate(self.specs):
            y = None if buffers is None else buffers[i]
            h = tbn.tbn_linear_forward(h, self.tiles[i], self.alphas[i], s.cout, self.k, y=y,
                                       flags=tbn.TBN_FLAG_RELU if s.relu else 0)
        return h

    def capture(self, x: torch.Tensor) -> Tuple[torch.cuda.CUDAGraph, torch.Tensor]:
        """One HIP graph for the whole chain on static buffers: replay() recomputes the returned tensor
        from the current contents of x without any host work between the layers."""
        buffers = [torch.empty((x.shape[0], s.cout), dtype=x.dtype, device=x.device) for s in self.specs]
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):   # warm-up outside the capture (first launches set kernel attributes)
            self.forward(x, buffers)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            out = self.forward(x, buffers)
        self._static = buffers   # keep the graph's buffers alive
        return graph, out


class DenseStack:
    """The same chain with ordinary float32 weight matrices (the full-precision row of the table)."""

    def __init__(self, specs: Sequence[LayerSpec], seed: int = 0, device: str = "cuda"):
        self.specs = list(specs)
        self.weights = [torch.from_numpy(wl.draw_w_real(s.cin * s.cout, 90 + seed, i)).to(device).view(s.cout, s.cin)
                        for i, s in enumerate(self.specs)]

    def param_bytes(self) -> int:
        return sum(w.numel() * 4 for w in self.weights)

    def forward(self, x: torch.Tensor) -> torch.Tensor:
        h = x
        for w, s in zip(self.weights, self.specs):
            h = torch.nn.functional.linear(h, w)
            if s.relu:
                h = torch.relu(h)
        return h


def _peak_during(fn) -> Tuple[int, int]:
    """(peak bytes allocated while fn runs, bytes allocated before it)."""
    torch.cuda.synchronize()
    base = torch.cuda.memory_allocated()
    torch.cuda.reset_peak_memory_stats()
    out = fn()
    torch.cuda.synchronize()
    peak = torch.cuda.max_memory_allocated()
    del out
    return peak, base


def _time_us(fn, iters: int = 50, warm: int = 5) -> float:
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / iters


def memory_report(dtype: torch.dtype = torch.float32) -> dict:
    """Peak and parameter memory of one forward pass over the ViT-shaped stack (one image = 64 tokens)."""
    specs = vit_stack_specs()
    x = torch.from_numpy(wl.draw_x((VIT_TOKENS, VIT_DIM), 91, 0, "f32")[0]).cuda().to(dtype)
    rows = {}
    n_weights = sum(s.cin * s.cout for s in specs)
    for name, build in (("full precision (float32 matrices, torch linear)", lambda: DenseStack(specs)),
                        ("binary weights, untiled (k = 1)", lambda: TiledStack(specs, 1)),
                        ("tiled bit network, k = 4", lambda: TiledStack(specs, 4)),
                        ("tiled bit network, k = 8", lambda: TiledStack(specs, 8))):
        if name.startswith("full") and dtype != torch.float32:
            continue
        torch.cuda.empty_cache()
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        model = build()
        params = model.param_bytes()
        resident = torch.cuda.memory_allocated() - before
        peak, base = _peak_during(lambda: model.forward(x))
        rows[name] = {"parameter_bytes": params, "resident_after_build_bytes": resident,
                      "peak_bytes": peak - before, "activation_peak_bytes": peak - base,
                      "parameter_share": params / max(peak - before, 1)}
        del model
    return {"weights": n_weights, "tokens": VIT_TOKENS, "dtype": str(dtype), "rows": rows}


def graph_report(dtype: torch.dtype = torch.bfloat16) -> dict:
    """Eager launches against one graph replay: the ViT-shaped stack at 64 tokens and a chain of eight
    4096 x 4096 layers (k = 8) at batch 1 and 16."""
    out = {}
    cases = [("vit stack, 36 layers, 64 tokens", vit_stack_specs(), 4, VIT_TOKENS, VIT_DIM),
             ("8 x (4096 -> 4096, k = 8), batch 1", [LayerSpec(4096, 4096, relu=True)] * 8, 8, 1, 4096),
             ("8 x (4096 -> 4096, k = 8), batch 16", [LayerSpec(4096, 4096, relu=True)] * 8, 8, 16, 4096)]
    for name, specs, k, M, cin in cases:
        model = TiledStack(specs, k)
        x = torch.from_numpy(wl.draw_x((M, cin), 92, 0, "f32")[0]).cuda().to(dtype)
        eager = _time_us(lambda: model.forward(x))
        graph, y = model.capture(x)
        ref = model.forward(x)
        graph.replay()
        torch.cuda.synchronize()
        same = bool(torch.equal(ref, y))
        replay = _time_us(graph.replay)
        out[name] = {"layers": len(specs), "eager_us": eager, "graph_us": replay, "graph_equals_eager": same}
        del model, graph
    return out


def main(argv: Sequence[str]) -> int:
    if not torch.cuda.is_available():
        print("this report needs a GPU", file=sys.stderr)
        return 1
    rep = {"memory_float32": memory_report(torch.float32), "memory_bfloat16": memory_report(torch.bfloat16),
           "graph": graph_report()}
    print(json.dumps(rep, indent=1))
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
