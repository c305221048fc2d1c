#!/usr/bin/env python3
"""Benchmark of the libtbn hot path on one MI355X.

A step is one pass of the whole path on the shape the headline metric is quoted on (tiled-bit
linear layer 4096 x 4096, k = 8, bfloat16 activations, one alpha per tile):

    tbn_pack_tile(W_real)  ->  tbn_linear_forward at batch 8192, 16 and 1

with all inputs resident in HBM.  `value` is the dense-equivalent rate of the three forward
passes, 2 * in * out * (8192 + 16 + 1) flop per step, over the wall time of the step (so the
packing pass and launch gaps count against it).  The `roofline` object describes the dominant
kernel, the batch-8192 forward, whose duration is measured with events on the launch stream
inside the timed steps.  `cpu_baseline` times the CPU oracle on a sample of the same batch.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline] [--all-configs]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16
MFMA_FP4_PEAK_TFLOPS = 10100.0  # dense 4-bit float (the binary-activation kernel multiplies +-1 in that format)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target CPU time of the oracle sample")
    ap.add_argument("--all-configs", action="store_true", help="also time the other layer shapes (extra lines on stderr)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a plain device copy of 256 MiB (for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--odd-shapes", action="store_true",
                    help="time shapes the matrix-core kernels decline (row lengths no multiple of 8, 5x5 / 7x7 windows, sign rows "
                         "no multiple of 256 bits): default dispatch against the one-thread-per-output kernels; prints one JSON object")
    ap.add_argument("--binact-only", action="store_true",
                    help="run only the binary-activation path on the metric shape: sign packing, the layer with bf16 outputs and "
                         "with sign-bit outputs, --steps times each (for rocprofv3 counter runs of these kernels)")
    return ap.parse_args()


def device_inputs(c, torch, wl):
    """Seeded synthetic tensors of workload c on the GPU (same recipe as the parity tests)."""
    w = torch.from_numpy(wl.draw_w_real(c.n, c.cfg, c.layer)).cuda()
    xv, xb = wl.draw_x((c.M, c.cin), c.cfg, c.layer, c.dtype)
    if xb is not None:
        import numpy as np
        x = torch.from_numpy(xb.view(np.int16)).cuda().view(torch.bfloat16)
    else:
        x = torch.from_numpy(xv).cuda()
    return w, x, xv


def event_pair(torch):
    return torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (the tiled-bit forward needs no second "
              "device); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2407_12075_amd import tbn, workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    tbn.lib()
    torch.cuda.set_device(0)

    if args.copy_calibration:
        a = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        b = torch.empty_like(a)
        for _ in range(5):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": a.numel(), "copy_bytes_written": b.numel(), "launches": 5}))
        return

    if args.odd_shapes:
        print(json.dumps(odd_shapes(torch, tbn, max(3, min(args.steps, 20)))))
        return

    if args.binact_only:
        c = wl.METRIC
        w, x, _ = device_inputs(c, torch, wl)
        tile, alpha = tbn.tbn_pack_tile(w, c.k, c.n_alpha)
        bits = tbn.tbn_sign_pack(x)
        y = torch.empty((c.M, c.cout), dtype=torch.bfloat16, device="cuda")
        yb = torch.empty((c.M, c.cout // 32), dtype=torch.int32, device="cuda")
        for _ in range(args.steps):
            tbn.tbn_sign_pack(x, xbits=bits)
            tbn.tbn_linear_forward_binact(bits, c.cin, tile, alpha, c.cout, c.k, y=y)
            tbn.tbn_linear_forward_binact(bits, c.cin, tile, alpha, c.cout, c.k, y=yb, flags=tbn.TBN_FLAG_SIGN_OUT)
        torch.cuda.synchronize()
        print(json.dumps({"workload": c.name, "calls_of_each": args.steps,
                          "algorithmic_bytes": {"sign_pack": c.M * c.cin * 2 + c.M * c.cin // 8,
                                                "layer_bf16_out": c.M * c.cin // 8 + c.p // 8 + c.M * c.cout * 2,
                                                "layer_sign_out": c.M * c.cin // 8 + c.p // 8 + c.M * c.cout // 8}}))
        return

    big = wl.METRIC                       # batch 8192
    mid, small = wl.CFG4[1], wl.CFG4[0]   # batch 16 and 1
    cin, cout, k, n_alpha = big.cin, big.cout, big.k, big.n_alpha
    n = big.n

    w_real, x_big, x_big_vals = device_inputs(big, torch, wl)
    _, x_mid, _ = device_inputs(mid, torch, wl)
    _, x_small, _ = device_inputs(small, torch, wl)
    tile = torch.empty(tbn.tbn_tile_words(n, k), dtype=torch.int32, device="cuda")
    alpha = torch.empty(n_alpha, dtype=torch.float32, device="cuda")
    workspace = torch.empty(tbn.tbn_pack_workspace_bytes(n, k, n_alpha) + 8, dtype=torch.uint8, device="cuda")
    y_big = torch.empty((big.M, cout), dtype=torch.bfloat16, device="cuda")
    y_mid = torch.empty((mid.M, cout), dtype=torch.bfloat16, device="cuda")
    y_small = torch.empty((small.M, cout), dtype=torch.bfloat16, device="cuda")

    # the four library calls of a step, marshalled once (tbn_bind): the same C calls on the same buffers every step, so
    # that the host issues a step well inside the time the GPU needs for it
    pack = tbn.tbn_bind(tbn.tbn_pack_tile, w_real, k, n_alpha, tile_out=tile, alpha_out=alpha, workspace=workspace)
    fwd_big = tbn.tbn_bind(tbn.tbn_linear_forward, x_big, tile, alpha, cout, k, y=y_big)
    fwd_mid = tbn.tbn_bind(tbn.tbn_linear_forward, x_mid, tile, alpha, cout, k, y=y_mid)
    fwd_small = tbn.tbn_bind(tbn.tbn_linear_forward, x_small, tile, alpha, cout, k, y=y_small)

    def step(ev=None):
        pack()
        if ev is not None:
            ev[0].record()
        fwd_big()
        if ev is not None:
            ev[1].record()
        fwd_mid()
        fwd_small()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    events = [event_pair(torch) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(events[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    flop_per_step = 2.0 * cin * cout * (big.M + mid.M + small.M)
    value = flop_per_step / (ms_per_step * 1e-3) / 1e12

    kern_ms = sorted(e0.elapsed_time(e1) for e0, e1 in events)
    kern_avg_ms = sum(kern_ms) / len(kern_ms)
    # algorithmic bytes of the batch-8192 forward: X read once, Y written once, packed tile and alpha read once
    alg_bytes = big.M * cin * 2 + big.M * cout * 2 + big.p // 8 + n_alpha * 4
    achieved = alg_bytes / (kern_avg_ms * 1e-3) / 1e9
    U = big.p // cin
    alg_flop = 2.0 * big.M * cin * U
    traffic, traffic_src = measured_traffic()
    roofline = {
        "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic, "traffic_source": traffic_src,
        "kernel": "linear_block_bf16_kernel (batch 8192)", "avg_kernel_ms": round(kern_avg_ms, 5),
        "median_kernel_ms": round(kern_ms[len(kern_ms) // 2], 5),
        "algorithmic_bytes": alg_bytes,
        "algorithmic_tflops": round(alg_flop / (kern_avg_ms * 1e-3) / 1e12, 1),
        "mfma_frac": round(alg_flop / (kern_avg_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
        "dense_equiv_tflops": round(2.0 * big.M * cin * cout / (kern_avg_ms * 1e-3) / 1e12, 1),
    }

    cpu_baseline = None
    if not args.no_cpu_baseline:
        from oracle import tbn_oracle as orc
        tile_h = tile.cpu().numpy().view(np.uint32)
        alpha_h = alpha.cpu().numpy()
        # Calibrate with two short calls (every call first materialises the dense weight, a fixed cost),
        # then time a sample sized for the requested CPU seconds.
        def timed_rows(r):
            t = time.perf_counter()
            orc.linear_forward(x_big_vals[:r], tile_h, alpha_h, cout, k)
            return time.perf_counter() - t
        timed_rows(8)
        t_a, t_b = timed_rows(16), timed_rows(80)
        per_row = max((t_b - t_a) / 64, 1e-6)
        fixed = max(t_a - 16 * per_row, 0.0)
        rows = int(min(big.M, max(64, (args.cpu_seconds - fixed) / per_row)))
        t = time.perf_counter()
        orc.linear_forward(x_big_vals[:rows], tile_h, alpha_h, cout, k)
        dt = time.perf_counter() - t
        cpu_baseline = {
            "value": round(2.0 * cin * cout * rows / dt / 1e12, 5), "unit": "dense-equiv TFLOP/s",
            "cores": orc.threads(), "kind": "oracle",
            "sample": f"first {rows} of the 8192 batch rows of the 4096x4096 k=8 forward "
                      f"(dense weight materialised from the tile, double accumulation), {dt:.1f} s",
        }

    line = {
        "metric": "dense-equiv TFLOP/s, TBN linear 4096x4096 k=8 at batch 1/16/8192 (pack + three forwards per step)",
        "value": round(value, 2), "unit": "TFLOP/s (dense-equivalent)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "metric: tiled-bit linear in=out=4096, k=8, 8 alphas, bf16, batch 8192 + 16 + 1, "
                               "preceded by tbn_pack_tile of the 4096x4096 real weight",
                   "n": n, "k": k, "p_bits": big.p, "unique_rows": U},
        "hbm_gbs": round(achieved, 1),
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
    }

    if args.all_configs:
        line["other_configs"] = time_other_configs(torch, tbn, wl)
    print(json.dumps(line))


def measured_traffic():
    """HBM bytes per launch of the batch-8192 forward from the committed rocprofv3 counter summary.

    bench.py cannot collect hardware counters itself; the figure is read from the summary that the
    documented rocprofv3 --pmc runs of this very command produced (FETCH_SIZE and WRITE_SIZE, each
    scaled by the same counter on a plain copy of known size).  None when no summary is there.
    """
    path = os.path.join(ROOT, "profiles", "linear_block_bf16_metric_4096x4096_k8_hbm_traffic.txt")
    try:
        vals = {}
        for ln in open(path):
            if "=" in ln and not ln.lstrip().startswith("#"):
                key, v = ln.split("=", 1)
                vals[key.strip()] = v.strip()
        return int(float(vals["fetch_bytes_per_launch"]) + float(vals["write_bytes_per_launch"])), \
            "profiles/" + os.path.basename(path)
    except (OSError, KeyError, ValueError):
        return None, None


MFMA_F32X3_NOTE = "float32 activations run as three exact bf16 terms: algorithmic flops x 3 on the bf16 matrix pipe"


def _timed_us(torch, fn, iters, warm=3):
    """Mean microseconds per call of fn(i), events around `iters` back-to-back calls on the current stream."""
    for i in range(warm):
        fn(i)
    torch.cuda.synchronize()
    e0, e1 = event_pair(torch)
    e0.record()
    for i in range(iters):
        fn(i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / iters


def _graph_us(torch, fn, calls=20, replays=20):
    """Microseconds per call when `calls` calls of fn(i) are captured in one HIP graph and the graph is replayed."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for i in range(3):
            fn(i)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for i in range(calls):
            fn(i)
    graph.replay()
    torch.cuda.synchronize()
    e0, e1 = event_pair(torch)
    e0.record()
    for _ in range(replays):
        graph.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / (replays * calls)


def measure_ceilings(torch, tbn):
    """What the chip gives kernels that do nothing else, measured like the layer kernels: the launch floor (eager
    and as graph replays), a streaming read and copy of 512 MiB (larger than the last-level cache), a loop of
    nothing but bf16 MFMAs."""
    out = {}
    out["empty_kernel_eager_us"] = round(_timed_us(torch, lambda i: tbn.tbn_diag_empty_launch(), 200, warm=20), 3)
    out["empty_kernel_graph_us"] = round(_graph_us(torch, lambda i: tbn.tbn_diag_empty_launch(), calls=50), 3)
    n = 512 << 20
    src = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty(n, dtype=torch.uint8, device="cuda")
    us = _timed_us(torch, lambda i: tbn.tbn_diag_stream(src), 10)
    out["stream_read_gbs"] = round(n / us / 1e3, 1)
    us = _timed_us(torch, lambda i: tbn.tbn_diag_stream(src, dst), 10)
    out["stream_copy_gbs"] = round(2 * n / us / 1e3, 1)   # bytes read + bytes written
    del src, dst
    blocks, iters = 1024, 2000
    us = _timed_us(torch, lambda i: tbn.tbn_diag_mfma(blocks, iters), 5, warm=2)
    out["mfma_bf16_loop_tflops"] = round(blocks * 4 * iters * 8 * 2.0 * 32 * 32 * 16 / us / 1e6, 1)
    us = _timed_us(torch, lambda i: tbn.tbn_diag_mfma_fp4(blocks, iters), 5, warm=2)
    out["mfma_fp4_loop_tflops"] = round(blocks * 4 * iters * 8 * 2.0 * 32 * 32 * 64 / us / 1e6, 1)
    return out


def _roof_fields(us, byts, alg_flop, ceil, flop_factor=1.0):
    """Fractions of the roofs for one timing: datasheet (HBM 8 TB/s, bf16 MFMA 2.5 PFLOP/s) and measured ceilings
    (streaming copy, MFMA-only loop).  The roof time is the larger of the memory and the matrix time."""
    t_hbm = byts / (HBM_PEAK_GBS * 1e3)
    t_mfma = alg_flop * flop_factor / (MFMA_BF16_PEAK_TFLOPS * 1e6)
    t_hbm_m = byts / (ceil["stream_copy_gbs"] * 1e3)
    t_mfma_m = alg_flop * flop_factor / (ceil["mfma_bf16_loop_tflops"] * 1e6)
    return {"roof_us": round(max(t_hbm, t_mfma), 2), "bound": "hbm" if t_hbm >= t_mfma else "mfma",
            "frac_of_roof": round(max(t_hbm, t_mfma) / us, 3),
            "frac_of_measured_ceiling": round(max(t_hbm_m, t_mfma_m) / us, 3)}


def time_other_configs(torch, tbn, wl, iters=30):
    """Kernel time of the remaining layer shapes: warm (one buffer set, which the 256 MiB last-level cache can
    hold) and cold (rotating buffer sets that total more than 320 MB), against the datasheet roofs and against
    the ceilings measured in the same process; launch floor and graph replays for the launch-bound rows."""
    import numpy as np
    out = {}
    ceil = measure_ceilings(torch, tbn)
    out["ceilings"] = ceil
    cold_target = 320e6

    def linear_row(c, flags=0, label=None):
        w, x, _ = device_inputs(c, torch, wl)
        tile, alpha = tbn.tbn_pack_tile(w, c.k, c.n_alpha)
        esz = x.element_size()
        byts = (c.M * c.cin + c.M * c.cout) * esz + c.p // 8
        U = min(c.cout, c.p // int(np.gcd(c.cin, c.p)))
        alg_flop = 2.0 * c.M * c.cin * U
        nsets = int(min(96, max(2, -(-cold_target // byts) + 1)))
        xs = [x] + [x.clone() for _ in range(nsets - 1)]
        ys = [torch.empty((c.M, c.cout), dtype=x.dtype, device="cuda") for _ in range(nsets)]
        # calls marshalled once (tbn_bind), so that an eager timing of a short kernel shows the launch rather than Python
        calls = [tbn.tbn_bind(tbn.tbn_linear_forward, xs[j], tile, alpha, c.cout, c.k, y=ys[j], flags=flags) for j in range(nsets)]
        warm = _timed_us(torch, lambda i: calls[0](), iters)
        cold = _timed_us(torch, lambda i: calls[i % nsets](), max(iters, nsets), warm=nsets)
        factor = 3.0 if c.dtype == "f32" else 1.0
        row = {"kernel": tbn.tbn_linear_forward_kernel(x.dtype, c.M, c.cin, c.cout, c.k, c.n_alpha, flags, x.data_ptr(), ys[0].data_ptr()),
               "us": round(warm, 2), "cold_us": round(cold, 2), "cold_sets": nsets, "cold_set_bytes_total": int(nsets * byts),
               "dense_equiv_tflops": round(2.0 * c.M * c.cin * c.cout / warm / 1e6, 1),
               "alg_gbs": round(byts / warm / 1e3, 1), "alg_gbs_cold": round(byts / cold / 1e3, 1),
               "warm": _roof_fields(warm, byts, alg_flop, ceil, factor), "cold": _roof_fields(cold, byts, alg_flop, ceil, factor)}
        if c.M <= 64:   # launch-bound rows: against the floor, eagerly and as graph replays
            g = _graph_us(torch, lambda i: tbn.tbn_linear_forward(xs[0], tile, alpha, c.cout, c.k, y=ys[0], flags=flags))
            row["graph_us"] = round(g, 2)
            row["eager_over_floor"] = round(warm / ceil["empty_kernel_eager_us"], 2)
            row["graph_over_floor"] = round(g / ceil["empty_kernel_graph_us"], 2)
        out[label or c.name] = row
        ws = torch.empty(tbn.tbn_pack_workspace_bytes(c.n, c.k, c.n_alpha) + 8, dtype=torch.uint8, device="cuda")
        if label is None:
            nw = int(min(16, max(2, -(-cold_target // (c.n * 4)) + 1)))
            wsets = [w] + [w.clone() for _ in range(nw - 1)]
            us = _timed_us(torch, lambda i: tbn.tbn_pack_tile(wsets[0], c.k, c.n_alpha, tile_out=tile, alpha_out=alpha, workspace=ws), iters)
            usc = _timed_us(torch, lambda i: tbn.tbn_pack_tile(wsets[i % nw], c.k, c.n_alpha, tile_out=tile, alpha_out=alpha, workspace=ws),
                            max(iters, nw), warm=nw)
            out[c.name + ":pack"] = {"us": round(us, 2), "cold_us": round(usc, 2), "alg_gbs": round(c.n * 4 / us / 1e3, 1),
                                     "alg_gbs_cold": round(c.n * 4 / usc / 1e3, 1),
                                     "cold_frac_of_hbm_peak": round(c.n * 4 / usc / 1e3 / HBM_PEAK_GBS, 3),
                                     "cold_frac_of_stream_read": round(c.n * 4 / usc / 1e3 / ceil["stream_read_gbs"], 3)}

    lin = [wl.CFG1, *wl.CFG2, *wl.CFG4, wl.METRIC, *wl.CFG5, *wl.CFG5_MISALIGNED]
    for c in lin:
        linear_row(c)
    out["float32_note"] = MFMA_F32X3_NOTE
    # the same layers in the column-tiled layout (fold of the k column blocks + one +-1 product on in / k inputs)
    for c in (wl.METRIC, *wl.CFG5):
        w, x, _ = device_inputs(c, torch, wl)
        tile, alpha = tbn.tbn_pack_coltile(w.view(c.cout, c.cin), c.k, c.k)
        y = torch.empty((c.M, c.cout), dtype=x.dtype, device="cuda")
        ws = torch.empty(tbn.tbn_linear_coltiled_workspace_bytes(x, c.k), dtype=torch.uint8, device="cuda")
        us = _timed_us(torch, lambda i: tbn.tbn_linear_coltiled_forward(x, tile, alpha, c.cout, c.k, y=y, workspace=ws), iters)
        byts = (c.M * c.cin + c.M * c.cout) * x.element_size() + c.p // 8
        out[c.name + ":column_tiled"] = {"us": round(us, 2), "dense_equiv_tflops": round(2.0 * c.M * c.cin * c.cout / us / 1e6, 1),
                                         "alg_gbs": round(byts / us / 1e3, 1)}
        del w, x, y, ws
    # batch sweep on the metric layer (bf16): which kernel family serves which batch size, and at what cost
    c = wl.METRIC
    w, x, _ = device_inputs(c, torch, wl)
    tile, alpha = tbn.tbn_pack_tile(w, c.k, c.n_alpha)
    sweep = {}
    for M in (1, 16, 64, 128, 256, 512, 1024, 2048, 4096, 8192):
        xm = x[:M].contiguous()
        ym = torch.empty((M, c.cout), dtype=x.dtype, device="cuda")
        call = tbn.tbn_bind(tbn.tbn_linear_forward, xm, tile, alpha, c.cout, c.k, y=ym)
        us = _timed_us(torch, lambda i: call(), iters)
        byts = (M * c.cin + M * c.cout) * 2 + c.p // 8
        roof = max(byts / (HBM_PEAK_GBS * 1e3), 2.0 * M * c.cin * (c.p // c.cin) / (MFMA_BF16_PEAK_TFLOPS * 1e6))
        sweep[str(M)] = {"kernel": tbn.tbn_linear_forward_kernel(x.dtype, M, c.cin, c.cout, c.k, c.n_alpha, 0, xm.data_ptr(), ym.data_ptr()),
                         "us": round(us, 2), "roof_us": round(roof, 2)}
    out["metric_layer_batch_sweep"] = sweep
    del w, x
    # long rows at a few hundred to a few thousand batch rows: the call without and with a workspace (split K)
    for c in wl.FFN_DOWN:
        w, x, _ = device_inputs(c, torch, wl)
        tile, alpha = tbn.tbn_pack_tile(w, c.k, c.n_alpha)
        y = torch.empty((c.M, c.cout), dtype=x.dtype, device="cuda")
        need = tbn.tbn_linear_forward_workspace_bytes(x.dtype, c.M, c.cin, c.cout, c.k)
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
        us = _timed_us(torch, lambda i: tbn.tbn_linear_forward(x, tile, alpha, c.cout, c.k, y=y), iters)
        usw = _timed_us(torch, lambda i: tbn.tbn_linear_forward_ws(x, tile, alpha, c.cout, c.k, ws, y=y), iters)
        byts = (c.M * c.cin + c.M * c.cout) * 2 + c.p // 8
        alg_flop = 2.0 * c.M * c.cin * (c.p // c.cin)
        out[c.name] = {"us": round(us, 2), "with_workspace_us": round(usw, 2), "workspace_bytes": need,
                       "warm": _roof_fields(us, byts, alg_flop, ceil), "with_workspace": _roof_fields(usw, byts, alg_flop, ceil)}
        del w, x, y, ws
    # binary activations (sign bits in, bfloat16 out): the sign packing of X and the layer on the bits; the matrix
    # time is priced at the 4-bit float rate (10.1 PFLOP/s dense), the format the kernel multiplies in
    for c in (wl.METRIC, *wl.CFG5):
        w, x, _ = device_inputs(c, torch, wl)
        tile, alpha = tbn.tbn_pack_tile(w, c.k, c.n_alpha)
        bits = tbn.tbn_sign_pack(x)
        y = torch.empty((c.M, c.cout), dtype=x.dtype, device="cuda")
        usp = _timed_us(torch, lambda i: tbn.tbn_sign_pack(x, xbits=bits), iters)
        us = _timed_us(torch, lambda i: tbn.tbn_linear_forward_binact(bits, c.cin, tile, alpha, c.cout, c.k, y=y), iters)
        yb = torch.empty((c.M, c.cout // 32), dtype=torch.int32, device="cuda")
        uss = _timed_us(torch, lambda i: tbn.tbn_linear_forward_binact(bits, c.cin, tile, alpha, c.cout, c.k, y=yb,
                                                                       flags=tbn.TBN_FLAG_SIGN_OUT), iters)
        byts = c.M * c.cin // 8 + c.M * c.cout * 2 + c.p // 8
        alg_flop = 2.0 * c.M * c.cin * (c.p // c.cin)
        t_hbm, t_mfma = byts / (HBM_PEAK_GBS * 1e3), alg_flop / (MFMA_FP4_PEAK_TFLOPS * 1e6)
        out[c.name + ":binary_activations"] = {
            "us": round(us, 2), "sign_pack_us": round(usp, 2), "sign_pack_gbs": round(c.M * c.cin * 2 / usp / 1e3, 1),
            "alg_gbs": round(byts / us / 1e3, 1), "roof_us": round(max(t_hbm, t_mfma), 2),
            "bound": "hbm" if t_hbm >= t_mfma else "mfma", "frac_of_roof": round(max(t_hbm, t_mfma) / us, 3),
            "sign_out_us": round(uss, 2), "real_valued_us": out[c.name]["us"]}
        del w, x, y, yb, bits
    for c in (wl.CFG3, wl.CFG3_MISALIGNED, *wl.CONV_MORE):
        w = torch.from_numpy(wl.draw_w_real(c.n, c.cfg, c.layer)).cuda()
        xv, xb = wl.draw_x((c.N, c.C, c.H, c.W), c.cfg, c.layer, c.dtype)
        x = torch.from_numpy(xv).cuda() if xb is None else torch.from_numpy(xb.view(np.int16)).cuda().view(torch.bfloat16)
        tile, alpha = tbn.tbn_pack_tile(w, c.k, c.n_alpha)
        Ho, Wo = tbn.conv_out_hw(c.H, c.W, c.kh, c.kw, c.stride, c.pad)
        byts = (x.numel() + c.N * c.O * Ho * Wo) * x.element_size() + c.p // 8
        nsets = int(max(2, -(-cold_target // byts) + 1))
        xs = [x] + [x.clone() for _ in range(nsets - 1)]
        ys = [torch.empty((c.N, c.O, Ho, Wo), dtype=x.dtype, device="cuda") for _ in range(nsets)]
        run = lambda i: tbn.tbn_conv2d_forward(xs[i % nsets], tile, alpha, c.O, c.kh, c.kw, c.k, stride=c.stride, pad=c.pad, y=ys[i % nsets])
        us = _timed_us(torch, lambda i: run(0), iters)
        usc = _timed_us(torch, run, max(iters, nsets), warm=nsets)
        flop = 2.0 * c.N * Ho * Wo * c.O * c.C * c.kh * c.kw
        filt = c.C * c.kh * c.kw
        U = min(c.O, c.p // int(np.gcd(filt, c.p)))
        alg_flop = flop * U / c.O
        out[c.name] = {"us": round(us, 2), "cold_us": round(usc, 2), "dense_equiv_tflops": round(flop / us / 1e6, 1),
                       "alg_gbs": round(byts / us / 1e3, 1), "warm": _roof_fields(us, byts, alg_flop, ceil, 3.0 if c.dtype == "f32" else 1.0),
                       "cold": _roof_fields(usc, byts, alg_flop, ceil, 3.0 if c.dtype == "f32" else 1.0)}
        del x, xs, ys
    return out


def odd_shapes(torch, tbn, iters):
    """Shapes outside the matrix-core kernels' range (seeded synthetic inputs, tiles of whole rows / filters):
    microseconds per call with the default dispatch (the direct kernels on the vector ALUs) and with
    TBN_FLAG_FORCE_GENERIC (one thread per output)."""
    g = torch.Generator(device="cuda")
    g.manual_seed(240712075)
    out = {}

    def both(fn):
        fn(0)
        fn(tbn.TBN_FLAG_FORCE_GENERIC)
        d = _timed_us(torch, lambda i: fn(0), iters, warm=1)
        f = _timed_us(torch, lambda i: fn(tbn.TBN_FLAG_FORCE_GENERIC), max(2, iters // 4), warm=1)
        return {"us": round(d, 1), "one_thread_per_output_us": round(f, 1), "ratio": round(f / d, 1)}

    for M, cin, cout, k, dt in ((8192, 196, 384, 4, torch.float32), (8192, 196, 384, 4, torch.bfloat16), (8192, 300, 300, 4, torch.float32),
                                (8192, 2050, 1026, 2, torch.bfloat16), (1024, 196, 384, 4, torch.float32)):
        w = torch.randn(cin * cout, device="cuda", generator=g) * 0.02
        x = torch.randn((M, cin), device="cuda", generator=g).to(dt)
        tile, alpha = tbn.tbn_pack_tile(w, k, k)
        y = torch.empty((M, cout), device="cuda", dtype=dt)
        out[f"linear_{M}x{cin}_to_{cout}_k{k}_{'f32' if dt == torch.float32 else 'bf16'}"] = both(
            lambda fl: tbn.tbn_linear_forward(x, tile, alpha, cout, k, y=y, flags=fl))
    for N, C, H, O, kk, st, pd, k, dt in ((32, 3, 224, 64, 7, 2, 3, 4, torch.float32), (32, 3, 224, 64, 7, 2, 3, 4, torch.bfloat16),
                                          (32, 64, 28, 64, 5, 1, 2, 4, torch.float32)):
        w = torch.randn(O * C * kk * kk, device="cuda", generator=g) * 0.02
        x = torch.randn((N, C, H, H), device="cuda", generator=g).to(dt)
        tile, alpha = tbn.tbn_pack_tile(w, k, 1)
        y = tbn.tbn_conv2d_forward(x, tile, alpha, O, kk, kk, k, (st, st), (pd, pd))
        out[f"conv{kk}x{kk}s{st}_{C}_{H}x{H}_to{O}_k{k}_b{N}_{'f32' if dt == torch.float32 else 'bf16'}"] = both(
            lambda fl: tbn.tbn_conv2d_forward(x, tile, alpha, O, kk, kk, k, (st, st), (pd, pd), y=y, flags=fl))
    for M, cin, cout, k in ((8192, 4128, 4096, 8), (8192, 3000, 3072, 6), (8192, 1024, 1000, 4)):
        w = torch.randn(cin * cout, device="cuda", generator=g) * 0.02
        x = torch.randn((M, cin), device="cuda", generator=g).bfloat16()
        tile, alpha = tbn.tbn_pack_tile(w, k, k)
        bits = tbn.tbn_sign_pack(x)
        y = torch.empty((M, cout), device="cuda", dtype=torch.bfloat16)
        out[f"binary_activations_{M}x{cin}_to_{cout}_k{k}"] = both(
            lambda fl: tbn.tbn_linear_forward_binact(bits, cin, tile, alpha, cout, k, y=y, flags=fl))
    return out


if __name__ == "__main__":
    main()
