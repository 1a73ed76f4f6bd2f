"""Layer sweep: every synthetic layer x {F2, F4} through the HIP path, timed on the GPU.

    python -m paper_2412_05781_amd.sweep [--layers A_conv_in,B_resblock,...] [--json out.json]

Per (layer, variant): microseconds per wino_conv2d_ex call (HIP-graph replay of `reps` calls on
rotating buffer sets, so neither host launch cost nor a warm cache flatters the number),
direct-equivalent TFLOP/s = 2*N*K*C*H*W*9 / t, the per-kernel durations, the GEMM stage as a
fraction of the dense MFMA peak and the transform kernels' GB/s.  No oracle here: parity is the
job of tests/.
"""
from __future__ import annotations

import argparse
import json
import sys

import torch

from . import binding as B
from . import synth

PEAK_TFLOPS = {"f16": 2500.0, "f32": 157.3}


def graph_time(fn, reps, replays=4):
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        for i in range(2):
            fn(i)
        side.synchronize()
        with torch.cuda.graph(g, stream=side):
            for i in range(reps):
                fn(i)
        g.replay()
        side.synchronize()
        best = float("inf")
        for _ in range(replays):
            a, z = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(side)
            g.replay()
            z.record(side)
            side.synchronize()
            best = min(best, a.elapsed_time(z))
    return best / reps * 1e-3


def run_layer(layer, variant, dev, layout=B.WINO_NCHW):
    N, C, K, H, W = layer.N, layer.C, layer.K, layer.H, layer.W
    tdt = synth.TORCH_DTYPE[layer.dtype]
    dt = B.DTYPE_OF[tdt]
    esz = 2 if layer.dtype == "f16" else 4
    alpha, Cp, T = B.wino_transformed_dims(N, C, H, W, K, variant)
    a2 = alpha * alpha
    g = torch.Generator(device=dev); g.manual_seed(layer.index)
    wd = (torch.randn((K, C, 3, 3), device=dev, generator=g) / (9.0 * C) ** 0.5).to(tdt)
    bd = torch.randn((K,), device=dev, generator=g) * 0.01
    set_bytes = (N * C * H * W + N * K * H * W) * esz + B.wino_filter_bytes(K, C, dt, variant)
    nsets = max(2, min(24, -(-(320 << 20) // set_bytes)))
    sets = []
    for _ in range(nsets):
        xs = (N, H, W, C) if layout == B.WINO_NHWC else (N, C, H, W)
        ys = (N, H, W, K) if layout == B.WINO_NHWC else (N, K, H, W)
        sets.append((torch.randn(xs, device=dev, generator=g).to(tdt), B.wino_filter_transform(wd, variant),
                     torch.empty(ys, device=dev, dtype=tdt)))
    ws = torch.empty(B.wino_workspace_bytes(N, C, H, W, K, dt, variant), dtype=torch.uint8, device=dev)
    V = torch.empty((a2, T, Cp), dtype=tdt, device=dev)
    M = torch.empty((a2, K, T), dtype=torch.float32, device=dev)
    reps = max(2, min(2 * nsets, 40))
    t_all = graph_time(lambda i: B.wino_conv2d_ex(sets[i % nsets][0], sets[i % nsets][1], bd, sets[i % nsets][2], ws, layout), reps)
    t_in = graph_time(lambda i: B.wino_input_transform(sets[i % nsets][0], variant, layout, out=V), reps)
    if layout == B.WINO_NHWC:       # channel-last keeps the product transposed: operands swapped
        t_g = graph_time(lambda i: B.wino_batched_gemm(V, sets[i % nsets][1].buf.view(tdt), T, C, K, variant, out=M), reps)
    else:
        t_g = graph_time(lambda i: B.wino_batched_gemm(sets[i % nsets][1].buf.view(tdt), V, K, C, T, variant, out=M), reps)
    t_out = graph_time(lambda i: B.wino_output_transform(M, bd, N, K, H, W, tdt, variant, layout, out=sets[i % nsets][2]), reps)
    fl = 2 * a2 * K * C * T
    return {
        "layer": layer.name, "variant": f"F{variant}", "dtype": layer.dtype, "us": t_all * 1e6,
        "direct_equiv_tflops": layer.direct_flops / t_all / 1e12,
        "us_input": t_in * 1e6, "us_gemm": t_g * 1e6, "us_output": t_out * 1e6,
        "gemm_tflops": fl / t_g / 1e12, "gemm_pct_mfma_peak": 100 * fl / t_g / 1e12 / PEAK_TFLOPS[layer.dtype],
        "gemm_operand_GBs": (a2 * (K + T) * Cp * esz + a2 * K * T * 4) / t_g / 1e9,
        "input_GBs": (N * C * H * W * esz + a2 * T * Cp * esz) / t_in / 1e9,
        "output_GBs": (a2 * K * T * 4 + N * K * H * W * esz) / t_out / 1e9,
        "auto_pick": B.wino_resolve_variant(N, C, H, W, K, dt, B.WINO_AUTO) == variant,
    }


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--layers", default=",".join(l.name for l in synth.ALL_LAYERS))
    ap.add_argument("--json", default=None)
    ap.add_argument("--layout", default="nchw", choices=["nchw", "nhwc"])
    args = ap.parse_args(argv)
    if not torch.cuda.is_available():
        sys.exit("sweep needs a GPU")
    dev = torch.device("cuda:0")
    rows = []
    print(f"{'layer':18s} {'var':3s} {'us':>9s} {'TFLOP/s':>8s} | {'in us':>8s} {'gemm us':>8s} {'out us':>8s} | {'gemm TF':>8s} {'%peak':>6s} {'in GB/s':>8s} {'out GB/s':>8s}")
    for name in args.layers.split(","):
        layer = synth.LAYERS[name]
        for variant in (B.WINO_F2, B.WINO_F4):
            r = run_layer(layer, variant, dev, B.WINO_NHWC if args.layout == "nhwc" else B.WINO_NCHW)
            rows.append(r)
            print(f"{r['layer']:18s} {r['variant']:3s} {r['us']:9.2f} {r['direct_equiv_tflops']:8.1f} | {r['us_input']:8.2f} {r['us_gemm']:8.2f} "
                  f"{r['us_output']:8.2f} | {r['gemm_tflops']:8.1f} {r['gemm_pct_mfma_peak']:6.1f} {r['input_GBs']:8.0f} {r['output_GBs']:8.0f}"
                  f"{'  <- AUTO' if r['auto_pick'] else ''}", flush=True)
            torch.cuda.empty_cache()
    if args.json:
        with open(args.json, "w") as f:
            json.dump(rows, f, indent=1)


if __name__ == "__main__":
    main()
