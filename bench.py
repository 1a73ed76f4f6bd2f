#!/usr/bin/env python3
"""Throughput of the Winograd 3x3 convolution path on one MI355X.

A step is one pass of the whole activation-side path over one synthetic layer:
activation transform -> alpha^2 batched MFMA GEMMs -> output transform + bias
(one wino_conv2d_ex call).  The filter transform runs once per weight tensor,
outside the timed region, and is reported separately.  Inputs are resident in
HBM before the timed region; by default the step rotates over enough (x, U, y)
sets to exceed the 256 MB Infinity Cache, so x and U come from HBM.

Prints ONE JSON line: direct-equivalent TFLOP/s = 2*N*K*C*H*W*9 / t, the
roofline of the dominant kernel (from per-kernel HIP-event timings taken on
the launch stream), and the CPU oracle timed on the host cores.
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

PEAK_TFLOPS = {"f16": 2500.0, "f32": 157.3}     # dense MFMA, published
PEAK_HBM_GBS = 8000.0
MALL_BYTES = 256 << 20
# HBM bytes per GEMM launch from rocprofv3 --pmc (FETCH_SIZE x 1.99 + WRITE_SIZE, both KiB per
# dispatch; the factors come from a plain copy kernel of known size in the same runs), see
# profiles/B_resblock_f4_pmc_traffic.txt.  Only for workloads that were profiled.
MEASURED_TRAFFIC = {("B_resblock", 4): int((10135.0 * 1.99 + 23040.0) * 1024)}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--layer", default="B_resblock", help="name from paper_2412_05781_amd.synth.LAYERS")
    ap.add_argument("--variant", default="auto", choices=["auto", "f2", "f4"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-rotate", action="store_true", help="reuse one buffer set (cache-warm x, U, y)")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is a single-GPU path (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2412_05781_amd import binding as B
    from paper_2412_05781_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    layer = synth.LAYERS[args.layer]
    N, C, K, H, W = layer.N, layer.C, layer.K, layer.H, layer.W
    dt = B.DTYPE_OF[synth.TORCH_DTYPE[layer.dtype]]
    esz = 2 if layer.dtype == "f16" else 4
    want = {"auto": B.WINO_AUTO, "f2": B.WINO_F2, "f4": B.WINO_F4}[args.variant]
    variant = B.wino_resolve_variant(N, C, H, W, K, dt, want)
    assert variant in (B.WINO_F2, B.WINO_F4)
    alpha, Cp, T = B.wino_transformed_dims(N, C, H, W, K, variant)
    a2 = alpha * alpha

    x, w, b = synth.make_layer_inputs(layer)
    xd, wd, bd = x.to(dev), w.to(dev), b.to(dev)

    # ---- filter transform: once per weight, timed on its own ----------------------------
    w_t = B.wino_filter_transform(wd, variant)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        B.wino_filter_transform(wd, variant)
    e1.record(); torch.cuda.synchronize()
    filter_ms = e0.elapsed_time(e1) / 10

    # ---- buffer sets: rotate so that x, U, y stream from HBM -----------------------------
    set_bytes = xd.numel() * esz + w_t.buf.numel() + N * K * H * W * esz
    nsets = 1 if args.no_rotate else max(2, -(-(MALL_BYTES + (64 << 20)) // set_bytes))
    sets = []
    for i in range(nsets):
        xi = xd if i == 0 else xd.clone()
        wti = w_t if i == 0 else B.Filter(w_t.buf.clone(), B.wino_filter())
        if i:
            d = wti.desc
            d.data, d.K, d.C, d.dtype, d.variant = wti.buf.data_ptr(), K, C, dt, variant
        yi = torch.empty((N, K, H, W), dtype=xd.dtype, device=dev)
        sets.append((xi, wti, yi))
    ws = torch.empty(B.wino_workspace_bytes(N, C, H, W, K, dt, variant), dtype=torch.uint8, device=dev)

    def step(i):
        xi, wti, yi = sets[i % nsets]
        B.wino_conv2d_ex(xi, wti, bd, yi, ws)

    # ---- the timed region ----------------------------------------------------------------------
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tflops = layer.direct_flops / (ms_per_step * 1e-3) / 1e12

    # ---- per-kernel durations: each kernel launched back to back between two HIP events
    #      on the launch stream (torch's current stream is the one handed to the library) --
    # V and M rotate like x, U and y do, so that no stage finds its input warm from its own previous launch
    Vbufs = [torch.empty((a2, T, Cp), dtype=xd.dtype, device=dev) for _ in range(nsets)]
    Mbufs = [torch.empty((a2, K, T), dtype=torch.float32, device=dev) for _ in range(nsets)]
    for i in range(nsets):                          # valid contents for the stages that read them
        B.wino_input_transform(sets[i][0], variant, out=Vbufs[i])
        B.wino_batched_gemm(sets[i][1].buf.view(xd.dtype), Vbufs[i], K, C, T, variant, out=Mbufs[i])
    torch.cuda.synchronize()
    reps = 2 * nsets                                # every buffer set twice per replay

    def time_kernel(fn):
        """Average GPU duration of one launch: `reps` launches captured in a HIP graph on a side
        stream (so the host's launch cost is out of the picture), replayed between two HIP events
        recorded on that same stream."""
        side = torch.cuda.Stream()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            for i in range(3):
                fn(i)
            side.synchronize()
            with torch.cuda.graph(g, stream=side):
                for i in range(reps):
                    fn(i)
            g.replay()
            side.synchronize()
            best = float("inf")
            for _ in range(5):
                a, z = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record(side)
                g.replay()
                z.record(side)
                side.synchronize()
                best = min(best, a.elapsed_time(z))
        return best / reps * 1e-3                   # seconds per launch

    t_in = time_kernel(lambda i: B.wino_input_transform(sets[i % nsets][0], variant, out=Vbufs[i % nsets]))
    t_gemm = time_kernel(lambda i: B.wino_batched_gemm(sets[i % nsets][1].buf.view(xd.dtype), Vbufs[i % nsets], K, C, T, variant,
                                                       out=Mbufs[i % nsets]))
    t_out = time_kernel(lambda i: B.wino_output_transform(Mbufs[i % nsets], bd, N, K, H, W, xd.dtype, variant, out=sets[i % nsets][2]))

    bytes_in = N * C * H * W * esz + a2 * T * Cp * esz
    flops_gemm = 2 * a2 * K * C * T
    bytes_gemm = a2 * K * Cp * esz + a2 * T * Cp * esz + a2 * K * T * 4
    bytes_out = a2 * K * T * 4 + N * K * H * W * esz + K * 4
    stages = {
        "input_transform": {"us": t_in * 1e6, "bound": "hbm", "achieved": bytes_in / t_in / 1e9,
                            "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": bytes_in / t_in / 1e9 / PEAK_HBM_GBS},
        "batched_gemm": {"us": t_gemm * 1e6, "bound": "mfma", "achieved": flops_gemm / t_gemm / 1e12,
                         "peak": PEAK_TFLOPS[layer.dtype], "unit": "TFLOP/s",
                         "frac": flops_gemm / t_gemm / 1e12 / PEAK_TFLOPS[layer.dtype],
                         "operand_GBs": bytes_gemm / t_gemm / 1e9},
        "output_transform": {"us": t_out * 1e6, "bound": "hbm", "achieved": bytes_out / t_out / 1e9,
                             "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": bytes_out / t_out / 1e9 / PEAK_HBM_GBS},
    }
    # The GEMM stage is the path's one dense contraction and the longest kernel.  Its binding roof
    # is the smaller of the MFMA roof and the HBM roof at its algorithmic intensity.
    g = stages["batched_gemm"]
    g["hbm_frac"] = bytes_gemm / t_gemm / 1e9 / PEAK_HBM_GBS
    t_mfma, t_hbm = flops_gemm / (PEAK_TFLOPS[layer.dtype] * 1e12), bytes_gemm / (PEAK_HBM_GBS * 1e9)
    if t_hbm >= t_mfma:
        roofline = {"bound": "hbm", "achieved": bytes_gemm / t_gemm / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": g["hbm_frac"]}
    else:
        roofline = {"bound": "mfma", "achieved": g["achieved"], "peak": g["peak"], "unit": "TFLOP/s", "frac": g["frac"]}
    roofline.update({"kernel": "wino_gemm_kernel", "avg_launch_us": g["us"], "mfma_frac": g["frac"],
                     "algorithmic_bytes": bytes_gemm, "algorithmic_flops": flops_gemm,
                     "traffic": MEASURED_TRAFFIC.get((layer.name, variant))})

    # ---- CPU baseline leg: the oracle, timed on the host cores; its first run also gives the parity figure of
    #      what was just timed (the oracle is test infrastructure: nothing outside this leg touches it) ------------
    cpu, rel = None, None
    if not args.no_cpu_baseline:
        import oracle
        xn, wn, bn = x.float().numpy(), w.float().numpy(), b.numpy()
        y_gpu = sets[0][2].float().cpu().numpy()
        t_or = time.perf_counter()
        ref = oracle.conv2d_direct(xn, wn, bn)
        first = time.perf_counter() - t_or
        rel = oracle.rel_l2(y_gpu, ref)
        best, spent, runs = first, first, 1
        while spent < 10.0 and runs < 200:       # about ten seconds of CPU work
            t_or = time.perf_counter()
            oracle.conv2d_direct(xn, wn, bn)
            d = time.perf_counter() - t_or
            best, spent, runs = min(best, d), spent + d, runs + 1
        cpu = {"value": layer.direct_flops / best / 1e12, "unit": "TFLOP/s (direct-equivalent)",
               "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"whole layer {layer.name}, fp64 direct correlation, best of {runs} runs ({best:.3f} s)"}

    out = {
        "metric": "direct-equivalent TFLOP/s per 3x3 conv layer; % of MFMA peak (GEMM stage)",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": layer.dtype, "data": "synthetic",
        "config": {"workload": f"{layer.name}: 3x3 s1 p1 conv N={N} C={C} K={K} H=W={H} {layer.dtype} NCHW",
                   "variant": f"F({variant}x{variant},3x3)", "rotating_buffer_sets": nsets,
                   "filter_transform_ms_once_per_weight": filter_ms},
        "gemm_pct_of_mfma_peak": 100.0 * stages["batched_gemm"]["frac"],
        "rel_l2_vs_oracle": rel,
        "roofline": roofline,
        "stages": stages,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
