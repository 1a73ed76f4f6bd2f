#!/usr/bin/env python3
"""Throughput of the Winograd 3x3 convolution path on one MI355X.

A step is one pass of the whole activation-side path over one synthetic layer (one wino_conv2d_ex call): activation
transform -> alpha^2 batched MFMA products -> output transform + bias, in the variant WINO_AUTO resolves to (for most
layers the last two run as ONE kernel).  The filter transform runs once per weight tensor, outside the timed region,
and is reported separately.  Inputs are resident in HBM before the timed region; every step rotates over enough
(x, U, y) sets to exceed the 256 MB Infinity Cache, so x and U come from HBM.

The headline (`value`, `ms_per_step`, `roofline`, `cpu_baseline`) is the SDv1.5 residual-block layer at batch 2, timed
with the host clock over exactly --steps steps.  `layers` then carries every layer of the workload groups (18), each
timed by HIP-graph replay with HIP events on the launch stream: microseconds per call, direct-equivalent TFLOP/s =
2*N*K*C*H*W*9 / t, the per-kernel durations, the kernel that holds the MFMA work as a fraction of the dense MFMA peak and
of its binding roof, and the whole-tensor relative L2 error against the CPU oracle.

Prints ONE JSON line.
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
HEADLINE = "B_resblock"
WORKLOAD_LAYERS = ["A_conv_in", "B_resblock", "C1_unet", "C2_unet", "C3_unet", "C4_unet", "C5_unet", "C6_unet", "C7_unet",
                   "C8_unet", "D1_sdxl", "D2_sdxl", "D3_sdxl", "E1_vae", "E2_vae", "E3_vae", "E4_vae", "E5_vae_out"]
# HBM bytes per launch of the headline's dominant kernel, from two rocprofv3 --pmc passes (FETCH_SIZE, WRITE_SIZE), scaled by
# what the same counters read for a plain copy of known size; typed in from the profile named beside it (not measured in
# this run).  Keyed by (layer, variant); absent -> null.
PROFILED_TRAFFIC = {
    ("B_resblock", "F4"): (int((10138.2 * 1.992 + 23040.0) * 1024), "profiles/B_resblock_f4_pmc_traffic.txt (rocprofv3 --pmc, not measured in this run)"),
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--layer", default=HEADLINE, help="headline layer, a name from paper_2412_05781_amd.synth.LAYERS")
    ap.add_argument("--layers", default="all", help="'all' (the 18 layers of the workload groups), 'none', or a comma-separated list")
    ap.add_argument("--variant", default="auto", choices=["auto", "f2", "f4", "fused_f2", "fused_f4"])
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip every oracle run (baseline timing and parity figures)")
    ap.add_argument("--no-rotate", action="store_true", help="reuse one buffer set (cache-warm x, U, y)")
    return ap.parse_args()


class LayerRun:
    """Device buffers of one layer in one variant: rotating (x, U, y) sets, workspace, per-stage buffers."""

    def __init__(self, layer, want, dev, rotate=True, cpu_inputs=None):
        import torch
        from paper_2412_05781_amd import binding as B
        from paper_2412_05781_amd import synth
        self.B, self.torch, self.layer = B, torch, layer
        N, C, K, H, W = layer.N, layer.C, layer.K, layer.H, layer.W
        self.tdt = synth.TORCH_DTYPE[layer.dtype]
        self.dt = B.DTYPE_OF[self.tdt]
        self.esz = 2 if layer.dtype == "f16" else 4
        self.variant = B.wino_resolve_variant(N, C, H, W, K, self.dt, want)
        assert self.variant in (B.WINO_F2, B.WINO_F4, B.WINO_FUSED_F2, B.WINO_FUSED_F4, B.WINO_DIRECT), self.variant
        if self.variant != B.WINO_DIRECT:            # the direct variant is only timed as a whole call (step)
            self.alpha, self.Cp, self.T = B.wino_transformed_dims(N, C, H, W, K, self.variant)
            self.a2 = self.alpha * self.alpha
        if cpu_inputs is not None:                   # the seeded CPU recipe (needed where the oracle checks the result)
            x, w, b = cpu_inputs
            xd, wd, self.bd = x.to(dev), w.to(dev), b.to(dev)
        else:                                        # same distributions, drawn on the device from the layer's seed
            g = torch.Generator(device=dev); g.manual_seed(synth.BASE_SEED + layer.index)
            xd = torch.randn((N, C, H, W), device=dev, generator=g).to(self.tdt)
            wd = (torch.randn((K, C, 3, 3), device=dev, generator=g) / (9.0 * C) ** 0.5).to(self.tdt)
            self.bd = torch.randn((K,), device=dev, generator=g) * 0.01
        self.wd = wd
        w_t = B.wino_filter_transform(wd, self.variant)
        set_bytes = (N * C * H * W + N * K * H * W) * self.esz + w_t.buf.numel()
        self.nsets = max(2, min(24, -(-(MALL_BYTES + (64 << 20)) // set_bytes))) if rotate else 1
        self.sets = []
        for i in range(self.nsets):
            xi = xd if i == 0 else xd.clone()
            wti = w_t if i == 0 else B.Filter(w_t.buf.clone(), B.wino_filter())
            if i:
                d = wti.desc
                d.data, d.K, d.C, d.dtype, d.variant = wti.buf.data_ptr(), K, C, self.dt, self.variant
            self.sets.append((xi, wti, torch.empty((N, K, H, W), dtype=self.tdt, device=dev)))
        self.ws = torch.empty(B.wino_workspace_bytes(N, C, H, W, K, self.dt, self.variant), dtype=torch.uint8, device=dev)
        self.dev = dev

    def step(self, i):
        xi, wti, yi = self.sets[i % self.nsets]
        self.B.wino_conv2d_ex(xi, wti, self.bd, yi, self.ws)

    def filter_ms(self):
        torch, B = self.torch, self.B
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(10):
            B.wino_filter_transform(self.wd, self.variant)
        e1.record(); torch.cuda.synchronize()
        return e0.elapsed_time(e1) / 10

    def stage_times(self):
        """Each kernel launched back to back on rotating buffers (its input comes from beyond the caches), averaged over a
        HIP-graph replay between two HIP events on the launch stream.  Returns ({kernel: seconds}, name of the kernel
        that holds the MFMA work)."""
        from paper_2412_05781_amd.gputime import graph_time
        torch, B, L = self.torch, self.B, self.layer
        N, C, K, H, W = L.N, L.C, L.K, L.H, L.W
        n, v = self.nsets, self.variant
        fused = v in (B.WINO_FUSED_F2, B.WINO_FUSED_F4)
        per_set = self.a2 * self.T * self.Cp * self.esz + (0 if fused else self.a2 * K * self.T * 4)
        nv = max(2, min(n, (8 << 30) // max(1, per_set)))          # V / M sets: rotate, within 8 GB
        Vb = [torch.empty((self.a2, self.T, self.Cp), dtype=self.tdt, device=self.dev) for _ in range(nv)]
        for i in range(nv):
            B.wino_input_transform(self.sets[i % n][0], v, out=Vb[i])
        out = {"input_transform": graph_time(lambda i: B.wino_input_transform(self.sets[i % n][0], v, out=Vb[i % nv]), 2 * n)}
        U = lambda i: self.sets[i % n][1].buf.view(self.tdt)
        if fused:
            out["fused_gemm_output"] = graph_time(
                lambda i: B.wino_fused_gemm_output(U(i), Vb[i % nv], self.bd, N, C, H, W, K, out=self.sets[i % n][2],
                                                   m=2 if v == B.WINO_FUSED_F2 else 4), 2 * n)
            return out, "fused_gemm_output"
        Mb = [torch.empty((self.a2, K, self.T), dtype=torch.float32, device=self.dev) for _ in range(nv)]
        for i in range(nv):
            B.wino_batched_gemm(U(i), Vb[i], K, C, self.T, v, out=Mb[i])
        out["batched_gemm"] = graph_time(lambda i: B.wino_batched_gemm(U(i), Vb[i % nv], K, C, self.T, v, out=Mb[i % nv]), 2 * n)
        out["output_transform"] = graph_time(
            lambda i: B.wino_output_transform(Mb[i % nv], self.bd, N, K, H, W, self.tdt, v, out=self.sets[i % n][2]), 2 * n)
        return out, "batched_gemm"

    def report(self, t_layer, stages, main_kernel):
        """Per-layer record: times, direct-equivalent rate, the MFMA kernel against both roofs."""
        B, L = self.B, self.layer
        N, C, K, H, W = L.N, L.C, L.K, L.H, L.W
        e, a2, T, Cp = self.esz, self.a2, self.T, self.Cp
        flops = 2 * a2 * K * C * T
        b_u, b_v, b_m, b_y = a2 * K * Cp * e, a2 * T * Cp * e, a2 * K * T * 4, N * K * H * W * e
        kbytes = {"input_transform": N * C * H * W * e + b_v, "batched_gemm": b_u + b_v + b_m,
                  "output_transform": b_m + b_y + 4 * K, "fused_gemm_output": b_u + b_v + b_y + 4 * K}
        t = stages[main_kernel]
        t_mfma, t_hbm = flops / (PEAK_TFLOPS[L.dtype] * 1e12), kbytes[main_kernel] / (PEAK_HBM_GBS * 1e9)
        mfma_frac, hbm_frac = t_mfma / t, t_hbm / t
        rec = {"name": L.name, "variant": {B.WINO_F2: "F2", B.WINO_F4: "F4", B.WINO_FUSED_F2: "FUSED_F2", B.WINO_FUSED_F4: "FUSED_F4"}[self.variant],
               "us": t_layer * 1e6, "tflops": L.direct_flops / t_layer / 1e12,
               "kernel_us": {k: v * 1e6 for k, v in stages.items()},
               "kernel_GBs": {k: kbytes[k] / v / 1e9 for k, v in stages.items()},
               "gemm_kernel": main_kernel, "gemm_us": t * 1e6, "gemm_tflops": flops / t / 1e12, "gemm_mfma_frac": mfma_frac,
               "bound": "hbm" if t_hbm >= t_mfma else "mfma", "frac": max(mfma_frac, hbm_frac),
               "rotating_buffer_sets": self.nsets}
        return rec, flops, kbytes[main_kernel]


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
    from paper_2412_05781_amd.gputime import graph_time

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    want = {"auto": B.WINO_AUTO, "f2": B.WINO_F2, "f4": B.WINO_F4, "fused_f2": B.WINO_FUSED_F2, "fused_f4": B.WINO_FUSED_F4}[args.variant]
    oracle = None
    if not args.no_cpu_baseline:
        import oracle                      # test infrastructure: only this leg of the bench touches it

    def parity(layer, cpu_inputs, y_dev):
        x, w, b = cpu_inputs
        t0 = time.perf_counter()
        ref = oracle.conv2d_direct(x.float().numpy(), w.float().numpy(), b.numpy())
        dt_or = time.perf_counter() - t0
        return oracle.rel_l2(y_dev.float().cpu().numpy(), ref), dt_or

    def int8_record(L, r, cpu_inputs):
        n = r.nsets
        qs = [B.wino_i8_filter_transform(r.wd) for _ in range(n)]
        ws8 = torch.empty(B.wino_i8_workspace_bytes(L.N, L.C, L.H, L.W, L.K), dtype=torch.uint8, device=dev)
        call = lambda i: B.wino_i8_conv2d(r.sets[i % n][0], qs[i % n], r.bd, r.sets[i % n][2], L.K, ws8)
        t8 = graph_time(call, 2 * n)
        out8 = {"us": t8 * 1e6, "tflops": L.direct_flops / t8 / 1e12}
        if oracle is not None:
            call(0)
            torch.cuda.synchronize()
            out8["rel_l2_vs_oracle"], _ = parity(L, cpu_inputs, r.sets[0][2])
        return out8

    # ---- headline: exactly --steps steps of the whole path, host clock, barrier = device synchronisation -----------
    layer = synth.LAYERS[args.layer]
    cpu_in = synth.make_layer_inputs(layer)
    run = LayerRun(layer, want, dev, rotate=not args.no_rotate, cpu_inputs=cpu_in)
    filter_ms = run.filter_ms()
    for i in range(args.warmup):
        run.step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        run.step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tflops = layer.direct_flops / (ms_per_step * 1e-3) / 1e12
    t_graph = graph_time(run.step, 2 * run.nsets)
    stages, main_kernel = run.stage_times()
    head, flops, kbytes = run.report(t_graph, stages, main_kernel)
    t = stages[main_kernel]
    if head["bound"] == "hbm":
        roofline = {"bound": "hbm", "achieved": kbytes / t / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": kbytes / t / 1e9 / PEAK_HBM_GBS}
    else:
        roofline = {"bound": "mfma", "achieved": flops / t / 1e12, "peak": PEAK_TFLOPS[layer.dtype], "unit": "TFLOP/s",
                    "frac": head["gemm_mfma_frac"]}
    prof = PROFILED_TRAFFIC.get((layer.name, head["variant"]))
    roofline.update({"kernel": main_kernel, "avg_launch_us": t * 1e6, "mfma_frac": head["gemm_mfma_frac"],
                     "algorithmic_bytes": kbytes, "algorithmic_flops": flops,
                     "traffic": prof[0] if prof else None, "traffic_source": prof[1] if prof else None})

    cpu, rel = None, None
    if oracle is not None:
        # CPU baseline: the oracle as it stands on the host cores, on the headline layer; its first run also gives the
        # parity figure of what was just timed
        run.step(0)
        torch.cuda.synchronize()
        rel, first = parity(layer, cpu_in, run.sets[0][2])
        xn, wn, bn = cpu_in[0].float().numpy(), cpu_in[1].float().numpy(), cpu_in[2].numpy()
        best, spent, runs = first, first, 1
        while spent < 10.0 and runs < 200:       # about ten seconds of CPU work
            t_or = time.perf_counter()
            oracle.conv2d_direct(xn, wn, bn)
            d = time.perf_counter() - t_or
            best, spent, runs = min(best, d), spent + d, runs + 1
        cpu = {"value": layer.direct_flops / best / 1e12, "unit": "TFLOP/s (direct-equivalent)",
               "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"whole layer {layer.name}, fp64 direct correlation, best of {runs} runs ({best:.3f} s)"}
    head["rel_l2_vs_oracle"] = rel
    del run
    torch.cuda.empty_cache()

    # ---- every layer of the workload groups, graph-timed --------------------------------------------------------------
    names = [] if args.layers == "none" else (WORKLOAD_LAYERS if args.layers == "all" else args.layers.split(","))
    layers_out = []
    for name in names:
        if name == layer.name:
            layers_out.append(head)
            continue
        L = synth.LAYERS[name]
        cin = synth.make_layer_inputs(L) if oracle is not None else None
        r = LayerRun(L, want, dev, rotate=not args.no_rotate, cpu_inputs=cin)
        tl = graph_time(r.step, 2 * r.nsets)
        st, mk = r.stage_times()
        rec, _, _ = r.report(tl, st, mk)
        if oracle is not None:
            r.step(0)
            torch.cuda.synchronize()
            rec["rel_l2_vs_oracle"], _ = parity(L, cin, r.sets[0][2])
        # where the library recommends its direct path over the Winograd variants (few channels on large images, or a
        # handful of output channels), that call is timed too, same inputs, same rotation
        if B.wino_recommend_variant(L.N, L.C, L.H, L.W, L.K, r.dt) == B.WINO_DIRECT:
            del r
            torch.cuda.empty_cache()
            r = LayerRun(L, B.WINO_DIRECT, dev, rotate=not args.no_rotate, cpu_inputs=cin)
            td = graph_time(r.step, 2 * r.nsets)
            rec["recommended"] = {"variant": "DIRECT", "us": td * 1e6, "tflops": L.direct_flops / td / 1e12}
            if oracle is not None:
                r.step(0)
                torch.cuda.synchronize()
                rec["recommended"]["rel_l2_vs_oracle"], _ = parity(L, cin, r.sets[0][2])
        # the layers whose step (ii) streams a large U against few tiles: the opt-in path with 8-bit integer U and V beside it
        # (lower precision: about 1.7e-2 against 5e-4; never what the headline or the `us` column runs)
        if L.dtype == "f16" and L.C >= 640 and L.N * ((L.H + 1) // 2) * ((L.W + 1) // 2) <= 128:
            rec["int8_uv"] = int8_record(L, r, cin)
        layers_out.append(rec)
        print(f"bench: {name} {rec['variant']} {rec['us']:.1f} us {rec['tflops']:.0f} TFLOP/s", file=sys.stderr, flush=True)
        del r, cin
        torch.cuda.empty_cache()

    N, C, K, H, W = layer.N, layer.C, layer.K, layer.H, layer.W
    out = {
        "metric": "direct-equivalent TFLOP/s per 3x3 conv layer; % of MFMA peak (GEMM stage)",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": layer.dtype, "data": "synthetic",
        "config": {"workload": f"{layer.name}: 3x3 s1 p1 conv N={N} C={C} K={K} H=W={H} {layer.dtype} NCHW",
                   "variant": head["variant"], "rotating_buffer_sets": head["rotating_buffer_sets"],
                   "filter_transform_ms_once_per_weight": filter_ms},
        "gemm_pct_of_mfma_peak": 100.0 * head["gemm_mfma_frac"],
        "rel_l2_vs_oracle": rel,
        "graph_replay_us_per_step": t_graph * 1e6,
        "roofline": roofline,
        "stages": head["kernel_us"],
        "cpu_baseline": cpu,
        "layers": layers_out,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
