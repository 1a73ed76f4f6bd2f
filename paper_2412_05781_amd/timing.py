"""Timing tables for the paths around the Winograd convolution, one MI355X, fp16, HIP-graph replay on rotating
buffer sets (so that x, filters and y come from beyond the 256 MB memory-side cache).  Each sub-command prints
the table that the file of the same topic under ``profiles/`` records:

    python -m paper_2412_05781_amd.timing fused          GroupNorm + SiLU + adds around the Winograd call
    python -m paper_2412_05781_amd.timing upsample       2x upsampling read inside the call (Winograd and direct)
    python -m paper_2412_05781_amd.timing flavours       1x1 and stride-2 convolutions through the implicit GEMM
    python -m paper_2412_05781_amd.timing direct         3x3 stride 1: Winograd vs direct vs 8-bit direct
    python -m paper_2412_05781_amd.timing half-product   the opt-in fp16 intermediate product
    python -m paper_2412_05781_amd.timing variants       every workload layer x {F(4x4), F(2x2), fused F(2x2), fused F(4x4)} x {NCHW, NHWC}
    python -m paper_2412_05781_amd.timing int8           F(2x2) with 8-bit integer U and V against the fp16 call, stage by stage

"framework" columns call the stock deep-learning framework's own operators on the same tensors, as context.
"""
from __future__ import annotations

import argparse
import sys

import torch

from . import binding as B
from . import synth
from .gputime import graph_time

DEV = "cuda:0"
DT = torch.float16
MALL = 320 << 20


def _w(K, C, R=3):
    return (torch.randn(K, C, R, R, device=DEV) / (R * R * C) ** 0.5).to(DT)


def _nsets(bytes_per_set, lo=2, hi=16):
    return max(lo, min(hi, MALL // max(1, bytes_per_set) + 1))


def _shape(N, C, H, W, layout):
    return (N, H, W, C) if layout == B.WINO_NHWC else (N, C, H, W)


def _vname(v):
    return {B.WINO_F2: "F2", B.WINO_F4: "F4", B.WINO_FUSED_F2: "fused-F2", B.WINO_FUSED_F4: "fused-F4", B.WINO_DIRECT: "direct"}.get(v, str(v))


def _lname(layout):
    return "NHWC" if layout == B.WINO_NHWC else "NCHW"


def cmd_fused(_):
    for name in ("B_resblock", "D2_sdxl", "E1_vae"):
        L = synth.LAYERS[name]
        N, C, K, H, W = L.N, L.C, L.K, L.H, L.W
        v = B.wino_resolve_variant(N, C, H, W, K, B.WINO_F16, B.WINO_AUTO)
        wd, bd = _w(K, C), torch.randn(K, device=DEV) * 0.01
        gamma, beta = torch.rand(C, device=DEV) + 0.5, torch.randn(C, device=DEV) * 0.1
        n = _nsets((N * C * H * W + 2 * N * K * H * W) * 2 + B.wino_filter_bytes(K, C, B.WINO_F16, v), hi=24)
        sets = [(torch.randn(N, C, H, W, device=DEV).to(DT), B.wino_filter_transform(wd, v), torch.empty(N, K, H, W, device=DEV, dtype=DT),
                 torch.randn(N, K, H, W, device=DEV).to(DT), torch.randn(N, K, device=DEV)) for _ in range(n)]
        ws = torch.empty(B.wino_workspace_bytes(N, C, H, W, K, B.WINO_F16, v), dtype=torch.uint8, device=DEV)
        st = torch.empty(B.wino_groupnorm_stats_bytes(N, 32), dtype=torch.uint8, device=DEV)
        t_plain = graph_time(lambda i: B.wino_conv2d_ex(sets[i % n][0], sets[i % n][1], bd, sets[i % n][2], ws), 2 * n)
        t_stats = graph_time(lambda i: B.wino_groupnorm_stats(sets[i % n][0], 32, out=st), 2 * n)

        def fused(i):
            x, wt, y, res, add = sets[i % n]
            B.wino_groupnorm_stats(x, 32, out=st)
            B.wino_conv2d_fused(x, wt, bd, y, ws, gn_stats=st, gn_gamma=gamma, gn_beta=beta, gn_groups=32, addvec=add, residual=res)
        t_fused = graph_time(fused, 2 * n)
        print(f"{name:12s} {_vname(v)}: plain call {t_plain*1e6:7.2f} us | groupnorm stats {t_stats*1e6:6.2f} us | stats + fused call "
              f"{t_fused*1e6:7.2f} us | extra for GN+SiLU+adds {1e6*(t_fused-t_plain):+.1f} us", flush=True)


def cmd_upsample(_):
    cases = [("UNet up 2x1280 16->32", 2, 1280, 1280, 16, 16), ("UNet up 2x640 32->64", 2, 640, 640, 32, 32),
             ("VAE up 512 128->256", 1, 512, 512, 128, 128), ("VAE up 256 256->512", 1, 256, 256, 256, 256)]
    for name, N, C, K, h, w in cases:
        H, W = 2 * h, 2 * w
        v = B.wino_resolve_variant(N, C, H, W, K, B.WINO_F16, B.WINO_AUTO)
        wd, bd = _w(K, C), torch.randn(K, device=DEV) * 0.01
        n = _nsets((N * C * h * w + N * C * H * W + N * K * H * W) * 2 + B.wino_filter_bytes(K, C, B.WINO_F16, v), hi=12)
        sets = [(torch.randn(N, C, h, w, device=DEV).to(DT), B.wino_filter_transform(wd, v), torch.empty(N, K, H, W, device=DEV, dtype=DT),
                 torch.randn(N, C, H, W, device=DEV).to(DT)) for _ in range(n)]
        ws = torch.empty(B.wino_workspace_bytes(N, C, H, W, K, B.WINO_F16, v), dtype=torch.uint8, device=DEV)
        t_f = graph_time(lambda i: B.wino_conv2d_fused(sets[i % n][0], sets[i % n][1], bd, sets[i % n][2], ws, upsample=True), 2 * n)
        t_c = graph_time(lambda i: B.wino_conv2d_ex(sets[i % n][3], sets[i % n][1], bd, sets[i % n][2], ws), 2 * n)
        t_u = graph_time(lambda i: torch.nn.functional.interpolate(sets[i % n][0], scale_factor=2, mode="nearest"), 2 * n)
        x, wt, y, _ = sets[0]
        B.wino_conv2d_fused(x, wt, bd, y, ws, upsample=True); torch.cuda.synchronize(); y1 = y.clone()
        B.wino_conv2d_ex(torch.nn.functional.interpolate(x, scale_factor=2, mode="nearest"), wt, bd, y, ws); torch.cuda.synchronize()
        same = torch.equal(y1, y)
        wtd = B.wino_filter_transform(wd, B.WINO_DIRECT)
        wsd = torch.empty(B.wino_workspace_bytes(N, C, H, W, K, B.WINO_F16, B.WINO_DIRECT), dtype=torch.uint8, device=DEV)
        t_d = graph_time(lambda i: B.wino_conv2d_fused(sets[i % n][0], wtd, bd, sets[i % n][2], wsd, upsample=True), 2 * n)
        xh = [s[0].permute(0, 2, 3, 1).contiguous() for s in sets]
        yh = [torch.empty(N, H, W, K, device=DEV, dtype=DT) for _ in sets]
        t_dh = graph_time(lambda i: B.wino_conv2d_fused(xh[i % n], wtd, bd, yh[i % n], wsd, B.WINO_NHWC, upsample=True), 2 * n)
        rec = B.wino_recommend_variant(N, C, H, W, K, B.WINO_F16)
        print(f"{name:22s} Winograd {_vname(v)} fused {t_f*1e6:8.2f} us | two-step: conv {t_c*1e6:8.2f} + framework upsample {t_u*1e6:6.2f} us "
              f"(bitwise equal: {same}) | direct variant fused NCHW {t_d*1e6:8.2f} NHWC {t_dh*1e6:8.2f} us | recommended variant {rec}",
              flush=True)


def _igemm_case(name, N, C, K, H, W, R, st, framework=True, fp8=False, winograd=False):
    pad = (R - 1) // 2
    Ho, Wo = (H + 2 * pad - R) // st + 1, (W + 2 * pad - R) // st + 1
    fl = 2 * N * K * C * Ho * Wo * R * R
    wd, bd = _w(K, C, R), torch.randn(K, device=DEV) * 0.01
    sw = 2.0 ** torch.floor(torch.log2(448.0 / wd.abs().max())).item()
    out = [f"{name:26s}"]
    for layout in (B.WINO_NCHW, B.WINO_NHWC):
        n = _nsets((N * C * H * W + N * K * Ho * Wo) * 2 + 2 * K * C * R * R, hi=12)
        sets = [(torch.randn(_shape(N, C, H, W, layout), device=DEV).to(DT), B.wino_igemm_filter_repack(wd), B.wino_fp8_filter_quantize(wd, sw),
                 torch.empty(_shape(N, K, Ho, Wo, layout), device=DEV, dtype=DT)) for _ in range(n)]
        ws = torch.empty(max(16, B.wino_igemm_workspace_bytes(N, C, H, W, K, R, st, B.WINO_F16, layout)), dtype=torch.uint8, device=DEV)
        t = graph_time(lambda i: B.wino_igemm_conv2d(sets[i % n][0], sets[i % n][1], bd, sets[i % n][3], K, R, st, ws, layout), 2 * n)
        out.append(f"direct {_lname(layout)} {t*1e6:8.2f} us ({fl/t/1e12:6.1f} TF)")
        if fp8:
            ws8 = torch.empty(max(16, B.wino_fp8_workspace_bytes(N, C, H, W, K, R, st)), dtype=torch.uint8, device=DEV)
            t8 = graph_time(lambda i: B.wino_fp8_conv2d(sets[i % n][0], sets[i % n][2], bd, sets[i % n][3], K, R, st, 64.0, sw, ws8, layout), 2 * n)
            out.append(f"8-bit {_lname(layout)} {t8*1e6:8.2f} us ({fl/t8/1e12:6.1f} TF)")
        if winograd and R == 3 and st == 1:
            v = B.wino_resolve_variant(N, C, H, W, K, B.WINO_F16, B.WINO_AUTO)
            wt = B.wino_filter_transform(wd, v)
            wsw = torch.empty(B.wino_workspace_bytes(N, C, H, W, K, B.WINO_F16, v), dtype=torch.uint8, device=DEV)
            tw = graph_time(lambda i: B.wino_conv2d_ex(sets[i % n][0], wt, bd, sets[i % n][3], wsw, layout), 2 * n)
            out.append(f"Winograd {_vname(v)} {_lname(layout)} {tw*1e6:8.2f} us")
        if framework and layout == B.WINO_NCHW:
            for _ in range(2):
                torch.nn.functional.conv2d(sets[0][0], wd, bd.to(DT), stride=st, padding=pad)
            tt = graph_time(lambda i: torch.nn.functional.conv2d(sets[i % n][0], wd, bd.to(DT), stride=st, padding=pad), 2 * n)
            out.append(f"framework conv2d {tt*1e6:8.2f} us")
    print(" | ".join(out), flush=True)


def cmd_flavours(_):
    for c in [("3x3 s2 2x320 64->32", 2, 320, 320, 64, 64, 3, 2), ("3x3 s2 2x640 32->16", 2, 640, 640, 32, 32, 3, 2),
              ("3x3 s2 2x1280 16->8", 2, 1280, 1280, 16, 16, 3, 2), ("3x3 s2 128 512->256", 1, 128, 128, 512, 512, 3, 2),
              ("1x1 2x320->640 @32", 2, 320, 640, 32, 32, 1, 1), ("1x1 2x640->1280 @16", 2, 640, 1280, 16, 16, 1, 1),
              ("1x1 2x1920->640 @32", 2, 1920, 640, 32, 32, 1, 1), ("1x1 512->512 @64", 1, 512, 512, 64, 64, 1, 1)]:
        _igemm_case(*c, framework=True, fp8=True)


def cmd_direct(_):
    for c in [("E5 128->3@1024", 1, 128, 3, 1024, 1024, 3, 1), ("E4 128@1024", 1, 128, 128, 1024, 1024, 3, 1), ("E3 256@512", 1, 256, 256, 512, 512, 3, 1),
              ("E2 512@256", 1, 512, 512, 256, 256, 3, 1), ("E1 512@128", 1, 512, 512, 128, 128, 3, 1),
              ("D2 2x640@64", 2, 640, 640, 64, 64, 3, 1), ("B 2x320@64", 2, 320, 320, 64, 64, 3, 1),
              ("C4 2x1280@16", 2, 1280, 1280, 16, 16, 3, 1)]:
        _igemm_case(*c, framework=False, fp8=True, winograd=True)


def cmd_half_product(_):
    for name in ("B_resblock", "C8_unet", "D2_sdxl", "E1_vae", "E2_vae", "E3_vae", "E4_vae"):
        L = synth.LAYERS[name]
        N, C, K, H, W = L.N, L.C, L.K, L.H, L.W
        v = B.wino_resolve_variant(N, C, H, W, K, B.WINO_F16, B.WINO_AUTO)
        wd, bd = _w(K, C), torch.randn(K, device=DEV) * 0.01
        n = _nsets((N * C * H * W + N * K * H * W) * 2 + B.wino_filter_bytes(K, C, B.WINO_F16, v))
        for layout in (B.WINO_NCHW, B.WINO_NHWC):
            sets = [(torch.randn(_shape(N, C, H, W, layout), device=DEV).to(DT), B.wino_filter_transform(wd, v),
                     torch.empty(_shape(N, K, H, W, layout), device=DEV, dtype=DT)) for _ in range(n)]
            ws = torch.empty(B.wino_workspace_bytes(N, C, H, W, K, B.WINO_F16, v), dtype=torch.uint8, device=DEV)
            t0 = graph_time(lambda i: B.wino_conv2d_fused(sets[i % n][0], sets[i % n][1], bd, sets[i % n][2], ws, layout), 2 * n)
            t1 = graph_time(lambda i: B.wino_conv2d_fused(sets[i % n][0], sets[i % n][1], bd, sets[i % n][2], ws, layout, product_fp16=True), 2 * n)
            print(f"{name:12s} {_vname(v)} {_lname(layout)}: fp32 product {t0*1e6:8.2f} us ({L.direct_flops/t0/1e12:7.1f} TF) | fp16 product "
                  f"{t1*1e6:8.2f} us ({L.direct_flops/t1/1e12:7.1f} TF)  x{t0/t1:.2f}", flush=True)


def cmd_variants(_):
    """Whole-call time (wino_conv2d_ex) of every synthetic layer (the workload groups and the paper's Table-1 shapes, in the
    layer's own storage type) in each Winograd variant and both layouts; '*' marks what WINO_AUTO resolves to.  The fused
    F(4x4) variant exists for the two-byte storage types only ('-' for the fp32 layers)."""
    tags = {B.WINO_F4: "F4", B.WINO_F2: "F2", B.WINO_FUSED_F2: "fused F2", B.WINO_FUSED_F4: "fused F4"}
    print(f"{'layer':18s} {'layout':5s} | " + " | ".join(f"{t + ' us':>11s}" for t in tags.values()) +
          " |  AUTO TF/s | fusedF2/F2 fusedF4/F4  workspace MB (F4 / F2 / fused F2 / fused F4)")
    for name, L in synth.LAYERS.items():
        N, C, K, H, W = L.N, L.C, L.K, L.H, L.W
        tdt = synth.TORCH_DTYPE[L.dtype]
        dt, e = B.DTYPE_OF[tdt], (4 if L.dtype == "f32" else 2)
        auto = B.wino_resolve_variant(N, C, H, W, K, dt, B.WINO_AUTO)
        wd, bd = _w(K, C).to(tdt), torch.randn(K, device=DEV) * 0.01
        for layout in (B.WINO_NCHW, B.WINO_NHWC):
            t = {}
            for v in tags:
                if B.wino_resolve_variant(N, C, H, W, K, dt, v) != v:
                    continue
                n = _nsets((N * C * H * W + N * K * H * W) * e + B.wino_filter_bytes(K, C, dt, v), hi=24)
                sets = [(torch.randn(_shape(N, C, H, W, layout), device=DEV).to(tdt), B.wino_filter_transform(wd, v),
                         torch.empty(_shape(N, K, H, W, layout), device=DEV, dtype=tdt)) for _ in range(n)]
                ws = torch.empty(B.wino_workspace_bytes(N, C, H, W, K, dt, v), dtype=torch.uint8, device=DEV)
                t[v] = graph_time(lambda i: B.wino_conv2d_ex(sets[i % n][0], sets[i % n][1], bd, sets[i % n][2], ws, layout), 2 * n) * 1e6
                del sets, ws
                torch.cuda.empty_cache()
            wsb = [B.wino_workspace_bytes(N, C, H, W, K, dt, v) / 1e6 for v in tags]
            cell = lambda v: (f"{t[v]:10.1f}{'*' if v == auto else ' '}" if v in t else f"{'-':>10s} ")
            r4 = f"{t[B.WINO_FUSED_F4] / t[B.WINO_F4]:5.2f}" if B.WINO_FUSED_F4 in t else "    -"
            print(f"{name:18s} {_lname(layout):5s} | " + " | ".join(cell(v) for v in tags) +
                  f" | {L.direct_flops / t[auto] / 1e6:10.1f} |    {t[B.WINO_FUSED_F2] / t[B.WINO_F2]:5.2f}      {r4}"
                  f"    {wsb[0]:7.1f} / {wsb[1]:7.1f} / {wsb[2]:7.1f} / {wsb[3]:7.1f}", flush=True)


def cmd_int8(_):
    """The layers whose step (ii) streams U (8x8 and 16x16 images) and two larger ones: whole call and the first two stages alone,
    fp16 (what WINO_AUTO runs) against the 8-bit integer path; every stage reads cold input (rotating sets)."""
    print(f"{'layer':10s} {'layout':5s} | fp16: {'call':>7s} {'K2':>6s} {'K3':>6s} | int8: {'call':>7s} {'K2':>6s} {'K3':>6s} | call x    K3 x   (us)")
    for name in ("C3_unet", "C4_unet", "C5_unet", "C6_unet", "D3_sdxl", "C7_unet", "B_resblock"):
        L = synth.LAYERS[name]
        N, C, K, H, W = L.N, L.C, L.K, L.H, L.W
        wd, bd = _w(K, C), torch.randn(K, device=DEV) * 0.01
        v = B.wino_resolve_variant(N, C, H, W, K, B.WINO_F16, B.WINO_AUTO)
        _, Cp, T = B.wino_transformed_dims(N, C, H, W, K, B.WINO_F2)
        for layout in (B.WINO_NCHW, B.WINO_NHWC):
            n = _nsets((N * C * H * W + N * K * H * W) * 2 + B.wino_i8_filter_bytes(K, C), hi=24)
            xs = [torch.randn(_shape(N, C, H, W, layout), device=DEV).to(DT) for _ in range(n)]
            ys = [torch.empty(_shape(N, K, H, W, layout), device=DEV, dtype=DT) for _ in range(n)]
            fs = [B.wino_filter_transform(wd, v) for _ in range(n)]
            qs = [B.wino_i8_filter_transform(wd) for _ in range(n)]
            ws = torch.empty(max(B.wino_workspace_bytes(N, C, H, W, K, B.WINO_F16, v), B.wino_i8_workspace_bytes(N, C, H, W, K)),
                             dtype=torch.uint8, device=DEV)
            t16 = graph_time(lambda i: B.wino_conv2d_ex(xs[i % n], fs[i % n], bd, ys[i % n], ws, layout), 2 * n) * 1e6
            t8 = graph_time(lambda i: B.wino_i8_conv2d(xs[i % n], qs[i % n], bd, ys[i % n], K, ws, layout), 2 * n) * 1e6
            # stages alone (F(2x2) geometry for both so that the columns compare like with like)
            f2 = [B.wino_filter_transform(wd, B.WINO_F2) for _ in range(n)]
            V16 = B.wino_input_transform(xs[0], B.WINO_F2, layout)
            k2_16 = graph_time(lambda i: B.wino_input_transform(xs[i % n], B.WINO_F2, layout, out=V16), 2 * n) * 1e6
            M = torch.empty((16, K, T), dtype=torch.float32, device=DEV)
            if layout == B.WINO_NHWC:
                k3_16 = graph_time(lambda i: B.wino_batched_gemm(V16, f2[i % n].buf.view(DT).view(16, K, Cp), T, C, K, B.WINO_F2, out=M.view(16, T, K)), 2 * n) * 1e6
            else:
                k3_16 = graph_time(lambda i: B.wino_batched_gemm(f2[i % n].buf.view(DT).view(16, K, Cp), V16, K, C, T, B.WINO_F2, out=M), 2 * n) * 1e6
            Vq, dV = B.wino_i8_input_transform(xs[0], layout)
            L_ = B.lib()
            k2_8 = graph_time(lambda i: B._check(L_.wino_i8_input_transform(B._ptr(xs[i % n]), B._ptr(Vq), B._ptr(dV), N, C, H, W, B.WINO_F16, layout,
                                                                             B._stream(None)), "k2"), 2 * n) * 1e6
            views = [B.i8_filter_views(q, K, C) for q in qs]
            if layout == B.WINO_NHWC:
                k3_8 = graph_time(lambda i: B._check(L_.wino_i8_batched_gemm(B._ptr(Vq), B._ptr(dV), B._ptr(views[i % n][0]), B._ptr(views[i % n][1]),
                                                                              B._ptr(M), T, C, K, -1, B._stream(None)), "k3"), 2 * n) * 1e6
            else:
                k3_8 = graph_time(lambda i: B._check(L_.wino_i8_batched_gemm(B._ptr(views[i % n][0]), B._ptr(views[i % n][1]), B._ptr(Vq), B._ptr(dV),
                                                                              B._ptr(M), K, C, T, -1, B._stream(None)), "k3"), 2 * n) * 1e6
            print(f"{name:10s} {_lname(layout):5s} | {_vname(v):>5s} {t16:7.1f} {k2_16:6.1f} {k3_16:6.1f} |       {t8:7.1f} {k2_8:6.1f} {k3_8:6.1f} |"
                  f"  {t16 / t8:5.2f}   {k3_16 / k3_8:5.2f}", flush=True)
            del xs, ys, fs, qs, f2, views, ws
            torch.cuda.empty_cache()


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("what", choices=["fused", "upsample", "flavours", "direct", "half-product", "variants", "int8"])
    a = ap.parse_args(argv)
    if not torch.cuda.is_available():
        print("timing: no GPU visible", file=sys.stderr)
        return 2
    {"fused": cmd_fused, "upsample": cmd_upsample, "flavours": cmd_flavours, "direct": cmd_direct,
     "half-product": cmd_half_product, "variants": cmd_variants, "int8": cmd_int8}[a.what](a)
    return 0


if __name__ == "__main__":
    sys.exit(main())
