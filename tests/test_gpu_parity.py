"""Parity of the HIP path (through the C ABI) against the CPU oracle, element by element.

Tolerances (relative L2 over the whole output tensor): 1e-5 for fp32 storage, 5e-3 for fp16
storage with fp32 accumulation.  Stage checks compare each kernel with the matching step of
the fp64 Winograd reference (Section "Techniques", steps (i)-(iii))."""
import numpy as np
import pytest
import torch

import os
import sys

import oracle
from oracle import winograd_ref as wr
from paper_2412_05781_amd import binding as B
from paper_2412_05781_amd import synth

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "f16": 5e-3}
DEV = "cuda:0"


def _run(x, w, b, variant):
    xd, wd = x.to(DEV), w.to(DEV)
    bd = None if b is None else b.to(DEV)
    y = B.conv2d(xd, wd, bd, variant)
    torch.cuda.synchronize()
    return y.float().cpu().numpy().astype(np.float64)


def _np(t):
    return t.float().numpy().astype(np.float64)


SMALL = [
    # N, C, K, H, W  — odd sizes, ragged tiles, channel counts off the MFMA tile
    (1, 1, 1, 1, 1), (1, 4, 3, 2, 3), (2, 5, 7, 5, 7), (3, 8, 16, 9, 13), (1, 33, 65, 17, 30),
    (2, 64, 130, 33, 9), (1, 100, 40, 12, 40), (2, 136, 200, 16, 16), (1, 72, 129, 70, 6),
]


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("variant", [B.WINO_F2, B.WINO_F4, B.WINO_DIRECT])
@pytest.mark.parametrize("shape", SMALL)
def test_small_shapes_full_tensor(shape, variant, dtype):
    N, C, K, H, W = shape
    x, w, b = synth.make_inputs(N, C, K, H, W, dtype, seed=1000 + sum(shape))
    ref = oracle.conv2d_direct(_np(x), _np(w), _np(b))
    y = _run(x, w, b, variant)
    assert y.shape == ref.shape
    err = oracle.rel_l2(y, ref)
    assert err <= TOL[dtype], (shape, variant, dtype, err)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("shape", SMALL)
def test_checking_kernel_small_shapes(shape, dtype):
    """wino_direct_conv2d, the one-lane-per-output kernel kept for checking (WINO_DIRECT through the filter-based
    entry points runs the implicit-GEMM kernel instead, covered by the test above)."""
    N, C, K, H, W = shape
    x, w, b = synth.make_inputs(N, C, K, H, W, dtype, seed=1000 + sum(shape))
    ref = oracle.conv2d_direct(_np(x), _np(w), _np(b))
    y = B.wino_direct_conv2d(x.to(DEV), w.to(DEV), b.to(DEV), torch.empty((N, K, H, W), dtype=x.dtype, device=DEV))
    torch.cuda.synchronize()
    assert oracle.rel_l2(y.float().cpu().numpy(), ref) <= (1e-5 if dtype == "f32" else 6e-4)


def test_direct_variant_through_every_entry_point():
    """A filter prepared with WINO_DIRECT: explicit workspace (both layouts), the stream-ordered entry point, and the
    fused entry point (which takes it with everything but GroupNorm; tests/test_gpu_fused.py covers those operators)."""
    import ctypes
    N, C, K, H, W = 2, 40, 72, 13, 18
    x, w, b = synth.make_inputs(N, C, K, H, W, "f16", seed=12)
    ref = oracle.conv2d_direct(_np(x), _np(w), _np(b))
    xd, wd, bd = x.to(DEV), w.to(DEV), b.to(DEV)
    w_t = B.wino_filter_transform(wd, B.WINO_DIRECT)
    assert w_t.desc.variant == B.WINO_DIRECT
    ws = torch.empty(B.wino_workspace_bytes(N, C, H, W, K, B.WINO_F16, B.WINO_DIRECT), dtype=torch.uint8, device=DEV)
    y1 = B.wino_conv2d_ex(xd, w_t, bd, torch.empty((N, K, H, W), dtype=xd.dtype, device=DEV), ws)
    y2 = B.wino_conv2d(xd, w_t, bd, torch.empty((N, K, H, W), dtype=xd.dtype, device=DEV))
    y3 = B.wino_conv2d_ex(xd.permute(0, 2, 3, 1).contiguous(), w_t, bd, torch.empty((N, H, W, K), dtype=xd.dtype, device=DEV), ws,
                          layout=B.WINO_NHWC)
    y4 = B.wino_conv2d_fused(xd, w_t, bd, torch.empty((N, K, H, W), dtype=xd.dtype, device=DEV), ws)
    torch.cuda.synchronize()
    for y in (y1, y2, y3.permute(0, 3, 1, 2), y4):
        err = oracle.rel_l2(y.float().cpu().numpy(), ref)
        assert FP16_BAND[B.WINO_DIRECT][0] <= err <= FP16_BAND[B.WINO_DIRECT][1], err
    assert torch.equal(y1, y2) and torch.equal(y1, y4)
    # the recommendation is what the binding's convenience call can be given directly
    v = B.wino_recommend_variant(1, 64, 256, 256, 64, B.WINO_F16)
    assert v == B.WINO_DIRECT


@pytest.mark.parametrize("variant", [B.WINO_F2, B.WINO_F4])
def test_no_bias_and_zero_input(variant):
    x, w, b = synth.make_inputs(2, 16, 24, 10, 11, "f32", seed=5)
    ref = oracle.conv2d_direct(_np(x), _np(w), None)
    assert oracle.rel_l2(_run(x, w, None, variant), ref) <= 1e-5
    # all-zero input: the output is exactly the bias
    y0 = _run(torch.zeros_like(x), w, b, variant)
    assert np.array_equal(y0, np.broadcast_to(_np(b).reshape(1, -1, 1, 1), y0.shape))


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("variant", [B.WINO_F2, B.WINO_F4])
def test_stage_by_stage(variant, dtype):
    m = variant
    N, C, K, H, W = 2, 40, 72, 13, 18
    x, w, b = synth.make_inputs(N, C, K, H, W, dtype, seed=77)
    xd, wd, bd = x.to(DEV), w.to(DEV), b.to(DEV)
    alpha, Cp, T = B.wino_transformed_dims(N, C, H, W, K, variant)
    a2 = alpha * alpha
    eps = 2.0 ** -11 if dtype == "f16" else 2.0 ** -24

    # step (i), filter
    filt = B.wino_filter_transform(wd, variant)
    U = filt.buf.view(x.dtype).view(a2, K, Cp)
    U_ref = wr.filter_transform(_np(w), m).reshape(a2, K, C)
    Uh = U.float().cpu().numpy().astype(np.float64)
    assert np.all(Uh[:, :, C:] == 0)
    assert np.abs(Uh[:, :, :C] - U_ref).max() <= 4 * eps * np.abs(U_ref).max()

    # step (i), activation
    V = B.wino_input_transform(xd, variant)
    V_ref = wr.input_transform(_np(x), m).reshape(a2, C, T).transpose(0, 2, 1)
    Vh = V.float().cpu().numpy().astype(np.float64)
    assert Vh.shape == (a2, T, Cp) and np.all(Vh[:, :, C:] == 0)
    assert np.abs(Vh[:, :, :C] - V_ref).max() <= 4 * eps * np.abs(V_ref).max()

    # step (ii): compare with the fp64 product of the *stored* U and V
    M = B.wino_batched_gemm(U, V, K, C, T, variant)
    M_ref = np.einsum("bkc,btc->bkt", Uh, Vh)
    Mh = M.cpu().numpy().astype(np.float64)
    assert oracle.rel_l2(Mh, M_ref) <= 1e-6

    # step (iii): compare with A^T M A of the stored M
    y = B.wino_output_transform(M, bd, N, K, H, W, x.dtype, variant)
    y_ref = wr.output_transform(Mh.reshape(alpha, alpha, K, T), _np(b), N, H, W, m)
    torch.cuda.synchronize()
    assert oracle.rel_l2(y.float().cpu().numpy(), y_ref) <= (1e-6 if dtype == "f32" else 6e-4)

    # channel-last stages: same V, the product formed with the operands swapped is the transpose
    # of M (the same sums in the same order), and the output transform reads it as [a2][T][K]
    V2 = B.wino_input_transform(xd.permute(0, 2, 3, 1).contiguous(), variant, layout=B.WINO_NHWC)
    assert torch.equal(V, V2)
    Mt = B.wino_batched_gemm(V, U, T, C, K, variant)
    assert tuple(Mt.shape) == (a2, T, K)
    assert oracle.rel_l2(Mt.cpu().numpy().astype(np.float64), M_ref.transpose(0, 2, 1)) <= 1e-6
    y2 = B.wino_output_transform(Mt, bd, N, K, H, W, x.dtype, variant, layout=B.WINO_NHWC)
    torch.cuda.synchronize()
    assert tuple(y2.shape) == (N, H, W, K)
    Mth = Mt.cpu().numpy().astype(np.float64).transpose(0, 2, 1)
    y2_ref = wr.output_transform(Mth.reshape(alpha, alpha, K, T), _np(b), N, H, W, m)
    assert oracle.rel_l2(y2.float().cpu().permute(0, 3, 1, 2).numpy(), y2_ref) <= (1e-6 if dtype == "f32" else 6e-4)


# what a correct path must show (tests/test_error_model.py derives the fp16 bands on the CPU);
# the direct fallback rounds only its output, so it sits an order of magnitude lower
FP16_BAND = {B.WINO_F2: (2.5e-4, 1.0e-3), B.WINO_F4: (1.5e-3, 4.5e-3), B.WINO_DIRECT: (1e-4, 4e-4)}


# ---- every full-size layer, whole tensor, element by element -------------------------------------------------------
# Beside the variant the library picks for the layer (what bench.py times), the variants listed here are run on the
# same oracle result: the fused variants everywhere (their block shapes differ from layer to layer; F(4x4) fused exists for the
# two-byte types), the other tile size
# on the largest workspaces (E4/F2: M alone is 2.1 GB, byte offsets pass 2^31) and the smallest images, the direct
# variant on VAE- and UNet-sized layers.
EXTRA_VARIANTS = {
    "E4_vae": [B.WINO_F2, B.WINO_DIRECT], "C5_unet": [B.WINO_F4], "D1_sdxl": [B.WINO_F2], "E5_vae_out": [B.WINO_F2],
    "E2_vae": [B.WINO_DIRECT], "C6_unet": [B.WINO_DIRECT], "B_resblock": [B.WINO_F2, B.WINO_F4, B.WINO_DIRECT],
    "A_conv_in": [B.WINO_F2, B.WINO_F4, B.WINO_DIRECT], "D3_sdxl": [B.WINO_F2, B.WINO_F4], "C8_unet": [B.WINO_F4],
}
TILE_EDGE = {B.WINO_F2: 2, B.WINO_F4: 4, B.WINO_FUSED_F2: 2, B.WINO_FUSED_F4: 4, B.WINO_DIRECT: 1}
FP16_BAND[B.WINO_FUSED_F2] = FP16_BAND[B.WINO_F2]
FP16_BAND[B.WINO_FUSED_F4] = FP16_BAND[B.WINO_F4]


@pytest.mark.parametrize("name", [l.name for l in synth.ALL_LAYERS])
def test_every_layer_whole_tensor(name):
    """All 18 layers of the workload groups and the ten Table-1 shapes: the whole output tensor against the oracle's
    defining sum, in the launch configuration the bench times (the variant WINO_AUTO resolves to) and in the variants
    listed above.  Acceptance per variant: relative L2 over the whole tensor within the tolerance AND inside the band
    of the variant that was asked for, every element finite, and no element further from the oracle than the
    element-wise bound allows (parity_util), so that a single wrong tile cannot hide in the norm."""
    import parity_util as pu
    layer = synth.LAYERS[name]
    x, w, b = synth.make_layer_inputs(layer)
    dt = B.DTYPE_OF[synth.TORCH_DTYPE[layer.dtype]]
    auto = B.wino_resolve_variant(layer.N, layer.C, layer.H, layer.W, layer.K, dt, B.WINO_AUTO)
    assert auto in (B.WINO_F2, B.WINO_F4, B.WINO_FUSED_F2, B.WINO_FUSED_F4)
    fused = [B.WINO_FUSED_F2] + ([B.WINO_FUSED_F4] if layer.dtype != "f32" else [])
    variants = [auto] + [v for v in fused + EXTRA_VARIANTS.get(name, []) if v != auto]
    ref = oracle.conv2d_direct(_np(x), _np(w), _np(b))
    for variant in variants:
        y = _run(x, w, b, variant)
        err = pu.check(y, ref, TOL[layer.dtype], TILE_EDGE[variant], layer.dtype, what=(name, variant), channels=layer.C)
        print(f"{name} variant {variant}{' (auto)' if variant == auto else ''}: relL2 {err:.3e}", flush=True)
        if layer.dtype == "f16":
            lo, hi = FP16_BAND[variant]
            assert lo <= err <= hi, (name, variant, err, "error outside the band of the requested variant: did another path run?")
        else:
            assert 1e-8 <= err, "fp32 result suspiciously exact"
        del y


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("variant", [B.WINO_F2, B.WINO_F4])
@pytest.mark.parametrize("shape", [(1, 1, 1, 1, 1), (2, 5, 7, 5, 7), (1, 33, 65, 17, 30), (2, 64, 130, 33, 9),
                                   (1, 100, 40, 12, 40), (2, 136, 200, 16, 16)])
def test_nhwc_layout(shape, variant, dtype):
    """Channels-last activations: same operator, x[N,H,W,C] -> y[N,H,W,K]."""
    N, C, K, H, W = shape
    x, w, b = synth.make_inputs(N, C, K, H, W, dtype, seed=2000 + sum(shape))
    ref = oracle.conv2d_direct(_np(x), _np(w), _np(b))
    x_nhwc = x.permute(0, 2, 3, 1).contiguous().to(DEV)
    y = B.conv2d(x_nhwc, w.to(DEV), b.to(DEV), variant, layout=B.WINO_NHWC)
    torch.cuda.synchronize()
    assert tuple(y.shape) == (N, H, W, K)
    y_nchw = y.float().cpu().permute(0, 3, 1, 2).numpy().astype(np.float64)
    err = oracle.rel_l2(y_nchw, ref)
    assert err <= TOL[dtype], (shape, variant, dtype, err)


def test_nhwc_stages_match_nchw_stages_bitwise():
    """Both layouts feed the same GEMM kernel (operands swapped for channel-last): V must be identical; y
    agrees to the last place or two (the 16 products of one MFMA step may be summed in another order)."""
    N, C, K, H, W = 2, 48, 40, 14, 19
    x, w, b = synth.make_inputs(N, C, K, H, W, "f16", seed=9)
    xd = x.to(DEV)
    for variant in (B.WINO_F2, B.WINO_F4):
        V1 = B.wino_input_transform(xd, variant)
        V2 = B.wino_input_transform(xd.permute(0, 2, 3, 1).contiguous(), variant, layout=B.WINO_NHWC)
        assert torch.equal(V1, V2)
        y1 = B.conv2d(xd, w.to(DEV), b.to(DEV), variant)
        y2 = B.conv2d(xd.permute(0, 2, 3, 1).contiguous(), w.to(DEV), b.to(DEV), variant, layout=B.WINO_NHWC)
        torch.cuda.synchronize()
        d = (y1.float() - y2.permute(0, 3, 1, 2).float()).abs().max().item()
        assert d <= 2.0 ** -9 * y1.float().abs().max().item(), d


def test_nhwc_full_layer():
    layer = synth.LAYERS["B_resblock"]
    x, w, b = synth.make_layer_inputs(layer)
    ref = oracle.conv2d_direct(_np(x), _np(w), _np(b))
    y = B.conv2d(x.permute(0, 2, 3, 1).contiguous().to(DEV), w.to(DEV), b.to(DEV), B.WINO_AUTO, layout=B.WINO_NHWC)
    torch.cuda.synchronize()
    err = oracle.rel_l2(y.float().cpu().permute(0, 3, 1, 2).numpy(), ref)
    assert err <= TOL["f16"] and FP16_BAND[B.WINO_F4][0] <= err


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("variant", [B.WINO_F2, B.WINO_F4])
@pytest.mark.parametrize("shape", [(2, 60, 8, 10, 216), (1, 128, 5, 7, 108), (1, 64, 4, 3, 40), (1, 64, 3, 9, 1000)])
def test_long_rows(shape, variant, dtype):
    """Rows of whole 16-byte chunks with C padded to a multiple of 64: the shapes on which the activation
    transform slides along a tile row in 64-byte bodies (ragged last step, clamped duplicate tiles, one or
    two steps per workgroup, channels beyond C)."""
    N, C, K, H, W = shape
    x, w, b = synth.make_inputs(N, C, K, H, W, dtype, seed=4000 + sum(shape))
    ref = oracle.conv2d_direct(_np(x), _np(w), _np(b))
    y = B.conv2d(x.to(DEV), w.to(DEV), b.to(DEV), variant)
    torch.cuda.synchronize()
    err = oracle.rel_l2(y.float().cpu().numpy(), ref)
    assert err <= TOL[dtype], (shape, variant, dtype, err)
    # stage check of V itself against the fp64 transform
    V = B.wino_input_transform(x.to(DEV), variant)
    alpha, Cp, T = B.wino_transformed_dims(N, C, H, W, K, variant)
    V_ref = wr.input_transform(_np(x), variant).reshape(alpha * alpha, C, T).transpose(0, 2, 1)
    Vh = V.float().cpu().numpy().astype(np.float64)
    eps = 2.0 ** -11 if dtype == "f16" else 2.0 ** -24
    assert np.all(Vh[:, :, C:] == 0)
    assert np.abs(Vh[:, :, :C] - V_ref).max() <= 4 * eps * np.abs(V_ref).max()


@pytest.mark.parametrize("layout", [B.WINO_NCHW, B.WINO_NHWC])
@pytest.mark.parametrize("dtype,shape", [("f16", (1, 1024, 256, 8, 8)), ("f16", (2, 576, 200, 8, 8)), ("f32", (1, 512, 160, 8, 8)),
                                         ("f16", (1, 640, 384, 16, 16))])
def test_deep_layers_split_reduction(dtype, shape, layout):
    """Small images with many channels: in NCHW the GEMM stage cuts the reduction over c into ranges and the output
    transform sums the partial products (F(2x2)); channel-last (operands swapped) keeps the reduction whole."""
    N, C, K, H, W = shape
    x, w, b = synth.make_inputs(N, C, K, H, W, dtype, seed=5000 + sum(shape))
    ref = oracle.conv2d_direct(_np(x), _np(w), _np(b))
    xd = (x.permute(0, 2, 3, 1).contiguous() if layout == B.WINO_NHWC else x).to(DEV)
    for variant in (B.WINO_F2, B.WINO_F4):
        y = B.conv2d(xd, w.to(DEV), b.to(DEV), variant, layout=layout)
        torch.cuda.synchronize()
        y = y.float().cpu()
        if layout == B.WINO_NHWC:
            y = y.permute(0, 3, 1, 2)
        err = oracle.rel_l2(y.numpy(), ref)
        assert err <= TOL[dtype], (shape, variant, dtype, layout, err)


def test_random_shapes_against_oracle():
    """Seeded random small problems (all variants, both dtypes, both layouts): ragged tiles in both
    directions, channel counts off every block size, batch > 1."""
    rng = np.random.default_rng(20241205)
    for trial in range(40):
        N = int(rng.integers(1, 4)); C = int(rng.integers(1, 150)); K = int(rng.integers(1, 150))
        H = int(rng.integers(1, 40)); W = int(rng.integers(1, 40))
        dtype = "f16" if trial % 2 else "f32"
        variant = [B.WINO_F2, B.WINO_F4][(trial // 2) % 2]
        layout = B.WINO_NHWC if (trial // 4) % 2 else B.WINO_NCHW
        x, w, b = synth.make_inputs(N, C, K, H, W, dtype, seed=5000 + trial, with_bias=bool(trial % 3))
        ref = oracle.conv2d_direct(_np(x), _np(w), None if b is None else _np(b))
        xd = (x.permute(0, 2, 3, 1).contiguous() if layout == B.WINO_NHWC else x).to(DEV)
        y = B.conv2d(xd, w.to(DEV), None if b is None else b.to(DEV), variant, layout=layout)
        torch.cuda.synchronize()
        y = y.float().cpu()
        if layout == B.WINO_NHWC:
            y = y.permute(0, 3, 1, 2)
        err = oracle.rel_l2(y.numpy(), ref)
        assert err <= TOL[dtype], (trial, (N, C, K, H, W), dtype, variant, layout, err)


def test_non_default_stream_and_unaligned_pointer():
    x, w, b = synth.make_inputs(1, 16, 16, 8, 8, "f16", seed=6)
    xd, wd, bd = x.to(DEV), w.to(DEV), b.to(DEV)
    ref = B.conv2d(xd, wd, bd, B.WINO_F4)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        y = B.conv2d(xd, wd, bd, B.WINO_F4)      # binding passes torch's current stream
    s.synchronize(); torch.cuda.synchronize()
    assert torch.equal(y, ref)
    # a view that starts 2 bytes into a buffer is rejected on the host, nothing is launched
    big = torch.zeros(xd.numel() + 8, dtype=torch.float16, device=DEV)
    x_off = big[1:1 + xd.numel()].view(xd.shape)
    with pytest.raises(B.WinoError) as e:
        B.conv2d(x_off, wd, bd, B.WINO_F4)
    assert e.value.status == B.WINO_ERR_ALIGN


def test_run_to_run_determinism():
    x, w, b = synth.make_inputs(2, 96, 80, 20, 20, "f16", seed=3)
    xd, wd, bd = x.to(DEV), w.to(DEV), b.to(DEV)
    y1 = B.conv2d(xd, wd, bd, B.WINO_F4).clone()
    y2 = B.conv2d(xd, wd, bd, B.WINO_F4)
    torch.cuda.synchronize()
    assert torch.equal(y1, y2)


def test_stream_ordered_entry_point_matches_explicit_workspace():
    x, w, b = synth.make_inputs(1, 32, 48, 12, 12, "f16", seed=4)
    xd, wd, bd = x.to(DEV), w.to(DEV), b.to(DEV)
    w_t = B.wino_filter_transform(wd, B.WINO_F4)
    y1 = torch.empty((1, 48, 12, 12), dtype=torch.float16, device=DEV)
    B.wino_conv2d(xd, w_t, bd, y1)
    y2 = B.conv2d(xd, wd, bd, B.WINO_F4)
    torch.cuda.synchronize()
    assert torch.equal(y1, y2)
