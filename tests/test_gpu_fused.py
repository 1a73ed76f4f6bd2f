"""Parity of the fused entry point (GroupNorm + SiLU on the way in, vector and residual adds on the
way out) against the fp64 oracle; same tolerances as the plain path (relative L2 <= 1e-5 fp32,
<= 5e-3 fp16)."""
import numpy as np
import pytest
import torch

import oracle
from oracle import fused_ops as fo
from paper_2412_05781_amd import binding as B
from paper_2412_05781_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = {"f32": 1e-5, "f16": 5e-3}


def _np(t):
    return None if t is None else t.float().numpy().astype(np.float64)


def _extras(N, C, K, H, W, dtype, seed):
    g = torch.Generator().manual_seed(seed)
    gamma = 1.0 + 0.2 * torch.randn(C, generator=g)
    beta = 0.3 * torch.randn(C, generator=g)
    addvec = 0.5 * torch.randn(N, K, generator=g)
    residual = torch.randn(N, K, H, W, generator=g).to(synth.TORCH_DTYPE[dtype])
    return gamma, beta, addvec, residual


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("groups", [1, 4])
def test_groupnorm_stats(dtype, groups):
    for layout in (B.WINO_NCHW, B.WINO_NHWC):
        for (N, C, H, W) in [(2, 8, 5, 7), (1, 32, 64, 64), (3, 12, 1, 1), (1, 64, 200, 200)]:
            x = (torch.randn(N, C, H, W, generator=torch.Generator().manual_seed(C + H)) * 1.7 + 0.4).to(synth.TORCH_DTYPE[dtype])
            xd = (x.permute(0, 2, 3, 1).contiguous() if layout == B.WINO_NHWC else x).to(DEV)
            st = B.stats_view(B.wino_groupnorm_stats(xd, groups, 1e-5, layout), N, groups).cpu().numpy().astype(np.float64)
            mean, rstd = fo.groupnorm_stats(_np(x), groups, 1e-5)
            assert np.abs(st[:, :, 0] - mean).max() <= 2e-6 * (1 + np.abs(mean).max())
            assert np.abs(st[:, :, 1] / rstd - 1).max() <= 5e-6


# the last two have rows long enough for the sliding-window activation kernel (C padded to 64, ragged last step)
CASES = [(1, 8, 8, 4, 4, 4), (2, 24, 40, 9, 13, 4), (1, 64, 130, 17, 30, 32), (2, 96, 40, 16, 16, 32), (1, 40, 33, 33, 6, 8),
         (2, 60, 8, 7, 216, 4), (1, 128, 6, 5, 108, 32)]


# every variant in fp32 and fp16; the fused F(4x4) kernel exists for the two-byte storage types only
VARIANT_DTYPE = [(v, d) for d in ("f32", "f16") for v in (B.WINO_F2, B.WINO_F4, B.WINO_FUSED_F2, B.WINO_FUSED_F4)
                 if not (v == B.WINO_FUSED_F4 and d == "f32")]


@pytest.mark.parametrize("variant,dtype", VARIANT_DTYPE)
@pytest.mark.parametrize("layout", [B.WINO_NCHW, B.WINO_NHWC])
@pytest.mark.parametrize("case", CASES)
def test_fused_full_tensor(case, layout, variant, dtype):
    N, C, K, H, W, G = case
    x, w, b = synth.make_inputs(N, C, K, H, W, dtype, seed=3000 + sum(case))
    gamma, beta, addvec, residual = _extras(N, C, K, H, W, dtype, 77 + sum(case))
    ref = fo.conv2d_fused(_np(x), _np(w), _np(b), _np(gamma), _np(beta), G, 1e-5, _np(addvec), _np(residual))
    perm = (lambda t: t.permute(0, 2, 3, 1).contiguous()) if layout == B.WINO_NHWC else (lambda t: t)
    y = B.conv2d_fused(perm(x).to(DEV), w.to(DEV), b.to(DEV), variant, layout, gamma.to(DEV), beta.to(DEV), G, 1e-5,
                       addvec.to(DEV), perm(residual).to(DEV))
    torch.cuda.synchronize()
    y = y.float().cpu()
    if layout == B.WINO_NHWC:
        y = y.permute(0, 3, 1, 2)
    err = oracle.rel_l2(y.numpy(), ref)
    assert err <= TOL[dtype], (case, layout, variant, dtype, err)


def test_each_part_alone_and_in_place_residual():
    N, C, K, H, W, G = 2, 32, 32, 12, 12, 8
    x, w, b = synth.make_inputs(N, C, K, H, W, "f16", seed=11)
    gamma, beta, addvec, residual = _extras(N, C, K, H, W, "f16", 12)
    xd, wd, bd = x.to(DEV), w.to(DEV), b.to(DEV)
    # nothing switched on: identical to the plain entry point
    assert torch.equal(B.conv2d_fused(xd, wd, bd, B.WINO_F4), B.conv2d(xd, wd, bd, B.WINO_F4))
    # only the pre-op
    y = B.conv2d_fused(xd, wd, bd, B.WINO_F4, gn_gamma=gamma.to(DEV), gn_beta=beta.to(DEV), gn_groups=G)
    ref = fo.conv2d_fused(_np(x), _np(w), _np(b), _np(gamma), _np(beta), G)
    assert oracle.rel_l2(y.float().cpu().numpy(), ref) <= 5e-3
    # only the post-ops
    y = B.conv2d_fused(xd, wd, bd, B.WINO_F4, addvec=addvec.to(DEV), residual=residual.to(DEV))
    ref = fo.conv2d_fused(_np(x), _np(w), _np(b), addvec=_np(addvec), residual=_np(residual))
    assert oracle.rel_l2(y.float().cpu().numpy(), ref) <= 5e-3
    # residual may be y itself
    w_t = B.wino_filter_transform(wd, B.WINO_F4)
    ws = torch.empty(B.wino_workspace_bytes(N, C, H, W, K, B.WINO_F16, B.WINO_F4), dtype=torch.uint8, device=DEV)
    acc = residual.to(DEV).clone()
    B.wino_conv2d_fused(xd, w_t, bd, acc, ws, residual=acc)
    torch.cuda.synchronize()
    assert torch.equal(acc, B.conv2d_fused(xd, wd, bd, B.WINO_F4, residual=residual.to(DEV)))


def test_fused_resblock_layer_full_size():
    """Layer B as it sits in a residual block: GroupNorm(32) + SiLU in, time-embedding vector and skip tensor out."""
    layer = synth.LAYERS["B_resblock"]
    x, w, b = synth.make_layer_inputs(layer)
    gamma, beta, addvec, residual = _extras(layer.N, layer.C, layer.K, layer.H, layer.W, "f16", 5)
    y = B.conv2d_fused(x.to(DEV), w.to(DEV), b.to(DEV), B.WINO_AUTO, B.WINO_NCHW, gamma.to(DEV), beta.to(DEV), 32, 1e-5,
                       addvec.to(DEV), residual.to(DEV))
    torch.cuda.synchronize()
    ref = fo.conv2d_fused(_np(x), _np(w), _np(b), _np(gamma), _np(beta), 32, 1e-5, _np(addvec), _np(residual))
    err = oracle.rel_l2(y.float().cpu().numpy(), ref)
    print(f"fused B layer: relL2 {err:.3e}")
    assert err <= 5e-3


# source shapes (N, C, K, h, w, groups); y is 2h x 2w.  They cover the scalar kernel (rows that are not whole
# 16-byte chunks), the chunked strip kernel, and the sliding-window kernel for long rows.
UP_CASES = [(1, 8, 8, 3, 5, 4), (2, 24, 16, 8, 12, 8), (1, 64, 8, 4, 108, 32), (1, 40, 6, 16, 16, 8)]


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("variant", [B.WINO_F2, B.WINO_F4, B.WINO_FUSED_F2])
@pytest.mark.parametrize("layout", [B.WINO_NCHW, B.WINO_NHWC])
@pytest.mark.parametrize("with_gn", [False, True])
@pytest.mark.parametrize("case", UP_CASES)
def test_upsample_fused(case, with_gn, layout, variant, dtype):
    """2x nearest-neighbour upsampling read inside the activation transform, alone and together with the
    GroupNorm + SiLU pre-op and both post-ops."""
    N, C, K, h, w_, G = case
    x, w, b = synth.make_inputs(N, C, K, h, w_, dtype, seed=6000 + sum(case))
    gamma, beta, addvec, residual = _extras(N, C, K, 2 * h, 2 * w_, dtype, 99 + sum(case))
    if with_gn:
        ref = fo.conv2d_fused(_np(x), _np(w), _np(b), _np(gamma), _np(beta), G, 1e-5, _np(addvec), _np(residual), upsample=True)
    else:
        ref = fo.conv2d_fused(_np(x), _np(w), _np(b), upsample=True)
    perm = (lambda t: t.permute(0, 2, 3, 1).contiguous()) if layout == B.WINO_NHWC else (lambda t: t)
    if with_gn:
        y = B.conv2d_fused(perm(x).to(DEV), w.to(DEV), b.to(DEV), variant, layout, gamma.to(DEV), beta.to(DEV), G, 1e-5,
                           addvec.to(DEV), perm(residual).to(DEV), upsample=True)
    else:
        y = B.conv2d_fused(perm(x).to(DEV), w.to(DEV), b.to(DEV), variant, layout, upsample=True)
    torch.cuda.synchronize()
    y = y.float().cpu()
    if layout == B.WINO_NHWC:
        y = y.permute(0, 3, 1, 2)
    assert tuple(y.shape) == (N, K, 2 * h, 2 * w_)
    err = oracle.rel_l2(y.numpy(), ref)
    assert err <= TOL[dtype], (case, with_gn, layout, variant, dtype, err)


def test_upsample_rejects_odd_output_size():
    x, w, b = synth.make_inputs(1, 8, 8, 4, 4, "f16", seed=1)
    w_t = B.wino_filter_transform(w.to(DEV), B.WINO_F2)
    y = torch.empty((1, 8, 7, 8), dtype=torch.float16, device=DEV)
    ws = torch.empty(1 << 20, dtype=torch.uint8, device=DEV)
    f = B.wino_fusion(); f.upsample = 1
    import ctypes
    rc = B.lib().wino_conv2d_fused(x.to(DEV).data_ptr(), ctypes.byref(w_t.desc), None, y.data_ptr(), 1, 8, 7, 8, 8, B.WINO_NCHW,
                                   ctypes.byref(f), ws.data_ptr(), ws.numel(), None)
    assert rc == B.WINO_ERR_DIM


# what a correct half-product path must show (tests/test_error_model.py derives these bands on the CPU)
HALF_PRODUCT_BAND = {B.WINO_F2: (4.0e-4, 1.0e-3), B.WINO_F4: (3.0e-3, 4.8e-3)}


@pytest.mark.parametrize("layout", [B.WINO_NCHW, B.WINO_NHWC])
@pytest.mark.parametrize("variant", [B.WINO_F2, B.WINO_F4])
@pytest.mark.parametrize("shape", [(2, 24, 40, 18, 22), (1, 64, 130, 33, 40), (2, 320, 64, 32, 32), (1, 136, 72, 7, 216)])
def test_half_product_mode(shape, variant, layout):
    """Opt-in fp16 intermediate product: inside the 5e-3 tolerance, above the plain path's error, inside the band
    the CPU model predicts (a path that silently kept M in fp32 would sit below it)."""
    N, C, K, H, W = shape
    x, w, b = synth.make_inputs(N, C, K, H, W, "f16", seed=9000 + sum(shape))
    ref = oracle.conv2d_direct(_np(x), _np(w), _np(b))
    perm = (lambda t: t.permute(0, 2, 3, 1).contiguous()) if layout == B.WINO_NHWC else (lambda t: t)
    unperm = (lambda t: t.permute(0, 3, 1, 2)) if layout == B.WINO_NHWC else (lambda t: t)
    y_hp = B.conv2d_fused(perm(x).to(DEV), w.to(DEV), b.to(DEV), variant, layout, product_fp16=True)
    y_fp = B.conv2d_fused(perm(x).to(DEV), w.to(DEV), b.to(DEV), variant, layout)
    torch.cuda.synchronize()
    e_hp = oracle.rel_l2(unperm(y_hp.float().cpu()).numpy(), ref)
    e_fp = oracle.rel_l2(unperm(y_fp.float().cpu()).numpy(), ref)
    lo, hi = HALF_PRODUCT_BAND[variant]
    assert e_hp <= TOL["f16"] and lo <= e_hp <= hi and e_hp > e_fp, (shape, variant, layout, e_hp, e_fp)


def test_half_product_mode_is_ignored_for_fp32_and_split_reductions():
    # fp32 storage: same bits as the plain call
    x, w, b = synth.make_inputs(1, 24, 16, 12, 12, "f32", seed=3)
    a = B.conv2d_fused(x.to(DEV), w.to(DEV), b.to(DEV), B.WINO_F4, product_fp16=True)
    c = B.conv2d(x.to(DEV), w.to(DEV), b.to(DEV), B.WINO_F4)
    assert torch.equal(a, c)
    # F(2x2) on an 8x8 image with 1024 channels splits its reduction: M stays fp32 there
    x, w, b = synth.make_inputs(1, 1024, 256, 8, 8, "f16", seed=4)
    a = B.conv2d_fused(x.to(DEV), w.to(DEV), b.to(DEV), B.WINO_F2, product_fp16=True)
    c = B.conv2d(x.to(DEV), w.to(DEV), b.to(DEV), B.WINO_F2)
    torch.cuda.synchronize()
    assert torch.equal(a, c)


# (N, C, K, h, w): the direct variant reads x through the upsampling by address arithmetic and adds the vector and the
# residual in its epilogue; the third shape has few pixels and a long reduction, so the adds happen in the kernel that
# sums the partial products
DIRECT_UP_CASES = [(1, 24, 40, 5, 7), (2, 64, 72, 8, 12), (1, 640, 96, 4, 4)]


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("layout", [B.WINO_NCHW, B.WINO_NHWC])
@pytest.mark.parametrize("upsample", [False, True])
@pytest.mark.parametrize("case", DIRECT_UP_CASES)
def test_direct_variant_fused(case, upsample, layout, dtype):
    N, C, K, h, w_ = case
    x, w, b = synth.make_inputs(N, C, K, h, w_, dtype, seed=12000 + sum(case))
    H, W = (2 * h, 2 * w_) if upsample else (h, w_)
    _, _, addvec, residual = _extras(N, C, K, H, W, dtype, 13 + sum(case))
    ref = fo.conv2d_fused(_np(x), _np(w), _np(b), addvec=_np(addvec), residual=_np(residual), upsample=upsample)
    perm = (lambda t: t.permute(0, 2, 3, 1).contiguous()) if layout == B.WINO_NHWC else (lambda t: t)
    y = B.conv2d_fused(perm(x).to(DEV), w.to(DEV), b.to(DEV), B.WINO_DIRECT, layout, addvec=addvec.to(DEV),
                       residual=perm(residual).to(DEV), upsample=upsample)
    torch.cuda.synchronize()
    y = y.float().cpu()
    if layout == B.WINO_NHWC:
        y = y.permute(0, 3, 1, 2)
    assert tuple(y.shape) == (N, K, H, W)
    err = oracle.rel_l2(y.numpy(), ref)
    assert err <= {"f32": 1e-5, "f16": 6e-4, "bf16": 3e-3}[dtype], (case, upsample, layout, dtype, err)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("layout", [B.WINO_NCHW, B.WINO_NHWC])
@pytest.mark.parametrize("case", [(2, 24, 40, 9, 13, 4, False), (1, 64, 72, 8, 16, 32, True), (1, 40, 16, 6, 6, 8, True), (1, 640, 96, 4, 4, 32, False)])
def test_direct_variant_groupnorm(case, layout, dtype):
    """GroupNorm + SiLU applied while the direct path re-lays x (rows of whole chunks and not, C padded to 8 and not,
    channel-last inputs that would otherwise be read in place, with and without the upsampling)."""
    N, C, K, h, w_, G, upsample = case
    x, w, b = synth.make_inputs(N, C, K, h, w_, dtype, seed=14000 + sum(case[:6]))
    H, W = (2 * h, 2 * w_) if upsample else (h, w_)
    gamma, beta, addvec, residual = _extras(N, C, K, H, W, dtype, 15 + sum(case[:6]))
    ref = fo.conv2d_fused(_np(x), _np(w), _np(b), _np(gamma), _np(beta), G, 1e-5, _np(addvec), _np(residual), upsample=upsample)
    perm = (lambda t: t.permute(0, 2, 3, 1).contiguous()) if layout == B.WINO_NHWC else (lambda t: t)
    y = B.conv2d_fused(perm(x).to(DEV), w.to(DEV), b.to(DEV), B.WINO_DIRECT, layout, gamma.to(DEV), beta.to(DEV), G, 1e-5,
                       addvec.to(DEV), perm(residual).to(DEV), upsample=upsample)
    torch.cuda.synchronize()
    y = y.float().cpu()
    if layout == B.WINO_NHWC:
        y = y.permute(0, 3, 1, 2)
    err = oracle.rel_l2(y.numpy(), ref)
    # the activated tensor is rounded once more than on the plain direct path
    assert err <= {"f32": 1e-5, "f16": 1.2e-3, "bf16": 5e-3}[dtype], (case, layout, dtype, err)


@pytest.mark.parametrize("path", ["winograd_f2", "winograd_f4", "direct", "fp8"])
def test_residual_block_composition(path):
    """A whole Stable-Diffusion residual block through the fused calls: h = conv1(SiLU(GN(x))) + b1 + temb[n, k];
    y = conv2(SiLU(GN(h))) + b2 + x.  The intermediate h stays on the GPU in fp16; the oracle runs the same two steps in fp64."""
    from oracle import fp8_model as f8
    N, C, H, W, G = 2, 64, 24, 24, 8
    g = torch.Generator().manual_seed(77)
    x = torch.randn(N, C, H, W, generator=g).to(torch.float16)
    w1 = (torch.randn(C, C, 3, 3, generator=g) / (9 * C) ** 0.5).to(torch.float16)
    w2 = (torch.randn(C, C, 3, 3, generator=g) / (9 * C) ** 0.5).to(torch.float16)
    b1, b2 = 0.1 * torch.randn(C, generator=g), 0.1 * torch.randn(C, generator=g)
    g1, be1 = 1 + 0.2 * torch.randn(C, generator=g), 0.2 * torch.randn(C, generator=g)
    g2, be2 = 1 + 0.2 * torch.randn(C, generator=g), 0.2 * torch.randn(C, generator=g)
    temb = 0.5 * torch.randn(N, C, generator=g)
    h_ref = fo.conv2d_fused(_np(x), _np(w1), _np(b1), _np(g1), _np(be1), G, 1e-5, addvec=_np(temb))
    y_ref = fo.conv2d_fused(h_ref, _np(w2), _np(b2), _np(g2), _np(be2), G, 1e-5, residual=_np(x))
    d = lambda t: t.to(DEV)
    xd = d(x)
    if path == "fp8":
        a1 = fo.silu(fo.groupnorm(_np(x), _np(g1), _np(be1), G, 1e-5))
        a2 = fo.silu(fo.groupnorm(h_ref, _np(g2), _np(be2), G, 1e-5))
        h = B.conv2d_fp8(xd, d(w1), d(b1), f8.power_of_two_scale(a1), f8.power_of_two_scale(_np(w1)), gn_gamma=d(g1), gn_beta=d(be1),
                         gn_groups=G, addvec=d(temb))
        y = B.conv2d_fp8(h, d(w2), d(b2), f8.power_of_two_scale(a2) / 2, f8.power_of_two_scale(_np(w2)), gn_gamma=d(g2), gn_beta=d(be2),
                         gn_groups=G, residual=xd)
        tol = 6e-2
    else:
        v = {"winograd_f2": B.WINO_F2, "winograd_f4": B.WINO_F4, "direct": B.WINO_DIRECT}[path]
        h = B.conv2d_fused(xd, d(w1), d(b1), v, B.WINO_NCHW, d(g1), d(be1), G, 1e-5, addvec=d(temb))
        y = B.conv2d_fused(h, d(w2), d(b2), v, B.WINO_NCHW, d(g2), d(be2), G, 1e-5, residual=xd)
        tol = {"winograd_f2": 2e-3, "winograd_f4": 8e-3, "direct": 2e-3}[path]
    torch.cuda.synchronize()
    err = oracle.rel_l2(y.float().cpu().numpy(), y_ref)
    print(f"residual block via {path}: relL2 {err:.3e}")
    assert err <= tol, (path, err)


def test_entry_points_replay_correctly_from_a_hip_graph():
    """Every entry point only enqueues kernels on the stream it is given (no allocation, no memset nodes), so a captured
    sequence can be replayed; each replay, with fresh inputs copied in and eager work in between, must equal the eager result."""
    N, C, K, H, W, G = 2, 64, 64, 16, 16, 8
    g = torch.Generator().manual_seed(5)
    wd = (torch.randn(K, C, 3, 3, generator=g) / (9 * C) ** 0.5).to(torch.float16).to(DEV)
    bd = (0.1 * torch.randn(K, generator=g)).to(DEV)
    gamma, beta = (1 + 0.2 * torch.randn(C, generator=g)).to(DEV), (0.2 * torch.randn(C, generator=g)).to(DEV)
    x = torch.empty(N, C, H, W, dtype=torch.float16, device=DEV)
    w_t, w_d, w_q = B.wino_filter_transform(wd, B.WINO_F4), B.wino_filter_transform(wd, B.WINO_DIRECT), B.wino_fp8_filter_quantize(wd, 1024.0)
    ys = [torch.empty(N, K, H, W, dtype=torch.float16, device=DEV) for _ in range(3)]
    ws = [torch.empty(max(B.wino_workspace_bytes(N, C, H, W, K, B.WINO_F16, B.WINO_F4), B.wino_workspace_bytes(N, C, H, W, K, B.WINO_F16, B.WINO_DIRECT),
                          B.wino_fp8_workspace_bytes(N, C, H, W, K, 3, 1)), dtype=torch.uint8, device=DEV) for _ in range(3)]
    st = torch.empty(B.wino_groupnorm_stats_bytes(N, G), dtype=torch.uint8, device=DEV)

    def run():
        B.wino_groupnorm_stats(x, G, out=st)
        B.wino_conv2d_fused(x, w_t, bd, ys[0], ws[0], gn_stats=st, gn_gamma=gamma, gn_beta=beta, gn_groups=G, residual=x)
        B.wino_conv2d_fused(x, w_d, bd, ys[1], ws[1], gn_stats=st, gn_gamma=gamma, gn_beta=beta, gn_groups=G)
        B.wino_fp8_conv2d(x, w_q, bd, ys[2], K, 3, 1, 32.0, 1024.0, ws[2])

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        x.copy_(torch.randn(N, C, H, W, generator=g).to(torch.float16))
        run()
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            run()
        for rep in range(3):
            xin = torch.randn(N, C, H, W, generator=g).to(torch.float16)
            x.copy_(xin)
            graph.replay()
            side.synchronize()
            got = [y.clone() for y in ys]
            for y in ys:
                y.zero_()                                   # eager work between the replays
            run()
            side.synchronize()
            for a, b in zip(got, ys):
                assert torch.equal(a, b), rep
