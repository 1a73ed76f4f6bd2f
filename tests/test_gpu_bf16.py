"""bfloat16 storage (fp32 accumulation) against the fp64 oracle.  Tolerances are this type's own, set from the
rounding model pinned in tests/test_error_model.py: F(2x2) <= 8e-3 (model 4.2e-3), F(4x4) <= 4e-2 (2.5e-2),
paths that round only their output (direct kernel, implicit GEMM) <= 3e-3 (1.7e-3).  The error must also sit
inside the band of the path that was asked for, so a silently different path fails."""
import numpy as np
import pytest
import torch

import oracle
from oracle import fused_ops as fo
from oracle import winograd_ref as wr
from paper_2412_05781_amd import binding as B
from paper_2412_05781_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = {B.WINO_F2: 8e-3, B.WINO_FUSED_F2: 8e-3, B.WINO_F4: 4e-2, B.WINO_DIRECT: 3e-3}
BAND = {B.WINO_F2: (3.0e-3, 6.0e-3), B.WINO_FUSED_F2: (3.0e-3, 6.0e-3), B.WINO_F4: (1.8e-2, 3.3e-2), B.WINO_DIRECT: (1.2e-3, 2.2e-3)}


def _np(t):
    return None if t is None else t.float().numpy().astype(np.float64)


SHAPES = [(2, 5, 7, 5, 7), (1, 33, 65, 17, 30), (2, 64, 130, 33, 16), (1, 136, 40, 12, 216), (1, 1024, 64, 8, 8)]


@pytest.mark.parametrize("variant", [B.WINO_F2, B.WINO_FUSED_F2, B.WINO_F4, B.WINO_DIRECT])
@pytest.mark.parametrize("shape", SHAPES)
def test_bf16_full_tensor(shape, variant):
    N, C, K, H, W = shape
    x, w, b = synth.make_inputs(N, C, K, H, W, "bf16", seed=10000 + sum(shape))
    ref = oracle.conv2d_direct(_np(x), _np(w), _np(b))
    xd, wd, bd = x.to(DEV), w.to(DEV), b.to(DEV)
    if variant == B.WINO_DIRECT:
        y = B.wino_direct_conv2d(xd, wd, bd, torch.empty((N, K, H, W), dtype=torch.bfloat16, device=DEV))
    else:
        y = B.conv2d(xd, wd, bd, variant)
    torch.cuda.synchronize()
    assert y.dtype == torch.bfloat16
    err = oracle.rel_l2(_np(y.cpu()), ref)
    assert err <= TOL[variant], (shape, variant, err)
    if C >= 33:                                   # enough terms for the rounding statistics to settle
        assert BAND[variant][0] <= err <= BAND[variant][1], (shape, variant, err)


@pytest.mark.parametrize("variant", [B.WINO_F2, B.WINO_F4])
def test_bf16_channel_last_and_stages(variant):
    N, C, K, H, W = 2, 40, 72, 13, 18
    x, w, b = synth.make_inputs(N, C, K, H, W, "bf16", seed=77)
    ref = oracle.conv2d_direct(_np(x), _np(w), _np(b))
    xd, wd, bd = x.to(DEV), w.to(DEV), b.to(DEV)
    y = B.conv2d(xd.permute(0, 2, 3, 1).contiguous(), wd, bd, variant, layout=B.WINO_NHWC)
    torch.cuda.synchronize()
    assert oracle.rel_l2(_np(y.cpu().permute(0, 3, 1, 2)), ref) <= TOL[variant]
    # the stored transforms are the fp64 transforms rounded once to bf16 (8 significant bits)
    alpha, Cp, T = B.wino_transformed_dims(N, C, H, W, K, variant)
    a2 = alpha * alpha
    eps = 2.0 ** -8
    U = B.wino_filter_transform(wd, variant).buf.view(torch.bfloat16).view(a2, K, Cp)
    U_ref = wr.filter_transform(_np(w), variant).reshape(a2, K, C)
    Uh = _np(U.cpu())
    assert np.all(Uh[:, :, C:] == 0) and np.abs(Uh[:, :, :C] - U_ref).max() <= 1.01 * eps * np.abs(U_ref).max()
    V = B.wino_input_transform(xd, variant)
    V_ref = wr.input_transform(_np(x), variant).reshape(a2, C, T).transpose(0, 2, 1)
    Vh = _np(V.cpu())
    assert np.all(Vh[:, :, C:] == 0) and np.abs(Vh[:, :, :C] - V_ref).max() <= 1.01 * eps * np.abs(V_ref).max()
    # the GEMM stage is exact up to fp32 accumulation on the stored operands
    M = B.wino_batched_gemm(U, V, K, C, T, variant)
    assert oracle.rel_l2(_np(M.cpu()), np.einsum("bkc,btc->bkt", Uh, Vh)) <= 1e-6


def test_bf16_auto_on_a_many_tile_layer_runs_the_fused_variant():
    """4096 F(2x2) tiles: WINO_AUTO resolves to the fused variant for bf16; whole tensor and element-wise against the oracle."""
    import os, sys
    sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
    import parity_util as pu
    N, C, K, H, W = 1, 64, 64, 128, 128
    assert B.wino_resolve_variant(N, C, H, W, K, B.WINO_BF16, B.WINO_AUTO) == B.WINO_FUSED_F2
    x, w, b = synth.make_inputs(N, C, K, H, W, "bf16", seed=10777)
    ref = oracle.conv2d_direct(_np(x), _np(w), _np(b))
    y = B.conv2d(x.to(DEV), w.to(DEV), b.to(DEV), B.WINO_AUTO)
    torch.cuda.synchronize()
    err = pu.check(_np(y.cpu()), ref, TOL[B.WINO_FUSED_F2], 2, "bf16", what="bf16 auto", channels=C)
    assert BAND[B.WINO_FUSED_F2][0] <= err <= BAND[B.WINO_FUSED_F2][1], err


def test_bf16_auto_never_picks_f4():
    for (N, C, K, H, W) in [(2, 320, 320, 64, 64), (1, 512, 512, 256, 256), (2, 1280, 1280, 8, 8)]:
        assert B.wino_resolve_variant(N, C, H, W, K, B.WINO_BF16, B.WINO_AUTO) in (B.WINO_F2, B.WINO_FUSED_F2)
    assert B.wino_resolve_variant(1, 512, 256, 256, 512, B.WINO_BF16, B.WINO_AUTO) == B.WINO_FUSED_F2      # 16384 tiles


@pytest.mark.parametrize("layout", [B.WINO_NCHW, B.WINO_NHWC])
def test_bf16_fused_ops(layout):
    N, C, K, h, w_, G = 1, 64, 24, 6, 108, 8          # long rows: the sliding-window kernel; y is 12 x 216
    x, w, b = synth.make_inputs(N, C, K, h, w_, "bf16", seed=31)
    g = torch.Generator().manual_seed(5)
    gamma, beta = 1.0 + 0.2 * torch.randn(C, generator=g), 0.3 * torch.randn(C, generator=g)
    addvec = 0.5 * torch.randn(N, K, generator=g)
    residual = torch.randn(N, K, 2 * h, 2 * w_, generator=g).to(torch.bfloat16)
    ref = fo.conv2d_fused(_np(x), _np(w), _np(b), _np(gamma), _np(beta), G, 1e-5, _np(addvec), _np(residual), upsample=True)
    perm = (lambda t: t.permute(0, 2, 3, 1).contiguous()) if layout == B.WINO_NHWC else (lambda t: t)
    y = B.conv2d_fused(perm(x).to(DEV), w.to(DEV), b.to(DEV), B.WINO_F2, layout, gamma.to(DEV), beta.to(DEV), G, 1e-5,
                       addvec.to(DEV), perm(residual).to(DEV), upsample=True)
    torch.cuda.synchronize()
    y = y.cpu()
    if layout == B.WINO_NHWC:
        y = y.permute(0, 3, 1, 2)
    assert oracle.rel_l2(_np(y), ref) <= TOL[B.WINO_F2]
    # the GroupNorm statistics of a bf16 tensor
    st = B.stats_view(B.wino_groupnorm_stats(x.to(DEV), G, 1e-5), N, G).cpu().numpy().astype(np.float64)
    mean, rstd = fo.groupnorm_stats(_np(x), G, 1e-5)
    assert np.abs(st[:, :, 0] - mean).max() <= 2e-6 * (1 + np.abs(mean).max()) and np.abs(st[:, :, 1] / rstd - 1).max() <= 5e-6


@pytest.mark.parametrize("layout", [B.WINO_NCHW, B.WINO_NHWC])
@pytest.mark.parametrize("R,stride,shape", [(1, 1, (2, 72, 136, 17, 15)), (3, 2, (1, 320, 200, 16, 16)), (3, 1, (1, 64, 64, 33, 40)),
                                            (3, 2, (2, 640, 96, 16, 16))])
def test_bf16_implicit_gemm(shape, R, stride, layout):
    N, C, K, H, W = shape
    g = torch.Generator().manual_seed(11000 + sum(shape))
    x = torch.randn(N, C, H, W, generator=g).to(torch.bfloat16)
    w = (torch.randn(K, C, R, R, generator=g) / (R * R * C) ** 0.5).to(torch.bfloat16)
    b = torch.randn(K, generator=g) * 0.1
    ref = oracle.conv2d_general(_np(x), _np(w), _np(b), stride)
    xd = (x.permute(0, 2, 3, 1).contiguous() if layout == B.WINO_NHWC else x).to(DEV)
    y = B.conv2d_igemm(xd, w.to(DEV), b.to(DEV), stride, layout)
    torch.cuda.synchronize()
    y = y.cpu()
    if layout == B.WINO_NHWC:
        y = y.permute(0, 3, 1, 2)
    err = oracle.rel_l2(_np(y), ref)
    assert BAND[B.WINO_DIRECT][0] <= err <= TOL[B.WINO_DIRECT], (shape, R, stride, layout, err)
