"""Parity of the implicit-GEMM convolution path (1x1, 3x3 stride 2, 3x3 stride 1) against the fp64 oracle:
relative L2 <= 1e-5 for fp32 storage, <= 5e-3 for fp16 storage with fp32 accumulation (the path rounds only its
output, so it sits far below that)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2412_05781_amd import binding as B
from paper_2412_05781_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = {"f32": 1e-5, "f16": 5e-3}


def _np(t):
    return None if t is None else t.float().numpy().astype(np.float64)


def _inputs(N, C, K, H, W, R, dtype, seed):
    g = torch.Generator().manual_seed(seed)
    tdt = synth.TORCH_DTYPE[dtype]
    x = torch.randn(N, C, H, W, generator=g).to(tdt)
    w = (torch.randn(K, C, R, R, generator=g) / (R * R * C) ** 0.5).to(tdt)
    b = torch.randn(K, generator=g) * 0.1
    return x, w, b


# (N, C, K, H, W): tiny, ragged channel counts (C not a multiple of 8 / of the 128-byte stage), several
# 64- and 128-wide blocks with ragged tails, odd image sizes
SHAPES = [(1, 1, 1, 1, 1), (2, 5, 7, 6, 9), (1, 24, 40, 13, 18), (2, 72, 136, 17, 15), (1, 320, 200, 16, 16), (1, 64, 64, 33, 40)]


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("layout", [B.WINO_NCHW, B.WINO_NHWC])
@pytest.mark.parametrize("R,stride", [(1, 1), (3, 2), (3, 1), (1, 2)])
@pytest.mark.parametrize("shape", SHAPES)
def test_igemm_full_tensor(shape, R, stride, layout, dtype):
    N, C, K, H, W = shape
    x, w, b = _inputs(N, C, K, H, W, R, dtype, seed=7000 + sum(shape) + 10 * R + stride)
    ref = oracle.conv2d_general(_np(x), _np(w), _np(b), stride)
    xd = (x.permute(0, 2, 3, 1).contiguous() if layout == B.WINO_NHWC else x).to(DEV)
    y = B.conv2d_igemm(xd, w.to(DEV), b.to(DEV), stride, layout)
    torch.cuda.synchronize()
    y = y.float().cpu()
    if layout == B.WINO_NHWC:
        y = y.permute(0, 3, 1, 2)
    assert tuple(y.shape) == ref.shape
    if not np.any(ref):
        assert not np.any(y.numpy())
        return
    err = oracle.rel_l2(y.numpy(), ref)
    assert err <= TOL[dtype], (shape, R, stride, layout, dtype, err)
    if dtype == "f16":
        assert err <= 6e-4          # only the output is rounded


def test_igemm_no_bias_large_block_and_determinism():
    N, C, K, H, W = 2, 128, 256, 48, 48          # 128x128 blocks
    x, w, _ = _inputs(N, C, K, H, W, 3, "f16", seed=5)
    ref = oracle.conv2d_general(_np(x), _np(w), None, 2)
    y1 = B.conv2d_igemm(x.to(DEV), w.to(DEV), None, 2)
    y2 = B.conv2d_igemm(x.to(DEV), w.to(DEV), None, 2)
    torch.cuda.synchronize()
    assert torch.equal(y1, y2)
    assert oracle.rel_l2(y1.float().cpu().numpy(), ref) <= 6e-4


@pytest.mark.parametrize("layout", [B.WINO_NCHW, B.WINO_NHWC])
@pytest.mark.parametrize("dtype,shape,R,stride", [("f16", (2, 640, 200, 16, 16), 3, 2), ("f16", (1, 2048, 96, 8, 8), 1, 1),
                                                  ("f32", (1, 264, 72, 12, 10), 3, 2), ("f16", (2, 328, 130, 9, 9), 3, 1)])
def test_igemm_split_reduction(dtype, shape, R, stride, layout):
    """Few output pixels and a long reduction: the stage is cut into ranges whose fp32 partial sums a second kernel
    adds (ragged block tails, a channel count that is not a whole number of stages, both layouts)."""
    N, C, K, H, W = shape
    x, w, b = _inputs(N, C, K, H, W, R, dtype, seed=8000 + sum(shape))
    ref = oracle.conv2d_general(_np(x), _np(w), _np(b), stride)
    xd = (x.permute(0, 2, 3, 1).contiguous() if layout == B.WINO_NHWC else x).to(DEV)
    assert B.wino_igemm_workspace_bytes(N, C, H, W, K, R, stride, B.DTYPE_OF[x.dtype], B.WINO_NHWC) > 0     # partial sums are in use
    y = B.conv2d_igemm(xd, w.to(DEV), b.to(DEV), stride, layout)
    torch.cuda.synchronize()
    y = y.float().cpu()
    if layout == B.WINO_NHWC:
        y = y.permute(0, 3, 1, 2)
    err = oracle.rel_l2(y.numpy(), ref)
    assert err <= (6e-4 if dtype == "f16" else 1e-5), (shape, R, stride, layout, dtype, err)


def test_igemm_matches_winograd_and_direct_kernels():
    """3x3 / stride 1: the same operator as the Winograd path and the checking kernel."""
    N, C, K, H, W = 1, 48, 56, 20, 24
    x, w, b = synth.make_inputs(N, C, K, H, W, "f32", seed=21)
    xd, wd, bd = x.to(DEV), w.to(DEV), b.to(DEV)
    yi = B.conv2d_igemm(xd, wd, bd, 1)
    yw = B.conv2d(xd, wd, bd, B.WINO_F2)
    yd = B.wino_direct_conv2d(xd, wd, bd, torch.empty_like(yw))
    torch.cuda.synchronize()
    assert (yi - yd).abs().max().item() <= 1e-5 * yd.abs().max().item()
    assert (yi - yw).abs().max().item() <= 1e-4 * yd.abs().max().item()


def test_igemm_argument_checks():
    x, w, b = _inputs(1, 8, 8, 8, 8, 3, "f16", seed=1)
    xd, wd = x.to(DEV), w.to(DEV)
    w_r = B.wino_igemm_filter_repack(wd)
    y = torch.empty((1, 8, 4, 4), dtype=torch.float16, device=DEV)
    L = B.lib()
    ws = torch.empty(B.wino_igemm_workspace_bytes(1, 8, 8, 8, 8, 3, 2, B.WINO_F16, B.WINO_NCHW), dtype=torch.uint8, device=DEV)
    args = lambda **kw: [kw.get("x", xd.data_ptr()), w_r.data_ptr(), None, y.data_ptr(), 1, 8, 8, 8, 8, kw.get("R", 3), kw.get("st", 2),
                         B.WINO_F16, kw.get("layout", B.WINO_NCHW), kw.get("ws", ws.data_ptr()), kw.get("wsb", ws.numel()), None]
    assert L.wino_igemm_conv2d(*args()) == B.WINO_OK
    assert L.wino_igemm_conv2d(*args(R=2)) == B.WINO_ERR_DIM
    assert L.wino_igemm_conv2d(*args(st=3)) == B.WINO_ERR_DIM
    assert L.wino_igemm_conv2d(*args(layout=5)) == B.WINO_ERR_LAYOUT
    assert L.wino_igemm_conv2d(*args(wsb=16)) == B.WINO_ERR_WORKSPACE
    assert L.wino_igemm_conv2d(*args(x=xd.data_ptr() + 2)) == B.WINO_ERR_ALIGN
    assert L.wino_igemm_conv2d(*args(x=None)) == B.WINO_ERR_NULL
    assert B.wino_igemm_workspace_bytes(1, 8, 8, 8, 8, 1, 1, B.WINO_F16, B.WINO_NHWC) == 0   # read in place, one stage: nothing to hold
    torch.cuda.synchronize()


# ---- very few output channels (K <= 4) on large images, fp16: the one-pass vector-ALU kernel behind the same entry points ----
# (N, C, K, H, W), each with at least 512 tiles of 8 x 64 pixels (below that the implicit-GEMM kernels take the call): one and
# several channel steps, heights that are not multiples of 8, widths that are multiples of 8 but not of 64 (and, channel-last,
# not even of 8), every K
FEWK_SHAPES = [(1, 16, 3, 517, 512), (2, 32, 4, 261, 520), (1, 48, 1, 1024, 256), (3, 16, 2, 200, 456)]


def _fewk_run(x, w, b, layout):
    xd = (x.permute(0, 2, 3, 1).contiguous() if layout == B.WINO_NHWC else x).to(DEV)
    y = B.conv2d_igemm(xd, w.to(DEV), None if b is None else b.to(DEV), 1, layout)
    torch.cuda.synchronize()
    y = y.cpu()
    return y.permute(0, 3, 1, 2) if layout == B.WINO_NHWC else y


@pytest.mark.parametrize("layout", [B.WINO_NCHW, B.WINO_NHWC])
@pytest.mark.parametrize("shape", FEWK_SHAPES)
def test_few_output_channels_full_tensor(shape, layout):
    """Whole tensor, element by element, against the fp64 oracle; every output is one rounding of an fp32 sum, so each
    element must be within fp16 rounding of the oracle plus the fp32 accumulation error."""
    N, C, K, H, W = shape
    if layout == B.WINO_NHWC:
        W += 3                                      # channel-last has no 8-column requirement
    x, w, b = _inputs(N, C, K, H, W, 3, "f16", seed=7700 + sum(shape))
    ref = oracle.conv2d_general(_np(x), _np(w), _np(b), 1)
    for use_bias in (True, False):
        r = ref if use_bias else ref - _np(b)[None, :, None, None]
        got = _np(_fewk_run(x, w, b if use_bias else None, layout))
        assert got.shape == r.shape
        err = oracle.rel_l2(got, r)
        assert err <= 6e-4, (shape, use_bias, err)
        # element-wise: half an fp16 ulp of the result plus a few fp32 ulps of the largest partial sum
        bound = 2.0 ** -11 * 1.001 * np.abs(r) + 2.0 ** -25 + 1e-5
        assert np.all(np.abs(got - r) <= bound), (shape, use_bias, float(np.abs(got - r).max()))
    if layout == B.WINO_NCHW:      # the same call through the direct variant of the Winograd entry points
        w_t = B.wino_filter_transform(w.to(DEV), B.WINO_DIRECT)
        ws = torch.empty(max(16, B.wino_workspace_bytes(N, C, H, W, K, B.WINO_F16, B.WINO_DIRECT)), dtype=torch.uint8, device=DEV)
        y2 = B.wino_conv2d_ex(x.to(DEV), w_t, b.to(DEV), torch.empty((N, K, H, W), dtype=torch.float16, device=DEV), ws)
        y1 = B.conv2d_igemm(x.to(DEV), w.to(DEV), b.to(DEV), 1, B.WINO_NCHW)
        torch.cuda.synchronize()
        assert torch.equal(y1, y2)


def test_few_output_channels_falls_back_where_the_kernel_does_not_apply():
    """Small images, a width that is not a multiple of 8, 24 channels, fp32: the implicit-GEMM kernels take the call; same
    tolerance."""
    for (N, C, K, H, W, dtype, layout) in [(1, 16, 3, 9, 16, "f16", B.WINO_NCHW), (1, 16, 3, 517, 509, "f16", B.WINO_NCHW),
                                           (1, 24, 3, 517, 512, "f16", B.WINO_NHWC), (1, 16, 3, 517, 512, "f32", B.WINO_NCHW)]:
        x, w, b = _inputs(N, C, K, H, W, 3, dtype, seed=7800 + C + W)
        ref = oracle.conv2d_general(_np(x), _np(w), _np(b), 1)
        y = _fewk_run(x, w, b, layout).float()
        assert oracle.rel_l2(y.numpy(), ref) <= TOL[dtype]
