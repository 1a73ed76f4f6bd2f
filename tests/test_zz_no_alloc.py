"""wino_conv2d_static: the entry point that allocates nothing (its scratch is a device array inside the library).
Two calls in a row, the second on a smaller input, each checked bit for bit against wino_conv2d_ex and against the
oracle; then the size limit."""
import os
import sys

import numpy as np
import pytest
import torch

import oracle
from paper_2412_05781_amd import binding as B
from paper_2412_05781_amd import synth

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
import parity_util as pu  # noqa: E402

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _np(t):
    return t.float().numpy().astype(np.float64)


@pytest.mark.parametrize("variant", [B.WINO_F4, B.WINO_F2, B.WINO_FUSED_F2, B.WINO_FUSED_F4, B.WINO_DIRECT])
def test_two_calls_in_a_row_second_smaller(variant):
    for (N, C, K, H, W) in [(2, 96, 80, 40, 44), (1, 40, 24, 9, 14)]:
        x, w, b = synth.make_inputs(N, C, K, H, W, "f16", seed=8000 + H)
        xd, wd, bd = x.to(DEV), w.to(DEV), b.to(DEV)
        w_t = B.wino_filter_transform(wd, variant)
        ws = torch.empty(max(16, B.wino_workspace_bytes(N, C, H, W, K, B.WINO_F16, variant)), dtype=torch.uint8, device=DEV)
        y_ex = B.wino_conv2d_ex(xd, w_t, bd, torch.empty((N, K, H, W), dtype=xd.dtype, device=DEV), ws)
        y_st = B.wino_conv2d_static(xd, w_t, bd, torch.full((N, K, H, W), float("nan"), dtype=xd.dtype, device=DEV))
        torch.cuda.synchronize()
        assert torch.equal(y_ex, y_st), (variant, (N, C, K, H, W))
        ref = oracle.conv2d_direct(_np(x), _np(w), _np(b))
        pu.check(y_st.float().cpu().numpy().astype(np.float64), ref, 5e-3, {B.WINO_F4: 4, B.WINO_FUSED_F4: 4, B.WINO_DIRECT: 1}.get(variant, 2), "f16")


def test_channel_last_and_fp32():
    N, C, K, H, W = 1, 24, 40, 18, 22
    x, w, b = synth.make_inputs(N, C, K, H, W, "f32", seed=8100)
    xd = x.permute(0, 2, 3, 1).contiguous().to(DEV)
    w_t = B.wino_filter_transform(w.to(DEV), B.WINO_F2)
    ws = torch.empty(B.wino_workspace_bytes(N, C, H, W, K, B.WINO_F32, B.WINO_F2), dtype=torch.uint8, device=DEV)
    y_ex = B.wino_conv2d_ex(xd, w_t, b.to(DEV), torch.empty((N, H, W, K), dtype=xd.dtype, device=DEV), ws, layout=B.WINO_NHWC)
    y_st = B.wino_conv2d_static(xd, w_t, b.to(DEV), torch.empty((N, H, W, K), dtype=xd.dtype, device=DEV), layout=B.WINO_NHWC)
    torch.cuda.synchronize()
    assert torch.equal(y_ex, y_st)


def test_limit_is_reported_and_enforced():
    assert B.wino_static_scratch_bytes() == 64 << 20
    # E1-sized layer: V + M far beyond 64 MiB -> refused on the host, nothing launched, y untouched
    N, C, K, H, W = 1, 512, 512, 128, 128
    assert B.wino_workspace_bytes(N, C, H, W, K, B.WINO_F16, B.WINO_F4) > B.wino_static_scratch_bytes()
    wd = torch.zeros((K, C, 3, 3), dtype=torch.float16, device=DEV)
    w_t = B.wino_filter_transform(wd, B.WINO_F4)
    xd = torch.zeros((N, C, H, W), dtype=torch.float16, device=DEV)
    y = torch.full((N, K, H, W), 3.0, dtype=torch.float16, device=DEV)
    with pytest.raises(B.WinoError) as e:
        B.wino_conv2d_static(xd, w_t, None, y)
    assert e.value.status == B.WINO_ERR_SCRATCH
    torch.cuda.synchronize()
    assert bool((y == 3.0).all())
    # the layer the bench times fits
    assert B.wino_workspace_bytes(2, 320, 64, 64, 320, B.WINO_F16, B.WINO_F4) <= B.wino_static_scratch_bytes()
