"""The Winograd F(2x2) path with 8-bit integer U and V against the oracle's model (oracle/int8_model.py).

Integer work is compared bit for bit: the codes and steps of the filter (decided in fp64 on both sides) and of the
activation (decided in fp32 on both sides, row combination first).  The product M is the exact integer sum times two fp32
steps; the kernel multiplies in fp32 where the model multiplies in fp64, so M may differ by two fp32 roundings.  The result
is checked (1) against the MODEL - only those roundings, the fp32 output transform and the rounding of y remain - and
(2) against the exact convolution, where the error must sit in the band the model's pins predict (1.3e-2 ... 2.2e-2;
tolerance of the path 3e-2)."""
import os
import sys

import numpy as np
import pytest
import torch

import oracle
from oracle import int8_model as i8
from oracle import winograd_ref as wr
from paper_2412_05781_amd import binding as B
from paper_2412_05781_amd import synth

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
import parity_util as pu  # noqa: E402

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
OUT_TOL = {"f32": 2e-6, "f16": 6e-4, "bf16": 3e-3}       # against the model: fp32 arithmetic after the integer sums + one rounding of y
FP32_SUM = 4e-6                                          # 16 products of |M| <= max|M|, each off by two fp32 roundings, summed in fp32
PATH_TOL = 3e-2


def _np(t):
    return None if t is None else t.float().numpy().astype(np.float64)


def _perm(t, layout):
    return t.permute(0, 2, 3, 1).contiguous() if layout == B.WINO_NHWC else t


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("KC", [(1, 1), (7, 5), (40, 33), (64, 130), (24, 1280), (3, 300)])
def test_i8_filter_codes_bit_exact(KC, dtype):
    K, C = KC
    _, w, _ = synth.make_inputs(1, C, K, 4, 4, dtype, seed=20000 + K + C)
    if K == 7:
        w[2] = 0                                        # an all-zero output channel: codes 0, step 0
    buf = B.wino_i8_filter_transform(w.to(DEV))
    Uq, dU = B.i8_filter_views(buf, K, C)
    torch.cuda.synchronize()
    Uq_ref, dU_ref = i8.filter_codes(_np(w))
    Uq_ref = Uq_ref.reshape(16, K, C)
    got = Uq.cpu().numpy()
    assert np.array_equal(got[:, :, :C], Uq_ref.astype(np.int8)) and np.all(got[:, :, C:] == 0)
    assert np.array_equal(dU.cpu().numpy(), dU_ref.reshape(16, K).astype(np.float32))


ACT_SHAPES = [(1, 1, 1, 1), (2, 5, 6, 9), (1, 24, 13, 18), (2, 72, 17, 15), (1, 130, 33, 40), (2, 640, 8, 8), (1, 1280, 16, 16),
              (1, 3300, 5, 4), (1, 3100, 24, 24)]       # the last two: more channel rounds than the kernel keeps in registers


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("layout", [B.WINO_NCHW, B.WINO_NHWC])
@pytest.mark.parametrize("shape", ACT_SHAPES)
def test_i8_activation_codes_bit_exact(shape, layout, dtype):
    N, C, H, W = shape
    x, _, _ = synth.make_inputs(N, C, 1, H, W, dtype, seed=21000 + sum(shape))
    if C >= 5:
        x[:, :, : min(H, 4), : min(W, 4)][0, :, :, :] *= 0.0       # some all-zero rows of V: codes 0, step 0
    Vq, dV = B.wino_i8_input_transform(_perm(x, layout).to(DEV), layout)
    torch.cuda.synchronize()
    Vq_ref, dV_ref = i8.activation_codes(_np(x))        # [4,4,C,T], [4,4,T]
    T = Vq_ref.shape[3]
    got = Vq.cpu().numpy()
    assert got.shape == (16, T, (C + 15) // 16 * 16)
    assert np.array_equal(got[:, :, :C], Vq_ref.reshape(16, C, T).transpose(0, 2, 1).astype(np.int8)) and np.all(got[:, :, C:] == 0)
    assert np.array_equal(dV.cpu().numpy(), dV_ref.reshape(16, T).astype(np.float32))


def _random_codes(rows, C, seed):
    g = torch.Generator().manual_seed(seed)
    Cq = (C + 15) // 16 * 16
    q = torch.randint(-127, 128, (16, rows, Cq), generator=g, dtype=torch.int32).to(torch.int8)
    q[:, :, C:] = 0
    d = (torch.rand(16, rows, generator=g) + 0.5) * 1e-2
    return q, d.float()


GEMM_DIMS = [(1, 1, 1), (33, 17, 50), (130, 128, 70), (64, 256, 31), (257, 384, 129), (96, 1280, 32), (40, 200, 300)]


@pytest.mark.parametrize("shape", [-1, 0, 1, 2, 3, 4, 5, 6, 7, 8])
@pytest.mark.parametrize("dims", GEMM_DIMS)
def test_i8_gemm_is_the_exact_integer_product_times_the_steps(dims, shape):
    K, C, T = dims
    Uq, dU = _random_codes(K, C, 22000 + K)
    Vq, dV = _random_codes(T, C, 23000 + T)
    M = B.wino_i8_batched_gemm(Uq.to(DEV), dU.to(DEV), Vq.to(DEV), dV.to(DEV), K, C, T, shape)
    Mt = B.wino_i8_batched_gemm(Vq.to(DEV), dV.to(DEV), Uq.to(DEV), dU.to(DEV), T, C, K, shape)      # operands swapped
    torch.cuda.synchronize()
    acc = np.einsum("bkc,btc->bkt", Uq.numpy().astype(np.int64), Vq.numpy().astype(np.int64))
    ref = acc.astype(np.float64) * dU.numpy().astype(np.float64)[:, :, None] * dV.numpy().astype(np.float64)[:, None, :]
    got = M.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - ref) <= 2.5e-7 * np.abs(ref)), (dims, shape)
    gott = Mt.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(gott - ref.transpose(0, 2, 1)) <= 2.5e-7 * np.abs(ref.transpose(0, 2, 1))), (dims, shape)


def test_i8_gemm_extreme_codes_do_not_overflow():
    """All codes +-127 over 4096 channels: |sum| = 66 064 384, far inside int32 and beyond fp32's exact integers."""
    K, C, T = 32, 4096, 32
    Uq = torch.full((16, K, C), 127, dtype=torch.int8)
    Vq = torch.full((16, T, C), -127, dtype=torch.int8)
    one = torch.ones(16, K)
    M = B.wino_i8_batched_gemm(Uq.to(DEV), one.to(DEV), Vq.to(DEV), torch.ones(16, T).to(DEV), K, C, T)
    torch.cuda.synchronize()
    assert torch.all(M.cpu() == float(np.float32(-127 * 127 * C)))


SHAPES = [(1, 1, 1, 1, 1), (2, 5, 7, 6, 9), (1, 24, 40, 13, 18), (2, 72, 136, 17, 15), (1, 320, 200, 16, 16), (1, 130, 64, 33, 40),
          (2, 640, 96, 8, 8), (1, 256, 72, 24, 20)]


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("layout", [B.WINO_NCHW, B.WINO_NHWC])
@pytest.mark.parametrize("shape", SHAPES)
def test_i8_conv_against_the_quantisation_model(shape, layout, dtype):
    N, C, K, H, W = shape
    x, w, b = synth.make_inputs(N, C, K, H, W, dtype, seed=24000 + sum(shape))
    M = i8.product(*i8.filter_codes(_np(w)), *i8.activation_codes(_np(x)))
    model = wr.output_transform(M, _np(b), N, H, W, 2)
    assert np.array_equal(model, i8.conv2d_winograd_int8(_np(x), _np(w), _np(b)))
    y = B.conv2d_i8(_perm(x, layout).to(DEV), w.to(DEV), b.to(DEV), layout)
    torch.cuda.synchronize()
    y = y.float().cpu()
    if layout == B.WINO_NHWC:
        y = y.permute(0, 3, 1, 2)
    assert tuple(y.shape) == model.shape
    yn = y.numpy().astype(np.float64)
    # the norm of the difference against the norm of what was summed (a tiny output can be the rest of a cancellation)
    scale = max(np.abs(M).max(), np.abs(model).max())
    err = np.linalg.norm(yn - model) / max(np.linalg.norm(model), scale)
    assert err <= OUT_TOL[dtype], (shape, layout, dtype, err)
    # element-wise: the fp32 arithmetic after the integer sums plus half a unit in the last place of y
    slack = FP32_SUM * scale + pu.HALF_ULP[dtype] * 1.001 * np.abs(model) + pu.SUBNORMAL_HALF_ULP[dtype]
    assert np.all(np.abs(yn - model) <= slack), (shape, layout, dtype)


@pytest.mark.parametrize("layout", [B.WINO_NCHW, B.WINO_NHWC])
def test_i8_error_band_against_the_exact_convolution(layout):
    N, C, K, H, W = 2, 320, 96, 24, 24
    x, w, b = synth.make_inputs(N, C, K, H, W, "f16", seed=3)
    ref = oracle.conv2d_direct(_np(x), _np(w), _np(b))
    y = B.conv2d_i8(_perm(x, layout).to(DEV), w.to(DEV), b.to(DEV), layout)
    torch.cuda.synchronize()
    y = y.float().cpu()
    if layout == B.WINO_NHWC:
        y = y.permute(0, 3, 1, 2)
    err = pu.check(y.numpy().astype(np.float64), ref, PATH_TOL, 2, "f16", what="int8 winograd", channels=C)
    assert 1.3e-2 <= err <= 2.2e-2, err


@pytest.mark.parametrize("layout", [B.WINO_NCHW, B.WINO_NHWC])
@pytest.mark.parametrize("name", ["C3_unet", "C4_unet", "C5_unet", "C6_unet"])
def test_i8_full_size_weight_streaming_layers(name, layout):
    """The layers the path is meant for, at full size: whole tensor against the model and against the exact convolution."""
    L = synth.LAYERS[name]
    x, w, b = synth.make_layer_inputs(L)
    model = i8.conv2d_winograd_int8(_np(x), _np(w), _np(b))
    ref = oracle.conv2d_direct(_np(x), _np(w), _np(b))
    y = B.conv2d_i8(_perm(x, layout).to(DEV), w.to(DEV), b.to(DEV), layout)
    torch.cuda.synchronize()
    y = y.float().cpu()
    if layout == B.WINO_NHWC:
        y = y.permute(0, 3, 1, 2)
    yn = y.numpy().astype(np.float64)
    assert oracle.rel_l2(yn, model) <= OUT_TOL[L.dtype], name
    err = pu.check(yn, ref, PATH_TOL, 2, L.dtype, what=name + " int8", channels=L.C)
    assert 1.3e-2 <= err <= 2.3e-2, (name, err)


def test_i8_zero_input_no_bias_determinism_and_scaling():
    N, C, K, H, W = 2, 40, 24, 10, 11
    x, w, b = synth.make_inputs(N, C, K, H, W, "f16", seed=5)
    xd, wd, bd = x.to(DEV), w.to(DEV), b.to(DEV)
    # an all-zero image: every row of V has step 0 and codes 0, so y is the bias, rounded once
    y0 = B.conv2d_i8(torch.zeros_like(xd), wd, bd)
    torch.cuda.synchronize()
    assert torch.equal(y0.float().cpu(), b.to(torch.float16).float().view(1, -1, 1, 1).expand(N, K, H, W))
    # no bias; the same call twice gives the same bits
    y1, y2 = B.conv2d_i8(xd, wd, None), B.conv2d_i8(xd, wd, None)
    torch.cuda.synchronize()
    assert torch.equal(y1, y2)
    model = i8.conv2d_winograd_int8(_np(x), _np(w), None)
    assert oracle.rel_l2(y1.float().cpu().numpy().astype(np.float64), model) <= OUT_TOL["f16"]
    # the steps follow the data: an image 16 times larger (exact in fp16 here) gives 16 times the result, the codes unchanged
    xs = (x * 16.0).to(torch.float16)
    assert torch.equal(xs.float(), x.float() * 16.0)
    Vq1, dV1 = B.wino_i8_input_transform(xd)
    Vq2, dV2 = B.wino_i8_input_transform(xs.to(DEV))
    torch.cuda.synchronize()
    assert torch.equal(Vq1, Vq2) and torch.equal(dV2, dV1 * 16.0)


def test_i8_rejects_bad_arguments():
    x = torch.zeros(1, 16, 8, 8, dtype=torch.float16, device=DEV)
    w = torch.zeros(8, 16, 3, 3, dtype=torch.float16, device=DEV)
    u_q = B.wino_i8_filter_transform(w)
    y = torch.empty(1, 8, 8, 8, dtype=torch.float16, device=DEV)
    small = torch.empty(16, dtype=torch.uint8, device=DEV)
    with pytest.raises(B.WinoError) as e:
        B.wino_i8_conv2d(x, u_q, None, y, 8, small)
    assert e.value.status == B.WINO_ERR_WORKSPACE
    ws = torch.empty(B.wino_i8_workspace_bytes(1, 16, 8, 8, 8), dtype=torch.uint8, device=DEV)
    with pytest.raises(B.WinoError) as e:
        B.wino_i8_conv2d(x, u_q, None, y, 8, ws, layout=7)
    assert e.value.status == B.WINO_ERR_LAYOUT
    Uq, dU = B.i8_filter_views(u_q, 8, 16)
    Vq, dV = B.wino_i8_input_transform(x)
    with pytest.raises(B.WinoError) as e:
        B.wino_i8_batched_gemm(Uq, dU, Vq, dV, 8, 16, 16, block_shape=9)
    assert e.value.status == B.WINO_ERR_VARIANT
    torch.cuda.synchronize()
