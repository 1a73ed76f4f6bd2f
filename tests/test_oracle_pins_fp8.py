"""Pins for the oracle's 8-bit floating-point model (CPU only)."""
import numpy as np
import pytest
import torch

import oracle
from oracle import fp8_model as f8


def test_every_e4m3_value_is_a_fixed_point_and_there_are_253_of_them():
    # all byte patterns through the library's decoder: 256 patterns, two NaNs, +0 and -0 coincide
    vals = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).float().numpy().astype(np.float64)
    finite = vals[np.isfinite(vals)]
    assert len(finite) == 254 and len(np.unique(finite)) == 253
    assert np.array_equal(f8.round_to_e4m3(finite), finite)
    assert finite.max() == 448.0 and np.min(np.abs(finite[finite != 0])) == 2.0 ** -9


def test_matches_library_conversion():
    rng = np.random.default_rng(0)
    a = np.concatenate([rng.standard_normal(50000) * 10.0 ** rng.integers(-4, 3, 50000), np.linspace(-448, 448, 4001),
                        [0.0, 2.0 ** -10, 3 * 2.0 ** -10, 2.0 ** -9, 17.0, 19.0, 21.0, 447.9, 1e-9]])
    a = a[np.abs(a) <= 448.0].astype(np.float32).astype(np.float64)
    ref = torch.tensor(a, dtype=torch.float32).to(torch.float8_e4m3fn).float().numpy().astype(np.float64)
    assert np.array_equal(f8.round_to_e4m3(a), ref)


def test_hand_cases():
    # binade [16, 32): spacing 2 -> 17 is a tie between 16 and 18 (even mantissa: 16), 19 a tie between 18 and 20 (20)
    assert list(f8.round_to_e4m3([17.0, 19.0, 21.0, 1.0625, 0.3])) == [16.0, 20.0, 20.0, 1.0, 0.3125]
    assert list(f8.round_to_e4m3([1000.0, -1e6, 2.0 ** -10, 3 * 2.0 ** -10])) == [448.0, -448.0, 0.0, 2.0 ** -8]   # saturation; subnormal ties
    assert f8.power_of_two_scale([0.02, -0.03]) == 8192.0 and f8.power_of_two_scale([0.0]) == 1.0
    assert f8.power_of_two_scale([448.0]) == 1.0 and f8.power_of_two_scale([449.0]) == 0.5


def test_quantised_convolution_properties_and_error_band():
    rng = np.random.default_rng(1)
    N, C, K, H, W = 1, 64, 8, 10, 12
    x = rng.standard_normal((N, C, H, W)); w = rng.standard_normal((K, C, 3, 3)) / np.sqrt(9 * C); b = rng.standard_normal(K)
    sx, sw = f8.power_of_two_scale(x), f8.power_of_two_scale(w)
    y = f8.conv2d_fp8(x, w, b, sx, sw)
    # operands that are already E4M3 numbers (after scaling) pass through unchanged: the model is then the exact convolution
    xq, wq = f8.round_to_e4m3(x * sx) / sx, f8.round_to_e4m3(w * sw) / sw
    assert np.abs(f8.conv2d_fp8(xq, wq, b, sx, sw) - oracle.conv2d_general(xq, wq, b)).max() < 1e-12
    assert np.abs(y - oracle.conv2d_general(xq, wq, b)).max() < 1e-12
    # a power of two moved between a tensor and its scale changes nothing: conv(4x; sx/4) = 4 conv(x; sx), exactly
    assert np.array_equal(f8.conv2d_fp8(4 * x, w, None, sx / 4, sw), 4 * f8.conv2d_fp8(x, w, None, sx, sw))
    # error against the unquantised convolution: about 3.8e-2 (two roundings of 3 mantissa bits per product)
    err = oracle.rel_l2(y - b[None, :, None, None], oracle.conv2d_general(x, w, None))
    assert 3.0e-2 <= err <= 4.5e-2, err
    # stride 2 and 1x1 go through the same definition
    w1 = rng.standard_normal((K, C, 1, 1)) / np.sqrt(C)
    s1 = f8.power_of_two_scale(w1)
    y1 = f8.conv2d_fp8(x, w1, None, sx, s1)
    assert np.abs(y1 - np.einsum("kc,nchw->nkhw", f8.round_to_e4m3(w1[:, :, 0, 0] * s1) / s1, xq)).max() < 1e-12
    assert np.array_equal(f8.conv2d_fp8(x, w, b, sx, sw, stride=2), y[:, :, ::2, ::2])
