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


def test_eight_bit_transformed_operands_error_bands():
    """What 8-bit storage of the TRANSFORMED tensors U and V would cost the Winograd path (the model is exact when the
    operands are already representable, see the first assertion).  E4M3 with per-tensor power-of-two scales: about
    6e-2 for F(2x2) - 1.7x the error of quantising x and w themselves on the direct path - and 0.4 for F(4x4); scales
    per tile position change nothing for a floating-point format.  int8 with one linear scale per tile position:
    about 2.2e-2 for F(2x2), 0.13 for F(4x4).  These figures decide which 8-bit variants are worth building."""
    rng = np.random.default_rng(3)
    N, C, K, H, W = 1, 64, 16, 12, 12
    x = rng.standard_normal((N, C, H, W)); w = rng.standard_normal((K, C, 3, 3)) / np.sqrt(9 * C); b = 0.1 * rng.standard_normal(K)
    ref = oracle.conv2d_direct(x, w, b)
    # operands whose transforms are small multiples of 1/2 need at most four significant bits: exact in E4M3 with a
    # power-of-two scale, so the model then returns the exact convolution
    xi = rng.integers(-2, 3, (1, 3, 6, 6)).astype(np.float64); wi = 2.0 * rng.integers(-1, 2, (2, 3, 3, 3)).astype(np.float64)
    for pp in (False, True):
        assert np.abs(f8.conv2d_winograd_8bit(xi, wi, None, 2, "e4m3", pp) - oracle.conv2d_direct(xi, wi, None)).max() < 1e-9
    band = {(2, "e4m3", False): (4.5e-2, 8e-2), (2, "e4m3", True): (4.5e-2, 8e-2), (2, "int8", True): (1.5e-2, 3e-2),
            (2, "int8", False): (1.8e-2, 3.5e-2), (4, "e4m3", False): (0.25, 0.6), (4, "int8", True): (0.08, 0.2)}
    for (m, fmt, pp), (lo, hi) in band.items():
        err = oracle.rel_l2(f8.conv2d_winograd_8bit(x, w, b, m, fmt, pp), ref)
        assert lo <= err <= hi, (m, fmt, pp, err)
    direct = oracle.rel_l2(f8.conv2d_fp8(x, w, b, f8.power_of_two_scale(x), f8.power_of_two_scale(w)), ref)
    assert oracle.rel_l2(f8.conv2d_winograd_8bit(x, w, b, 2, "e4m3"), ref) > 1.4 * direct
