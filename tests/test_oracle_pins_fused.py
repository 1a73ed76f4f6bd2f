"""Pins for the oracle's GroupNorm / SiLU / fused-convolution functions (CPU only)."""
import numpy as np
import pytest
import torch

import oracle
from oracle import fused_ops as fo


def test_groupnorm_matches_library_routine():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((2, 12, 5, 7)); g = rng.standard_normal(12); b = rng.standard_normal(12)
    ref = torch.nn.functional.group_norm(torch.from_numpy(x), 4, torch.from_numpy(g), torch.from_numpy(b), eps=1e-5).numpy()
    assert np.abs(fo.groupnorm(x, g, b, 4, 1e-5) - ref).max() < 1e-12
    ref_s = torch.nn.functional.silu(torch.from_numpy(ref)).numpy()
    assert np.abs(fo.silu(ref) - ref_s).max() < 1e-13


def test_groupnorm_hand_case():
    # one group holding the values {1, 3}: mean 2, biased variance 1 -> +-1/sqrt(1+eps), then *2 + 0.5
    x = np.array([1.0, 3.0]).reshape(1, 2, 1, 1)
    v = fo.groupnorm(x, [2.0, 2.0], [0.5, 0.5], groups=1, eps=0.25)
    s = 1.0 / np.sqrt(1.25)
    assert np.allclose(v.ravel(), [0.5 - 2 * s, 0.5 + 2 * s], atol=1e-15)
    mean, rstd = fo.groupnorm_stats(x, 1, eps=0.25)
    assert mean[0, 0] == 2.0 and abs(rstd[0, 0] - s) < 1e-15


def test_groupnorm_closed_forms_and_invariants():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((3, 8, 6, 6))
    v = fo.groupnorm(x, np.ones(8), np.zeros(8), groups=2, eps=0.0)
    vg = v.reshape(3, 2, -1)
    assert np.abs(vg.mean(axis=2)).max() < 1e-14 and np.abs(vg.var(axis=2) - 1).max() < 1e-13
    # affine input changes nothing (eps = 0): GN(a*x + b) = GN(x) for a > 0
    assert np.abs(fo.groupnorm(3.5 * x - 2.0, np.ones(8), np.zeros(8), 2, 0.0) - v).max() < 1e-12
    # a constant group normalises to zero, so only beta survives
    c = np.full((1, 4, 3, 3), 7.0)
    beta = np.array([0.1, -0.2, 0.3, 0.0])
    assert np.allclose(fo.groupnorm(c, np.ones(4), beta, 2, 1e-5), beta.reshape(1, 4, 1, 1))
    # groups are independent: changing group 1 leaves group 0 untouched
    x2 = x.copy(); x2[:, 4:] *= 9.0
    assert np.array_equal(fo.groupnorm(x2, np.ones(8), np.zeros(8), 2, 1e-5)[:, :4], fo.groupnorm(x, np.ones(8), np.zeros(8), 2, 1e-5)[:, :4])


def test_silu_closed_forms():
    v = np.linspace(-6, 6, 25)
    assert fo.silu(0.0) == 0.0
    assert np.allclose(fo.silu(v) - fo.silu(-v), v, atol=1e-15)      # s(v) - s(-v) = v
    assert abs(fo.silu(1.0) - 1.0 / (1.0 + np.exp(-1.0))) < 1e-16
    assert np.all(fo.silu(v) >= -0.2785)                                 # global minimum of SiLU


def test_fused_conv_reduces_to_its_parts():
    rng = np.random.default_rng(2)
    N, C, K, H, W = 2, 8, 5, 6, 7
    x = rng.standard_normal((N, C, H, W)); w = rng.standard_normal((K, C, 3, 3)); b = rng.standard_normal(K)
    g = rng.standard_normal(C); be = rng.standard_normal(C)
    add = rng.standard_normal((N, K)); res = rng.standard_normal((N, K, H, W))
    plain = oracle.conv2d_direct(x, w, b)
    assert np.array_equal(fo.conv2d_fused(x, w, b), plain)
    assert np.allclose(fo.conv2d_fused(x, w, b, addvec=add, residual=res), plain + add[:, :, None, None] + res, atol=1e-14)
    a = torch.nn.functional.silu(torch.nn.functional.group_norm(torch.from_numpy(x), 4, torch.from_numpy(g), torch.from_numpy(be), eps=1e-5))
    ref = torch.nn.functional.conv2d(a, torch.from_numpy(w), torch.from_numpy(b), padding=1).numpy()
    assert np.abs(fo.conv2d_fused(x, w, b, g, be, groups=4) - ref).max() < 1e-12
    # padding is applied AFTER the activation: with beta != 0 the border differs from activating a padded image
    big = np.zeros((N, C, H + 2, W + 2)); big[:, :, 1:-1, 1:-1] = x
    wrong = fo.silu(fo.groupnorm(big, g, be, 4))
    assert not np.allclose(oracle.conv2d_direct(wrong, w, b)[:, :, 1:-1, 1:-1], fo.conv2d_fused(x, w, b, g, be, groups=4))


def test_upsample_matches_library_routine_and_hand_case():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((2, 3, 4, 5))
    ref = torch.nn.functional.interpolate(torch.from_numpy(x), scale_factor=2, mode="nearest").numpy()
    u = fo.upsample_nearest2x(x)
    assert u.shape == (2, 3, 8, 10) and np.array_equal(u, ref)
    h = fo.upsample_nearest2x(np.array([[1.0, 2.0], [3.0, 4.0]]).reshape(1, 1, 2, 2))[0, 0]
    assert np.array_equal(h, [[1, 1, 2, 2], [1, 1, 2, 2], [3, 3, 4, 4], [3, 3, 4, 4]])
    # every 2x2 block is constant and sub-sampling undoes it
    assert np.array_equal(u[:, :, ::2, ::2], x) and np.array_equal(u[:, :, 1::2, 1::2], x)


def test_fused_upsample_conv_properties():
    rng = np.random.default_rng(6)
    N, C, K, H, W = 1, 3, 2, 4, 3
    x = rng.standard_normal((N, C, H, W)); w = rng.standard_normal((K, C, 3, 3)); b = rng.standard_normal(K)
    y = fo.conv2d_fused(x, w, b, upsample=True)
    assert y.shape == (N, K, 2 * H, 2 * W)
    # the same thing through the library: interpolate, then conv2d
    xu = torch.nn.functional.interpolate(torch.from_numpy(x), scale_factor=2, mode="nearest")
    ref = torch.nn.functional.conv2d(xu, torch.from_numpy(w), torch.from_numpy(b), padding=1).numpy()
    assert np.abs(y - ref).max() < 1e-12
    # an interior output of a constant image sees nine equal taps: y = c * sum(w) + b
    c = np.full((1, C, H, W), 0.5)
    yc = fo.conv2d_fused(c, w, b, upsample=True)
    assert np.allclose(yc[0, :, 3, 2], 0.5 * w.sum(axis=(1, 2, 3)) + b, atol=1e-13)
    # GroupNorm statistics do not change under upsampling, and the point-wise steps commute with it
    g = rng.standard_normal(C); be = rng.standard_normal(C)
    a = fo.conv2d_fused(x, w, b, g, be, groups=1, upsample=True)
    bb = fo.conv2d_fused(fo.upsample_nearest2x(x), w, b, g, be, groups=1)
    assert np.abs(a - bb).max() < 1e-12
