"""Pins for the oracle's general convolution (R x R filter, stride, padding): CPU only."""
import numpy as np
import pytest
import torch

import oracle


@pytest.mark.parametrize("R,stride,pad", [(1, 1, 0), (3, 2, 1), (3, 1, 1), (1, 2, 0), (3, 2, 0), (5, 3, 2)])
def test_matches_library_routine(R, stride, pad):
    rng = np.random.default_rng(R * 10 + stride)
    N, C, K, H, W = 2, 5, 4, 9, 11
    x = rng.standard_normal((N, C, H, W)); w = rng.standard_normal((K, C, R, R)); b = rng.standard_normal(K)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x), torch.from_numpy(w), torch.from_numpy(b), stride=stride, padding=pad).numpy()
    y = oracle.conv2d_general(x, w, b, stride, pad)
    assert y.shape == ref.shape
    assert np.abs(y - ref).max() < 1e-12


def test_reduces_to_the_3x3_stride1_oracle_and_to_a_matrix_product():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((2, 6, 7, 5)); w = rng.standard_normal((4, 6, 3, 3)); b = rng.standard_normal(4)
    assert np.abs(oracle.conv2d_general(x, w, b, 1, 1) - oracle.conv2d_direct(x, w, b)).max() < 1e-13
    # 1x1: a matrix product over channels at every pixel
    w1 = rng.standard_normal((4, 6, 1, 1))
    y1 = oracle.conv2d_general(x, w1, b)
    assert np.abs(y1 - (np.einsum("kc,nchw->nkhw", w1[:, :, 0, 0], x) + b[None, :, None, None])).max() < 1e-13
    # stride 2 is stride 1 sub-sampled (same padding)
    y2 = oracle.conv2d_general(x, w, b, 2, 1)
    assert np.array_equal(y2, oracle.conv2d_general(x, w, b, 1, 1)[:, :, ::2, ::2])


def test_hand_case_stride2():
    # 4x4 ramp, one channel, filter that picks the tap above-left of the centre (r = s = 0): with pad 1
    # and stride 2, y[i][j] = xhat[2i - 1][2j - 1]
    x = np.arange(16, dtype=np.float64).reshape(1, 1, 4, 4)
    w = np.zeros((1, 1, 3, 3)); w[0, 0, 0, 0] = 1.0
    y = oracle.conv2d_general(x, w, None, 2, 1)[0, 0]
    assert np.array_equal(y, [[0.0, 0.0], [0.0, 5.0]])
    w[0, 0, 0, 0] = 0.0; w[0, 0, 2, 2] = 2.0          # below-right tap: y[i][j] = 2 * xhat[2i + 1][2j + 1]
    y = oracle.conv2d_general(x, w, np.array([0.5]), 2, 1)[0, 0]
    assert np.array_equal(y, [[10.5, 14.5], [26.5, 30.5]])


def test_output_size_and_argument_checks():
    x = np.zeros((1, 1, 5, 6)); w = np.zeros((1, 1, 3, 3))
    assert oracle.conv2d_general(x, w, None, 2, 1).shape == (1, 1, 3, 3)
    assert oracle.conv2d_general(x, w, None, 2, 0).shape == (1, 1, 2, 2)
    with pytest.raises(ValueError):
        oracle.conv2d_general(x, np.zeros((1, 2, 3, 3)))
