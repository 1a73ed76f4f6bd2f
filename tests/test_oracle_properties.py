"""Property tests of the oracles over random shapes (hypothesis, CPU only): identities that hold for any input and that a
dropped term, a wrong sign or index, or a transposed operand would break."""
import numpy as np
from hypothesis import given, settings, strategies as st

import oracle
from oracle import fp8_model as f8
from oracle import fused_ops as fo
from oracle import winograd_ref as wr

dims = st.tuples(st.integers(1, 2), st.integers(1, 5), st.integers(1, 4), st.integers(1, 9), st.integers(1, 9))


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


@settings(max_examples=25, deadline=None)
@given(dims, st.integers(0, 10 ** 6))
def test_direct_conv_is_bilinear_and_matches_the_general_oracle(d, seed):
    N, C, K, H, W = d
    x, x2 = _rand((N, C, H, W), seed), _rand((N, C, H, W), seed + 1)
    w, w2 = _rand((K, C, 3, 3), seed + 2), _rand((K, C, 3, 3), seed + 3)
    b = _rand((K,), seed + 4)
    y = oracle.conv2d_direct(x, w, None)
    assert np.allclose(oracle.conv2d_direct(2 * x - 3 * x2, w, None), 2 * y - 3 * oracle.conv2d_direct(x2, w, None), atol=1e-10)
    assert np.allclose(oracle.conv2d_direct(x, w + w2, None), y + oracle.conv2d_direct(x, w2, None), atol=1e-10)
    assert np.allclose(oracle.conv2d_direct(x, w, b), y + b[None, :, None, None], atol=1e-12)
    assert np.allclose(oracle.conv2d_general(x, w, b, 1, 1), oracle.conv2d_direct(x, w, b), atol=1e-12)
    # flipping image and filter together flips the output (cross-correlation, symmetric padding)
    assert np.allclose(oracle.conv2d_direct(x[:, :, ::-1, ::-1], w[:, :, ::-1, ::-1], None), y[:, :, ::-1, ::-1], atol=1e-12)
    # transposing both spatial axes of image and filter transposes the output
    assert np.allclose(oracle.conv2d_direct(x.transpose(0, 1, 3, 2), w.transpose(0, 1, 3, 2), None), y.transpose(0, 1, 3, 2), atol=1e-12)


@settings(max_examples=20, deadline=None)
@given(dims, st.sampled_from([2, 4]), st.integers(0, 10 ** 6))
def test_winograd_reference_equals_the_definition(d, m, seed):
    N, C, K, H, W = d
    x, w, b = _rand((N, C, H, W), seed), _rand((K, C, 3, 3), seed + 1), _rand((K,), seed + 2)
    ref = oracle.conv2d_direct(x, w, b)
    y = wr.conv2d_winograd(x, w, b, m)
    assert np.abs(y - ref).max() <= 1e-10 * max(1.0, np.abs(ref).max())


@settings(max_examples=20, deadline=None)
@given(dims, st.sampled_from([(1, 1), (3, 1), (3, 2), (1, 2)]), st.integers(0, 10 ** 6))
def test_general_conv_sampled_definition(d, rs, seed):
    """Every output element against the defining sum written inline."""
    N, C, K, H, W = d
    R, stride = rs
    pad = (R - 1) // 2
    x, w = _rand((N, C, H, W), seed), _rand((K, C, R, R), seed + 1)
    y = oracle.conv2d_general(x, w, None, stride)
    xp = np.pad(x, ((0, 0), (0, 0), (pad, pad), (pad, pad)))
    Ho, Wo = y.shape[2], y.shape[3]
    assert Ho == (H + 2 * pad - R) // stride + 1 and Wo == (W + 2 * pad - R) // stride + 1
    rng = np.random.default_rng(seed)
    for _ in range(8):
        n, k, i, j = rng.integers(N), rng.integers(K), rng.integers(Ho), rng.integers(Wo)
        want = np.sum(xp[n, :, i * stride:i * stride + R, j * stride:j * stride + R] * w[k])
        assert abs(y[n, k, i, j] - want) <= 1e-10 * max(1.0, abs(want))


@settings(max_examples=15, deadline=None)
@given(st.tuples(st.integers(1, 2), st.sampled_from([2, 4, 6]), st.integers(1, 3), st.integers(1, 6), st.integers(1, 6)), st.integers(0, 10 ** 6))
def test_fused_oracle_pieces(d, seed):
    N, C, K, H, W = d
    x, w, b = _rand((N, C, H, W), seed) * 2 + 0.5, _rand((K, C, 3, 3), seed + 1), _rand((K,), seed + 2)
    gamma, beta = _rand((C,), seed + 3), _rand((C,), seed + 4)
    G = 2 if C % 2 == 0 else 1
    a = fo.silu(fo.groupnorm(x, gamma, beta, G, 1e-5))
    assert np.allclose(fo.conv2d_fused(x, w, b, gamma, beta, G, 1e-5), oracle.conv2d_direct(a, w, b), atol=1e-12)
    # statistics: mean / rstd reproduce the normalised tensor
    mean, rstd = fo.groupnorm_stats(x, G, 1e-5)
    xn = (x.reshape(N, G, -1) - mean[:, :, None]) * rstd[:, :, None]
    assert np.allclose(xn.reshape(N, C, H, W) * gamma[None, :, None, None] + beta[None, :, None, None], fo.groupnorm(x, gamma, beta, G, 1e-5), atol=1e-10)
    # upsampling then convolving = convolving the explicitly repeated tensor
    xu = np.repeat(np.repeat(x, 2, axis=2), 2, axis=3)
    assert np.array_equal(fo.upsample_nearest2x(x), xu)
    assert np.allclose(fo.conv2d_fused(x, w, b, upsample=True), oracle.conv2d_direct(xu, w, b), atol=1e-12)


@settings(max_examples=30, deadline=None)
@given(st.lists(st.floats(-500, 500, allow_nan=False), min_size=1, max_size=64))
def test_e4m3_rounding_is_nearest_monotone_and_idempotent(vals):
    a = np.array(vals, dtype=np.float64)
    q = f8.round_to_e4m3(a)
    assert np.array_equal(f8.round_to_e4m3(q), q)                       # idempotent
    order = np.argsort(a)
    assert np.all(np.diff(q[order]) >= 0)                               # monotone
    inside = np.abs(a) <= 448
    # nearest: no representable neighbour (one step up or down) is closer
    e = np.maximum(np.floor(np.log2(np.maximum(np.abs(q), 2.0 ** -9))), -6.0)
    step = 2.0 ** (e - 3)
    assert np.all(np.abs(a - q)[inside] <= step[inside] / 2 + 1e-12)
    assert np.all(np.abs(q) <= 448)
