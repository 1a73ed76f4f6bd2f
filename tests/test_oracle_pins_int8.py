"""Pins for the oracle's model of the Winograd F(2x2) path with 8-bit integer U and V (CPU only)."""
from fractions import Fraction as Fr

import numpy as np
import torch

import oracle
from oracle import int8_model as i8
from oracle import winograd_ref as wr


def _half(a):
    return np.asarray(a, dtype=np.float64).astype(np.float16).astype(np.float64)


def _inputs(N, C, K, H, W, seed):
    rng = np.random.default_rng(seed)
    x = _half(rng.standard_normal((N, C, H, W)))
    w = _half(rng.standard_normal((K, C, 3, 3)) / np.sqrt(9 * C))
    b = rng.standard_normal(K) * 0.1
    return x, w, b


def test_one_input_channel_reduces_to_the_exact_convolution():
    """C = 1: every row of U and of V has a single entry, its code is +-127 and code * step gives the entry back (up to the
    fp32 rounding of the step), so the quantised result is the exact convolution - ragged image, several images and filters."""
    x, w, b = _inputs(2, 1, 3, 7, 9, seed=1)
    y = i8.conv2d_winograd_int8(x, w, b)
    ref = oracle.conv2d_direct(x, w, b)
    assert y.shape == ref.shape
    assert np.abs(y - ref).max() <= 4e-7 * np.abs(ref).max()
    Uq, dU = i8.filter_codes(w)
    assert set(np.unique(np.abs(Uq))) <= {0.0, 127.0}


def test_codes_against_exact_rational_arithmetic():
    """Small-integer data: every transform value is an exact small rational.  The codes are recomputed with Fractions
    (scaling by 127 / max, rounding half to even on the rational) and the product with Python integers."""
    rng = np.random.default_rng(2)
    N, C, K, H, W = 1, 5, 2, 4, 6
    x = rng.integers(-8, 9, (N, C, H, W)).astype(np.float64)
    w = rng.integers(-4, 5, (K, C, 3, 3)).astype(np.float64)
    at, g, bt = wr.exact_matrices(2)

    def rint_fr(v):                       # nearest integer, halves to even
        fl = v.numerator // v.denominator
        r = v - fl
        if r > Fr(1, 2) or (r == Fr(1, 2) and fl % 2 == 1):
            fl += 1
        return fl

    def mat(A, X, B):                     # A X B^T on nested lists of Fractions
        AX = [[sum(A[i][k] * X[k][j] for k in range(len(X))) for j in range(len(X[0]))] for i in range(len(A))]
        return [[sum(AX[i][k] * B[j][k] for k in range(len(B[0]))) for j in range(len(B))] for i in range(len(AX))]

    U = {(k, c): mat(g, [[Fr(int(v)) for v in row] for row in w[k, c]], g) for k in range(K) for c in range(C)}
    th, tw = 2, 3
    xp = np.zeros((C, 2 * th + 2, 2 * tw + 2)); xp[:, 1:H + 1, 1:W + 1] = x[0]
    V = {(c, t): mat(bt, [[Fr(int(v)) for v in row] for row in xp[c, 2 * (t // tw):2 * (t // tw) + 4, 2 * (t % tw):2 * (t % tw) + 4]], bt)
         for c in range(C) for t in range(th * tw)}
    Uq, dU = i8.filter_codes(w)
    Vq, dV = i8.activation_codes(x)
    M = i8.product(Uq, dU, Vq, dV)
    for xi in range(4):
        for nu in range(4):
            for k in range(K):
                mu = max(abs(U[(k, c)][xi][nu]) for c in range(C))
                uq = [rint_fr(U[(k, c)][xi][nu] * 127 / mu) if mu else 0 for c in range(C)]
                assert uq == [int(v) for v in Uq[xi, nu, k]], (xi, nu, k)
                assert dU[xi, nu, k] == float(np.float32(float(mu) / 127.0))
                for t in range(th * tw):
                    mv = max(abs(V[(c, t)][xi][nu]) for c in range(C))
                    # the activation side decides in fp32: its scale is the fp32 quotient, not the rational one
                    s = Fr(float(np.float32(127.0) / np.float32(float(mv)))) if mv else Fr(0)
                    vq = [rint_fr(Fr(float(np.float32(float(V[(c, t)][xi][nu] * s))))) for c in range(C)]
                    assert vq == [int(v) for v in Vq[xi, nu, :, t]], (xi, nu, t)
                    acc = sum(a * b for a, b in zip(uq, vq))
                    assert M[xi, nu, k, t] == acc * dU[xi, nu, k] * dV[xi, nu, t]


def test_rounding_rule_and_range():
    # one row with a maximum of 127: the scale is exactly 1, codes are rint of the values, halves go to the even neighbour
    row = np.array([127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.49, -126.5, 0.0])
    w = np.zeros((1, row.size, 3, 3)); w[0, :, 0, 0] = row          # U[0,0,k,c] = g[0][0]
    Uq, dU = i8.filter_codes(w)
    assert list(Uq[0, 0, 0]) == [127.0, 0.0, 2.0, 2.0, -0.0, -2.0, -2.0, 3.0, -126.0, 0.0]
    assert dU[0, 0, 0] == 1.0
    # an all-zero row: codes 0 and step 0, no division by zero
    assert np.all(Uq[3, 3] == 0) and np.all(dU[3, 3] == 0)
    # the activation side, centre position of one tile: V[1,1] = d11 + d12 + d21 + d22 of the window = the four pixels of a 2x2 image
    x = np.zeros((1, row.size, 2, 2)); x[0, :, 0, 0] = row
    Vq, dV = i8.activation_codes(x)
    assert list(Vq[1, 1, :, 0]) == [127.0, 0.0, 2.0, 2.0, -0.0, -2.0, -2.0, 3.0, -126.0, 0.0] and dV[1, 1, 0] == 1.0


def test_quantiser_against_library_fake_quantisation():
    """torch's per-channel fake quantisation (round(v / step) clamped to +-127, times step) on the same rows; it divides by
    the step where the definition multiplies by 127 / max, so single codes may differ by one at near-ties - nothing else may."""
    x, w, _ = _inputs(1, 96, 8, 8, 8, seed=3)
    V = i8.activation_transform_f32(x)                                # [4,4,C,T]
    Vq, dV = i8.activation_codes(x)
    rows = torch.tensor(V.transpose(0, 1, 3, 2).reshape(-1, V.shape[2]))          # one row per (xi, nu, t)
    step = torch.tensor(dV.reshape(-1), dtype=torch.float32)
    fq = torch.fake_quantize_per_channel_affine(rows, step, torch.zeros(len(step), dtype=torch.int32), 0, -127, 127)
    mine = (Vq * dV[:, :, None, :]).transpose(0, 1, 3, 2).reshape(-1, V.shape[2])
    diff = np.abs(fq.numpy().astype(np.float64) - mine) / step.numpy().astype(np.float64)[:, None]
    assert diff.max() <= 1.0 + 1e-6 and np.mean(diff > 1e-3) < 1e-3


def test_properties():
    x, w, b = _inputs(2, 40, 6, 9, 10, seed=4)
    Uq, dU = i8.filter_codes(w)
    Vq, dV = i8.activation_codes(x)
    U, V = wr.filter_transform(w, 2), wr.input_transform(x, 2)
    # the fp32 activation transform of 16-bit data is the exact transform but for the rare entry whose four terms span more
    # than 24 bits (then it is within one fp32 rounding of it)
    V32 = i8.activation_transform_f32(x).astype(np.float64)
    assert np.mean(V32 != V) < 1e-3 and np.all(np.abs(V32 - V) <= 2.0 ** -23 * np.abs(V).max())
    # codes are integers in [-127, 127], every non-zero row reaches 127, and code * step is within half a step of the value
    for q in (Uq, Vq):
        assert np.array_equal(q, np.rint(q)) and np.abs(q).max() == 127
    assert np.all(np.abs(Uq).max(axis=3) == 127) and np.all(np.abs(Vq).max(axis=2)[dV > 0] == 127)
    assert np.all(np.abs(Uq * dU[..., None] - U) <= 0.5 * dU[..., None] * (1 + 1e-6))
    assert np.all(np.abs(Vq * dV[:, :, None, :] - V) <= 0.5 * dV[:, :, None, :] * (1 + 1e-5))
    y, y0 = i8.conv2d_winograd_int8(x, w, b), i8.conv2d_winograd_int8(x, w, None)
    # the steps absorb a power of two exactly (no overflow or underflow here)
    assert np.array_equal(i8.conv2d_winograd_int8(4 * x, 0.5 * w, None), 2 * y0)
    # the order of the input channels does not matter (integer sums are exact)
    p = np.random.default_rng(0).permutation(x.shape[1])
    assert np.array_equal(i8.conv2d_winograd_int8(x[:, p], w[:, p], b), y)
    # with the codes replaced by the unrounded scaled values the three steps are the exact convolution
    M = wr.multiply(U, V)
    assert np.abs(wr.output_transform(M, b, 2, 9, 10, 2) - oracle.conv2d_direct(x, w, b)).max() < 1e-12
    # bias is added after everything else
    assert np.allclose(y - y0, b[None, :, None, None], rtol=0, atol=1e-12)


def test_error_band_against_the_exact_convolution():
    """Unit-variance data: relative L2 error 1.3e-2 ... 2.2e-2 (it falls slowly as rows get shorter); tolerance of the path 3e-2."""
    for (N, C, K, H, W), (lo, hi) in [((2, 320, 16, 16, 16), (1.4e-2, 2.1e-2)), ((1, 1280, 8, 8, 8), (1.6e-2, 2.3e-2)),
                                      ((1, 64, 16, 24, 20), (1.1e-2, 1.8e-2))]:
        x, w, b = _inputs(N, C, K, H, W, seed=5 + C)
        err = oracle.rel_l2(i8.conv2d_winograd_int8(x, w, b), oracle.conv2d_direct(x, w, b))
        assert lo <= err <= hi, ((N, C, K, H, W), err)
