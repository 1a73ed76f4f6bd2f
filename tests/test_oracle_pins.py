"""Pins for the oracle: things the mathematics fixes, none of them the oracle itself.

Operator: 3x3, stride 1, zero-pad 1 cross-correlation (the convolution operator of the
paper's Section "Techniques"; shapes per Table 1's header) and the three Winograd steps
named there.  CPU only.
"""
import itertools
import os
from fractions import Fraction as Fr

import numpy as np
import pytest
import torch

import oracle
from oracle import winograd_ref as wr


# ----------------------------------------------------------------------------------------
# helpers that are NOT the oracle: pure-Python exact arithmetic, element by element
# ----------------------------------------------------------------------------------------
def brute_conv(x, w, b):
    """Seven nested loops over Python ints/Fractions; x[N][C][H][W], w[K][C][3][3]."""
    N, C, H, W = len(x), len(x[0]), len(x[0][0]), len(x[0][0][0])
    K = len(w)
    y = [[[[Fr(b[k]) for _ in range(W)] for _ in range(H)] for k in range(K)] for _ in range(N)]
    for n in range(N):
        for k in range(K):
            for i in range(H):
                for j in range(W):
                    for c in range(C):
                        for r in range(3):
                            for s in range(3):
                                ii, jj = i + r - 1, j + s - 1
                                if 0 <= ii < H and 0 <= jj < W:
                                    y[n][k][i][j] += Fr(x[n][c][ii][jj]) * Fr(w[k][c][r][s])
    return y


def matmul(A, B):
    return [[sum(A[i][k] * B[k][j] for k in range(len(B))) for j in range(len(B[0]))] for i in range(len(A))]


def transpose(A):
    return [list(r) for r in zip(*A)]


def hadamard(A, B):
    return [[a * b for a, b in zip(ra, rb)] for ra, rb in zip(A, B)]


def rand_fr(rng, shape):
    if len(shape) == 1:
        return [Fr(int(rng.integers(-9, 10)), int(rng.integers(1, 7))) for _ in range(shape[0])]
    return [rand_fr(rng, shape[1:]) for _ in range(shape[0])]


def to_np(a):
    return np.array(a, dtype=object).astype(np.float64)


# ----------------------------------------------------------------------------------------
# p1: hand-computed cases
# ----------------------------------------------------------------------------------------
def test_hand_ones_3x3_counts_in_bounds_taps():
    y = oracle.conv2d_direct(np.ones((1, 1, 3, 3)), np.ones((1, 1, 3, 3)), np.zeros(1))
    assert np.array_equal(y[0, 0], np.array([[4, 6, 4], [6, 9, 6], [4, 6, 4]], dtype=np.float64))


def test_hand_1x1_image_uses_centre_tap_only():
    w = np.arange(1, 10, dtype=np.float64).reshape(1, 1, 3, 3)
    y = oracle.conv2d_direct(np.full((1, 1, 1, 1), 3.0), w, np.array([0.5]))
    assert y.shape == (1, 1, 1, 1) and y[0, 0, 0, 0] == 3.0 * 5.0 + 0.5


def test_hand_worked_case_from_golden_file(golden_dir):
    vals = {}
    with open(os.path.join(golden_dir, "hand_case_c2_k2_2x2.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            key, *nums = line.split()
            vals[key] = np.array([float(v) for v in nums])
    x = vals["x"].reshape(1, 2, 2, 2)
    w = vals["w"].reshape(2, 2, 3, 3)
    y = oracle.conv2d_direct(x, w, vals["bias"])
    assert np.array_equal(y.ravel(), vals["y"])
    assert np.array_equal(oracle.conv2d_direct_at(x, w, vals["bias"], np.arange(8)), vals["y"])


# ----------------------------------------------------------------------------------------
# p2: exact brute force on small integer inputs (fp64 is exact there)
# ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("N,C,K,H,W", [(1, 1, 1, 1, 1), (1, 2, 3, 2, 5), (2, 3, 2, 4, 3), (2, 1, 3, 6, 6), (1, 3, 1, 5, 1)])
def test_brute_force_exact(N, C, K, H, W):
    rng = np.random.default_rng(N * 1000 + C * 100 + K * 10 + H + W)
    x = rng.integers(-8, 9, size=(N, C, H, W))
    w = rng.integers(-8, 9, size=(K, C, 3, 3))
    b = rng.integers(-8, 9, size=(K,))
    ref = to_np(brute_conv(x.tolist(), w.tolist(), b.tolist()))
    y = oracle.conv2d_direct(x, w, b)
    assert np.array_equal(y, ref)
    idx = np.arange(y.size)[::-1].copy()
    assert np.array_equal(oracle.conv2d_direct_at(x, w, b, idx), ref.ravel()[idx])


# ----------------------------------------------------------------------------------------
# p3/p4: delta filters (identity and shifts) — catch flips, pad side, transposed r/s
# ----------------------------------------------------------------------------------------
def _delta_w(C, r, s):
    w = np.zeros((C, C, 3, 3))
    for c in range(C):
        w[c, c, r, s] = 1.0
    return w


def test_delta_centre_is_identity_plus_bias():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((2, 3, 5, 7))
    b = rng.standard_normal(3)
    y = oracle.conv2d_direct(x, _delta_w(3, 1, 1), b)
    assert np.array_equal(y, x + b.reshape(1, 3, 1, 1))


@pytest.mark.parametrize("r,s", list(itertools.product(range(3), range(3))))
def test_shifted_delta(r, s):
    rng = np.random.default_rng(10 + 3 * r + s)
    x = rng.standard_normal((1, 2, 6, 5))
    y = oracle.conv2d_direct(x, _delta_w(2, r, s), None)
    # y[i,j] = xhat[i+r-1, j+s-1]
    exp = np.zeros_like(x)
    H, W = 6, 5
    for i in range(H):
        for j in range(W):
            ii, jj = i + r - 1, j + s - 1
            if 0 <= ii < H and 0 <= jj < W:
                exp[:, :, i, j] = x[:, :, ii, jj]
    assert np.array_equal(y, exp)
    sel = np.arange(0, y.size, 3)
    assert np.array_equal(oracle.conv2d_direct_at(x, _delta_w(2, r, s), None, sel), exp.ravel()[sel])


# ----------------------------------------------------------------------------------------
# p5: linearity in x and in w
# ----------------------------------------------------------------------------------------
def test_linearity():
    rng = np.random.default_rng(5)
    x1, x2 = rng.standard_normal((2, 2, 3, 6, 7))
    w1, w2 = rng.standard_normal((2, 4, 3, 3, 3))
    a = 1.75
    f = lambda x, w: oracle.conv2d_direct(x, w, None)
    assert np.allclose(f(a * x1 + x2, w1), a * f(x1, w1) + f(x2, w1), rtol=0, atol=1e-13)
    assert np.allclose(f(x1, a * w1 + w2), a * f(x1, w1) + f(x1, w2), rtol=0, atol=1e-13)
    b = rng.standard_normal(4)
    assert np.allclose(oracle.conv2d_direct(x1, w1, b) - f(x1, w1), b.reshape(1, 4, 1, 1), atol=1e-14)


# ----------------------------------------------------------------------------------------
# p6: zero-padding boundary invariant
# ----------------------------------------------------------------------------------------
def test_zero_canvas_embedding():
    rng = np.random.default_rng(6)
    N, C, K, H, W = 2, 3, 2, 4, 5
    x = rng.integers(-5, 6, size=(N, C, H, W)).astype(np.float64)
    w = rng.integers(-5, 6, size=(K, C, 3, 3)).astype(np.float64)
    small = oracle.conv2d_direct(x, w, None)
    big_x = np.zeros((N, C, H + 2, W + 2))
    big_x[:, :, 1:-1, 1:-1] = x
    big = oracle.conv2d_direct(big_x, w, None)
    assert np.array_equal(big[:, :, 1:-1, 1:-1], small)
    # the ring is the partial sum of the taps that still reach the image: top-left corner of
    # the canvas sees only x[0,0] through tap (2,2)
    exp_corner = np.einsum("nc,kc->nk", x[:, :, 0, 0], w[:, :, 2, 2])
    assert np.array_equal(big[:, :, 0, 0], exp_corner)
    exp_bottom_right = np.einsum("nc,kc->nk", x[:, :, -1, -1], w[:, :, 0, 0])
    assert np.array_equal(big[:, :, -1, -1], exp_bottom_right)


# ----------------------------------------------------------------------------------------
# p7: constant input closed form
# ----------------------------------------------------------------------------------------
def test_constant_input_closed_form():
    rng = np.random.default_rng(7)
    C, K, H, W = 3, 2, 5, 6
    w = rng.integers(-4, 5, size=(K, C, 3, 3)).astype(np.float64)
    b = rng.integers(-4, 5, size=(K,)).astype(np.float64)
    y = oracle.conv2d_direct(np.ones((1, C, H, W)), w, b)
    ws = w.sum(axis=1)  # [K,3,3]
    for k in range(K):
        assert y[0, k, 2, 2] == b[k] + ws[k].sum()                       # interior
        assert y[0, k, 0, 2] == b[k] + ws[k, 1:, :].sum()                # top edge drops filter row 0
        assert y[0, k, H - 1, 3] == b[k] + ws[k, :2, :].sum()            # bottom edge drops row 2
        assert y[0, k, 2, 0] == b[k] + ws[k, :, 1:].sum()                # left edge drops col 0
        assert y[0, k, 2, W - 1] == b[k] + ws[k, :, :2].sum()            # right edge drops col 2
        assert y[0, k, 0, 0] == b[k] + ws[k, 1:, 1:].sum()               # corner
        assert y[0, k, H - 1, W - 1] == b[k] + ws[k, :2, :2].sum()


# ----------------------------------------------------------------------------------------
# p8: batch independence, channel permutation, translation equivariance
# ----------------------------------------------------------------------------------------
def test_structural_invariants():
    rng = np.random.default_rng(8)
    x = rng.standard_normal((3, 4, 7, 6))
    w = rng.standard_normal((5, 4, 3, 3))
    b = rng.standard_normal(5)
    y = oracle.conv2d_direct(x, w, b)
    for n in range(3):
        assert np.array_equal(oracle.conv2d_direct(x[n:n + 1], w, b)[0], y[n])
    perm = np.array([2, 0, 3, 1])
    assert np.allclose(oracle.conv2d_direct(x[:, perm], w[:, perm], b), y, atol=1e-13)
    kperm = np.array([4, 2, 0, 1, 3])
    assert np.array_equal(oracle.conv2d_direct(x, w[kperm], b[kperm]), y[:, kperm])
    # shift the image content down-right by (1,2) inside a larger zero canvas: interior shifts along
    canvas = np.zeros((3, 4, 12, 12)); canvas[:, :, 2:9, 2:8] = x
    shifted = np.zeros_like(canvas); shifted[:, :, 3:10, 4:10] = x
    yc = oracle.conv2d_direct(canvas, w, None)
    ys = oracle.conv2d_direct(shifted, w, None)
    assert np.array_equal(ys[:, :, 2:11, 3:11], yc[:, :, 1:10, 1:9])


# ----------------------------------------------------------------------------------------
# p9: reduces to a library routine
# ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("N,C,K,H,W", [(1, 4, 8, 9, 13), (2, 5, 7, 17, 3), (3, 1, 1, 1, 30), (1, 16, 12, 33, 32)])
def test_against_torch_conv2d(N, C, K, H, W):
    rng = np.random.default_rng(9 + H)
    x = rng.standard_normal((N, C, H, W)); w = rng.standard_normal((K, C, 3, 3)); b = rng.standard_normal(K)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x), torch.from_numpy(w), torch.from_numpy(b), padding=1).numpy()
    y = oracle.conv2d_direct(x, w, b)
    assert np.abs(y - ref).max() < 1e-12
    sel = rng.integers(0, y.size, size=64)
    assert np.abs(oracle.conv2d_direct_at(x, w, b, sel) - ref.ravel()[sel]).max() < 1e-12


def test_promotes_fp16_inputs_exactly():
    rng = np.random.default_rng(11)
    x = rng.standard_normal((1, 3, 4, 4)).astype(np.float16)
    w = rng.standard_normal((2, 3, 3, 3)).astype(np.float16)
    assert np.array_equal(oracle.conv2d_direct(x, w, None),
                          oracle.conv2d_direct(x.astype(np.float64), w.astype(np.float64), None))


# ----------------------------------------------------------------------------------------
# p10: exact-rational Winograd identity — pins the (A,G,B) triples and the tiling rule
# ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("m", [2, 4])
def test_rational_identity_one_tile(m):
    AT, G, BT = wr.exact_matrices(m)
    al = m + 2
    assert len(AT) == m and len(AT[0]) == al and len(G) == al and len(G[0]) == 3 and len(BT) == al
    rng = np.random.default_rng(100 + m)
    for _ in range(20):
        d = rand_fr(rng, (al, al))
        g = rand_fr(rng, (3, 3))
        U = matmul(matmul(G, g), transpose(G))
        V = matmul(matmul(BT, d), transpose(BT))
        Y = matmul(matmul(AT, hadamard(U, V)), transpose(AT))
        for a in range(m):
            for b in range(m):
                direct = sum(d[a + r][b + s] * g[r][s] for r in range(3) for s in range(3))
                assert Y[a][b] == direct


def rational_winograd_image(x, w, bias, m):
    """Whole-image Winograd in Fractions, element loops only (no numpy, no oracle code)."""
    AT, G, BT = wr.exact_matrices(m)
    al = m + 2
    N, C, H, W = len(x), len(x[0]), len(x[0][0]), len(x[0][0][0])
    K = len(w)
    th, tw = -(-H // m), -(-W // m)
    y = [[[[None] * W for _ in range(H)] for _ in range(K)] for _ in range(N)]
    xhat = lambda n, c, i, j: Fr(x[n][c][i][j]) if (0 <= i < H and 0 <= j < W) else Fr(0)
    for n in range(N):
        for ti in range(th):
            for tj in range(tw):
                for k in range(K):
                    Msum = [[Fr(0)] * al for _ in range(al)]
                    for c in range(C):
                        d = [[xhat(n, c, m * ti - 1 + a, m * tj - 1 + b) for b in range(al)] for a in range(al)]
                        g = [[Fr(v) for v in row] for row in w[k][c]]
                        U = matmul(matmul(G, g), transpose(G))
                        V = matmul(matmul(BT, d), transpose(BT))
                        UV = hadamard(U, V)
                        Msum = [[p + q for p, q in zip(r1, r2)] for r1, r2 in zip(Msum, UV)]
                    Y = matmul(matmul(AT, Msum), transpose(AT))
                    for a in range(m):
                        for b in range(m):
                            i, j = m * ti + a, m * tj + b
                            if i < H and j < W:
                                y[n][k][i][j] = Y[a][b] + Fr(bias[k])
    return y


@pytest.mark.parametrize("m,H,W", [(2, 3, 5), (2, 4, 4), (4, 5, 7), (4, 4, 8), (4, 1, 2), (2, 1, 1)])
def test_rational_winograd_whole_image_matches_brute_force(m, H, W):
    rng = np.random.default_rng(200 + m + H * 10 + W)
    N, C, K = 2, 2, 2
    x = rng.integers(-6, 7, size=(N, C, H, W)).tolist()
    w = rng.integers(-6, 7, size=(K, C, 3, 3)).tolist()
    b = rng.integers(-6, 7, size=(K,)).tolist()
    assert rational_winograd_image(x, w, b, m) == brute_conv(x, w, b)


# ----------------------------------------------------------------------------------------
# the fp64 Winograd stage reference: each stage against element-wise exact arithmetic, and
# the pipeline against the direct definition
# ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("m", [2, 4])
def test_winograd_ref_stages_elementwise(m):
    AT, G, BT = wr.exact_matrices(m)
    al = m + 2
    rng = np.random.default_rng(300 + m)
    N, C, K, H, W = 2, 2, 3, 2 * m + 1, m + 3          # ragged in both directions
    x = rng.integers(-6, 7, size=(N, C, H, W))
    w = rng.integers(-6, 7, size=(K, C, 3, 3))
    th, tw = -(-H // m), -(-W // m)
    T = N * th * tw
    U = wr.filter_transform(w, m)
    V = wr.input_transform(x, m)
    assert U.shape == (al, al, K, C) and V.shape == (al, al, C, T)
    xhat = lambda n, c, i, j: Fr(int(x[n, c, i, j])) if (0 <= i < H and 0 <= j < W) else Fr(0)
    for k in range(K):
        for c in range(C):
            for xi in range(al):
                for nu in range(al):
                    e = sum(G[xi][r] * int(w[k, c, r, s]) * G[nu][s] for r in range(3) for s in range(3))
                    assert abs(U[xi, nu, k, c] - float(e)) < 1e-12
    for n in range(N):
        for ti in range(th):
            for tj in range(tw):
                t = (n * th + ti) * tw + tj
                for c in range(C):
                    for xi in range(al):
                        for nu in range(al):
                            e = sum(BT[xi][a] * xhat(n, c, m * ti - 1 + a, m * tj - 1 + b) * BT[nu][b]
                                    for a in range(al) for b in range(al))
                            assert V[xi, nu, c, t] == float(e)        # integer-valued: exact
    M = wr.multiply(U, V)
    assert M.shape == (al, al, K, T)
    e = sum(U[1, 2, 1, c] * V[1, 2, c, 3] for c in range(C))
    assert abs(M[1, 2, 1, 3] - e) < 1e-12
    # output transform, element by element, on an integer-valued M
    Mi = rng.integers(-5, 6, size=(al, al, K, T)).astype(np.float64)
    bias = rng.integers(-5, 6, size=(K,)).astype(np.float64)
    y = wr.output_transform(Mi, bias, N, H, W, m)
    assert y.shape == (N, K, H, W)
    for n in range(N):
        for k in range(K):
            for i in range(H):
                for j in range(W):
                    ti, a, tj, b = i // m, i % m, j // m, j % m
                    t = (n * th + ti) * tw + tj
                    e = sum(AT[a][xi] * int(Mi[xi, nu, k, t]) * AT[b][nu] for xi in range(al) for nu in range(al))
                    assert y[n, k, i, j] == float(e) + bias[k]


@pytest.mark.parametrize("m", [2, 4])
@pytest.mark.parametrize("N,C,K,H,W", [(1, 3, 2, 8, 8), (2, 5, 7, 9, 13), (1, 2, 3, 1, 1), (1, 4, 4, 3, 30)])
def test_winograd_ref_pipeline_equals_direct(m, N, C, K, H, W):
    rng = np.random.default_rng(400 + m + H)
    x = rng.standard_normal((N, C, H, W)); w = rng.standard_normal((K, C, 3, 3)); b = rng.standard_normal(K)
    y = oracle.conv2d_direct(x, w, b)
    yw = wr.conv2d_winograd(x, w, b, m)
    assert oracle.rel_l2(yw, y) < 1e-13


def test_rel_l2_metric():
    a = np.array([3.0, 4.0])
    assert oracle.rel_l2(a, a) == 0.0
    assert abs(oracle.rel_l2(a + np.array([0.3, 0.4]), a) - 0.1) < 1e-15
    with pytest.raises(ValueError):
        oracle.rel_l2(a, np.zeros(2))
