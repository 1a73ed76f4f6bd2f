"""ORACLE — test infrastructure only.

The Winograd minimal-filtering convolution F(m x m, 3 x 3), m in {2, 4}, in fp64
numpy, taking the steps in the order the paper's Section "Techniques" names
them: (i) preprocess of the filter and of the activation, (ii) element-wise
multiplication of the preprocessed tensors (summed over input channels),
(iii) postprocess of the intermediate result.  No blocking, no layout tricks:
each stage returns a plain array so that the HIP kernels can be checked stage
by stage.

The paper prints no transform matrices; it cites the minimal-filtering
construction.  The triples (A^T, G, B^T) below are the standard ones for the
interpolation points {0, +-1, inf} (m=2) and {0, +-1, +-2, inf} (m=4).  They
are held as exact fractions; ``tests/test_oracle_pins.py`` proves with rational
arithmetic that A^T[(G g G^T) .* (B^T d B)]A equals the direct m x m
correlation, so the identity — not this listing — is the authority.

Array conventions (alpha = m + 2, th = ceil(H/m), tw = ceil(W/m), T = N*th*tw,
tile index t = (n*th + ti)*tw + tj, xi = 0..alpha-1 row, nu = 0..alpha-1 col):
  U[xi, nu, k, c]   V[xi, nu, c, t]   M[xi, nu, k, t]
"""
from __future__ import annotations

from fractions import Fraction as Fr

import numpy as np

_F = Fr
MATRICES = {
    2: dict(
        BT=[[1, 0, -1, 0],
            [0, 1, 1, 0],
            [0, -1, 1, 0],
            [0, 1, 0, -1]],
        G=[[_F(1), _F(0), _F(0)],
           [_F(1, 2), _F(1, 2), _F(1, 2)],
           [_F(1, 2), _F(-1, 2), _F(1, 2)],
           [_F(0), _F(0), _F(1)]],
        AT=[[1, 1, 1, 0],
            [0, 1, -1, -1]],
    ),
    4: dict(
        BT=[[4, 0, -5, 0, 1, 0],
            [0, -4, -4, 1, 1, 0],
            [0, 4, -4, -1, 1, 0],
            [0, -2, -1, 2, 1, 0],
            [0, 2, -1, -2, 1, 0],
            [0, 4, 0, -5, 0, 1]],
        G=[[_F(1, 4), _F(0), _F(0)],
           [_F(-1, 6), _F(-1, 6), _F(-1, 6)],
           [_F(-1, 6), _F(1, 6), _F(-1, 6)],
           [_F(1, 24), _F(1, 12), _F(1, 6)],
           [_F(1, 24), _F(-1, 12), _F(1, 6)],
           [_F(0), _F(0), _F(1)]],
        AT=[[1, 1, 1, 1, 1, 0],
            [0, 1, -1, 2, -2, 0],
            [0, 1, 1, 4, 4, 0],
            [0, 1, -1, 8, -8, 1]],
    ),
}


def exact_matrices(m: int):
    """(AT, G, BT) as nested lists of Fraction."""
    mm = MATRICES[m]
    conv = lambda M: [[Fr(v) for v in row] for row in M]
    return conv(mm["AT"]), conv(mm["G"]), conv(mm["BT"])


def matrices(m: int):
    """(AT, G, BT) as fp64 arrays."""
    at, g, bt = exact_matrices(m)
    f = lambda M: np.array([[float(v) for v in row] for row in M], dtype=np.float64)
    return f(at), f(g), f(bt)


def tile_counts(H: int, W: int, m: int):
    return (H + m - 1) // m, (W + m - 1) // m


def filter_transform(w, m: int) -> np.ndarray:
    """Step (i), filter:  U[xi,nu,k,c] = (G g[k,c] G^T)[xi,nu]."""
    _, G, _ = matrices(m)
    w = np.asarray(w, dtype=np.float64)
    return np.einsum("ar,kcrs,bs->abkc", G, w, G)


def input_tiles(x, m: int) -> np.ndarray:
    """d[c, t, a, b] = xhat[n, c, m*ti-1+a, m*tj-1+b], zeros outside the image."""
    x = np.asarray(x, dtype=np.float64)
    N, C, H, W = x.shape
    al = m + 2
    th, tw = tile_counts(H, W, m)
    xp = np.zeros((N, C, m * th + 2, m * tw + 2), dtype=np.float64)
    xp[:, :, 1:H + 1, 1:W + 1] = x
    d = np.empty((C, N * th * tw, al, al), dtype=np.float64)
    for n in range(N):
        for ti in range(th):
            for tj in range(tw):
                t = (n * th + ti) * tw + tj
                d[:, t] = xp[n, :, m * ti:m * ti + al, m * tj:m * tj + al]
    return d


def input_transform(x, m: int) -> np.ndarray:
    """Step (i), activation:  V[xi,nu,c,t] = (B^T d[c,t] B)[xi,nu]."""
    _, _, BT = matrices(m)
    d = input_tiles(x, m)
    return np.einsum("xa,ctab,nb->xnct", BT, d, BT)


def multiply(U, V) -> np.ndarray:
    """Step (ii):  M[xi,nu,k,t] = sum_c U[xi,nu,k,c] * V[xi,nu,c,t]."""
    return np.einsum("xnkc,xnct->xnkt", U, V)


def output_transform(M, bias, N: int, H: int, W: int, m: int) -> np.ndarray:
    """Step (iii):  y tile = A^T M[:,:,k,t] A, cropped to H x W, plus bias[k]."""
    AT, _, _ = matrices(m)
    al = m + 2
    K = M.shape[2]
    th, tw = tile_counts(H, W, m)
    Y = np.einsum("ax,xnkt,bn->ktab", AT, M, AT)            # [K, T, m, m]
    Y = Y.reshape(K, N, th, tw, m, m).transpose(1, 0, 2, 4, 3, 5).reshape(N, K, th * m, tw * m)
    y = np.ascontiguousarray(Y[:, :, :H, :W])
    if bias is not None:
        y = y + np.asarray(bias, dtype=np.float64).reshape(1, K, 1, 1)
    return y


def conv2d_winograd(x, w, bias, m: int) -> np.ndarray:
    """All three steps in order; equals conv2d_direct up to fp64 rounding."""
    x = np.asarray(x, dtype=np.float64)
    N, C, H, W = x.shape
    U = filter_transform(w, m)
    V = input_transform(x, m)
    M = multiply(U, V)
    return output_transform(M, bias, N, H, W, m)


def round_to_bf16(a) -> np.ndarray:
    """Round to the nearest bfloat16 (8 exponent bits, 7 stored mantissa bits), ties to even, written on the
    bit pattern of the fp32 value: add 0x7fff plus the lowest kept bit, drop the low 16 bits.  Returned as fp64.
    (Finite inputs only; the error model never feeds it anything else.)"""
    bits = np.asarray(a, dtype=np.float64).astype(np.float32).view(np.uint32).astype(np.uint64)
    bits = (bits + 0x7FFF + ((bits >> 16) & 1)) & 0xFFFF0000
    return bits.astype(np.uint32).view(np.float32).astype(np.float64)


def conv2d_winograd_storage_model(x, w, bias, m: int, store_dtype=np.float16, product_dtype=None) -> np.ndarray:
    """Error model of a low-precision Winograd path (not the definition of the result): the
    same three steps, with U and V rounded once to `store_dtype` as a kernel that keeps them
    in that type would, the products accumulated exactly (fp64 stands in for fp32), and the
    output rounded once to `store_dtype`.  Used to predict the relative L2 error a correct
    fp16-storage implementation must show - far above or far below means a different path ran.
    `product_dtype` (None = exact) additionally rounds the intermediate product M once, as a path
    that stores M in that type between its second and third step would."""
    x = np.asarray(x, dtype=np.float64)
    N, C, H, W = x.shape
    if isinstance(store_dtype, str) and store_dtype == "bf16":
        q = round_to_bf16
    elif np.dtype(store_dtype).itemsize >= 8:
        q = lambda a: a
    else:                       # the kernels transform in fp32, then round once to the storage type
        q = lambda a: a.astype(np.float32).astype(store_dtype).astype(np.float64)
    U = q(filter_transform(w, m))
    V = q(input_transform(x, m))
    M = multiply(U, V)
    if product_dtype is not None:
        M = M.astype(np.float32).astype(product_dtype).astype(np.float64)
    return q(output_transform(M, bias, N, H, W, m))
