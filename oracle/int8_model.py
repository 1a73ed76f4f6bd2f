"""ORACLE — test infrastructure only.

Winograd F(2x2, 3x3) convolution whose TRANSFORMED operands are held as 8-bit integers.  The paper's Section
"Techniques" only remarks that its stack supports quantised operators and defines no scheme; this one is this build's
own, the plainest symmetric linear quantisation with one step per row of each matrix product of step (ii):

    U = G g G^T  (exact)                       mU[xi,nu,k] = max_c |U[xi,nu,k,c]|
    V = (B^T d) B                              mV[xi,nu,t] = max_c |V[xi,nu,c,t]|
    Uq = rint(U * (127 / mU)),  Vq = rint(V * (127 / mV))         codes in [-127, 127], ties to even, 0 where m = 0
    dU = mU / 127,  dV = mV / 127                                  the quantisation steps, kept as fp32 numbers
    M[xi,nu,k,t] = (sum_c Uq[xi,nu,k,c] * Vq[xi,nu,c,t]) * dU[xi,nu,k] * dV[xi,nu,t]
    y = A^T M A + bias

Where floating point decides an integer code the precision is part of the definition, and it is the one a kernel can
reproduce bit for bit:
  * the filter side works in fp64: U of a 16- or 32-bit filter is exact there (nine terms, coefficients 1, 1/2, 1/4),
    so are the row maxima; 127 / mU, the product U * (127 / mU) and rint are single IEEE operations;
    dU = fp32(mU / 127) (fp64 division, rounded once to fp32);
  * the activation side works in fp32 (it runs on every call): B^T has one +1 and one -1 (or two +1) per row, so every
    entry of B^T d and then of (B^T d) B is ONE IEEE addition or subtraction - the result is fixed by taking the row
    combination (B^T d) first and the column combination second, whatever a kernel names its temporaries;
    127 / mV, V * (127 / mV) and mV / 127 are single fp32 operations.
The products of codes and their sums are integers and exact.  The two steps multiply the integer sum in fp64 here; a
kernel does it in fp32 (two roundings, ~1e-7 relative), which is what a comparison has to allow.
"""
from __future__ import annotations

import numpy as np

from . import winograd_ref as wr

QMAX = 127.0


def filter_codes(w):
    """(Uq, dU): Uq[xi,nu,k,c] integer codes as fp64, dU[xi,nu,k] fp32 steps as fp64, decided in fp64 as defined above."""
    U = wr.filter_transform(w, 2)                                   # exact in fp64 for 16-bit and fp32 filters
    mU = np.max(np.abs(U), axis=3)
    with np.errstate(divide="ignore"):
        s = np.where(mU > 0, QMAX / np.where(mU > 0, mU, 1.0), 0.0)
    Uq = np.rint(U * s[..., None])
    dU = (mU / QMAX).astype(np.float32).astype(np.float64)
    return Uq, dU


def activation_transform_f32(x) -> np.ndarray:
    """V[xi,nu,c,t] = ((B^T d) B)[xi,nu] in fp32, one addition or subtraction per entry and pass, rows first."""
    d = wr.input_tiles(x, 2).astype(np.float32)                     # [C, T, 4, 4]; 16- and 32-bit inputs are exact in fp32
    r0, r1, r2, r3 = d[:, :, 0, :], d[:, :, 1, :], d[:, :, 2, :], d[:, :, 3, :]
    t = np.stack([r0 - r2, r1 + r2, r2 - r1, r1 - r3], axis=2)      # B^T d: combinations of the window's rows
    c0, c1, c2, c3 = t[:, :, :, 0], t[:, :, :, 1], t[:, :, :, 2], t[:, :, :, 3]
    v = np.stack([c0 - c2, c1 + c2, c2 - c1, c1 - c3], axis=3)      # (B^T d) B: combinations of its columns
    assert v.dtype == np.float32
    return np.ascontiguousarray(v.transpose(2, 3, 0, 1))            # [xi, nu, c, t]


def activation_codes(x):
    """(Vq, dV): Vq[xi,nu,c,t] integer codes as fp64, dV[xi,nu,t] fp32 steps as fp64, decided in fp32 as defined above."""
    V = activation_transform_f32(x)
    mV = np.max(np.abs(V), axis=2)                                  # [xi, nu, t], fp32
    one = np.float32(1.0)
    s = np.where(mV > 0, np.float32(QMAX) / np.where(mV > 0, mV, one), np.float32(0.0)).astype(np.float32)
    Vq = np.rint(V * s[:, :, None, :])
    assert Vq.dtype == np.float32
    dV = (mV / np.float32(QMAX)).astype(np.float32)
    return Vq.astype(np.float64), dV.astype(np.float64)


def product(Uq, dU, Vq, dV) -> np.ndarray:
    """Step (ii) on the codes: M[xi,nu,k,t] = (sum_c Uq Vq) * dU[xi,nu,k] * dV[xi,nu,t]; the sum is an exact integer."""
    acc = np.einsum("xnkc,xnct->xnkt", Uq, Vq)
    return acc * dU[:, :, :, None] * dV[:, :, None, :]


def conv2d_winograd_int8(x, w, bias) -> np.ndarray:
    """The whole quantised convolution defined in the header; x[N][C][H][W], w[K][C][3][3], fp64 result."""
    x = np.asarray(x, dtype=np.float64)
    N, C, H, W = x.shape
    Uq, dU = filter_codes(w)
    Vq, dV = activation_codes(x)
    return wr.output_transform(product(Uq, dU, Vq, dV), bias, N, H, W, 2)
