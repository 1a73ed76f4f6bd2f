"""ORACLE — test infrastructure only.

The operators that sit on either side of the 3x3 convolution inside a Stable-Diffusion residual
block, in fp64 numpy, so that the fused entry point of the library can be checked: GroupNorm
followed by SiLU on the way in, a per-(image, channel) vector and a residual tensor added on the
way out.  The paper's Section "Techniques" motivates keeping dependent steps local; it defines
none of these operators, so the textbook definitions are written out here:

  GroupNorm:  channels are cut into G equal groups; per (n, group) the mean and the biased
              variance are taken over the group's channels and all pixels;
              v = (x - mean) / sqrt(var + eps) * gamma[c] + beta[c]
  SiLU:       s(v) = v / (1 + exp(-v))

  Nearest-neighbour 2x upsampling (the step before the 3x3 convolution in the UNet's and the
  VAE decoder's up-sampling blocks): u[n, c, i, j] = x[n, c, floor(i / 2), floor(j / 2)].

Pinned by tests/test_oracle_pins_fused.py (library routine, closed forms, invariants).
"""
from __future__ import annotations

import numpy as np

from . import conv2d_direct


def groupnorm(x, gamma, beta, groups: int, eps: float = 1e-5) -> np.ndarray:
    x = np.asarray(x, dtype=np.float64)
    N, C, H, W = x.shape
    if C % groups:
        raise ValueError("C must be a multiple of groups")
    xg = x.reshape(N, groups, C // groups, H, W)
    mean = xg.mean(axis=(2, 3, 4), keepdims=True)
    var = ((xg - mean) ** 2).mean(axis=(2, 3, 4), keepdims=True)
    v = ((xg - mean) / np.sqrt(var + eps)).reshape(N, C, H, W)
    return v * np.asarray(gamma, dtype=np.float64).reshape(1, C, 1, 1) + np.asarray(beta, dtype=np.float64).reshape(1, C, 1, 1)


def groupnorm_stats(x, groups: int, eps: float = 1e-5):
    """(mean, rstd), each [N, groups]; rstd = 1 / sqrt(var + eps)."""
    x = np.asarray(x, dtype=np.float64)
    N, C, H, W = x.shape
    xg = x.reshape(N, groups, -1)
    mean = xg.mean(axis=2)
    var = ((xg - mean[:, :, None]) ** 2).mean(axis=2)
    return mean, 1.0 / np.sqrt(var + eps)


def silu(v) -> np.ndarray:
    v = np.asarray(v, dtype=np.float64)
    return v / (1.0 + np.exp(-v))


def upsample_nearest2x(x) -> np.ndarray:
    """u[n, c, i, j] = x[n, c, i // 2, j // 2], written as that index expression."""
    x = np.asarray(x, dtype=np.float64)
    N, C, H, W = x.shape
    ii = np.arange(2 * H) // 2
    jj = np.arange(2 * W) // 2
    return x[:, :, ii[:, None], jj[None, :]]


def conv2d_fused(x, w, bias, gamma=None, beta=None, groups: int = 32, eps: float = 1e-5,
                 addvec=None, residual=None, upsample: bool = False) -> np.ndarray:
    """y = conv3x3(up(SiLU(GroupNorm(x)))) + bias + addvec[n,k] + residual; every extra is optional
    (gamma None = no GroupNorm/SiLU, upsample False = no 2x nearest-neighbour upsampling).  Zero
    padding applies to the tensor the convolution sees; with upsampling y, addvec's image and the
    residual have twice the height and width of x."""
    a = np.asarray(x, dtype=np.float64)
    if gamma is not None:
        a = silu(groupnorm(a, gamma, beta, groups, eps))
    if upsample:
        a = upsample_nearest2x(a)
    y = conv2d_direct(a, w, bias)
    if addvec is not None:
        y = y + np.asarray(addvec, dtype=np.float64)[:, :, None, None]
    if residual is not None:
        y = y + np.asarray(residual, dtype=np.float64)
    return y
