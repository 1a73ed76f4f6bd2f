"""ORACLE — test infrastructure only.

Model of a convolution whose operands are quantised to 8-bit floating point (OCP "E4M3": 1 sign, 4 exponent
and 3 mantissa bits, bias 7, no infinities, largest finite value 448, subnormals down to 2^-9) with one
power-of-two scale per tensor, products accumulated exactly and the sum divided by the two scales.  The paper
only remarks that its stack supports quantised operators; it defines no scheme, so this is this build's own:

    xq = e4m3(clamp(x * sx, -448, 448)),  wq = e4m3(clamp(w * sw, -448, 448))
    y  = conv(xq, wq) / (sx * sw) + bias

`round_to_e4m3` is written on the number line (spacing 2^(e-3) in binade e, ties to even, fixed spacing 2^-9
below 2^-6), not by calling a library conversion; tests pin it against one.
"""
from __future__ import annotations

import numpy as np

from . import conv2d_general

E4M3_MAX = 448.0


def round_to_e4m3(a) -> np.ndarray:
    """Nearest E4M3 value (ties to even) of every element after clamping to [-448, 448]; fp64 in, fp64 out."""
    a = np.clip(np.asarray(a, dtype=np.float64), -E4M3_MAX, E4M3_MAX)
    mag = np.abs(a)
    # binade exponent, clamped at the smallest normal binade (2^-6): below it the spacing stays 2^-9
    with np.errstate(divide="ignore"):
        e = np.floor(np.log2(np.where(mag > 0, mag, 1.0)))
    e = np.maximum(e, -6.0)
    step = 2.0 ** (e - 3.0)
    q = np.rint(mag / step) * step              # numpy's rint rounds halves to even
    return np.sign(a) * np.minimum(q, E4M3_MAX)


def power_of_two_scale(a) -> float:
    """Largest power of two s with max|a| * s <= 448 (1.0 for an all-zero tensor)."""
    m = float(np.max(np.abs(np.asarray(a, dtype=np.float64))))
    return 1.0 if m == 0.0 else float(2.0 ** np.floor(np.log2(E4M3_MAX / m)))


def conv2d_fp8(x, w, bias, sx: float, sw: float, stride: int = 1) -> np.ndarray:
    """The quantised convolution defined above (R x R filter, pad (R-1)/2), in fp64."""
    xq = round_to_e4m3(np.asarray(x, dtype=np.float64) * sx)
    wq = round_to_e4m3(np.asarray(w, dtype=np.float64) * sw)
    y = conv2d_general(xq, wq, None, stride) / (sx * sw)
    if bias is not None:
        y = y + np.asarray(bias, dtype=np.float64)[None, :, None, None]
    return y


def conv2d_winograd_8bit(x, w, bias, m: int, fmt: str = "e4m3", per_position: bool = False) -> np.ndarray:
    """Error model (not the definition of a result): the three Winograd steps with the TRANSFORMED tensors U and V held
    in 8 bits - E4M3 with a power-of-two scale, or int8 with a symmetric linear scale - per tensor, or one scale per
    position (xi, nu) of the transformed tile; products accumulated exactly, y kept in fp64.  Answers whether 8-bit
    operands for step (ii) of the Winograd path could meet a useful tolerance: the transforms mix values of very
    different size into one tensor and the inverse transform amplifies what the rounding leaves behind."""
    from . import winograd_ref as wr
    x = np.asarray(x, dtype=np.float64)
    N, C, H, W = x.shape
    U = wr.filter_transform(w, m)
    V = wr.input_transform(x, m)

    def q(a):
        axes = (2, 3) if per_position else None
        mx = np.max(np.abs(a), axis=axes, keepdims=True)
        mx = np.where(mx == 0, 1.0, mx)
        if fmt == "e4m3":
            s = 2.0 ** np.floor(np.log2(E4M3_MAX / mx))
            return round_to_e4m3(a * s) / s
        if fmt == "int8":
            s = 127.0 / mx
            return np.clip(np.rint(a * s), -127, 127) / s
        raise ValueError(fmt)

    return wr.output_transform(wr.multiply(q(U), q(V)), bias, N, H, W, m)
