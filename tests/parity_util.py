"""Acceptance checks shared by the GPU parity tests: the whole-tensor relative L2 error AND an element-wise bound,
so that one wrong tile cannot hide in the norm.

Element-wise bound.  The error e = y - ref of a correct low-precision Winograd path is, per position (a, b) inside
the m x m output tile, close to Gaussian (sums of many independent operand roundings; the positions differ in
variance because the rows of A^T differ in weight), plus the final rounding of y, which is at most half a unit in the
last place of the storage type.  So, per position class (i mod m, j mod m):

    |e| <= C_SIGMA * rms_class(e) + 2^-p * |ref|        p = 11 (fp16), 8 (bf16), 24 (fp32)

with C_SIGMA = 8: tests/test_error_model.py pins, on the CPU storage model, that a correct path stays below 6 (the
expected maximum of 10^8 Gaussian samples is 5.9 sigma) and that one element that is wrong by the size of a typical
output, planted in a correct result, breaks the bound.  The direct variant (m = 1 here) only rounds y, so for it the
second term alone has to cover the error.  With fewer than 32 input channels an output's error is a sum of only a few
products of Gaussians, whose tails are heavier (the same pin shows up to 9 class-rms at C = 4): C_SIGMA_FEW = 16 there.
With fp32 storage the error is that of the fp32 accumulation itself, whose size follows the running sums and not a
fixed variance (an emulation of fp32 accumulation in the same pin file shows 7.4 class-rms on 2.6e5 outputs where
rounded operands show 5): C_SIGMA_F32 = 12.
"""
import numpy as np

C_SIGMA = 8.0
C_SIGMA_FEW = 16.0          # fewer than FEW_CHANNELS input channels
C_SIGMA_F32 = 12.0          # fp32 storage
FEW_CHANNELS = 32
HALF_ULP = {"f16": 2.0 ** -11, "bf16": 2.0 ** -8, "f32": 2.0 ** -24}
SUBNORMAL_HALF_ULP = {"f16": 2.0 ** -25, "bf16": 0.0, "f32": 0.0}      # fp16 spacing stops shrinking below 2^-14


def rel_l2(y, ref) -> float:
    d = np.subtract(y, ref, dtype=np.float64).ravel()
    return float(np.sqrt(d @ d) / np.linalg.norm(np.asarray(ref, dtype=np.float64).ravel()))


def elementwise_excess(y, ref, m: int, dtype: str) -> float:
    """max over elements of (|e| - half-ulp slack) / rms of the element's tile-position class; NCHW arrays.
    A correct path gives <= ~6; the tests require <= C_SIGMA."""
    worst = 0.0
    for a in range(m):
        for b in range(m):
            r = ref[:, :, a::m, b::m]
            if r.size == 0:
                continue
            e = y[:, :, a::m, b::m] - r
            rms = float(np.sqrt(np.mean(e * e)))
            over = np.abs(e) - HALF_ULP[dtype] * 1.001 * np.abs(r) - SUBNORMAL_HALF_ULP[dtype]
            mx = float(over.max())
            if mx <= 0.0:
                continue
            if rms == 0.0:
                return float("inf")
            worst = max(worst, mx / rms)
    return worst


def check(y, ref, tol: float, m: int, dtype: str, what="", channels: int = FEW_CHANNELS) -> float:
    """relL2 <= tol, every element finite, and the element-wise bound (`channels` = input channels of the layer).
    Returns relL2."""
    assert y.shape == ref.shape, (what, y.shape, ref.shape)
    assert np.isfinite(y).all(), what
    err = rel_l2(y, ref)
    assert err <= tol, (what, "relL2", err)
    ex = elementwise_excess(y, ref, m, dtype)
    lim = C_SIGMA_FEW if channels < FEW_CHANNELS else (C_SIGMA_F32 if dtype == "f32" else C_SIGMA)
    assert ex <= lim, (what, "an element is %.1f class-rms away from the oracle (relL2 %.2e)" % (ex, err))
    return err
