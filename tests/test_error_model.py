"""The rounding-error model of the fp16-storage Winograd path (CPU only).

The paper gives no accuracy figure; the tolerance (relative L2 <= 5e-3 for fp16 storage with fp32
accumulation) is this build's target.  These tests fix what a CORRECT fp16-storage path must show,
from the arithmetic alone: F(2x2) rounds to about 5e-4, F(4x4) to about 3e-3 (its transforms
amplify the rounding of V), both independent of the channel count.  The GPU tests use the same
bands to detect a path that silently ran something else."""
import numpy as np
import pytest

import oracle
from oracle import winograd_ref as wr

# expected relative-L2 band of a correct fp16-storage path, per output tile size
BANDS = {2: (2.5e-4, 1.0e-3), 4: (1.5e-3, 4.5e-3)}


@pytest.mark.parametrize("C", [32, 320])
@pytest.mark.parametrize("m", [2, 4])
def test_fp16_storage_error_band(m, C):
    rng = np.random.default_rng(C + m)
    N, K, H, W = 1, 16, 16, 16
    x = rng.standard_normal((N, C, H, W)).astype(np.float16)
    w = (rng.standard_normal((K, C, 3, 3)) / np.sqrt(9 * C)).astype(np.float16)
    b = (0.01 * rng.standard_normal(K)).astype(np.float32)
    ref = oracle.conv2d_direct(x, w, b)
    y = wr.conv2d_winograd_storage_model(x.astype(np.float64), w.astype(np.float64), b.astype(np.float64), m)
    err = oracle.rel_l2(y, ref)
    lo, hi = BANDS[m]
    assert lo <= err <= hi, (m, C, err)
    assert err <= 5e-3


# with the intermediate product M also kept in fp16 (the library's opt-in "half product" mode)
BANDS_HALF_PRODUCT = {2: (4.0e-4, 1.0e-3), 4: (3.0e-3, 4.8e-3)}


@pytest.mark.parametrize("C", [32, 320, 1280])
@pytest.mark.parametrize("m", [2, 4])
def test_fp16_product_error_band(m, C):
    """Rounding M to fp16 as well costs F(4x4) about a quarter more error (3.1e-3 -> 3.8..4.2e-3): still inside
    5e-3, with less room - which is why the mode is opt-in."""
    rng = np.random.default_rng(C + m)
    N, K, H, W = 1, 16, 16, 16
    x = rng.standard_normal((N, C, H, W)).astype(np.float16)
    w = (rng.standard_normal((K, C, 3, 3)) / np.sqrt(9 * C)).astype(np.float16)
    b = (0.01 * rng.standard_normal(K)).astype(np.float32)
    ref = oracle.conv2d_direct(x, w, b)
    x64, w64, b64 = x.astype(np.float64), w.astype(np.float64), b.astype(np.float64)
    err = oracle.rel_l2(wr.conv2d_winograd_storage_model(x64, w64, b64, m, product_dtype=np.float16), ref)
    base = oracle.rel_l2(wr.conv2d_winograd_storage_model(x64, w64, b64, m), ref)
    lo, hi = BANDS_HALF_PRODUCT[m]
    assert lo <= err <= hi and err > base and err <= 5e-3, (m, C, err, base)


# bfloat16 storage (7 stored mantissa bits): F(2x2) about 4.2e-3, F(4x4) about 2.5e-2, a direct path that
# rounds only its output about 1.7e-3.  The library's tolerances for that type are set from these: 8e-3, 4e-2, 3e-3.
BANDS_BF16 = {2: (3.0e-3, 6.0e-3), 4: (1.8e-2, 3.3e-2), "direct": (1.2e-3, 2.2e-3)}


def test_round_to_bf16_matches_the_library_conversion():
    import torch
    rng = np.random.default_rng(0)
    a = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-6, 6, 20000),
                        [1.0, 1.00390625, 1.01171875, 1.0078125, 0.0, -0.0, 3.0e38, -1.0e-38]])   # ties both ways included
    ref = torch.tensor(a, dtype=torch.float32).to(torch.bfloat16).float().numpy().astype(np.float64)
    assert np.array_equal(wr.round_to_bf16(a), ref)
    assert wr.round_to_bf16([1.00390625])[0] == 1.0 and wr.round_to_bf16([1.01171875])[0] == 1.015625   # ties go to even


@pytest.mark.parametrize("C", [32, 320])
@pytest.mark.parametrize("m", [2, 4])
def test_bf16_storage_error_band(m, C):
    rng = np.random.default_rng(C + m)
    N, K, H, W = 1, 16, 16, 16
    x = wr.round_to_bf16(rng.standard_normal((N, C, H, W)))
    w = wr.round_to_bf16(rng.standard_normal((K, C, 3, 3)) / np.sqrt(9 * C))
    b = (0.01 * rng.standard_normal(K)).astype(np.float32).astype(np.float64)
    ref = oracle.conv2d_direct(x, w, b)
    err = oracle.rel_l2(wr.conv2d_winograd_storage_model(x, w, b, m, store_dtype="bf16"), ref)
    lo, hi = BANDS_BF16[m]
    assert lo <= err <= hi, (m, C, err)
    d = oracle.rel_l2(wr.round_to_bf16(ref), ref)
    assert BANDS_BF16["direct"][0] <= d <= BANDS_BF16["direct"][1]


def test_model_without_rounding_is_exact():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((1, 8, 9, 10)); w = rng.standard_normal((4, 8, 3, 3)); b = rng.standard_normal(4)
    y = wr.conv2d_winograd_storage_model(x, w, b, 4, store_dtype=np.float64)
    assert oracle.rel_l2(y, oracle.conv2d_direct(x, w, b)) < 1e-13


# ---- the element-wise acceptance bound of the GPU parity tests (tests/parity_util.py) ------------------------------
@pytest.mark.parametrize("shape", [(2, 320, 48, 32, 32), (1, 96, 64, 63, 66)])
@pytest.mark.parametrize("m", [2, 4])
def test_elementwise_bound_holds_for_a_correct_path_and_catches_one_wrong_element(m, shape):
    """Per tile-position class the error of the storage model is close to Gaussian: no element further than 6 class-rms
    from the exact result (beyond the half-ulp of the output rounding), so the GPU tests' bound of 8 passes a correct
    path.  One element wrong by the size of a typical output (planted here, on the CPU, in a correct result) is
    hundreds of class-rms away and fails it, although the relative L2 error of the tensor hardly moves."""
    import sys, os
    sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
    import parity_util as pu
    N, C, K, H, W = shape
    rng = np.random.default_rng(sum(shape) + m)
    x = rng.standard_normal((N, C, H, W)).astype(np.float16).astype(np.float64)
    w = (rng.standard_normal((K, C, 3, 3)) / np.sqrt(9 * C)).astype(np.float16).astype(np.float64)
    b = (0.01 * rng.standard_normal(K)).astype(np.float32).astype(np.float64)
    ref = oracle.conv2d_direct(x, w, b)
    y = wr.conv2d_winograd_storage_model(x, w, b, m)
    ex = pu.elementwise_excess(y, ref, m, "f16")
    assert ex <= 6.0, ex
    assert pu.check(y, ref, 5e-3, m, "f16") <= 5e-3
    # uniform grouping (m = 1) would NOT do for F(4x4): the tile positions differ in variance
    if m == 4:
        assert pu.elementwise_excess(y, ref, 1, "f16") > 8.0
    bad = y.copy()
    bad[N - 1, K // 2, H // 2, W // 3] += 1.0
    assert oracle.rel_l2(bad, ref) <= 5e-3                      # the norm alone lets it through
    assert pu.elementwise_excess(bad, ref, m, "f16") > 50.0
    with pytest.raises(AssertionError):
        pu.check(bad, ref, 5e-3, m, "f16")
    # a path that only rounds its output (the direct variant) is covered by the half-ulp term alone
    yd = ref.astype(np.float32).astype(np.float16).astype(np.float64)
    assert pu.elementwise_excess(yd, ref, 1, "f16") == 0.0
    # ... and a path that silently ran that variant where F(4x4) was asked for is still flagged by the error band


def test_elementwise_bound_with_few_channels():
    """Four input channels (the conv_in layer): heavier tails, up to ~10 class-rms on a correct path (fp32 and fp16
    storage models), hence the wider limit below 32 channels; a planted wrong element is still far outside it."""
    import sys, os
    sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
    import parity_util as pu
    rng = np.random.default_rng(4)
    x = rng.standard_normal((1, 4, 64, 64)).astype(np.float32).astype(np.float64)
    w = (rng.standard_normal((64, 4, 3, 3)) / 6.0).astype(np.float32).astype(np.float64)
    b = (0.01 * rng.standard_normal(64)).astype(np.float64)
    ref = oracle.conv2d_direct(x, w, b)
    for m in (2, 4):
        for store, name, tol in ((np.float32, "f32", 1e-5), (np.float16, "f16", 5e-3)):
            xs, ws = x.astype(store).astype(np.float64), w.astype(store).astype(np.float64)
            r = oracle.conv2d_direct(xs, ws, b)
            y = wr.conv2d_winograd_storage_model(xs, ws, b, m, store_dtype=store)
            assert pu.elementwise_excess(y, r, m, name) <= 12.0
            pu.check(y, r, tol, m, name, channels=4)
            bad = y.copy(); bad[0, 7, 9, 11] += 0.5
            with pytest.raises(AssertionError):
                pu.check(bad, r, 1.0, m, name, channels=4)


def test_elementwise_bound_with_fp32_accumulation():
    """fp32 storage: what is left is the rounding of the fp32 accumulation, emulated here by adding the products of
    two channels at a time into an fp32 array.  Its tails are heavier than those of rounded operands (about 7 class-rms
    on 6.5e4 outputs against 4.5), which is why the GPU tests allow 12 for fp32 storage."""
    import sys, os
    sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
    import parity_util as pu
    rng = np.random.default_rng(1)
    N, C, K, H, W = 1, 160, 16, 64, 64
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    w = (rng.standard_normal((K, C, 3, 3)) / np.sqrt(9 * C)).astype(np.float32)
    b = np.zeros(K)
    ref = oracle.conv2d_direct(x.astype(np.float64), w.astype(np.float64), b)
    for m in (2, 4):
        U = wr.filter_transform(w.astype(np.float64), m).astype(np.float32)
        V = wr.input_transform(x.astype(np.float64), m).astype(np.float32)
        M = np.zeros(U.shape[:3] + V.shape[3:], dtype=np.float32)
        for c0 in range(0, C, 2):
            M += np.einsum("xnkc,xnct->xnkt", U[..., c0:c0 + 2], V[:, :, c0:c0 + 2, :]).astype(np.float32)
        y = wr.output_transform(M.astype(np.float64), b, N, H, W, m).astype(np.float32).astype(np.float64)
        assert oracle.rel_l2(y, ref) <= 1e-5
        ex = pu.elementwise_excess(y, ref, m, "f32")
        assert 4.0 <= ex <= 10.0, ex
        pu.check(y, ref, 1e-5, m, "f32", channels=C)
