"""Every block shape of the step (ii) kernel (Section "Techniques": the element-wise multiplication summed over
input channels, i.e. alpha^2 matrix products) on small ragged inputs, through wino_batched_gemm_shape: the large
blocks (256x256, 256x128) are otherwise reached only by full-size layers.  Compared element by element with the fp64
product of the stored operands."""
import numpy as np
import pytest
import torch

from paper_2412_05781_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("dtype", [torch.float16, torch.float32, torch.bfloat16])
@pytest.mark.parametrize("variant", [B.WINO_F2, B.WINO_F4])
@pytest.mark.parametrize("block_shape", list(range(9)))
# reduction lengths: ragged last stage (40, 136, 72) and whole stages (64, 192, 320), which take different kernels
@pytest.mark.parametrize("dims", [(70, 40, 33), (300, 136, 290), (129, 72, 513), (70, 64, 33), (300, 192, 290), (129, 320, 513)])
def test_named_block_shape_against_fp64_product(dims, block_shape, variant, dtype):
    K, C, T = dims
    a2 = (variant + 2) ** 2
    Cp = (C + 7) // 8 * 8
    g = torch.Generator().manual_seed(K + C + T + block_shape)
    U = torch.randn(a2, K, Cp, generator=g).to(dtype)
    V = torch.randn(a2, T, Cp, generator=g).to(dtype)
    U[:, :, C:] = 0
    V[:, :, C:] = 0
    M = B.wino_batched_gemm(U.to(DEV), V.to(DEV), K, C, T, variant, block_shape=block_shape)
    M_auto = B.wino_batched_gemm(U.to(DEV), V.to(DEV), K, C, T, variant)
    torch.cuda.synchronize()
    ref = np.einsum("bkc,btc->bkt", U.double().numpy(), V.double().numpy())
    got = M.cpu().numpy().astype(np.float64)
    assert got.shape == (a2, K, T)
    # fp32 accumulation of <= 320 products of magnitude ~1: each element within a few fp32 ulps of sqrt(C)
    tol = 2e-5 * np.sqrt(C) * 4
    assert np.abs(got - ref).max() <= tol, (dims, block_shape, np.abs(got - ref).max())
    # the shapes differ only in the order of the fp32 sums (one or two partial accumulators per sub-tile)
    assert np.abs(got - M_auto.cpu().numpy().astype(np.float64)).max() <= tol


def test_block_shape_out_of_range_is_rejected():
    U = torch.zeros(16 * 8 * 8, dtype=torch.float16, device=DEV)
    for bad in (-1, 9, 100):
        with pytest.raises(B.WinoError) as e:
            B.wino_batched_gemm(U, U, 8, 8, 8, B.WINO_F2, block_shape=bad)
        assert e.value.status == B.WINO_ERR_VARIANT
