"""Host-side checks of the C-ABI boundary that need no GPU: the library loads, exports every
symbol the header declares, answers size queries, and rejects bad arguments before any launch."""
import ctypes
import os
import re

import pytest

from paper_2412_05781_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(B.LIB_PATH):
        from paper_2412_05781_amd.build import build_libwino
        build_libwino()
    return B.lib()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "wino.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(wino_[a-z0-9_]+)\s*\(", text)))


def test_header_and_library_agree(L):
    names = declared_functions()
    assert set(names) == set(B.EXPORTS), (names, B.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_version_and_status_strings(L):
    assert B.wino_version() >= 100
    seen = {B.status_string(s) for s in range(0, 11)}
    assert len(seen) == 11 and "ok" in seen
    assert B.status_string(12345) == "unknown status"


def test_sizes(L):
    # U[alpha^2][K][Cp]
    assert B.wino_filter_bytes(320, 320, B.WINO_F16, B.WINO_F4) == 36 * 320 * 320 * 2
    assert B.wino_filter_bytes(320, 4, B.WINO_F32, B.WINO_F2) == 16 * 320 * 8 * 4      # C padded to 8
    assert B.wino_filter_bytes(320, 320, B.WINO_F16, B.WINO_AUTO) == 0
    assert B.wino_filter_bytes(0, 320, B.WINO_F16, B.WINO_F2) == 0
    assert B.wino_filter_bytes(8, 8, 7, B.WINO_F2) == 0
    assert B.wino_transformed_dims(2, 320, 64, 64, 320, B.WINO_F4) == (6, 320, 512)
    assert B.wino_transformed_dims(2, 320, 64, 64, 320, B.WINO_F2) == (4, 320, 2048)
    assert B.wino_transformed_dims(1, 5, 7, 9, 3, B.WINO_F4) == (6, 8, 2 * 3)
    ws = B.wino_workspace_bytes(2, 320, 64, 64, 320, B.WINO_F16, B.WINO_F4)
    assert ws == 36 * 512 * 320 * 2 + 36 * 320 * 512 * 4
    # the direct variant: the channel-last copy of x (2*64*64*320 fp16 elements), no partial sums for this shape
    assert B.wino_workspace_bytes(2, 320, 64, 64, 320, B.WINO_F16, B.WINO_DIRECT) == 2 * 64 * 64 * 320 * 2
    assert B.wino_filter_bytes(320, 320, B.WINO_F16, B.WINO_DIRECT) == (9 * 320 * 320 + 320) * 2
    # what the library recommends: Winograd for the UNet layers, the direct path for few channels on huge images
    assert B.wino_recommend_variant(2, 320, 64, 64, 320, B.WINO_F16) == B.WINO_F4
    assert B.wino_recommend_variant(1, 128, 1024, 1024, 128, B.WINO_F16) == B.WINO_FUSED_F4      # the fused variant beats the direct path there
    assert B.wino_recommend_variant(1, 128, 256, 256, 128, B.WINO_F16) == B.WINO_DIRECT
    assert B.wino_recommend_variant(1, 512, 256, 256, 512, B.WINO_F16) == B.WINO_FUSED_F4
    assert B.wino_recommend_variant(1, 256, 512, 512, 256, B.WINO_BF16) == B.WINO_DIRECT
    assert B.wino_recommend_variant(2, 1280, 8, 8, 1280, B.WINO_F16) == B.WINO_F2
    assert B.wino_recommend_variant(0, 1, 1, 1, 1, B.WINO_F16) == -1
    assert B.wino_workspace_bytes(2, 320, 64, -1, 320, B.WINO_F16, B.WINO_F4) == 0


def test_resolve_variant(L):
    assert B.wino_resolve_variant(2, 320, 64, 64, 320, B.WINO_F16, B.WINO_F2) == B.WINO_F2
    assert B.wino_resolve_variant(2, 320, 64, 64, 320, B.WINO_F16, B.WINO_AUTO) == B.WINO_F4
    # 8x8 images with wide channels: the transformed filter dominates the traffic, F2's is 2.25x smaller
    assert B.wino_resolve_variant(2, 1280, 8, 8, 1280, B.WINO_F16, B.WINO_AUTO) == B.WINO_F2
    # the fused variants where they measured faster: F(4x4) from 4096 tiles on with <= 512 channels and >= 512 blocks (fp16), many-tile layers in bf16
    assert B.wino_resolve_variant(1, 128, 1024, 1024, 128, B.WINO_F16, B.WINO_AUTO) == B.WINO_FUSED_F4
    assert B.wino_resolve_variant(1, 128, 1024, 1024, 3, B.WINO_F16, B.WINO_AUTO) == B.WINO_F4
    assert B.wino_resolve_variant(1, 256, 512, 512, 256, B.WINO_F16, B.WINO_AUTO) == B.WINO_FUSED_F4
    assert B.wino_resolve_variant(1, 512, 256, 256, 512, B.WINO_F16, B.WINO_AUTO) == B.WINO_FUSED_F4
    assert B.wino_resolve_variant(1, 512, 128, 128, 512, B.WINO_F16, B.WINO_AUTO) == B.WINO_F4          # 1024 tiles
    assert B.wino_resolve_variant(1, 64, 256, 256, 64, B.WINO_F16, B.WINO_AUTO) == B.WINO_F4            # 64 blocks
    assert B.wino_resolve_variant(1, 1024, 256, 256, 1024, B.WINO_F16, B.WINO_AUTO) == B.WINO_F4
    assert B.wino_resolve_variant(2, 320, 128, 128, 320, B.WINO_BF16, B.WINO_AUTO) == B.WINO_FUSED_F2
    assert B.wino_resolve_variant(2, 320, 64, 64, 320, B.WINO_BF16, B.WINO_AUTO) == B.WINO_F2
    assert B.wino_recommend_variant(1, 128, 1024, 1024, 3, B.WINO_F16) == B.WINO_DIRECT      # few output channels, large image
    assert B.wino_recommend_variant(2, 320, 64, 64, 4, B.WINO_F16) == B.WINO_F4               # ... but not on a 64x64 latent
    assert B.wino_resolve_variant(2, 320, 64, 64, 320, B.WINO_F16, 3) == -1
    assert B.wino_resolve_variant(2, 320, 64, 64, 320, 9, B.WINO_AUTO) == -1
    assert B.wino_resolve_variant(0, 320, 64, 64, 320, B.WINO_F16, B.WINO_AUTO) == -1


def test_argument_validation_happens_before_any_launch(L):
    vp = ctypes.c_void_p
    desc = B.wino_filter()
    good = vp(0x1000)
    # filter transform
    assert L.wino_filter_transform(None, good, 8, 8, B.WINO_F16, B.WINO_F4, ctypes.byref(desc), None) == B.WINO_ERR_NULL
    assert L.wino_filter_transform(good, good, 8, 8, B.WINO_F16, B.WINO_F4, None, None) == B.WINO_ERR_NULL
    assert L.wino_filter_transform(good, good, 8, 8, 5, B.WINO_F4, ctypes.byref(desc), None) == B.WINO_ERR_DTYPE
    assert L.wino_filter_transform(good, good, 8, 8, B.WINO_F16, B.WINO_AUTO, ctypes.byref(desc), None) == B.WINO_ERR_VARIANT
    assert L.wino_filter_transform(good, good, 0, 8, B.WINO_F16, B.WINO_F4, ctypes.byref(desc), None) == B.WINO_ERR_DIM
    assert L.wino_filter_transform(vp(0x1004), good, 8, 8, B.WINO_F16, B.WINO_F4, ctypes.byref(desc), None) == B.WINO_ERR_ALIGN
    # conv
    desc.data, desc.K, desc.C, desc.dtype, desc.variant = 0x2000, 8, 8, B.WINO_F16, B.WINO_F4
    args = dict(N=1, C=8, H=4, W=4, K=8)
    call = lambda x, y, d=desc, ws=vp(0x100000), wsb=1 << 30, layout=0, **kw: L.wino_conv2d_ex(
        x, ctypes.byref(d), None, y, kw.get("N", 1), kw.get("C", 8), kw.get("H", 4), kw.get("W", 4), kw.get("K", 8),
        layout, ws, wsb, None)
    assert call(None, vp(0x9000)) == B.WINO_ERR_NULL
    assert call(vp(0x8000), None) == B.WINO_ERR_NULL
    assert call(vp(0x8000), vp(0x9000), H=0) == B.WINO_ERR_DIM
    assert call(vp(0x8000), vp(0x9000), C=16) == B.WINO_ERR_DIM           # mismatches the transformed filter
    assert call(vp(0x8008), vp(0x9000)) == B.WINO_ERR_ALIGN
    assert call(vp(0x8000), vp(0x8010)) == B.WINO_ERR_ALIAS               # 1*8*4*4*2 = 256 bytes each
    assert call(vp(0x8000), vp(0x9000), wsb=16) == B.WINO_ERR_WORKSPACE
    assert call(vp(0x8000), vp(0x9000), ws=None) == B.WINO_ERR_WORKSPACE
    assert call(vp(0x8000), vp(0x9000), layout=3) == B.WINO_ERR_LAYOUT
    assert L.wino_input_transform(good, good, 1, 8, 4, 4, B.WINO_F16, B.WINO_F4, 2, None) == B.WINO_ERR_LAYOUT
    bad = B.wino_filter(); bad.data, bad.K, bad.C, bad.dtype, bad.variant = 0x2000, 8, 8, B.WINO_F16, B.WINO_AUTO
    assert call(vp(0x8000), vp(0x9000), d=bad) == B.WINO_ERR_VARIANT
    assert L.wino_conv2d(None, ctypes.byref(desc), None, vp(0x9000), 1, 8, 4, 4, 8, None) == B.WINO_ERR_NULL
    # stages and direct fallback
    assert L.wino_input_transform(None, good, 1, 8, 4, 4, B.WINO_F16, B.WINO_F4, 0, None) == B.WINO_ERR_NULL
    assert L.wino_input_transform(good, good, 1, 8, 4, 4, B.WINO_F16, B.WINO_DIRECT, 0, None) == B.WINO_ERR_VARIANT
    assert L.wino_batched_gemm(good, good, None, 8, 8, 4, B.WINO_F16, B.WINO_F4, None) == B.WINO_ERR_NULL
    assert L.wino_batched_gemm(good, good, good, 8, 8, 0, B.WINO_F16, B.WINO_F4, None) == B.WINO_ERR_DIM
    assert L.wino_output_transform(good, None, None, 1, 8, 4, 4, B.WINO_F16, B.WINO_F4, 0, None) == B.WINO_ERR_NULL
    assert L.wino_output_transform(good, None, good, 1, 8, 4, 4, 7, B.WINO_F4, 0, None) == B.WINO_ERR_DTYPE
    assert L.wino_direct_conv2d(good, None, None, good, 1, 8, 4, 4, 8, B.WINO_F16, None) == B.WINO_ERR_NULL
    assert L.wino_direct_conv2d(vp(0x8000), good, None, vp(0x8000), 1, 8, 4, 4, 8, B.WINO_F16, None) == B.WINO_ERR_ALIAS


def test_fused_entry_points_validate_on_the_host(L):
    vp = ctypes.c_void_p
    assert B.wino_groupnorm_stats_bytes(2, 32) >= 2 * 32 * 8
    assert B.wino_groupnorm_stats_bytes(0, 32) == 0
    good = vp(0x1000)
    f32 = ctypes.c_float(1e-5)
    assert L.wino_groupnorm_stats(None, good, 1, 8, 4, 4, 2, f32, B.WINO_F16, 0, None) == B.WINO_ERR_NULL
    assert L.wino_groupnorm_stats(good, good, 1, 8, 4, 4, 3, f32, B.WINO_F16, 0, None) == B.WINO_ERR_DIM      # 3 does not divide 8
    assert L.wino_groupnorm_stats(good, good, 1, 8, 4, 4, 2, f32, B.WINO_F16, 5, None) == B.WINO_ERR_LAYOUT
    desc = B.wino_filter(); desc.data, desc.K, desc.C, desc.dtype, desc.variant = 0x2000, 8, 8, B.WINO_F16, B.WINO_F4
    f = B.wino_fusion()
    call = lambda fus, y=vp(0x9000): L.wino_conv2d_fused(vp(0x8000), ctypes.byref(desc), None, y, 1, 8, 4, 4, 8, 0,
                                                        fus, vp(0x100000), 1 << 30, None)
    assert call(None) == B.WINO_ERR_NULL
    f.gn_stats = 0x3000                                   # GroupNorm on, gamma/beta missing
    assert call(ctypes.byref(f)) == B.WINO_ERR_NULL
    f.gn_gamma, f.gn_beta, f.gn_groups = 0x4000, 0x5000, 3
    assert call(ctypes.byref(f)) == B.WINO_ERR_DIM
    f.gn_groups = 2; f.residual = 0x9010                  # overlaps y without being y
    assert call(ctypes.byref(f)) == B.WINO_ERR_ALIAS
    f.residual = 0x9004
    assert call(ctypes.byref(f)) == B.WINO_ERR_ALIGN


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        B.lib()


def test_measurement_tools_import_without_a_gpu():
    """The timing tables and the programs that measure the roofline denominators (a plain copy, register-only MFMA
    rates, the fill rate of a compute unit, the operand access pattern as a pure stream) are part of the package: they
    import on a CPU-only box, and the sources they name exist."""
    from paper_2412_05781_amd import calibrate, gputime, timing
    assert calibrate.names() == ["l2_to_lds", "mfma_rates", "operand_stream", "stream"]
    assert callable(timing.main) and callable(gputime.graph_time)


def test_fused_variant_sizes_and_the_entry_points_added_for_it(L):
    """WINO_FUSED_F2 keeps U and V of F(2x2) and has no stored product; the block-shape arguments and the scratch-free
    entry point reject bad input on the host, before any HIP call (this test runs without a GPU)."""
    assert B.WINO_FUSED_F2 == 12
    assert B.wino_filter_bytes(320, 320, B.WINO_F16, B.WINO_FUSED_F2) == B.wino_filter_bytes(320, 320, B.WINO_F16, B.WINO_F2)
    assert B.wino_transformed_dims(2, 320, 64, 64, 320, B.WINO_FUSED_F2) == (4, 320, 2048)
    assert B.wino_workspace_bytes(2, 320, 64, 64, 320, B.WINO_F16, B.WINO_FUSED_F2) == 16 * 2048 * 320 * 2      # V only
    assert B.wino_resolve_variant(2, 320, 64, 64, 320, B.WINO_F16, B.WINO_FUSED_F2) == B.WINO_FUSED_F2
    assert B.wino_resolve_variant(2, 320, 64, 64, 320, B.WINO_F16, 13) == -1
    # WINO_FUSED_F4: U and V of F(4x4), no stored product, two-byte storage types only
    assert B.WINO_FUSED_F4 == 14
    assert B.wino_filter_bytes(320, 320, B.WINO_F16, B.WINO_FUSED_F4) == B.wino_filter_bytes(320, 320, B.WINO_F16, B.WINO_F4)
    assert B.wino_transformed_dims(2, 320, 64, 64, 320, B.WINO_FUSED_F4) == (6, 320, 512)
    assert B.wino_workspace_bytes(2, 320, 64, 64, 320, B.WINO_BF16, B.WINO_FUSED_F4) == 36 * 512 * 320 * 2      # V only
    assert B.wino_resolve_variant(2, 320, 64, 64, 320, B.WINO_F16, B.WINO_FUSED_F4) == B.WINO_FUSED_F4
    assert B.wino_resolve_variant(2, 320, 64, 64, 320, B.WINO_F32, B.WINO_FUSED_F4) == -1
    assert B.wino_filter_bytes(320, 320, B.WINO_F32, B.WINO_FUSED_F4) == 0
    assert B.wino_workspace_bytes(2, 320, 64, 64, 320, B.WINO_F32, B.WINO_FUSED_F4) == 0
    vp = ctypes.c_void_p
    a = vp(0x1000)
    # named block shapes out of range; null and misaligned pointers
    assert L.wino_batched_gemm_shape(a, a, a, 8, 8, 8, B.WINO_F16, B.WINO_F2, 9, None) == B.WINO_ERR_VARIANT
    assert L.wino_batched_gemm_shape(a, a, a, 8, 8, 8, B.WINO_F16, B.WINO_F2, -1, None) == B.WINO_ERR_VARIANT
    assert L.wino_batched_gemm_shape(None, a, a, 8, 8, 8, B.WINO_F16, B.WINO_F2, 0, None) == B.WINO_ERR_NULL
    assert L.wino_batched_gemm_shape(a, a, a, 8, 8, 8, B.WINO_F16, B.WINO_FUSED_F2, 0, None) == B.WINO_ERR_VARIANT
    assert L.wino_batched_gemm(a, a, a, 8, 8, 8, B.WINO_F16, B.WINO_FUSED_F2, None) == B.WINO_ERR_VARIANT
    assert L.wino_fused_gemm_output(a, a, None, a, 1, 8, 4, 4, 8, B.WINO_F16, B.WINO_NCHW, 7, None) == B.WINO_ERR_VARIANT
    assert L.wino_fused_gemm_output(a, None, None, a, 1, 8, 4, 4, 8, B.WINO_F16, B.WINO_NCHW, 0, None) == B.WINO_ERR_NULL
    assert L.wino_fused_gemm_output(a, a, None, a, 1, 8, 4, 4, 8, B.WINO_F16, 5, 0, None) == B.WINO_ERR_LAYOUT
    assert L.wino_fused_gemm_output(a, a, None, vp(0x1008), 1, 8, 4, 4, 8, B.WINO_F16, B.WINO_NCHW, 0, None) == B.WINO_ERR_ALIGN
    assert L.wino_fused_f4_gemm_output(a, a, None, a, 1, 8, 4, 4, 8, B.WINO_F16, B.WINO_NCHW, 2, None) == B.WINO_ERR_VARIANT
    assert L.wino_fused_f4_gemm_output(a, a, None, a, 1, 8, 4, 4, 8, B.WINO_F32, B.WINO_NCHW, 0, None) == B.WINO_ERR_DTYPE
    assert L.wino_fused_f4_gemm_output(a, None, None, a, 1, 8, 4, 4, 8, B.WINO_F16, B.WINO_NCHW, 0, None) == B.WINO_ERR_NULL
    assert L.wino_fused_f4_gemm_output(a, a, None, a, 1, 8, 4, 4, 8, B.WINO_BF16, 5, 0, None) == B.WINO_ERR_LAYOUT
    assert L.wino_fused_gemm_output(a, a, None, a, 0, 8, 4, 4, 8, B.WINO_F16, B.WINO_NCHW, 0, None) == B.WINO_ERR_DIM
    # the scratch-free entry point: limit, and the same validation as wino_conv2d_ex
    assert B.wino_static_scratch_bytes() == 64 << 20
    f = B.wino_filter()
    f.data, f.K, f.C, f.dtype, f.variant = 0x2000, 512, 512, B.WINO_F16, B.WINO_F4
    x, y = vp(0x10000000), vp(0x20000000)
    assert L.wino_conv2d_static(x, ctypes.byref(f), None, y, 1, 512, 128, 128, 512, B.WINO_NCHW, None) == B.WINO_ERR_SCRATCH
    assert L.wino_conv2d_static(None, ctypes.byref(f), None, y, 1, 512, 128, 128, 512, B.WINO_NCHW, None) == B.WINO_ERR_NULL
    assert L.wino_conv2d_static(x, ctypes.byref(f), None, y, 1, 512, 128, 128, 500, B.WINO_NCHW, None) == B.WINO_ERR_DIM
    assert L.wino_conv2d_static(x, ctypes.byref(f), None, y, 1, 512, 8, 8, 512, 7, None) == B.WINO_ERR_LAYOUT
    assert L.wino_conv2d_static(x, ctypes.byref(f), None, x, 1, 512, 8, 8, 512, B.WINO_NCHW, None) == B.WINO_ERR_ALIAS
