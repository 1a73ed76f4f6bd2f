// Host sanitizer run of the C-ABI layer (csrc/wino_api.hip compiled with AddressSanitizer and
// UndefinedBehaviorSanitizer on the host side): every size query and every pre-launch error path, i.e. all the code
// that runs before a kernel is enqueued.  No call here reaches a HIP launch, so it runs without a GPU.
// Built and run by tests/test_sanitizers.py; test infrastructure only.
#include <cstdio>
#include <cstdint>
#include "wino.h"

#define CHECK(expr, want) do { long long got_ = (long long)(expr); if (got_ != (long long)(want)) { \
    std::printf("line %d: %s = %lld, expected %lld\n", __LINE__, #expr, got_, (long long)(want)); return 1; } } while (0)

int main() {
    void* a = reinterpret_cast<void*>(0x10000000);
    void* b = reinterpret_cast<void*>(0x20000000);
    void* odd = reinterpret_cast<void*>(0x10000008);
    CHECK(wino_version() >= 100, 1);
    for (int s = -2; s < 14; ++s) if (!wino_status_string(s)) return 2;
    // sizes
    CHECK(wino_filter_bytes(320, 320, WINO_F16, WINO_F4), 36LL * 320 * 320 * 2);
    CHECK(wino_filter_bytes(320, 320, WINO_F16, WINO_FUSED_F2), 16LL * 320 * 320 * 2);
    CHECK(wino_filter_bytes(320, 320, WINO_F16, WINO_AUTO), 0);
    CHECK(wino_filter_bytes(-1, 320, WINO_F16, WINO_F2), 0);
    CHECK(wino_filter_bytes(1 << 30, 1 << 30, WINO_F32, WINO_F4), 0);
    CHECK(wino_workspace_bytes(2, 320, 64, 64, 320, WINO_F16, WINO_F4), 36LL * 512 * 320 * 2 + 36LL * 320 * 512 * 4);
    CHECK(wino_workspace_bytes(2, 320, 64, 64, 320, WINO_F16, WINO_FUSED_F2), 16LL * 2048 * 320 * 2);
    CHECK(wino_workspace_bytes(2, 320, 64, 64, 320, 9, WINO_F4), 0);
    CHECK(wino_workspace_bytes(1 << 20, 1 << 20, 1 << 20, 1 << 20, 1 << 20, WINO_F16, WINO_F4), 0);
    CHECK(wino_workspace_bytes(2, 320, 64, 64, 320, WINO_F16, WINO_DIRECT) > 0, 1);
    CHECK(wino_igemm_filter_bytes(64, 40, 3, WINO_F16), (9LL * 64 * 40 + 40) * 2);
    CHECK(wino_igemm_workspace_bytes(1, 40, 9, 9, 64, 3, 2, WINO_F16, WINO_NCHW) > 0, 1);
    CHECK(wino_igemm_workspace_bytes(1, 40, 9, 9, 64, 5, 2, WINO_F16, WINO_NCHW), 0);
    CHECK(wino_fp8_filter_bytes(64, 40, 3), 9LL * 64 * 48 + 48);
    CHECK(wino_fp8_workspace_bytes(1, 40, 9, 9, 64, 3, 1) > 0, 1);
    CHECK(wino_i8_filter_bytes(64, 40), 16LL * 64 * 48 + 16LL * 64 * 4);
    CHECK(wino_i8_filter_bytes(64, 70000), 0);
    CHECK(wino_i8_workspace_bytes(1, 40, 8, 8, 64), 16LL * 16 * 48 + 16LL * 16 * 4 + 16LL * 64 * 16 * 4);
    CHECK(wino_i8_workspace_bytes(1, 40, 0, 8, 64), 0);
    CHECK(wino_groupnorm_stats_bytes(2, 32) > 0, 1);
    CHECK(wino_groupnorm_stats_bytes(0, 32), 0);
    CHECK(wino_static_scratch_bytes(), 64LL << 20);
    int alpha = 0, Cp = 0, T = 0;
    CHECK(wino_transformed_dims(1, 5, 7, 9, 3, WINO_F4, &alpha, &Cp, &T), WINO_OK);
    CHECK(alpha == 6 && Cp == 8 && T == 6, 1);
    CHECK(wino_transformed_dims(1, 5, 7, 9, 3, WINO_F4, nullptr, nullptr, nullptr), WINO_OK);
    CHECK(wino_transformed_dims(1, 5, 7, 9, 3, WINO_AUTO, &alpha, &Cp, &T), WINO_ERR_VARIANT);
    CHECK(wino_resolve_variant(2, 320, 64, 64, 320, WINO_F16, WINO_AUTO) > 0, 1);
    CHECK(wino_resolve_variant(2, 320, 64, 64, 320, WINO_F16, 13), -1);
    CHECK(wino_recommend_variant(1, 128, 1024, 1024, 128, WINO_F16), WINO_FUSED_F4);
    CHECK(wino_recommend_variant(1, 128, 256, 256, 128, WINO_F16), WINO_DIRECT);
    CHECK(wino_resolve_variant(1, 128, 1024, 1024, 128, WINO_F32, WINO_FUSED_F4), -1);
    CHECK(wino_workspace_bytes(1, 128, 64, 64, 128, WINO_F16, WINO_FUSED_F4), 36LL * 256 * 128 * 2);
    CHECK(wino_fused_f4_gemm_output(a, a, nullptr, b, 1, 8, 4, 4, 8, WINO_F32, WINO_NCHW, 0, nullptr), WINO_ERR_DTYPE);
    // pre-launch error paths of every entry point
    wino_filter f{a, 320, 320, WINO_F16, WINO_F4};
    CHECK(wino_filter_transform(nullptr, a, 8, 8, WINO_F16, WINO_F2, &f, nullptr), WINO_ERR_NULL);
    CHECK(wino_filter_transform(a, b, 8, 8, 7, WINO_F2, &f, nullptr), WINO_ERR_DTYPE);
    CHECK(wino_filter_transform(a, b, 8, 8, WINO_F16, WINO_AUTO, &f, nullptr), WINO_ERR_VARIANT);
    CHECK(wino_filter_transform(a, odd, 8, 8, WINO_F16, WINO_F2, &f, nullptr), WINO_ERR_ALIGN);
    CHECK(wino_filter_transform(a, b, 0, 8, WINO_F16, WINO_F2, &f, nullptr), WINO_ERR_DIM);
    f = wino_filter{a, 320, 320, WINO_F16, WINO_F4};
    CHECK(wino_conv2d(nullptr, &f, nullptr, b, 2, 320, 64, 64, 320, nullptr), WINO_ERR_NULL);
    CHECK(wino_conv2d(a, &f, nullptr, b, 2, 320, 64, 64, 321, nullptr), WINO_ERR_DIM);
    CHECK(wino_conv2d(a, &f, nullptr, a, 2, 320, 64, 64, 320, nullptr), WINO_ERR_ALIAS);
    CHECK(wino_conv2d_ex(a, &f, nullptr, b, 2, 320, 64, 64, 320, WINO_NCHW, nullptr, 0, nullptr), WINO_ERR_WORKSPACE);
    CHECK(wino_conv2d_ex(a, &f, nullptr, b, 2, 320, 64, 64, 320, 5, a, 1, nullptr), WINO_ERR_LAYOUT);
    CHECK(wino_conv2d_ex(a, &f, reinterpret_cast<const float*>(0x30000002), b, 2, 320, 64, 64, 320, WINO_NCHW, a, 1, nullptr), WINO_ERR_ALIGN);
    CHECK(wino_conv2d_static(a, &f, nullptr, b, 1, 320, 256, 256, 320, WINO_NCHW, nullptr), WINO_ERR_SCRATCH);
    wino_fusion fu{};
    fu.upsample = 2;
    CHECK(wino_conv2d_fused(a, &f, nullptr, b, 2, 320, 64, 64, 320, WINO_NCHW, &fu, a, 1, nullptr), WINO_ERR_DIM);
    fu.upsample = 0; fu.gn_stats = reinterpret_cast<const float*>(a);
    CHECK(wino_conv2d_fused(a, &f, nullptr, b, 2, 320, 64, 64, 320, WINO_NCHW, &fu, a, 1, nullptr), WINO_ERR_NULL);
    CHECK(wino_conv2d_fused(a, &f, nullptr, b, 2, 320, 64, 64, 320, WINO_NCHW, nullptr, a, 1, nullptr), WINO_ERR_NULL);
    CHECK(wino_input_transform(a, nullptr, 1, 8, 8, 8, WINO_F16, WINO_F2, WINO_NCHW, nullptr), WINO_ERR_NULL);
    CHECK(wino_batched_gemm(a, a, reinterpret_cast<float*>(b), 8, 8, 8, WINO_F16, WINO_FUSED_F2, nullptr), WINO_ERR_VARIANT);
    CHECK(wino_batched_gemm_shape(a, a, reinterpret_cast<float*>(b), 8, 8, 8, WINO_F16, WINO_F2, 9, nullptr), WINO_ERR_VARIANT);
    CHECK(wino_output_transform(reinterpret_cast<const float*>(a), nullptr, b, 1, 8, 0, 8, WINO_F16, WINO_F2, WINO_NCHW, nullptr), WINO_ERR_DIM);
    CHECK(wino_fused_gemm_output(a, a, nullptr, b, 1, 8, 4, 4, 8, WINO_F16, WINO_NCHW, 7, nullptr), WINO_ERR_VARIANT);
    CHECK(wino_direct_conv2d(a, a, nullptr, a, 1, 8, 8, 8, 8, WINO_F16, nullptr), WINO_ERR_ALIAS);
    CHECK(wino_groupnorm_stats(a, reinterpret_cast<float*>(b), 1, 30, 8, 8, 4, 1e-5f, WINO_F16, WINO_NCHW, nullptr), WINO_ERR_DIM);
    CHECK(wino_igemm_filter_repack(a, b, 8, 8, 2, WINO_F16, nullptr), WINO_ERR_DIM);
    CHECK(wino_igemm_conv2d(a, a, nullptr, b, 1, 8, 8, 8, 8, 3, 3, WINO_F16, WINO_NCHW, nullptr, 0, nullptr), WINO_ERR_DIM);
    CHECK(wino_igemm_conv2d(a, a, nullptr, b, 1, 8, 8, 8, 8, 3, 1, WINO_F16, WINO_NCHW, nullptr, 0, nullptr), WINO_ERR_WORKSPACE);
    CHECK(wino_fp8_filter_quantize(a, b, 8, 8, 3, WINO_F16, -1.f, nullptr), WINO_ERR_DIM);
    CHECK(wino_fp8_conv2d(a, a, nullptr, b, 1, 8, 8, 8, 8, 3, 1, WINO_F16, WINO_NCHW, 0.f, 1.f, nullptr, a, 1 << 20, nullptr), WINO_ERR_DIM);
    CHECK(wino_i8_filter_transform(a, nullptr, 8, 8, WINO_F16, nullptr), WINO_ERR_NULL);
    CHECK(wino_i8_filter_transform(a, b, 8, 70000, WINO_F16, nullptr), WINO_ERR_DIM);
    CHECK(wino_i8_input_transform(a, b, reinterpret_cast<float*>(b), 1, 8, 8, 8, 7, WINO_NCHW, nullptr), WINO_ERR_DTYPE);
    CHECK(wino_i8_batched_gemm(a, reinterpret_cast<const float*>(a), a, reinterpret_cast<const float*>(a), reinterpret_cast<float*>(b), 8, 8, 8, 9, nullptr), WINO_ERR_VARIANT);
    CHECK(wino_i8_conv2d(a, a, nullptr, b, 1, 8, 8, 8, 8, WINO_F16, WINO_NCHW, nullptr, 0, nullptr), WINO_ERR_WORKSPACE);
    CHECK(wino_i8_conv2d(a, a, nullptr, a, 1, 8, 8, 8, 8, WINO_F16, WINO_NCHW, b, 1 << 20, nullptr), WINO_ERR_ALIAS);
    CHECK(wino_i8_conv2d(a, a, nullptr, b, 1, 8, 8, 8, 8, WINO_F16, 5, b, 1 << 20, nullptr), WINO_ERR_LAYOUT);
    std::printf("abi sanitizer run ok\n");
    return 0;
}
