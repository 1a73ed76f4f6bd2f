// Calibration: register-only MFMA rates (no memory traffic besides one guarded store): the fp16 32x32x16 step the
// GEMM stages use, the legacy 8-bit 32x32x16 step, and the scaled 8-bit 32x32x64 step the quantised path uses.
#include <hip/hip_runtime.h>
#include <cstdio>
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));
typedef int int8v __attribute__((ext_vector_type(8)));
template <int MODE>
__global__ void __launch_bounds__(256) k(float* out, int iters) {
    half8_t ah, bh;
    for (int i = 0; i < 8; ++i) { ah[i] = (_Float16)1.0f; bh[i] = (_Float16)0.5f; }
    long a = 0x3838383838383838L, b = 0x3030303030303030L;     // E4M3: 1.0 = 0x38, 0.5 = 0x30
    int8v a8, b8;
    for (int i = 0; i < 8; ++i) { a8[i] = 0x38383838; b8[i] = 0x30303030; }
    float16_t c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
    for (int it = 0; it < iters; ++it) {
        if (MODE == 0) {
            c0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bh, c0, 0, 0, 0);
            c1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bh, c1, 0, 0, 0);
            c2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bh, c2, 0, 0, 0);
            c3 = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah, bh, c3, 0, 0, 0);
        } else if (MODE == 1) {
            c0 = __builtin_amdgcn_mfma_f32_32x32x16_fp8_fp8(a, b, c0, 0, 0, 0);
            c1 = __builtin_amdgcn_mfma_f32_32x32x16_fp8_fp8(a, b, c1, 0, 0, 0);
            c2 = __builtin_amdgcn_mfma_f32_32x32x16_fp8_fp8(a, b, c2, 0, 0, 0);
            c3 = __builtin_amdgcn_mfma_f32_32x32x16_fp8_fp8(a, b, c3, 0, 0, 0);
        } else {
            c0 = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, c0, 0, 0, 0, 0x7f7f7f7f, 0, 0x7f7f7f7f);
            c1 = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, c1, 0, 0, 0, 0x7f7f7f7f, 0, 0x7f7f7f7f);
            c2 = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, c2, 0, 0, 0, 0x7f7f7f7f, 0, 0x7f7f7f7f);
            c3 = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, c3, 0, 0, 0, 0x7f7f7f7f, 0, 0x7f7f7f7f);
        }
    }
    float s = 0; for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
    if (s == 12345.678f) out[0] = s;
    if (blockIdx.x == 0 && threadIdx.x == 0 && iters == 1) out[1] = c0[0];      // one step of all-ones x all-halves: K * 0.5
}
template <int MODE> static void run(const char* name, double kdim, float* out) {
    hipEvent_t e0, e1; (void)hipEventCreate(&e0); (void)hipEventCreate(&e1);
    hipLaunchKernelGGL(k<MODE>, dim3(1), dim3(256), 0, 0, out, 1);
    float h[2]; (void)hipMemcpy(h, out, 8, hipMemcpyDeviceToHost);
    printf("%-24s one step of 1.0 x 0.5 -> %g (expected %g)\n", name, h[1], kdim * 0.5);
    for (int blocks : {256, 1024}) {
        const int iters = 20000; float best = 1e9f;
        for (int rep = 0; rep < 3; ++rep) {
            (void)hipEventRecord(e0); hipLaunchKernelGGL(k<MODE>, dim3(blocks), dim3(256), 0, 0, out, iters); (void)hipEventRecord(e1);
            (void)hipEventSynchronize(e1);
            float ms; (void)hipEventElapsedTime(&ms, e0, e1); if (ms < best) best = ms;
        }
        const double flops = (double)blocks * 4 * iters * 4 * 32.0 * 32.0 * kdim * 2.0;
        printf("%-24s %4d workgroups: %9.1f us  %7.1f TFLOP/s\n", name, blocks, best * 1e3, flops / (best * 1e-3) / 1e12);
    }
}
// The same fp16 loop with pseudo-random operands (uniform in [-1, 1], four different register sets in rotation): the
// switching activity of real data.  The chip holds a lower clock under it than with constant operands.
__global__ void __launch_bounds__(256) k_random(float* out, int iters) {
    half8_t a[4], b[4];
    unsigned s = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
    for (int r = 0; r < 4; ++r) for (int i = 0; i < 8; ++i) {
        s = s * 1664525u + 1013904223u; a[r][i] = (_Float16)(((int)(s >> 9) % 2001 - 1000) * 1e-3f);
        s = s * 1664525u + 1013904223u; b[r][i] = (_Float16)(((int)(s >> 9) % 2001 - 1000) * 1e-3f);
    }
    float16_t c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
    for (int it = 0; it < iters; ++it) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[0], b[1], c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[1], b[2], c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[2], b[3], c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[3], b[0], c3, 0, 0, 0);
    }
    float t = 0; for (int i = 0; i < 16; ++i) t += c0[i] + c1[i] + c2[i] + c3[i];
    if (t == 12345.678f) out[0] = t;
}
static void run_random(float* out) {
    hipEvent_t e0, e1; (void)hipEventCreate(&e0); (void)hipEventCreate(&e1);
    for (int blocks : {256, 1024}) {
        const int iters = 20000; float best = 1e9f;
        for (int rep = 0; rep < 3; ++rep) {
            (void)hipEventRecord(e0); hipLaunchKernelGGL(k_random, dim3(blocks), dim3(256), 0, 0, out, iters); (void)hipEventRecord(e1);
            (void)hipEventSynchronize(e1);
            float ms; (void)hipEventElapsedTime(&ms, e0, e1); if (ms < best) best = ms;
        }
        const double flops = (double)blocks * 4 * iters * 4 * 32768.0;
        printf("%-24s %4d workgroups: %9.1f us  %7.1f TFLOP/s\n", "fp16, random operands", blocks, best * 1e3, flops / (best * 1e-3) / 1e12);
    }
}
int main() {
    float* out; (void)hipMalloc(&out, 64); (void)hipMemset(out, 0, 64);
    run<0>("fp16 32x32x16", 16.0, out);
    run_random(out);
    run<1>("fp8 32x32x16 (legacy)", 16.0, out);
    run<2>("fp8 32x32x64 scaled", 64.0, out);
    return 0;
}
