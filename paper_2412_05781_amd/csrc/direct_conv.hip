// Checking fallback: direct 3x3 / stride 1 / zero-pad 1 cross-correlation on the
// GPU from the untransformed filter — the operator the Winograd path replaces
// (Section "Techniques").  One thread per output element, fp32 accumulation in
// the order c, r, s.  Not a fast path.
#include "wino_internal.h"

namespace wino {

template <typename E>
__global__ void __launch_bounds__(256)
direct_conv2d_kernel(const E* __restrict__ x, const E* __restrict__ w, const float* __restrict__ bias,
                     E* __restrict__ y, int N, int C, int H, int W, int K) {
    const size_t total = (size_t)N * K * H * W;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t f = (size_t)blockIdx.x * blockDim.x + threadIdx.x; f < total; f += stride) {
        size_t q = f;
        const int j = (int)(q % W); q /= W;
        const int i = (int)(q % H); q /= H;
        const int k = (int)(q % K); q /= K;
        const int n = (int)q;
        float acc = bias ? bias[k] : 0.f;
        for (int c = 0; c < C; ++c) {
            const E* xp = x + ((size_t)n * C + c) * H * W;
            const E* wp = w + ((size_t)k * C + c) * 9;
#pragma unroll
            for (int r = 0; r < 3; ++r) {
                const int ii = i + r - 1;
                if (ii < 0 || ii >= H) continue;
#pragma unroll
                for (int s = 0; s < 3; ++s) {
                    const int jj = j + s - 1;
                    if (jj < 0 || jj >= W) continue;
                    acc = fmaf(to_f32<E>(xp[(size_t)ii * W + jj]), to_f32<E>(wp[r * 3 + s]), acc);
                }
            }
        }
        y[f] = from_f32<E>(acc);
    }
}

hipError_t launch_direct_conv2d(const void* x, const void* w, const float* bias, void* y,
                                int N, int C, int H, int W, int K, int dt, hipStream_t s) {
    const size_t total = (size_t)N * K * H * W;
    size_t blocks = (total + 255) / 256;
    if (blocks > (size_t)1 << 20) blocks = (size_t)1 << 20;   // grid-stride beyond that
    dim3 block(256), grid((unsigned)blocks);
    return with_dtype(dt, [&](auto* tag) {
        using E = std::remove_pointer_t<decltype(tag)>;
        hipLaunchKernelGGL((direct_conv2d_kernel<E>), grid, block, 0, s, (const E*)x, (const E*)w, bias, (E*)y, N, C, H, W, K);
        return hipGetLastError();
    });
}

}  // namespace wino
