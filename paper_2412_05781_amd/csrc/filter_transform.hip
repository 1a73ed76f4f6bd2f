// Step (i), filter side (Section "Techniques"): U = G g G^T for every (k,c),
// written tile-major as U[alpha^2][K][Cp] so each of the alpha^2 matrices is a
// dense row-major [K x Cp] GEMM operand with the reduction index contiguous.
// Runs once per weight tensor; bound by HBM traffic (reads 9, writes alpha^2 values).
#include "wino_internal.h"
#include "wino_transforms.h"

namespace wino {

template <int M, typename E>
__global__ void __launch_bounds__(256)
filter_transform_kernel(const E* __restrict__ w, E* __restrict__ U, int K, int C, int Cp) {
    constexpr int A = M + 2;
    const int c = blockIdx.x * blockDim.x + threadIdx.x;   // fastest: contiguous stores along c
    const int k = blockIdx.y;
    if (c >= Cp) return;
    float g[3][3];
    if (c < C) {
        const E* p = w + ((size_t)k * C + c) * 9;
#pragma unroll
        for (int r = 0; r < 3; ++r)
#pragma unroll
            for (int s = 0; s < 3; ++s) g[r][s] = to_f32<E>(p[r * 3 + s]);
    } else {
#pragma unroll
        for (int r = 0; r < 3; ++r)
#pragma unroll
            for (int s = 0; s < 3; ++s) g[r][s] = 0.f;   // padded reduction columns must be exact zeros
    }
    // columns: tmp[:, s] = G * g[:, s]
    float tmp[A][3];
#pragma unroll
    for (int s = 0; s < 3; ++s) {
        float in[3] = {g[0][s], g[1][s], g[2][s]}, out[A];
        g_1d<M>(in, out);
#pragma unroll
        for (int a = 0; a < A; ++a) tmp[a][s] = out[a];
    }
    // rows: U[xi, :] = G * tmp[xi, :]
    const size_t plane = (size_t)K * Cp;
    E* dst = U + (size_t)k * Cp + c;
#pragma unroll
    for (int xi = 0; xi < A; ++xi) {
        float out[A];
        g_1d<M>(tmp[xi], out);
#pragma unroll
        for (int nu = 0; nu < A; ++nu) dst[(size_t)(xi * A + nu) * plane] = from_f32<E>(out[nu]);
    }
}

hipError_t launch_filter_transform(const void* w, void* U, int K, int C, int Cp, int m, int dt, hipStream_t s) {
    dim3 block(256), grid((Cp + 255) / 256, K);
    return with_dtype(dt, [&](auto* tag) {
        using E = std::remove_pointer_t<decltype(tag)>;
        if (m == 2) hipLaunchKernelGGL((filter_transform_kernel<2, E>), grid, block, 0, s, (const E*)w, (E*)U, K, C, Cp);
        else        hipLaunchKernelGGL((filter_transform_kernel<4, E>), grid, block, 0, s, (const E*)w, (E*)U, K, C, Cp);
        return hipGetLastError();
    });
}

}  // namespace wino
