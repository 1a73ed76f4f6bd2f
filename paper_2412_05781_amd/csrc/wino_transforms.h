// 1-D Winograd transforms F(m,3), m in {2,4}, as straight-line fp32 code.
// The 2-D transforms of steps (i) and (iii) (Section "Techniques") apply these
// along columns, then along rows.  Matrices: the minimal-filtering triples for
// the points {0,+-1,inf} (m=2) and {0,+-1,+-2,inf} (m=4).
#pragma once
#include <hip/hip_runtime.h>

namespace wino {

// out = B^T * in   (in, out: alpha values, stride 1 in registers)
template <int M> __device__ __forceinline__ void bt_1d(const float* in, float* out);
template <> __device__ __forceinline__ void bt_1d<2>(const float* d, float* o) {
    o[0] = d[0] - d[2];
    o[1] = d[1] + d[2];
    o[2] = d[2] - d[1];
    o[3] = d[1] - d[3];
}
template <> __device__ __forceinline__ void bt_1d<4>(const float* d, float* o) {
    o[0] = 4.f * d[0] - 5.f * d[2] + d[4];
    o[1] = -4.f * (d[1] + d[2]) + d[3] + d[4];
    o[2] = 4.f * (d[1] - d[2]) - d[3] + d[4];
    o[3] = 2.f * (d[3] - d[1]) - d[2] + d[4];
    o[4] = 2.f * (d[1] - d[3]) - d[2] + d[4];
    o[5] = 4.f * d[1] - 5.f * d[3] + d[5];
}

// out = G * in   (in: 3 values, out: alpha values)
template <int M> __device__ __forceinline__ void g_1d(const float* in, float* out);
template <> __device__ __forceinline__ void g_1d<2>(const float* g, float* o) {
    o[0] = g[0];
    o[1] = 0.5f * (g[0] + g[1] + g[2]);
    o[2] = 0.5f * (g[0] - g[1] + g[2]);
    o[3] = g[2];
}
template <> __device__ __forceinline__ void g_1d<4>(const float* g, float* o) {
    const float s = g[0] + g[2];
    o[0] = 0.25f * g[0];
    o[1] = (-1.f / 6.f) * (s + g[1]);
    o[2] = (-1.f / 6.f) * (s - g[1]);
    const float q = (1.f / 24.f) * g[0] + (1.f / 6.f) * g[2];
    o[3] = q + (1.f / 12.f) * g[1];
    o[4] = q - (1.f / 12.f) * g[1];
    o[5] = g[2];
}

// out = A^T * in   (in: alpha values, out: m values)
template <int M> __device__ __forceinline__ void at_1d(const float* in, float* out);
template <> __device__ __forceinline__ void at_1d<2>(const float* v, float* o) {
    o[0] = v[0] + v[1] + v[2];
    o[1] = v[1] - v[2] - v[3];
}
template <> __device__ __forceinline__ void at_1d<4>(const float* v, float* o) {
    const float p = v[1] + v[2], q = v[1] - v[2];
    const float r = v[3] + v[4], s = v[3] - v[4];
    o[0] = v[0] + p + r;
    o[1] = q + 2.f * s;
    o[2] = p + 4.f * r;
    o[3] = q + 8.f * s + v[5];
}

}  // namespace wino
