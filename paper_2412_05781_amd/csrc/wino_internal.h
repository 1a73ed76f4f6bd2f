// Internal declarations shared by the HIP sources of libwino (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stddef.h>
#include <stdint.h>

namespace wino {

// Geometry of one Winograd problem (Section "Techniques": steps (i)-(iii)).
struct Geom {
    int N, C, H, W, K;
    int m;        // output tile edge: 2 or 4
    int alpha;    // m + 2
    int th, tw;   // tiles per image column / row
    int T;        // N * th * tw
    int Cp;       // C rounded up to 8 (16-byte rows of U and V)
};

inline int round_up(int v, int q) { return (v + q - 1) / q * q; }

inline Geom make_geom(int N, int C, int H, int W, int K, int m) {
    Geom g;
    g.N = N; g.C = C; g.H = H; g.W = W; g.K = K;
    g.m = m; g.alpha = m + 2;
    g.th = (H + m - 1) / m; g.tw = (W + m - 1) / m;
    g.T = N * g.th * g.tw;
    g.Cp = round_up(C, 8);
    return g;
}

// element conversion helpers usable in kernels
template <typename E> __device__ __forceinline__ float to_f32(E v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<__half>(__half v) { return __half2float(v); }
template <typename E> __device__ __forceinline__ E from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ __half from_f32<__half>(float v) { return __float2half_rn(v); }

// launchers (each enqueues on `s`, returns the launch status)
hipError_t launch_filter_transform(const void* w, void* U, int K, int C, int Cp, int m, bool f16, hipStream_t s);
hipError_t launch_input_transform(const void* x, void* V, const Geom& g, bool f16, bool nhwc, hipStream_t s);
hipError_t launch_batched_gemm(const void* U, const void* V, float* M, int K, int Cp, int T, int nbatch, bool f16, hipStream_t s);
hipError_t launch_output_transform(const float* M, const float* bias, void* y, const Geom& g, bool f16, bool nhwc, hipStream_t s);
hipError_t launch_direct_conv2d(const void* x, const void* w, const float* bias, void* y,
                                int N, int C, int H, int W, int K, bool f16, hipStream_t s);

}  // namespace wino
