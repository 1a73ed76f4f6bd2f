// Step (iii) (Section "Techniques"): y tile = A^T M A per (k, tile), plus bias,
// cropped to the image, rounded once to the storage type.
// NCHW: one lane per (k, t), t fastest, so the alpha^2 reads of M[alpha^2][K][T] are
// contiguous across lanes and the m-wide row stores of neighbouring tiles abut.
// Channel-last: the product arrives transposed, M[alpha^2][T][K], one lane per
// (t, channel pair), so reads and writes both run along k.
// Both also add the optional per-(image, channel) vector and the residual, sum the
// partial products of a split reduction, and can read M stored as fp16.
// Bound by HBM/L2 traffic: reads alpha^2 fp32 per m^2 outputs.
#include "wino_internal.h"
#include <type_traits>
#include "wino_transforms.h"

namespace wino {

template <typename E, int M> struct RowVec;
template <> struct RowVec<float, 2> { using type = float2; };
template <> struct RowVec<float, 4> { using type = float4; };
template <> struct RowVec<__half, 2> { using type = uint32_t; };
template <> struct RowVec<__half, 4> { using type = uint2; };
template <> struct RowVec<bf16_t, 2> { using type = uint32_t; };
template <> struct RowVec<bf16_t, 4> { using type = uint2; };
// two 16-bit elements in one word, first element in the low half
template <typename E> __device__ __forceinline__ uint32_t pack2(float a, float b) {
    const E ea = from_f32<E>(a), eb = from_f32<E>(b);
    return (uint32_t)*reinterpret_cast<const uint16_t*>(&ea) | ((uint32_t)*reinterpret_cast<const uint16_t*>(&eb) << 16);
}
template <typename E> __device__ __forceinline__ float unpack_lo(uint32_t w) { const uint16_t h = (uint16_t)(w & 0xffffu); return to_f32<E>(*reinterpret_cast<const E*>(&h)); }
template <typename E> __device__ __forceinline__ float unpack_hi(uint32_t w) { const uint16_t h = (uint16_t)(w >> 16); return to_f32<E>(*reinterpret_cast<const E*>(&h)); }

template <typename E, int M>
__device__ __forceinline__ void store_row(E* p, const float* v) {
    typename RowVec<E, M>::type r;
    if constexpr (sizeof(E) == 4) {
        if constexpr (M == 2) { r.x = v[0]; r.y = v[1]; }
        else { r.x = v[0]; r.y = v[1]; r.z = v[2]; r.w = v[3]; }
    } else {
        if constexpr (M == 2) { r = pack2<E>(v[0], v[1]); }
        else { r.x = pack2<E>(v[0], v[1]); r.y = pack2<E>(v[2], v[3]); }
    }
    *reinterpret_cast<typename RowVec<E, M>::type*>(p) = r;
}

// residual row of m elements (same vector type as the store), added in fp32
template <typename E, int M>
__device__ __forceinline__ void add_row(const E* p, float* v) {
    const typename RowVec<E, M>::type r = *reinterpret_cast<const typename RowVec<E, M>::type*>(p);
    if constexpr (sizeof(E) == 4) {
        if constexpr (M == 2) { v[0] += r.x; v[1] += r.y; }
        else { v[0] += r.x; v[1] += r.y; v[2] += r.z; v[3] += r.w; }
    } else {
        if constexpr (M == 2) { v[0] += unpack_lo<E>(r); v[1] += unpack_hi<E>(r); }
        else { v[0] += unpack_lo<E>(r.x); v[1] += unpack_hi<E>(r.x); v[2] += unpack_lo<E>(r.y); v[3] += unpack_hi<E>(r.y); }
    }
}

template <int TPT> struct FVec;
template <> struct FVec<1> { using type = float; };
template <> struct FVec<2> { using type = float2; };
template <> struct FVec<4> { using type = float4; };

// One lane handles TPT consecutive tiles of one output channel (TPT divides T), so each of the
// alpha^2 reads is a TPT*4-byte vector and a wave reads TPT*256 contiguous bytes per plane.
// MT = type the product is stored in (float; __half in the half-product mode, one tile per lane only).
template <int M, typename E, int TPT, typename MT>
__global__ void __launch_bounds__(256)
output_transform_nchw_kernel(const MT* __restrict__ Mt, const float* __restrict__ bias, E* __restrict__ y,
                             int N, int K, int H, int W, int th, int tw, int T, int vec_ok, int nsplit, PostOp post) {
    constexpr int A = M + 2;
    const size_t KT = (size_t)K * T;
    const int Tq = T / TPT;
    const size_t fq = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (fq >= (size_t)K * Tq) return;
    const int k = (int)(fq / Tq);
    const int t0 = (int)(fq - (size_t)k * Tq) * TPT;
    const size_t f = (size_t)k * T + t0;

    float v[A * A][TPT];
    if constexpr (sizeof(MT) == 2) {
        static_assert(sizeof(MT) == 4 || TPT == 1, "half product: one tile per lane");
#pragma unroll
        for (int p = 0; p < A * A; ++p) {
            const unsigned short h = load_stream(reinterpret_cast<const unsigned short*>(Mt + (size_t)p * KT + f));   // read once
            v[p][0] = to_f32<MT>(*reinterpret_cast<const MT*>(&h));
        }
    } else {
#pragma unroll
        for (int p = 0; p < A * A; ++p) {
            if constexpr (TPT == 1) {
                v[p][0] = load_stream(Mt + (size_t)p * KT + f);          // the product is read once
            } else {
                const typename FVec<TPT>::type q = *reinterpret_cast<const typename FVec<TPT>::type*>(Mt + (size_t)p * KT + f);
                const float* qf = reinterpret_cast<const float*>(&q);
#pragma unroll
                for (int u = 0; u < TPT; ++u) v[p][u] = qf[u];
            }
        }
        // partial products of a reduction cut into nsplit ranges: summed here, in a fixed order
        for (int sp = 1; sp < nsplit; ++sp) {
            const MT* Ms = Mt + (size_t)sp * (A * A) * KT + f;
#pragma unroll
            for (int p = 0; p < A * A; ++p) {
                const typename FVec<TPT>::type q = *reinterpret_cast<const typename FVec<TPT>::type*>(Ms + (size_t)p * KT);
                const float* qf = reinterpret_cast<const float*>(&q);
#pragma unroll
                for (int u = 0; u < TPT; ++u) v[p][u] += qf[u];
            }
        }
    }
    const float b = bias ? bias[k] : 0.f;
#pragma unroll
    for (int u = 0; u < TPT; ++u) {
        int t = t0 + u;
        const int tj = t % tw; t /= tw;
        const int ti = t % th;
        const int n = t / th;
        // columns: tmp[:, nu] = A^T v[:, nu]
        float tmp[M][A];
#pragma unroll
        for (int nu = 0; nu < A; ++nu) {
            float in[A], out[M];
#pragma unroll
            for (int xi = 0; xi < A; ++xi) in[xi] = v[xi * A + nu][u];
            at_1d<M>(in, out);
#pragma unroll
            for (int a = 0; a < M; ++a) tmp[a][nu] = out[a];
        }
        const int i0 = M * ti, j0 = M * tj;
        const size_t yoff = (((size_t)n * K + k) * H + i0) * W + j0;
        E* yp = y + yoff;
        const E* rp = post.residual ? static_cast<const E*>(post.residual) + yoff : nullptr;
        const float bb = b + (post.addvec ? post.addvec[(size_t)n * K + k] : 0.f);
#pragma unroll
        for (int a = 0; a < M; ++a) {
            float out[M];
            at_1d<M>(tmp[a], out);
#pragma unroll
            for (int q = 0; q < M; ++q) out[q] += bb;
            if (i0 + a < H) {
                if (vec_ok) {
                    if (rp) add_row<E, M>(rp + (size_t)a * W, out);
                    store_row<E, M>(yp + (size_t)a * W, out);
                } else {
#pragma unroll
                    for (int q = 0; q < M; ++q)
                        if (j0 + q < W) yp[(size_t)a * W + q] = from_f32<E>(out[q] + (rp ? to_f32<E>(rp[(size_t)a * W + q]) : 0.f));
                }
            }
        }
    }
}

template <int M, typename E, int TPT, typename MT = float>
static hipError_t launch_ot_cfg(const MT* Mt, const float* bias, void* y, const Geom& g, int nsplit, const PostOp& post, hipStream_t s) {
    const size_t items = (size_t)g.K * (g.T / TPT);
    dim3 block(256), grid((unsigned)((items + 255) / 256));
    const int vec_ok = (g.W % M == 0) && ((reinterpret_cast<uintptr_t>(y) & 15u) == 0) &&
                       ((reinterpret_cast<uintptr_t>(post.residual) & 15u) == 0);
    hipLaunchKernelGGL((output_transform_nchw_kernel<M, E, TPT, MT>), grid, block, 0, s,
                       Mt, bias, (E*)y, g.N, g.K, g.H, g.W, g.th, g.tw, g.T, vec_ok, nsplit, post);
    return hipGetLastError();
}

template <int M, typename E>
static hipError_t launch_ot(const float* Mt, const float* bias, void* y, const Geom& g, int nsplit, const PostOp& post, hipStream_t s) {
    // measured over the layer sweep: one tile per lane is never worse than two or four in the chained path
    return launch_ot_cfg<M, E, 1>(Mt, bias, y, g, nsplit, post, s);
}

// NHWC output (y[N][H][W][K], channels contiguous).  Here the product arrives transposed,
// Mt[alpha^2][T][K] (the batched GEMM is symmetric in its operands: called with V and U swapped it
// leaves the channel index contiguous), so reads and writes both run along k and nothing has to be
// transposed on the way.  One lane owns KPT adjacent channels of one tile.
template <int M, typename E, int KPT, typename MT>
__global__ void __launch_bounds__(256)
output_transform_nhwc_kernel(const MT* __restrict__ Mt, const float* __restrict__ bias, E* __restrict__ y,
                             int N, int K, int H, int W, int th, int tw, int T, int nsplit, PostOp post) {
    constexpr int A = M + 2;
    const int groups = (K + KPT - 1) / KPT;
    const size_t item = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (item >= (size_t)T * groups) return;
    const int k = (int)(item % groups) * KPT;                  // KPT divides K on this path
    const int t = (int)(item / groups);
    const int tj = t % tw; const int q0 = t / tw;
    const int ti = q0 % th;
    const int n = q0 / th;
    const size_t TK = (size_t)T * K;
    const MT* src = Mt + (size_t)t * K + k;
    float v[KPT][A][A];
#pragma unroll
    for (int xi = 0; xi < A; ++xi)
#pragma unroll
        for (int nu = 0; nu < A; ++nu) {
            const MT* p = src + (size_t)(xi * A + nu) * TK;
            // the product is read once: streaming loads
            if constexpr (sizeof(MT) == 2) {
                if constexpr (KPT == 2) {
                    const uint32_t w = load_stream(reinterpret_cast<const uint32_t*>(p));
                    const float2 f = __half22float2(*reinterpret_cast<const __half2*>(&w));
                    v[0][xi][nu] = f.x; v[1][xi][nu] = f.y;
                } else {
                    const unsigned short h = load_stream(reinterpret_cast<const unsigned short*>(p));
                    v[0][xi][nu] = to_f32<MT>(*reinterpret_cast<const MT*>(&h));
                }
            } else {
                if constexpr (KPT == 2) {
                    typedef float f32x2_t __attribute__((ext_vector_type(2)));
                    const f32x2_t f = load_stream(reinterpret_cast<const f32x2_t*>(p));
                    v[0][xi][nu] = f.x; v[1][xi][nu] = f.y;
                } else v[0][xi][nu] = load_stream(reinterpret_cast<const float*>(p));
            }
        }
    if constexpr (sizeof(MT) == 4) {
        for (int sp = 1; sp < nsplit; ++sp) {                  // partial products, summed in a fixed order
            const float* ss = src + (size_t)sp * (A * A) * TK;
#pragma unroll
            for (int xi = 0; xi < A; ++xi)
#pragma unroll
                for (int nu = 0; nu < A; ++nu) {
                    const float* p = ss + (size_t)(xi * A + nu) * TK;
                    if constexpr (KPT == 2) { const float2 f = *reinterpret_cast<const float2*>(p); v[0][xi][nu] += f.x; v[1][xi][nu] += f.y; }
                    else v[0][xi][nu] += p[0];
                }
        }
    }
    // residual: loaded up front from clamped (always valid) positions so that the loads overlap;
    // positions outside the image are never stored
    // KPT channels move as one 4- or 8-byte word
    union Pack { E e[KPT]; typename std::conditional<sizeof(E) * KPT == 8, uint2, typename std::conditional<sizeof(E) * KPT == 4, uint32_t, uint16_t>::type>::type w; };
    Pack res[M][M];
    if (post.residual) {
        const E* rb = static_cast<const E*>(post.residual) + (size_t)n * H * W * K + k;
#pragma unroll
        for (int a = 0; a < M; ++a)
#pragma unroll
            for (int q = 0; q < M; ++q) {
                const E* p = rb + ((size_t)min(M * ti + a, H - 1) * W + min(M * tj + q, W - 1)) * K;
                res[a][q].w = *reinterpret_cast<const decltype(Pack::w)*>(p);
            }
    }
    float b[KPT];
#pragma unroll
    for (int u = 0; u < KPT; ++u)
        b[u] = (bias ? bias[k + u] : 0.f) + (post.addvec ? post.addvec[(size_t)n * K + k + u] : 0.f);
    float out[KPT][M][M];
#pragma unroll
    for (int u = 0; u < KPT; ++u) {
        float tmp[M][A];
#pragma unroll
        for (int nu = 0; nu < A; ++nu) {
            float in[A], o[M];
#pragma unroll
            for (int xi = 0; xi < A; ++xi) in[xi] = v[u][xi][nu];
            at_1d<M>(in, o);
#pragma unroll
            for (int a = 0; a < M; ++a) tmp[a][nu] = o[a];
        }
#pragma unroll
        for (int a = 0; a < M; ++a) at_1d<M>(tmp[a], out[u][a]);
    }
    E* yb = y + (size_t)n * H * W * K + k;
#pragma unroll
    for (int a = 0; a < M; ++a) {
        const int i = M * ti + a;
#pragma unroll
        for (int q = 0; q < M; ++q) {
            const int j = M * tj + q;
            if (i < H && j < W) {
                Pack o;
#pragma unroll
                for (int u = 0; u < KPT; ++u) {
                    float f = out[u][a][q] + b[u];
                    if (post.residual) f += to_f32<E>(res[a][q].e[u]);
                    o.e[u] = from_f32<E>(f);
                }
                *reinterpret_cast<decltype(Pack::w)*>(yb + ((size_t)i * W + j) * K) = o.w;
            }
        }
    }
}

template <int M, typename E, typename MT = float>
static hipError_t launch_ot_nhwc(const MT* Mt, const float* bias, void* y, const Geom& g, int nsplit, const PostOp& post, hipStream_t s) {
    const bool pair = g.K % 2 == 0;               // rows of Mt, y and the residual then keep channel pairs aligned
    const size_t items = (size_t)g.T * ((g.K + (pair ? 1 : 0)) / (pair ? 2 : 1));
    const size_t blocks = (items + 255) / 256;
    if (blocks > 0x7fffffffULL) return hipErrorInvalidValue;
    if (pair) hipLaunchKernelGGL((output_transform_nhwc_kernel<M, E, 2, MT>), dim3((unsigned)blocks), dim3(256), 0, s,
                                 Mt, bias, (E*)y, g.N, g.K, g.H, g.W, g.th, g.tw, g.T, nsplit, post);
    else      hipLaunchKernelGGL((output_transform_nhwc_kernel<M, E, 1, MT>), dim3((unsigned)blocks), dim3(256), 0, s,
                                 Mt, bias, (E*)y, g.N, g.K, g.H, g.W, g.th, g.tw, g.T, nsplit, post);
    return hipGetLastError();
}

hipError_t launch_output_transform(const void* Mv, const float* bias, void* y, const Geom& g, int nsplit, int dt, bool nhwc,
                                   bool half_product, const PostOp* postp, hipStream_t s) {
    const PostOp post = postp ? *postp : PostOp();
    if (half_product) {
        if (dt != DT_F16 || nsplit != 1) return hipErrorInvalidValue;
        const __half* Mh = static_cast<const __half*>(Mv);
        if (nhwc) return g.m == 2 ? launch_ot_nhwc<2, __half, __half>(Mh, bias, y, g, 1, post, s) : launch_ot_nhwc<4, __half, __half>(Mh, bias, y, g, 1, post, s);
        return g.m == 2 ? launch_ot_cfg<2, __half, 1, __half>(Mh, bias, y, g, 1, post, s) : launch_ot_cfg<4, __half, 1, __half>(Mh, bias, y, g, 1, post, s);
    }
    const float* M = static_cast<const float*>(Mv);
    return with_dtype(dt, [&](auto* tag) {
        using E = std::remove_pointer_t<decltype(tag)>;
        if (nhwc) return g.m == 2 ? launch_ot_nhwc<2, E>(M, bias, y, g, nsplit, post, s) : launch_ot_nhwc<4, E>(M, bias, y, g, nsplit, post, s);
        return g.m == 2 ? launch_ot<2, E>(M, bias, y, g, nsplit, post, s) : launch_ot<4, E>(M, bias, y, g, nsplit, post, s);
    });
}

}  // namespace wino
