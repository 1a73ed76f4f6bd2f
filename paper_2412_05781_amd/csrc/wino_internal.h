// Internal declarations shared by the HIP sources of libwino (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <hip/hip_bf16.h>
#include <type_traits>
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

// Storage types (values of wino_dtype).  `with_dtype` calls f with a null pointer of the element
// type, so that a generic lambda can name it:  using E = std::remove_pointer_t<decltype(tag)>.
typedef __hip_bfloat16 bf16_t;
enum { DT_F32 = 0, DT_F16 = 1, DT_BF16 = 2, DT_I8 = 3 };     // DT_I8: internal only (operands of the quantised Winograd path)
inline bool two_byte(int dt) { return dt != DT_F32; }
template <typename F> inline hipError_t with_dtype(int dt, F&& f) {
    if (dt == DT_F16) return f(static_cast<__half*>(nullptr));
    if (dt == DT_BF16) return f(static_cast<bf16_t*>(nullptr));
    return f(static_cast<float*>(nullptr));
}

// 8-bit floating-point operand (OCP E4M3) of the quantised direct path: storage only.
struct fp8_t { uint8_t v; };
// 8-bit integer code of the quantised Winograd path (symmetric, -127..127): storage only.
struct i8_t { int8_t v; };
// nearest E4M3 value of v after clamping to the format's range (+-448), ties to even
__device__ __forceinline__ uint32_t quant_e4m3(float v) {
    v = fminf(fmaxf(v, -448.f), 448.f);
    return (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(v, v, 0, false) & 0xffu;
}

// element conversion helpers usable in kernels
template <typename E> __device__ __forceinline__ float to_f32(E v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<__half>(__half v) { return __half2float(v); }
template <> __device__ __forceinline__ float to_f32<bf16_t>(bf16_t v) { return __bfloat162float(v); }
template <typename E> __device__ __forceinline__ E from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ __half from_f32<__half>(float v) { return __float2half_rn(v); }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return __float2bfloat16(v); }   // round to nearest even

// Streaming read: data that a kernel reads exactly once carries the non-temporal hint, so that it does not displace what
// the kernel re-reads from L2.  Used for the product M in the output transform (chain time -2 % on the 128x128-image
// layers, -6...-8 % on the VAE-sized ones).  The same hint on the STORES of V and M makes each kernel faster on its own
// (activation transform -25...-35 %) but the chain no faster or slower: the next kernel then finds its input in HBM
// instead of the memory-side cache.  So intermediates are stored with ordinary stores.
template <typename T> __device__ __forceinline__ T load_stream(const T* p) { return __builtin_nontemporal_load(p); }

// Optional operators fused around the convolution.  PreOp: x' = SiLU(GroupNorm(x)) applied as the
// activation transform loads x (stats = (mean, rstd) per (n, group)); PostOp: y += addvec[n][k] +
// residual in the output transform.  Null pointers switch a part off.
struct PreOp {
    const float* stats = nullptr;     // [N][groups][2]
    const float* gamma = nullptr;     // [C]
    const float* beta = nullptr;      // [C]
    int groups = 1;
    int cpg = 1;                      // channels per group
    int up = 0;                       // 1: x holds [H/2][W/2] pixels and is read as its 2x nearest-neighbour upsampling
};
// 16 bytes of an upsampled row from the 8 source bytes under them: every element twice
template <typename E> __device__ __forceinline__ uint4 dup_elements(uint2 s);
template <> __device__ __forceinline__ uint4 dup_elements<float>(uint2 s) { return make_uint4(s.x, s.x, s.y, s.y); }
__device__ __forceinline__ uint4 dup_elements_16bit(uint2 s) {
    const uint32_t a = s.x & 0xffffu, b = s.x >> 16, c = s.y & 0xffffu, d = s.y >> 16;
    return make_uint4(a | (a << 16), b | (b << 16), c | (c << 16), d | (d << 16));
}
template <> __device__ __forceinline__ uint4 dup_elements<__half>(uint2 s) { return dup_elements_16bit(s); }
template <> __device__ __forceinline__ uint4 dup_elements<bf16_t>(uint2 s) { return dup_elements_16bit(s); }
struct PostOp {
    const float* addvec = nullptr;    // [N][K]
    const void* residual = nullptr;   // like y
};

// per-lane constants of the fused GroupNorm: v = x*sc + sh, then SiLU; zero outside the image
struct PreLane { float sc, sh; bool on; };
__device__ __forceinline__ PreLane pre_lane(const PreOp& pre, int n, int c, int C) {
    PreLane l; l.on = c < C; l.sc = 0.f; l.sh = 0.f;
    if (l.on) {
        const float* st = pre.stats + ((size_t)n * pre.groups + c / pre.cpg) * 2;
        l.sc = pre.gamma[c] * st[1];
        l.sh = pre.beta[c] - st[0] * l.sc;
    }
    return l;
}
__device__ __forceinline__ float pre_apply(float x, const PreLane& l, bool in_image) {
    if (!(l.on && in_image)) return 0.f;
    const float v = fmaf(x, l.sc, l.sh);
    return __fdividef(v, 1.f + __expf(-v));
}

// Direct 3x3 / stride 1 kernel for K <= 4 output channels on large images (fp16, conv_fewk.hip): whether it applies, and the launch.
// Wr is the tap-major filter of the implicit-GEMM path.
bool fewk_conv_ok(const void* x, int N, int C, int H, int W, int K, int R, int st, int dt, bool nhwc, int up, bool pre, bool post);
hipError_t launch_fewk_conv3x3(const void* x, const void* Wr, const float* bias, void* y, int N, int C, int H, int W, int K, bool nhwc, hipStream_t s);

// launchers (each enqueues on `s`, returns the launch status)
hipError_t launch_filter_transform(const void* w, void* U, int K, int C, int Cp, int m, int dt, hipStream_t s);
hipError_t launch_input_transform(const void* x, void* V, const Geom& g, int dt, bool nhwc, const PreOp* pre, hipStream_t s);
// nsplit > 1: the reduction is cut into nsplit ranges and M holds nsplit partial products
// [nsplit][nbatch][K][T], which launch_output_transform sums.  gemm_split() is the policy the
// whole path uses for a shape (rows = rows of the first operand, cols = rows of the second).
// half_product: M is stored as fp16 (fp16 storage and an unsplit reduction only)
// shape: -1 = the library's choice for the problem size, 0..8 = a named block shape (see wino_gemm.hip)
hipError_t launch_batched_gemm(const void* U, const void* V, void* M, int K, int Cp, int T, int nbatch, int nsplit, int dt, bool half_product,
                               hipStream_t s, int shape = -1);
// the same product on 8-bit integer codes (rows of 16-byte multiples, Cq % 16 == 0) with one quantisation step per row of each
// operand: M[b][k][t] = float(sum_c Uq[b][k][c] * Vq[b][t][c]) * dU[b][k] * dV[b][t]; int32 accumulation, exact
hipError_t launch_batched_gemm_i8(const void* Uq, const float* dU, const void* Vq, const float* dV, float* M, int K, int Cq, int T,
                                  int nbatch, int nsplit, hipStream_t s, int shape = -1);
// step (i) of the quantised F(2x2) path (wino_int8.hip): codes and steps of the filter (once per weight tensor, fp64 decisions)
// and of the activation (fp32 decisions); Uq[16][K][Cq], dU[16][K], Vq[16][T][Cq], dV[16][T], Cq % 16 == 0, padded channels zero
hipError_t launch_filter_quant_i8(const void* w, void* Uq, float* dU, int K, int C, int Cq, int dt, hipStream_t s);
hipError_t launch_input_transform_i8(const void* x, void* Vq, float* dV, const Geom& g, int Cq, int dt, bool nhwc, hipStream_t s);
int gemm_max_split(int Cp, int dt);
int gemm_split(int rows, int cols, int Cp, int nbatch, int dt);
hipError_t launch_output_transform(const void* M, const float* bias, void* y, const Geom& g, int nsplit, int dt, bool nhwc,
                                   bool half_product, const PostOp* post, hipStream_t s);
// steps (ii) and (iii) in one kernel, F(2x2,3x3) only: U, V as for launch_batched_gemm, y written directly.
// shape: -1 = chosen from the problem size, 0..3 = a named block shape (see wino_fused.hip)
hipError_t launch_fused_gemm_output(const void* U, const void* V, const float* bias, void* y, const Geom& g, int dt, bool nhwc,
                                    const PostOp* post, int shape, hipStream_t s);
int fused_pick_shape(int rows, int cols);
// the same for F(4x4,3x3) (wino_fused_f4.hip), two-byte storage types; shape: -1 = chosen from the problem size, 0..1 = a named block shape
hipError_t launch_fused4_gemm_output(const void* U, const void* V, const float* bias, void* y, const Geom& g, int dt, bool nhwc,
                                     const PostOp* post, int shape, hipStream_t s);
hipError_t launch_groupnorm_stats(const void* x, float* stats, int N, int C, int H, int W, int groups, float eps,
                                  int dt, bool nhwc, hipStream_t s);
size_t groupnorm_stats_bytes(int N, int groups);
hipError_t launch_igemm_filter_repack(const void* w, void* Wr, int K, int C, int R, int dt, hipStream_t s);
hipError_t launch_igemm_conv2d(const void* x, const void* Wr, const float* bias, void* y,
                               int N, int C, int H, int W, int K, int R, int st, int dt, bool nhwc,
                               void* workspace, size_t xh_bytes, int up, const PreOp* pre, const float* addvec, const void* residual,
                               hipStream_t s);
int igemm_split(int T, int K, int Cp, int R, int dt);   // number of partial products the path writes for a shape (dt < 0: 8-bit operands)
hipError_t launch_igemm_fp8_filter_quant(const void* w, void* Wq, int K, int C, int R, int dt, float sw, hipStream_t s);
hipError_t launch_igemm_fp8_conv2d(const void* x, const void* Wq, const float* bias, void* y,
                                   int N, int C, int H, int W, int K, int R, int st, int dt, bool nhwc,
                                   void* workspace, size_t xq_bytes, int up, const PreOp* pre, const float* addvec,
                                   const void* residual, float sx, float sw, hipStream_t s);
hipError_t launch_direct_conv2d(const void* x, const void* w, const float* bias, void* y,
                                int N, int C, int H, int W, int K, int dt, hipStream_t s);

}  // namespace wino
