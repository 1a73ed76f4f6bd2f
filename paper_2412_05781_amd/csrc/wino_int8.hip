// Step (i) of the Winograd F(2x2,3x3) path (Section "Techniques") with the transformed tensors held as 8-bit integer
// codes, one quantisation step per row of each of the 16 matrix products of step (ii):
//     Uq[b][k][c] = rint(U[b][k][c] * (127 / mU[b][k])),  mU[b][k] = max_c |U[b][k][c]|,  dU[b][k] = mU / 127
//     Vq[b][t][c] = rint(V[b][t][c] * (127 / mV[b][t])),  mV[b][t] = max_c |V[b][t][c]|,  dV[b][t] = mV / 127
// (the paper only remarks that quantised operators are supported; the scheme is this library's).  The precision in which
// a code is decided is part of the definition so that results can be reproduced bit for bit: the filter side, which runs
// once per weight tensor, works in fp64 (U is exact there); the activation side works in fp32 with the row combination
// B^T d taken first and the column combination second, each entry one addition or subtraction; the scale, the scaled value
// and the step are single correctly rounded operations.
//
// A row's maximum needs the whole row, so a workgroup owns whole rows: the filter kernel one output channel k (all 16
// positions), the activation kernel one tile t and one row xi of the transformed tile (4 positions, which need only two
// rows of the 4x4 window).  Both make two passes over their inputs (maximum, then codes); the second pass of the
// activation kernel re-reads at most a few KB that the first pass has just brought into the cache.
#include "wino_internal.h"

namespace wino {

namespace {

constexpr int kMaxWaves = 16;

// maximum over the workgroup of NV values per thread; every thread gets the result.  red: NV * kMaxWaves floats of LDS.
template <int NV, typename F>
__device__ __forceinline__ void block_max(F (&v)[NV], F* red) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        F m = v[i];
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const F o = __shfl_xor(m, off, 64);
            m = o > m ? o : m;
        }
        if (lane == 0) red[i * kMaxWaves + wave] = m;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        F m = red[i * kMaxWaves];
        for (int w = 1; w < nw; ++w) { const F o = red[i * kMaxWaves + w]; m = o > m ? o : m; }
        v[i] = m;
    }
}

// U = G g G^T of one (k, c) in fp64: exact for 16- and 32-bit filters, whatever the order of the additions
template <typename E>
__device__ __forceinline__ void filter_tile_f64(const E* __restrict__ w, int k, int c, int C, double (&U)[16]) {
    double g[3][3];
    const E* p = w + ((size_t)k * C + c) * 9;
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int s = 0; s < 3; ++s) g[r][s] = c < C ? (double)to_f32<E>(p[r * 3 + s]) : 0.0;
    double t[4][3];
#pragma unroll
    for (int s = 0; s < 3; ++s) {
        t[0][s] = g[0][s];
        t[1][s] = 0.5 * (g[0][s] + g[1][s] + g[2][s]);
        t[2][s] = 0.5 * (g[0][s] - g[1][s] + g[2][s]);
        t[3][s] = g[2][s];
    }
#pragma unroll
    for (int xi = 0; xi < 4; ++xi) {
        U[xi * 4 + 0] = t[xi][0];
        U[xi * 4 + 1] = 0.5 * (t[xi][0] + t[xi][1] + t[xi][2]);
        U[xi * 4 + 2] = 0.5 * (t[xi][0] - t[xi][1] + t[xi][2]);
        U[xi * 4 + 3] = t[xi][2];
    }
}

template <typename E>
__global__ void __launch_bounds__(256)
filter_quant_i8_kernel(const E* __restrict__ w, int8_t* __restrict__ Uq, float* __restrict__ dU, int K, int C, int Cq) {
    __shared__ double red[16 * kMaxWaves];
    const int k = blockIdx.x;
    double mx[16];
#pragma unroll
    for (int b = 0; b < 16; ++b) mx[b] = 0.0;
    for (int c = threadIdx.x; c < C; c += blockDim.x) {
        double U[16];
        filter_tile_f64<E>(w, k, c, C, U);
#pragma unroll
        for (int b = 0; b < 16; ++b) mx[b] = fmax(mx[b], fabs(U[b]));
    }
    block_max<16>(mx, red);
    double sc[16];
#pragma unroll
    for (int b = 0; b < 16; ++b) sc[b] = mx[b] > 0.0 ? __ddiv_rn(127.0, mx[b]) : 0.0;
    for (int c = threadIdx.x; c < Cq; c += blockDim.x) {
        double U[16];
        filter_tile_f64<E>(w, k, c, C, U);           // zeros for the padded channels c >= C
#pragma unroll
        for (int b = 0; b < 16; ++b)
            Uq[((size_t)b * K + k) * Cq + c] = (int8_t)(int)rint(__dmul_rn(U[b], sc[b]));
    }
    if (threadIdx.x < 16) {
        // the value of mx for b = threadIdx.x without a dynamically indexed register array
        double m = 0.0;
#pragma unroll
        for (int b = 0; b < 16; ++b) m = threadIdx.x == b ? mx[b] : m;
        dU[(size_t)threadIdx.x * K + k] = (float)__ddiv_rn(m, 127.0);
    }
}

// the two window rows that row xi of B^T combines, and whether they are added: B^T = [1 0 -1 0; 0 1 1 0; 0 -1 1 0; 0 1 0 -1]
__device__ __forceinline__ void bt_row(int xi, int& ia, int& ib, bool& add) {
    ia = xi == 0 ? 0 : (xi == 2 ? 2 : 1);
    ib = xi == 0 ? 2 : (xi == 1 ? 2 : (xi == 2 ? 1 : 3));
    add = xi == 1;
}

// the four entries V[xi][0..3] of channel c of one tile: (B^T d) first - one addition or subtraction of two window rows
// per column - then the column combination, again one operation per entry.  Pixels outside the image and channels
// c >= C read as zero.
template <typename E, bool NHWC>
__device__ __forceinline__ void activation_row(const E* __restrict__ x, int n, int c, int C, int H, int W, int h0, int w0,
                                               int ia, int ib, bool add, float (&v)[4]) {
    float ra[4], rb[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int wj = w0 + j, ha = h0 + ia, hb = h0 + ib;
        const bool okw = c < C && wj >= 0 && wj < W;
        const bool oka = okw && ha >= 0 && ha < H, okb = okw && hb >= 0 && hb < H;
        const size_t offa = NHWC ? (((size_t)n * H + ha) * W + wj) * C + c : (((size_t)n * C + c) * H + ha) * W + wj;
        const size_t offb = NHWC ? (((size_t)n * H + hb) * W + wj) * C + c : (((size_t)n * C + c) * H + hb) * W + wj;
        ra[j] = oka ? to_f32<E>(x[offa]) : 0.f;
        rb[j] = okb ? to_f32<E>(x[offb]) : 0.f;
    }
    float t[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) t[j] = add ? __fadd_rn(ra[j], rb[j]) : __fsub_rn(ra[j], rb[j]);
    v[0] = __fsub_rn(t[0], t[2]);
    v[1] = __fadd_rn(t[1], t[2]);
    v[2] = __fsub_rn(t[2], t[1]);
    v[3] = __fsub_rn(t[1], t[3]);
}

// grid.x = 4 * T: workgroup = (tile t, row xi of the transformed tile); threads stride over the channels.
// KEEP channel rounds are held in registers between the two passes; longer rows are recomputed in the second pass.
template <typename E, bool NHWC, int KEEP>
__global__ void __launch_bounds__(1024)
input_transform_i8_kernel(const E* __restrict__ x, int8_t* __restrict__ Vq, float* __restrict__ dV,
                          int N, int C, int H, int W, int th, int tw, int T, int Cq) {
    __shared__ float red[4 * kMaxWaves];
    const int t = blockIdx.x >> 2, xi = blockIdx.x & 3;
    const int n = t / (th * tw), rem = t - n * th * tw, ti = rem / tw, tj = rem - ti * tw;
    const int h0 = 2 * ti - 1, w0 = 2 * tj - 1;
    int ia, ib; bool add;
    bt_row(xi, ia, ib, add);
    const int nt = blockDim.x;
    float kept[KEEP][4];
    float mx[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int r = 0; r < KEEP; ++r) {
        const int c = threadIdx.x + r * nt;
        if (c < Cq) {
            activation_row<E, NHWC>(x, n, c, C, H, W, h0, w0, ia, ib, add, kept[r]);
#pragma unroll
            for (int nu = 0; nu < 4; ++nu) mx[nu] = fmaxf(mx[nu], fabsf(kept[r][nu]));
        }
    }
    for (int c = threadIdx.x + KEEP * nt; c < Cq; c += nt) {
        float v[4];
        activation_row<E, NHWC>(x, n, c, C, H, W, h0, w0, ia, ib, add, v);
#pragma unroll
        for (int nu = 0; nu < 4; ++nu) mx[nu] = fmaxf(mx[nu], fabsf(v[nu]));
    }
    block_max<4>(mx, red);
    float sc[4];
#pragma unroll
    for (int nu = 0; nu < 4; ++nu) sc[nu] = mx[nu] > 0.f ? __fdiv_rn(127.f, mx[nu]) : 0.f;
    int8_t* dst = Vq + ((size_t)(xi * 4) * T + t) * Cq;
    const size_t plane = (size_t)T * Cq;
#pragma unroll
    for (int r = 0; r < KEEP; ++r) {
        const int c = threadIdx.x + r * nt;
        if (c < Cq) {
#pragma unroll
            for (int nu = 0; nu < 4; ++nu) dst[nu * plane + c] = (int8_t)(int)rintf(__fmul_rn(kept[r][nu], sc[nu]));
        }
    }
    for (int c = threadIdx.x + KEEP * nt; c < Cq; c += nt) {
        float v[4];
        activation_row<E, NHWC>(x, n, c, C, H, W, h0, w0, ia, ib, add, v);
#pragma unroll
        for (int nu = 0; nu < 4; ++nu) dst[nu * plane + c] = (int8_t)(int)rintf(__fmul_rn(v[nu], sc[nu]));
    }
    if (threadIdx.x < 4) {
        float m = 0.f;
#pragma unroll
        for (int nu = 0; nu < 4; ++nu) m = threadIdx.x == nu ? mx[nu] : m;
        dV[(size_t)(xi * 4 + threadIdx.x) * T + t] = __fdiv_rn(m, 127.f);
    }
}

}  // namespace

hipError_t launch_filter_quant_i8(const void* w, void* Uq, float* dU, int K, int C, int Cq, int dt, hipStream_t s) {
    if (K < 1 || C < 1 || Cq < C || Cq % 16 != 0) return hipErrorInvalidValue;
    return with_dtype(dt, [&](auto* tag) {
        using E = std::remove_pointer_t<decltype(tag)>;
        hipLaunchKernelGGL((filter_quant_i8_kernel<E>), dim3((unsigned)K), dim3(256), 0, s, (const E*)w, (int8_t*)Uq, dU, K, C, Cq);
        return hipGetLastError();
    });
}

hipError_t launch_input_transform_i8(const void* x, void* Vq, float* dV, const Geom& g, int Cq, int dt, bool nhwc, hipStream_t s) {
    if (g.m != 2 || Cq < g.C || Cq % 16 != 0 || (long long)g.T * 4 > 0x7fffffffLL) return hipErrorInvalidValue;
    int threads = round_up(Cq, 64);
    if (threads > 1024) threads = 1024;
    const dim3 grid((unsigned)(4 * g.T)), block((unsigned)threads);
    return with_dtype(dt, [&](auto* tag) {
        using E = std::remove_pointer_t<decltype(tag)>;
        if (nhwc) hipLaunchKernelGGL((input_transform_i8_kernel<E, true, 3>), grid, block, 0, s, (const E*)x, (int8_t*)Vq, dV,
                                     g.N, g.C, g.H, g.W, g.th, g.tw, g.T, Cq);
        else      hipLaunchKernelGGL((input_transform_i8_kernel<E, false, 3>), grid, block, 0, s, (const E*)x, (int8_t*)Vq, dV,
                                     g.N, g.C, g.H, g.W, g.th, g.tw, g.T, Cq);
        return hipGetLastError();
    });
}

}  // namespace wino
