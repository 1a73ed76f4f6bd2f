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
// rows of the 4x4 window).  The filter kernel makes two passes over its input (maximum, then codes); the activation kernel
// keeps a row's entries in registers between the two and recomputes only what exceeds them (more than 3072 channels).
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

// x[n][c][h][w] (or [n][h][w][c]) as fp32, zero outside the image and for c >= C.  The load itself is unconditional (a
// clamped, always valid address), so that a thread's loads can all be in flight together.
template <typename E, bool NHWC>
__device__ __forceinline__ float load_x(const E* __restrict__ x, int n, int c, int h, int w, int C, int H, int W) {
    const bool ok = c < C && h >= 0 && h < H && w >= 0 && w < W;
    const size_t off = NHWC ? (((size_t)n * H + h) * W + w) * C + c : (((size_t)n * C + c) * H + h) * W + w;
    const float v = to_f32<E>(x[ok ? off : 0]);
    return ok ? v : 0.f;
}

__device__ __forceinline__ int8_t code_of(float v, float scale) { return (int8_t)(int)rintf(__fmul_rn(v, scale)); }

// The activation transform defined in the header of this file.  grid.x = 4 * T: a workgroup owns tile t and row xi of the
// transformed tile, i.e. the four rows V[xi*4 + nu][t][:] of the products' second operand, over all channels.  (B^T d)
// first - one addition or subtraction of two window rows per column - then the column combination, again one operation per entry.
//
// Channel-last: a lane owns a channel (a wave's loads are 128 contiguous bytes), computes all four nu and keeps them in
// registers for KEEP rounds of blockDim.x channels; rows longer than that are recomputed in the second pass.
template <typename E, int KEEP>
__global__ void __launch_bounds__(1024)
input_transform_i8_nhwc_kernel(const E* __restrict__ x, int8_t* __restrict__ Vq, float* __restrict__ dV,
                               int N, int C, int H, int W, int th, int tw, int T, int Cq) {
    __shared__ float red[4 * kMaxWaves];
    const int t = blockIdx.x >> 2, xi = blockIdx.x & 3;
    const int n = t / (th * tw), rem = t - n * th * tw, ti = rem / tw, tj = rem - ti * tw;
    const int h0 = 2 * ti - 1, w0 = 2 * tj - 1;
    int ia, ib; bool add;
    bt_row(xi, ia, ib, add);
    const int nt = blockDim.x;
    auto row = [&](int c, float (&v)[4]) {
        float tt[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float a = load_x<E, true>(x, n, c, h0 + ia, w0 + j, C, H, W), b = load_x<E, true>(x, n, c, h0 + ib, w0 + j, C, H, W);
            tt[j] = add ? __fadd_rn(a, b) : __fsub_rn(a, b);
        }
        v[0] = __fsub_rn(tt[0], tt[2]);
        v[1] = __fadd_rn(tt[1], tt[2]);
        v[2] = __fsub_rn(tt[2], tt[1]);
        v[3] = __fsub_rn(tt[1], tt[3]);
    };
    float kept[KEEP][4];
    float mx[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int r = 0; r < KEEP; ++r) row(threadIdx.x + r * nt, kept[r]);      // channels >= C give zeros
#pragma unroll
    for (int r = 0; r < KEEP; ++r)
#pragma unroll
        for (int nu = 0; nu < 4; ++nu) mx[nu] = fmaxf(mx[nu], fabsf(kept[r][nu]));
    for (int c = threadIdx.x + KEEP * nt; c < Cq; c += nt) {
        float v[4];
        row(c, v);
#pragma unroll
        for (int nu = 0; nu < 4; ++nu) mx[nu] = fmaxf(mx[nu], fabsf(v[nu]));
    }
    // maximum over the workgroup: lanes of a wave, then the waves through LDS (unused wave slots hold 0, a neutral value)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (threadIdx.x < 4 * kMaxWaves) red[threadIdx.x] = 0.f;
    __syncthreads();
#pragma unroll
    for (int nu = 0; nu < 4; ++nu) {
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) mx[nu] = fmaxf(mx[nu], __shfl_xor(mx[nu], off, 64));
        if (lane == 0) red[nu * kMaxWaves + wave] = mx[nu];
    }
    __syncthreads();
    float sc[4];
#pragma unroll
    for (int nu = 0; nu < 4; ++nu) {
        float m = 0.f;
#pragma unroll
        for (int w = 0; w < kMaxWaves; ++w) m = fmaxf(m, red[nu * kMaxWaves + w]);
        mx[nu] = m;
        sc[nu] = m > 0.f ? __fdiv_rn(127.f, m) : 0.f;
    }
    int8_t* dst = Vq + ((size_t)(xi * 4) * T + t) * Cq;
    const size_t plane = (size_t)T * Cq;
#pragma unroll
    for (int r = 0; r < KEEP; ++r) {
        const int c = threadIdx.x + r * nt;
        if (c < Cq) {
#pragma unroll
            for (int nu = 0; nu < 4; ++nu) dst[nu * plane + c] = code_of(kept[r][nu], sc[nu]);
        }
    }
    for (int c = threadIdx.x + KEEP * nt; c < Cq; c += nt) {
        float v[4];
        row(c, v);
#pragma unroll
        for (int nu = 0; nu < 4; ++nu) dst[nu * plane + c] = code_of(v[nu], sc[nu]);
    }
    if (threadIdx.x < 4) {
        float m = 0.f;
#pragma unroll
        for (int nu = 0; nu < 4; ++nu) m = threadIdx.x == nu ? mx[nu] : m;
        dV[(size_t)(xi * 4 + threadIdx.x) * T + t] = __fdiv_rn(m, 127.f);
    }
}

// NCHW: the only contiguity is along the image row, so eight adjacent lanes own the 2 x 4 entries of the window that row xi
// needs of one channel (one load per lane; a wave's load touches 8 channel planes - on 8x8 images a plane is a single
// 128-byte line, and how many lines a compute unit has to fetch is what this kernel's time follows).  The two rows are
// exchanged between the halves of the octet, the entries of B^T d between the lanes of a quad; both quads of an octet hold
// the same values, lane 8q + nu stores V[xi*4 + nu] of its channel.  A round covers blockDim.x / 8 channels.
template <typename E, int KEEP>
__global__ void __launch_bounds__(1024)
input_transform_i8_nchw_kernel(const E* __restrict__ x, int8_t* __restrict__ Vq, float* __restrict__ dV,
                               int N, int C, int H, int W, int th, int tw, int T, int Cq) {
    __shared__ float red[4 * kMaxWaves];
    const int t = blockIdx.x >> 2, xi = blockIdx.x & 3;
    const int n = t / (th * tw), rem = t - n * th * tw, ti = rem / tw, tj = rem - ti * tw;
    const int h0 = 2 * ti - 1, w0 = 2 * tj - 1;
    int ia, ib; bool add;
    bt_row(xi, ia, ib, add);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nu = threadIdx.x & 3, second = (threadIdx.x >> 2) & 1, cl = threadIdx.x >> 3, cpr = blockDim.x >> 3;   // channels per round
    const int hrow = h0 + (second ? ib : ia);
    // sources of this lane's column combination inside its quad: nu 0: t0 - t2, 1: t1 + t2, 2: t2 - t1, 3: t1 - t3
    const int qa = (lane & ~3) + (nu == 0 ? 0 : (nu == 2 ? 2 : 1));
    const int qb = (lane & ~3) + (nu == 0 ? 2 : (nu == 1 ? 2 : (nu == 2 ? 1 : 3)));
    auto entry = [&](int c) -> float {
        const float mine = load_x<E, false>(x, n, c, hrow, w0 + nu, C, H, W);
        const float other = __shfl_xor(mine, 4, 64);                   // the same column of the other window row
        const float a = second ? other : mine, b = second ? mine : other;
        const float tt = add ? __fadd_rn(a, b) : __fsub_rn(a, b);
        const float ta = __shfl(tt, qa, 64), tb = __shfl(tt, qb, 64);
        return nu == 1 ? __fadd_rn(ta, tb) : __fsub_rn(ta, tb);
    };
    float kept[KEEP];
    float mx = 0.f;
#pragma unroll
    for (int r = 0; r < KEEP; ++r) kept[r] = entry(cl + r * cpr);
#pragma unroll
    for (int r = 0; r < KEEP; ++r) mx = fmaxf(mx, fabsf(kept[r]));
    const int rounds = (Cq + cpr - 1) / cpr;                 // the same for every thread: the exchanges inside entry() need whole octets
    for (int r = KEEP; r < rounds; ++r) mx = fmaxf(mx, fabsf(entry(cl + r * cpr)));
    if (threadIdx.x < 4 * kMaxWaves) red[threadIdx.x] = 0.f;
    __syncthreads();
#pragma unroll
    for (int off = 32; off >= 8; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));       // lanes with the same nu
    if (lane < 4) red[lane * kMaxWaves + wave] = mx;
    __syncthreads();
    float m = 0.f;
#pragma unroll
    for (int w = 0; w < kMaxWaves; ++w) m = fmaxf(m, red[nu * kMaxWaves + w]);
    const float sc = m > 0.f ? __fdiv_rn(127.f, m) : 0.f;
    int8_t* dst = Vq + ((size_t)(xi * 4 + nu) * T + t) * Cq;
#pragma unroll
    for (int r = 0; r < KEEP; ++r) {
        const int c = cl + r * cpr;
        if (c < Cq && !second) dst[c] = code_of(kept[r], sc);
    }
    for (int r = KEEP; r < rounds; ++r) {
        const int c = cl + r * cpr;
        const float v = entry(c);
        if (c < Cq && !second) dst[c] = code_of(v, sc);
    }
    if (threadIdx.x < 4) dV[(size_t)(xi * 4 + nu) * T + t] = __fdiv_rn(m, 127.f);
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

template <typename E, int KEEP>
static void launch_i8_nhwc(const void* x, void* Vq, float* dV, const Geom& g, int Cq, int threads, hipStream_t s) {
    hipLaunchKernelGGL((input_transform_i8_nhwc_kernel<E, KEEP>), dim3((unsigned)(4 * g.T)), dim3((unsigned)threads), 0, s,
                       (const E*)x, (int8_t*)Vq, dV, g.N, g.C, g.H, g.W, g.th, g.tw, g.T, Cq);
}
template <typename E, int KEEP>
static void launch_i8_nchw(const void* x, void* Vq, float* dV, const Geom& g, int Cq, int threads, hipStream_t s) {
    hipLaunchKernelGGL((input_transform_i8_nchw_kernel<E, KEEP>), dim3((unsigned)(4 * g.T)), dim3((unsigned)threads), 0, s,
                       (const E*)x, (int8_t*)Vq, dV, g.N, g.C, g.H, g.W, g.th, g.tw, g.T, Cq);
}

hipError_t launch_input_transform_i8(const void* x, void* Vq, float* dV, const Geom& g, int Cq, int dt, bool nhwc, hipStream_t s) {
    if (g.m != 2 || Cq < g.C || Cq % 16 != 0 || (long long)g.T * 4 > 0x7fffffffLL) return hipErrorInvalidValue;
    // a round = the channels one pass of the workgroup covers (a lane per channel, or eight lanes per channel); the
    // workgroup is sized so that its rounds are full, and rows of up to 3 (24) rounds stay in registers between the passes
    const int per_round_max = nhwc ? 1024 : 128;
    const int rounds = (Cq + per_round_max - 1) / per_round_max;
    const int per_round = round_up((Cq + rounds - 1) / rounds, nhwc ? 64 : 8);
    const int threads = nhwc ? per_round : 8 * per_round;
    return with_dtype(dt, [&](auto* tag) {
        using E = std::remove_pointer_t<decltype(tag)>;
        if (nhwc) {
            if (rounds <= 1) launch_i8_nhwc<E, 1>(x, Vq, dV, g, Cq, threads, s);
            else if (rounds == 2) launch_i8_nhwc<E, 2>(x, Vq, dV, g, Cq, threads, s);
            else launch_i8_nhwc<E, 3>(x, Vq, dV, g, Cq, threads, s);
        } else {
            if (rounds <= 3) launch_i8_nchw<E, 3>(x, Vq, dV, g, Cq, threads, s);
            else if (rounds <= 6) launch_i8_nchw<E, 6>(x, Vq, dV, g, Cq, threads, s);
            else if (rounds <= 12) launch_i8_nchw<E, 12>(x, Vq, dV, g, Cq, threads, s);
            else launch_i8_nchw<E, 24>(x, Vq, dV, g, Cq, threads, s);
        }
        return hipGetLastError();
    });
}

}  // namespace wino
