// Direct 3x3 / stride 1 / pad 1 correlation for layers with very few output channels (K <= 4: the VAE's last layer
// 128 -> 3) on large images, fp16, either layout.  There the Winograd path writes and re-reads a transformed activation
// tensor many times the size of x for a handful of outputs, and the implicit-GEMM path pads K to a 32-wide MFMA tile
// after re-laying x; the operator itself is one pass over x with 9*K multiply-adds per input element.
// A workgroup owns 8 x 64 output pixels (a lane: one column, two rows) and walks the channels 16 at a time: the
// 10 x 80 patch of each channel is fetched with 16-byte loads (along W for NCHW, whose channels are interleaved in pairs on
// the way into LDS; along C for channel-last, where a load already holds four pairs of one pixel) so that one 32-bit LDS
// word = the same pixel of channels 2p and 2p+1, and the sum runs on v_dot2_f32_f16: two channels per
// instruction, fp32 accumulation, weights as wave-uniform (scalar) operands read from the tap-major filter
// Wr[9][K][Cp] that the implicit-GEMM path already keeps.  The next 16 channels are in flight while these are used.
// Algorithmic work: reads x once (plus halo), writes y; 18*C*K flops per pixel on the vector ALU.
#include "wino_internal.h"

namespace wino {

typedef _Float16 h2_t __attribute__((ext_vector_type(2)));

template <int KO, bool NHWC>
__global__ void __launch_bounds__(256)
conv3x3_fewk_kernel(const __half* __restrict__ x, const uint32_t* __restrict__ W2, const float* __restrict__ bias,
                         __half* __restrict__ y, int C, int H, int W, int Cp) {
    constexpr int TH = 8, TW = 64;                    // output tile
    constexpr int PR = TH + 2;                        // patch rows
    constexpr int PC = TW + 16;                       // patch columns staged: image columns col0-8 .. col0+71 (whole 16-byte chunks)
    constexpr int NQ = PC / 8;                        // chunks per patch row
    constexpr int CC = 16, NP = CC / 2;               // channels / channel pairs per step
    constexpr int PLANE = PR * PC;                    // words per channel pair
    constexpr int ITEMS = NP * PR * NQ;               // (pair, row, chunk) items per step
    constexpr int PASSES = (ITEMS + 255) / 256;
    __shared__ __attribute__((aligned(16))) uint32_t patch[2][NP * PLANE];

    const int tid = threadIdx.x;
    const int col0 = blockIdx.x * TW, row0 = blockIdx.y * TH, n = blockIdx.z;
    const __half* xn = x + (size_t)n * C * H * W;

    // ---- staging.  NCHW: a lane owns (pair, row, chunk) items; both channels of the pair are loaded, then interleaved.
    // Channel-last: a lane owns (half of the 16 channels, row, column) items; its 16 bytes are four pairs of one pixel.
    constexpr int NCOL = TW + 2;                                  // channel-last stages image columns col0-1 .. col0+64 only
    constexpr int ITEMS_CL = 2 * PR * NCOL;
    constexpr int PASSES_CL = (ITEMS_CL + 255) / 256;
    constexpr int NREG = NHWC ? PASSES_CL : 2 * PASSES;
    uint4 reg[NREG];
    auto fetch = [&](int c0) {
        if constexpr (NHWC) {
#pragma unroll
            for (int ps = 0; ps < PASSES_CL; ++ps) {
                const int item = tid + ps * 256;
                const int h = item / (PR * NCOL), rem = item - h * (PR * NCOL);
                const int row = rem / NCOL, cl = rem - row * NCOL;
                const int r = row0 - 1 + row, col = col0 - 1 + cl;
                reg[ps] = make_uint4(0, 0, 0, 0);
                if (item < ITEMS_CL && r >= 0 && r < H && col >= 0 && col < W)
                    reg[ps] = *reinterpret_cast<const uint4*>(xn + ((size_t)r * W + col) * C + c0 + 8 * h);
            }
        } else {
#pragma unroll
            for (int ps = 0; ps < PASSES; ++ps) {
                const int item = tid + ps * 256;
                const int p = item / (PR * NQ), rem = item - p * (PR * NQ);
                const int row = rem / NQ, q = rem - row * NQ;
                const int r = row0 - 1 + row, col = col0 - 8 + 8 * q;
                reg[2 * ps] = make_uint4(0, 0, 0, 0);
                reg[2 * ps + 1] = make_uint4(0, 0, 0, 0);
                if (item < ITEMS && r >= 0 && r < H && col >= 0 && col + 8 <= W) {     // W is a multiple of 8: a chunk is inside or outside
                    const __half* src = xn + ((size_t)(c0 + 2 * p) * H + r) * W + col;
                    reg[2 * ps] = *reinterpret_cast<const uint4*>(src);
                    reg[2 * ps + 1] = *reinterpret_cast<const uint4*>(src + (size_t)H * W);
                }
            }
        }
    };
    auto stash = [&](int buf) {
        if constexpr (NHWC) {
#pragma unroll
            for (int ps = 0; ps < PASSES_CL; ++ps) {
                const int item = tid + ps * 256;
                if (item < ITEMS_CL) {
                    const int h = item / (PR * NCOL), rem = item - h * (PR * NCOL);
                    const int row = rem / NCOL, cl = rem - row * NCOL;
                    uint32_t* dst = &patch[buf][(4 * h) * PLANE + row * PC + 7 + cl];      // image column col0-1+cl sits at word 7+cl
                    dst[0] = reg[ps].x; dst[PLANE] = reg[ps].y; dst[2 * PLANE] = reg[ps].z; dst[3 * PLANE] = reg[ps].w;
                }
            }
        } else {
#pragma unroll
            for (int ps = 0; ps < PASSES; ++ps) {
                const int item = tid + ps * 256;
                if (item < ITEMS) {
                    const int p = item / (PR * NQ), rem = item - p * (PR * NQ);
                    const int row = rem / NQ, q = rem - row * NQ;
                    const uint4 ra = reg[2 * ps], rb = reg[2 * ps + 1];
                    const uint32_t a[4] = {ra.x, ra.y, ra.z, ra.w}, b[4] = {rb.x, rb.y, rb.z, rb.w};
                    uint32_t o[8];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        o[2 * i] = (a[i] & 0xffffu) | (b[i] << 16);
                        o[2 * i + 1] = (a[i] >> 16) | (b[i] & 0xffff0000u);
                    }
                    uint4* dst = reinterpret_cast<uint4*>(&patch[buf][p * PLANE + row * PC + q * 8]);
                    dst[0] = make_uint4(o[0], o[1], o[2], o[3]);
                    dst[1] = make_uint4(o[4], o[5], o[6], o[7]);
                }
            }
        }
    };

    const int j = tid & 63, rp = tid >> 6;            // output column and row pair of this lane
    float acc[KO][2];
#pragma unroll
    for (int k = 0; k < KO; ++k) { acc[k][0] = 0.f; acc[k][1] = 0.f; }

    const int nsteps = C / CC;
    const int Cq = Cp / 2;                            // channel pairs per filter row
    fetch(0);
    stash(0);
    __syncthreads();
    for (int st = 0; st < nsteps; ++st) {
        if (st + 1 < nsteps) fetch((st + 1) * CC);    // in flight while this step is summed
        const uint32_t* pb = &patch[st & 1][(2 * rp) * PC + 7 + j];
        // two pairs per trip: the 9*KO weights of a pair live in scalar registers, and unrolling all eight pairs would need
        // more of those than a wave has
#pragma unroll 2
        for (int p = 0; p < NP; ++p) {
            uint32_t xv[4][3];
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 3; ++b) xv[a][b] = pb[p * PLANE + a * PC + b];
            const uint32_t* wp = W2 + (st * NP + p);  // wave-uniform
#pragma unroll
            for (int k = 0; k < KO; ++k)
#pragma unroll
                for (int dr = 0; dr < 3; ++dr)
#pragma unroll
                    for (int dc = 0; dc < 3; ++dc) {
                        const uint32_t wv = wp[(size_t)((dr * 3 + dc) * KO + k) * Cq];
                        const h2_t w2 = __builtin_bit_cast(h2_t, wv);
                        const h2_t x0 = __builtin_bit_cast(h2_t, xv[dr][dc]), x1 = __builtin_bit_cast(h2_t, xv[dr + 1][dc]);
                        // mixed-precision multiply-adds (fp16 operands taken from either half of a register, fp32 sum):
                        // the two-element dot product instruction runs at a quarter of their rate on this chip
                        acc[k][0] = __builtin_fmaf((float)x0.x, (float)w2.x, acc[k][0]);
                        acc[k][0] = __builtin_fmaf((float)x0.y, (float)w2.y, acc[k][0]);
                        acc[k][1] = __builtin_fmaf((float)x1.x, (float)w2.x, acc[k][1]);
                        acc[k][1] = __builtin_fmaf((float)x1.y, (float)w2.y, acc[k][1]);
                    }
        }
        if (st + 1 < nsteps) stash((st + 1) & 1);     // the buffer step st-1 used; everyone left it before the last barrier
        __syncthreads();
    }

    const int col = col0 + j;
    if (col < W) {
#pragma unroll
        for (int k = 0; k < KO; ++k) {
            const float b = bias ? bias[k] : 0.f;
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int r = row0 + 2 * rp + u;
                if (r < H) {
                    const size_t o = NHWC ? (((size_t)n * H + r) * W + col) * KO + k : (((size_t)n * KO + k) * H + r) * W + col;
                    y[o] = __float2half_rn(acc[k][u] + b);
                }
            }
        }
    }
}

// Whether the kernel above can take the call (everything else goes the implicit-GEMM way): the sizes it is written for, and
// enough 8 x 64 tiles to fill the chip - a workgroup walks all channels of its tile, so on small images (the UNet's 320 -> 4
// layer on a 64 x 64 latent has 16 tiles) the other paths are several times faster.
bool fewk_conv_ok(const void* x, int N, int C, int H, int W, int K, int R, int st, int dt, bool nhwc, int up, bool pre, bool post) {
    if (!(dt == DT_F16 && R == 3 && st == 1 && up == 0 && !pre && !post && K >= 1 && K <= 4 && C >= 16 && C % 16 == 0)) return false;
    if ((reinterpret_cast<uintptr_t>(x) & 15u) != 0 || N > 65535 || (H + 7) / 8 > 65535) return false;
    if (!nhwc && W % 8 != 0) return false;
    return (long long)N * ((H + 7) / 8) * ((W + 63) / 64) >= 512;
}

hipError_t launch_fewk_conv3x3(const void* x, const void* Wr, const float* bias, void* y, int N, int C, int H, int W, int K, bool nhwc, hipStream_t s) {
    const dim3 grid((unsigned)((W + 63) / 64), (unsigned)((H + 7) / 8), (unsigned)N), block(256);
    const int Cp = (C + 7) / 8 * 8;
    const __half* xh = static_cast<const __half*>(x);
    const uint32_t* W2 = static_cast<const uint32_t*>(Wr);
    __half* yh = static_cast<__half*>(y);
#define WINO_FEWK(KO)                                                                                                          \
    case KO:                                                                                                                   \
        if (nhwc) hipLaunchKernelGGL((conv3x3_fewk_kernel<KO, true>), grid, block, 0, s, xh, W2, bias, yh, C, H, W, Cp);     \
        else hipLaunchKernelGGL((conv3x3_fewk_kernel<KO, false>), grid, block, 0, s, xh, W2, bias, yh, C, H, W, Cp);         \
        break;
    switch (K) {
        WINO_FEWK(1) WINO_FEWK(2) WINO_FEWK(3) WINO_FEWK(4)
        default: return hipErrorInvalidValue;
    }
#undef WINO_FEWK
    return hipGetLastError();
}

}  // namespace wino
