// Direct convolution as an implicit GEMM on the MFMA units, for the convolution flavours of a
// Stable-Diffusion UNet / VAE that the Winograd path does not cover (1x1 projections, 3x3 with
// stride 2), so that the library can stand in for the whole 2-D convolution operator the paper's
// Section "Techniques" replaces.  Square R x R filter, stride st, zero padding (R-1)/2:
//
//   y[n,k,i,j] = bias[k] + sum_{tap=(r,s)} sum_c  xhat[n, i*st + r - pad, j*st + s - pad, c] * w[k,c,r,s]
//
// i.e. R*R accumulated matrix products  Y[k][t] += Wr[tap][k][:] . P_tap[t][:]  in which row t of
// P_tap is the channel vector of one input pixel (or a row of zeros in the padding).  The kernel
// has the structure of the Winograd GEMM stage (128-byte reduction stages, global -> LDS transfers
// into a ring, XOR-swizzled chunks, 32x32 MFMA tiles, fp32 accumulation); what differs is that the
// rows of the pixel operand are found by address arithmetic per filter tap instead of being stored,
// and that the epilogue adds the bias and writes y in its storage type.
//
// The pixel operand needs the channel index contiguous: x[N][H][W][Cp].  Channel-last inputs with
// C a multiple of 8 are used in place; otherwise (NCHW, or C not a multiple of 8) a re-layout
// kernel writes that tensor into the workspace first.  That kernel is also where the optional
// SiLU(GroupNorm(x)) is applied (the GEMM kernel's loads go straight to LDS and cannot), so with it
// even a channel-last input is copied once.  The optional 2x upsampling is pure address arithmetic.
#include "wino_internal.h"
#include "wino_mma.h"

namespace wino {

struct ConvGeom {
    int N, C, Cp, H, W, K, R, st, pad, Ho, Wo, T;      // T = N*Ho*Wo output pixels
    int up, Hs, Ws;                                    // up = 1: x is stored at Hs x Ws = H/2 x W/2 and read upsampled
};
// Optional additions in the epilogue (fp32, before the one rounding): a per-(image, channel) vector and a
// tensor of y's shape and layout.
struct IgemmPost {
    const float* addvec = nullptr;    // [N][K]
    const void* residual = nullptr;   // like y
    float scale = 1.f;                // the accumulated sum is multiplied by this first (quantised operands: 1 / (sx * sw))
};

// PIX_A: the pixel operand supplies the rows of the block (outputs [t][k], channel-last y);
// otherwise the filter does (outputs [k][t], NCHW y).
// E = operand type (fp16, bf16, fp32, or fp8_t for the quantised path), EO = type of y and of the residual.
template <typename E, typename EO, int BM, int BN, int NST, bool PIX_A, int WGM = 2, int WGN = 2>
__global__ void __launch_bounds__(WGM * WGN * 64)
conv_igemm_kernel(const E* __restrict__ xh, const E* __restrict__ Wr, const E* __restrict__ zero_row,
                  const float* __restrict__ bias, EO* __restrict__ y, float* __restrict__ part, ConvGeom g, IgemmPost post,
                  int tiles_m, int tiles_n, int total_blocks, int blocks_per_xcd, int nsplit) {
    constexpr int RB = 128;
    constexpr int CPR = RB / 16;                          // 16-byte chunks per row per stage
    constexpr int BKE = RB / (int)sizeof(E);              // reduction elements per stage
    constexpr int EPC = 16 / (int)sizeof(E);
    constexpr int ROWS = BM + BN;
    constexpr int RPL = 1024 / RB;                        // rows covered by one wave-wide load
    constexpr int NW = WGM * WGN;                         // waves per workgroup
    constexpr int LPW = ROWS / RPL / NW;                  // wave-wide loads per wave per stage
    constexpr int WTM = BM / WGM, WTN = BN / WGN;
    constexpr int FM = WTM / 32, FN = WTN / 32;
    constexpr int STAGE_BYTES = ROWS * RB;
    static_assert(WTM % 32 == 0 && WTN % 32 == 0 && ROWS % (RPL * NW) == 0 && BM % RPL == 0, "tile shape");
    static_assert(NST >= 2 && LPW * (NST - 1) < 64, "ring depth / vmcnt range");

    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];

    const int bid = blockIdx.x;
    const int logical = (bid % 8) * blocks_per_xcd + bid / 8;   // one contiguous range per XCD
    if (logical >= total_blocks) return;                        // uniform, before any barrier
    // With nsplit > 1 the reduction (taps x channel stages) is cut into nsplit ranges of whole stages;
    // split i leaves its fp32 partial sums in the i-th copy of `part` and a second kernel adds them up.
    const int split = logical % nsplit;
    const int tile = logical / nsplit;
    int tm, tn;
    if (tiles_m <= tiles_n) { tm = tile % tiles_m; tn = tile / tiles_m; }
    else { tn = tile % tiles_n; tm = tile / tiles_n; }

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int row_a0 = tm * BM, row_b0 = tn * BN;
    const int rowsA = PIX_A ? g.T : g.K, rowsB = PIX_A ? g.K : g.T;

    // Per-lane description of its LPW loads.  Filter rows: a pointer that advances with the tap and
    // the stage.  Pixel rows: the image, and the top-left input coordinate of the output pixel.
    const int lrow = lane / CPR, lchunk = lane % CPR;
    const E* fptr[LPW];                                   // filter row: Wr + k*Cp + chunk (tap 0, stage 0)
    int pn[LPW], pi0[LPW], pj0[LPW];                       // pixel row: image offset (pixels), first input row / column
    int chunk_of[LPW];
    bool is_pix[LPW];
    const int HoWo = g.Ho * g.Wo;
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
        const int row = (wave + NW * i) * RPL + lrow;       // row inside the stage, A rows first
        const int chunk = lchunk ^ ((row >> 1) & (CPR - 1));
        chunk_of[i] = chunk;
        const bool in_a = row < BM;
        int gr = in_a ? row_a0 + row : row_b0 + (row - BM);
        const int lim = in_a ? rowsA : rowsB;
        gr = gr < lim ? gr : lim - 1;                       // rows beyond the end repeat the last one; never stored
        is_pix[i] = (in_a == PIX_A);
        fptr[i] = Wr + (size_t)gr * g.Cp + chunk * EPC;
        const int n = gr / HoWo, p = gr - n * HoWo;
        const int oi = p / g.Wo, oj = p - oi * g.Wo;
        pn[i] = n * g.Hs * g.Ws; pi0[i] = oi * g.st - g.pad; pj0[i] = oj * g.st - g.pad;
    }

    const int nkc = (g.Cp + BKE - 1) / BKE;
    const bool ragged = (g.Cp % BKE) != 0;
    const int taps = g.R * g.R;
    const int nstage_all = taps * nkc;
    const int q0 = (int)((long long)split * nstage_all / nsplit), q1 = (int)((long long)(split + 1) * nstage_all / nsplit);
    const int nstage = q1 - q0;

    // issue side: the (tap, stage-in-tap) of the next stage to fetch, and that tap's row pointers
    int itap = q0 / nkc, ikc = q0 - (q0 / nkc) * nkc, iq = 0;
    bool tap_set = false;
    const E* src[LPW];
    auto set_tap = [&](int tap) {
        const int r = tap / g.R, s = tap - r * g.R;
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            if (is_pix[i]) {
                const int ii = pi0[i] + r, jj = pj0[i] + s;
                const bool in = ii >= 0 && ii < g.H && jj >= 0 && jj < g.W;
                src[i] = in ? xh + ((size_t)pn[i] + (size_t)(ii >> g.up) * g.Ws + (jj >> g.up)) * g.Cp + chunk_of[i] * EPC
                            : zero_row + chunk_of[i] * EPC;
            } else {
                src[i] = fptr[i] + (size_t)tap * g.K * g.Cp;
            }
        }
    };
    auto issue_next = [&]() {
        if (ikc == 0 || !tap_set) { set_tap(itap); tap_set = true; }
        unsigned char* slot = lds + (iq % NST) * STAGE_BYTES;
        if (ragged && ikc == nkc - 1) {
            // last, partial stage of a tap: through registers, chunks beyond Cp become zeros
#pragma unroll
            for (int i = 0; i < LPW; ++i) {
                const int gk = ikc * BKE + chunk_of[i] * EPC;
                uint4 v = make_uint4(0, 0, 0, 0);
                if (gk < g.Cp) v = *reinterpret_cast<const uint4*>(src[i] + ikc * BKE);
                *reinterpret_cast<uint4*>(slot + (wave + NW * i) * 1024 + lane * 16) = v;
            }
        } else {
#pragma unroll
            for (int i = 0; i < LPW; ++i) dma_load_1k(src[i] + ikc * BKE, slot + (wave + NW * i) * 1024);
        }
        ++iq;
        if (++ikc == nkc) { ikc = 0; ++itap; }
    };

    float16_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

#pragma unroll
    for (int s = 0; s < NST - 1; ++s)
        if (s < nstage) issue_next();

    const int frag_row = lane & 31, frag_half = lane >> 5;
    for (int q = 0; q < nstage; ++q) {
        // transfers complete in issue order: allow as many outstanding as were issued after stage q
        if (q + NST - 1 >= nstage) wait_vmcnt<0>();
        else wait_vmcnt<(NST - 2) * LPW>();
        __syncthreads();            // stage q visible to all waves; everyone is done with stage q-1
        if (q + NST - 1 < nstage) issue_next();             // refills the slot stage q-1 used

        const unsigned char* slot = lds + (q % NST) * STAGE_BYTES;
        constexpr int KCH = MmaChunks<E>::value;          // chunks per lane and MFMA step
        constexpr int STEPS = CPR / (2 * KCH);
        uint4 fa[STEPS][FM][KCH], fb[STEPS][FN][KCH];
#pragma unroll
        for (int ks = 0; ks < STEPS; ++ks) {
#pragma unroll
            for (int c = 0; c < KCH; ++c) {
#pragma unroll
                for (int i = 0; i < FM; ++i) {
                    const int row = wm * WTM + i * 32 + frag_row;
                    const int chunk = (2 * KCH * ks + KCH * frag_half + c) ^ ((row >> 1) & (CPR - 1));
                    fa[ks][i][c] = *reinterpret_cast<const uint4*>(slot + row * RB + chunk * 16);
                }
#pragma unroll
                for (int j = 0; j < FN; ++j) {
                    const int row = BM + wn * WTN + j * 32 + frag_row;
                    const int chunk = (2 * KCH * ks + KCH * frag_half + c) ^ ((row >> 1) & (CPR - 1));
                    fb[ks][j][c] = *reinterpret_cast<const uint4*>(slot + row * RB + chunk * 16);
                }
            }
        }
#pragma unroll
        for (int ks = 0; ks < STEPS; ++ks)
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j) {
                    if constexpr (KCH == 2) Mma<E>::run2(fa[ks][i][0], fa[ks][i][1], fb[ks][j][0], fb[ks][j][1], acc[i][j]);
                    else Mma<E>::run(fa[ks][i][0], fb[ks][j][0], acc[i][j]);
                }
    }

    // 32x32 accumulator layout: register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32.
    if (nsplit > 1) {
        // partial sums, [split][rowsA][rowsB] fp32
        float* pb = part + (size_t)split * rowsA * rowsB;
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                const int cb = row_b0 + wn * WTN + j * 32 + frag_row;
                if (cb >= rowsB) continue;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int ra = row_a0 + wm * WTM + i * 32 + 8 * (r / 4) + 4 * frag_half + (r % 4);
                    if (ra < rowsA) pb[(size_t)ra * rowsB + cb] = acc[i][j][r];
                }
            }
        return;
    }
    // Bias is added in fp32 and the sum rounded once to the storage type.
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            const int cb = row_b0 + wn * WTN + j * 32 + frag_row;      // column of this lane
            if (cb >= rowsB) continue;
            if (PIX_A) {
                // rows are output pixels, the column is k: y[t][k], lanes along k
                const float b = bias ? bias[cb] : 0.f;
                const EO* res = static_cast<const EO*>(post.residual);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int t = row_a0 + wm * WTM + i * 32 + 8 * (r / 4) + 4 * frag_half + (r % 4);
                    if (t < g.T) {
                        float v = acc[i][j][r] * post.scale + b;
                        if (post.addvec) v += post.addvec[(size_t)(t / HoWo) * g.K + cb];
                        if (res) v += to_f32<EO>(res[(size_t)t * g.K + cb]);
                        y[(size_t)t * g.K + cb] = from_f32<EO>(v);
                    }
                }
            } else {
                // rows are k, the column is an output pixel: y[n][k][p], lanes along p
                const int n = cb / HoWo, p = cb - n * HoWo;
                EO* yp = y + (size_t)n * g.K * HoWo + p;
                const EO* rp = post.residual ? static_cast<const EO*>(post.residual) + (size_t)n * g.K * HoWo + p : nullptr;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int k = row_a0 + wm * WTM + i * 32 + 8 * (r / 4) + 4 * frag_half + (r % 4);
                    if (k < g.K) {
                        float v = acc[i][j][r] * post.scale + (bias ? bias[k] : 0.f);
                        if (post.addvec) v += post.addvec[(size_t)n * g.K + k];
                        if (rp) v += to_f32<EO>(rp[(size_t)k * HoWo]);
                        yp[(size_t)k * HoWo] = from_f32<EO>(v);
                    }
                }
            }
        }
}

// Sum of the nsplit partial products (fixed order), bias, one rounding, y in its layout.
// part is [nsplit][rowsA][rowsB]; PIX_A: (t, k) -> y[t][k]; otherwise (k, t) -> y[n][k][p].
template <typename E, bool PIX_A>
__global__ void __launch_bounds__(256)
igemm_reduce_kernel(const float* __restrict__ part, const float* __restrict__ bias, E* __restrict__ y,
                    int K, int T, int HoWo, int nsplit, IgemmPost post) {
    const size_t total = (size_t)K * T;
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    float acc = 0.f;
    for (int sp = 0; sp < nsplit; ++sp) acc += part[(size_t)sp * total + e];
    acc *= post.scale;
    const E* res = static_cast<const E*>(post.residual);
    if (PIX_A) {
        const int k = (int)(e % K), t = (int)(e / K);
        acc += bias ? bias[k] : 0.f;
        if (post.addvec) acc += post.addvec[(size_t)(t / HoWo) * K + k];
        if (res) acc += to_f32<E>(res[e]);
        y[e] = from_f32<E>(acc);
    } else {
        const int t = (int)(e % T), k = (int)(e / T);
        const int n = t / HoWo, p = t - n * HoWo;
        const size_t o = ((size_t)n * K + k) * HoWo + p;
        acc += bias ? bias[k] : 0.f;
        if (post.addvec) acc += post.addvec[(size_t)n * K + k];
        if (res) acc += to_f32<E>(res[o]);
        y[o] = from_f32<E>(acc);
    }
}

// w[K][C][R][R] -> Wr[R*R][K][Cp] (channel index contiguous, zero-filled to Cp), followed by one row
// of Cp zeros that stands in for the pixels of the padding.
template <typename E>
__global__ void __launch_bounds__(256)
igemm_filter_repack_kernel(const E* __restrict__ w, E* __restrict__ Wr, int K, int C, int Cp, int taps) {
    const size_t total = (size_t)taps * K * Cp + Cp;
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    E v = from_f32<E>(0.f);
    if (e < (size_t)taps * K * Cp) {
        const int c = (int)(e % Cp);
        const size_t q = e / Cp;
        const int k = (int)(q % K), tap = (int)(q / K);
        if (c < C) v = w[((size_t)k * C + c) * taps + tap];
    }
    Wr[e] = v;
}

// x -> xh[N][H][W][Cp], zero-filled channels.  NCHW source: a 32 (w) x 64 (c) tile goes through LDS so
// that reads run along w and writes along c.  Channel-last source (C not a multiple of 8): plain copy.
template <typename E>
__global__ void __launch_bounds__(256)
igemm_relayout_nchw_kernel(const E* __restrict__ x, E* __restrict__ xh, int N, int C, int Cp, int H, int W, int wtiles, PreOp pre) {
    __shared__ E tile[64][33];
    int b = blockIdx.x;
    const int wt = b % wtiles; b /= wtiles;
    const int h = b % H; const int n = b / H;
    const int c0 = blockIdx.y * 64, w0 = wt * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;     // 32 x 8
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const int c = c0 + ty + 8 * k, wq = w0 + tx;
        E v = (c < C && wq < W) ? x[(((size_t)n * C + c) * H + h) * W + wq] : from_f32<E>(0.f);
        if (pre.stats && c < C) v = from_f32<E>(pre_apply(to_f32<E>(v), pre_lane(pre, n, c, C), true));   // SiLU(GroupNorm(x)), rounded once
        tile[ty + 8 * k][tx] = v;
    }
    __syncthreads();
    const int cx = threadIdx.x & 63, wy = threadIdx.x >> 6;     // 64 x 4
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const int wq = w0 + wy + 4 * k, c = c0 + cx;
        if (wq < W && c < Cp) xh[(((size_t)n * H + h) * W + wq) * Cp + c] = tile[cx][wy + 4 * k];
    }
}

// The same re-layout with 16-byte accesses on both sides, for rows of whole 16-byte chunks: a tile of
// 64 channels x TW pixels (TW = 8 chunks) of one image row goes through LDS; a lane reads one chunk
// along w, and writes one chunk of EPC adjacent channels of one pixel, gathered element by element
// from LDS (row pitch an odd number of words: conflict-free both ways).
template <typename E>
__global__ void __launch_bounds__(256)
igemm_relayout_nchw_vec_kernel(const E* __restrict__ x, E* __restrict__ xh, int N, int C, int Cp, int H, int W, int wtiles, PreOp pre) {
    constexpr int EPC = 16 / (int)sizeof(E);
    constexpr int EPW = 4 / (int)sizeof(E);
    constexpr int TW = 8 * EPC;                            // pixels per tile
    constexpr int PITCHW = TW / EPW + 1;                   // words per channel row, odd
    __shared__ uint32_t tile[64 * PITCHW];
    int b = blockIdx.x;
    const int wt = b % wtiles; b /= wtiles;
    const int h = b % H; const int n = b / H;
    const int c0 = blockIdx.y * 64, w0 = wt * TW;
    // in: 64 channels x 8 chunks = 512 chunks, two per lane
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int item = threadIdx.x + 256 * k;
        const int cl = item >> 3, ch = item & 7;
        const int c = c0 + cl, wq = w0 + ch * EPC;
        union { uint4 q; E e[EPC]; } v;
        v.q = make_uint4(0, 0, 0, 0);
        if (c < C && wq < W) {
            v.q = *reinterpret_cast<const uint4*>(x + (((size_t)n * C + c) * H + h) * W + wq);
            if (pre.stats) {                                  // SiLU(GroupNorm(x)), rounded once to the storage type
                const PreLane pl = pre_lane(pre, n, c, C);
#pragma unroll
                for (int i = 0; i < EPC; ++i) v.e[i] = from_f32<E>(pre_apply(to_f32<E>(v.e[i]), pl, true));
            }
        }
        uint32_t* d = tile + cl * PITCHW + ch * 4;
        d[0] = v.q.x; d[1] = v.q.y; d[2] = v.q.z; d[3] = v.q.w;
    }
    __syncthreads();
    // out: TW pixels x (64 / EPC) channel chunks
    const E* te = reinterpret_cast<const E*>(tile);
    constexpr int CCH = 64 / EPC;                          // chunks per pixel
    for (int item = threadIdx.x; item < TW * CCH; item += 256) {
        const int cg = item % CCH, wl = item / CCH;
        const int wq = w0 + wl, c = c0 + cg * EPC;
        if (wq >= W || c >= Cp) continue;
        union { E e[EPC]; uint4 v; } o;
#pragma unroll
        for (int i = 0; i < EPC; ++i) o.e[i] = te[(cg * EPC + i) * (PITCHW * EPW) + wl];
        *reinterpret_cast<uint4*>(xh + (((size_t)n * H + h) * W + wq) * Cp + c) = o.v;
    }
}

template <typename E>
__global__ void __launch_bounds__(256)
igemm_pad_nhwc_kernel(const E* __restrict__ x, E* __restrict__ xh, size_t pixels, size_t pixels_per_image, int C, int Cp, PreOp pre) {
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= pixels * Cp) return;
    const int c = (int)(e % Cp);
    const size_t p = e / Cp;
    E v = c < C ? x[p * C + c] : from_f32<E>(0.f);
    if (pre.stats && c < C) v = from_f32<E>(pre_apply(to_f32<E>(v), pre_lane(pre, (int)(p / pixels_per_image), c, C), true));
    xh[e] = v;
}

template <typename E, typename EO, int BM, int BN, int NST, bool PIX_A, int WGM = 2, int WGN = 2>
static hipError_t launch_igemm_cfg(const E* xh, const E* Wr, const float* bias, EO* y, float* part, int nsplit,
                                   const ConvGeom& g, const IgemmPost& post, hipStream_t s) {
    const int rowsA = PIX_A ? g.T : g.K, rowsB = PIX_A ? g.K : g.T;
    const int tiles_m = (rowsA + BM - 1) / BM, tiles_n = (rowsB + BN - 1) / BN;
    const long long total = (long long)tiles_m * tiles_n * nsplit;
    if (total > 0x3fffffffLL) return hipErrorInvalidValue;
    const int per_xcd = (int)((total + 7) / 8);
    constexpr int lds_bytes = (BM + BN) * 128 * NST;
    static_assert(lds_bytes <= 160 * 1024, "LDS budget");
    auto kern = conv_igemm_kernel<E, EO, BM, BN, NST, PIX_A, WGM, WGN>;
    // once per instantiation; a function-local static is initialised under the language's own lock
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (attr != hipSuccess) return attr;
    const E* zero_row = Wr + (size_t)g.R * g.R * g.K * g.Cp;
    hipLaunchKernelGGL(kern, dim3((unsigned)(per_xcd * 8)), dim3(WGM * WGN * 64), lds_bytes, s,
                       xh, Wr, zero_row, bias, y, part, g, post, tiles_m, tiles_n, (int)total, per_xcd, nsplit);
    if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
    if (nsplit > 1) {
        const size_t blocks = ((size_t)g.K * g.T + 255) / 256;
        if (blocks > 0x7fffffffULL) return hipErrorInvalidValue;
        hipLaunchKernelGGL((igemm_reduce_kernel<EO, PIX_A>), dim3((unsigned)blocks), dim3(256), 0, s, part, bias, y, g.K, g.T, g.Ho * g.Wo, nsplit, post);
    }
    return hipGetLastError();
}

// Block shape as (pixels x output channels).  The stage is bound by what a compute unit can pull from L2
// into LDS (26-37 bytes per clock measured), so the block with the fewest operand bytes per flop that
// still fills the chip wins: 256x256 (16 waves; 1.0 PFLOP/s on 512 channels at 256x256) when K is a
// multiple of 256, 256x128 (8 waves) when K is a multiple of 128, each while >= 256 blocks remain;
// then 128x128 while >= 256 blocks remain, else 64x64.
struct IgemmShape { int tp, tk; };
static IgemmShape igemm_shape(int T, int K) {
    static const IgemmShape menu[5] = {{128, 128}, {64, 64}, {256, 256}, {256, 128}, {128, 256}};
    auto blocks = [&](int tp, int tk) { return (long long)((T + tp - 1) / tp) * ((K + tk - 1) / tk); };
    if (K % 256 == 0 && blocks(256, 256) >= 256) return menu[2];
    if (K % 128 == 0 && blocks(256, 128) >= 256) return menu[3];
    if (blocks(128, 128) >= 256) return menu[0];
    return menu[1];
}

// Few blocks and a long reduction (deep down-sampling layers: 8x8 outputs, 9 x 1280 channels): cut the
// reduction so that about two workgroups per compute unit are in flight, at least eight stages each
// (the second kernel costs ~3 us, more than a short reduction gains).
int igemm_split(int T, int K, int Cp, int R, int dt) {
    // dt < 0: 8-bit operands, 128 reduction elements per stage
    const bool f16 = two_byte(dt);
    if (dt < 0) Cp = (Cp + 1) / 2;                        // same stage count as 64-element stages over half the channels
    const int bke = f16 ? 64 : 32;
    const int nstage = R * R * ((Cp + bke - 1) / bke);
    int sp = 1;
    {
        const IgemmShape sh = igemm_shape(T, K);
        const long long blocks = (long long)((T + sh.tp - 1) / sh.tp) * ((K + sh.tk - 1) / sh.tk);
        if (blocks < 256) sp = (int)((512 + blocks - 1) / blocks);
        if (sp > 16) sp = 16;
        if (sp > nstage / 8) sp = nstage / 8;
    }
    if (sp > nstage) sp = nstage;
    return sp < 1 ? 1 : sp;
}

template <typename E, typename EO, bool PIX_A>
static hipError_t launch_igemm_t(const E* xh, const E* Wr, const float* bias, EO* y, float* part, int nsplit,
                                 const ConvGeom& g, const IgemmPost& post, hipStream_t s) {
    // rows of the block: pixels when y is channel-last, output channels otherwise
    const IgemmShape sh = igemm_shape(g.T, g.K);
    const int bm = PIX_A ? sh.tp : sh.tk, bn = PIX_A ? sh.tk : sh.tp;
    if (bm == 256 && bn == 256) return launch_igemm_cfg<E, EO, 256, 256, 2, PIX_A, 4, 4>(xh, Wr, bias, y, part, nsplit, g, post, s);
    if (bm == 256 && bn == 128) return launch_igemm_cfg<E, EO, 256, 128, 2, PIX_A, 4, 2>(xh, Wr, bias, y, part, nsplit, g, post, s);
    if (bm == 128 && bn == 256) return launch_igemm_cfg<E, EO, 128, 256, 2, PIX_A, 2, 4>(xh, Wr, bias, y, part, nsplit, g, post, s);
    if (bm == 128) return launch_igemm_cfg<E, EO, 128, 128, 2, PIX_A>(xh, Wr, bias, y, part, nsplit, g, post, s);
    return launch_igemm_cfg<E, EO, 64, 64, 2, PIX_A>(xh, Wr, bias, y, part, nsplit, g, post, s);
}

hipError_t launch_igemm_filter_repack(const void* w, void* Wr, int K, int C, int R, int dt, hipStream_t s) {
    const int Cp = (C + 7) / 8 * 8, taps = R * R;
    const size_t total = (size_t)taps * K * Cp + Cp;
    const size_t blocks = (total + 255) / 256;
    if (blocks > 0x7fffffffULL) return hipErrorInvalidValue;
    return with_dtype(dt, [&](auto* tag) {
        using E = std::remove_pointer_t<decltype(tag)>;
        hipLaunchKernelGGL(igemm_filter_repack_kernel<E>, dim3((unsigned)blocks), dim3(256), 0, s, (const E*)w, (E*)Wr, K, C, Cp, taps);
        return hipGetLastError();
    });
}

template <typename E>
static hipError_t igemm_conv_t(const void* x, const void* Wr, const float* bias, void* y, const ConvGeom& g, const IgemmPost& post,
                               const PreOp& pre, bool nhwc, void* workspace, size_t xh_bytes, hipStream_t s) {
    const E* xh = static_cast<const E*>(x);
    const int nsplit = igemm_split(g.T, g.K, g.Cp, g.R, sizeof(E) == 2 ? DT_F16 : DT_F32);
    float* part = reinterpret_cast<float*>(static_cast<unsigned char*>(workspace) + xh_bytes);   // only used when nsplit > 1
    if (!nhwc) {
        constexpr int EPC = 16 / (int)sizeof(E);
        const bool chunks = g.Ws % EPC == 0;                 // x and the workspace are 16-byte aligned, so every row then is
        const int tw = chunks ? 8 * EPC : 32;
        const int wtiles = (g.Ws + tw - 1) / tw;
        const long long bx = (long long)g.N * g.Hs * wtiles;
        if (bx > 0x7fffffffLL || (g.Cp + 63) / 64 > 65535) return hipErrorInvalidValue;
        if (chunks)
            hipLaunchKernelGGL(igemm_relayout_nchw_vec_kernel<E>, dim3((unsigned)bx, (unsigned)((g.Cp + 63) / 64)), dim3(256), 0, s,
                               (const E*)x, (E*)workspace, g.N, g.C, g.Cp, g.Hs, g.Ws, wtiles, pre);
        else
            hipLaunchKernelGGL(igemm_relayout_nchw_kernel<E>, dim3((unsigned)bx, (unsigned)((g.Cp + 63) / 64)), dim3(256), 0, s,
                               (const E*)x, (E*)workspace, g.N, g.C, g.Cp, g.Hs, g.Ws, wtiles, pre);
        if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
        xh = static_cast<const E*>(workspace);
    } else if (g.C != g.Cp || pre.stats) {               // padding needed, or GroupNorm + SiLU to apply: a copy in the workspace
        const size_t pixels = (size_t)g.N * g.Hs * g.Ws;
        const size_t blocks = (pixels * g.Cp + 255) / 256;
        if (blocks > 0x7fffffffULL) return hipErrorInvalidValue;
        hipLaunchKernelGGL(igemm_pad_nhwc_kernel<E>, dim3((unsigned)blocks), dim3(256), 0, s, (const E*)x, (E*)workspace, pixels, (size_t)g.Hs * g.Ws, g.C, g.Cp, pre);
        if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
        xh = static_cast<const E*>(workspace);
    }
    return nhwc ? launch_igemm_t<E, E, true>(xh, (const E*)Wr, bias, (E*)y, part, nsplit, g, post, s)
                : launch_igemm_t<E, E, false>(xh, (const E*)Wr, bias, (E*)y, part, nsplit, g, post, s);
}

hipError_t launch_igemm_conv2d(const void* x, const void* Wr, const float* bias, void* y,
                               int N, int C, int H, int W, int K, int R, int st, int dt, bool nhwc,
                               void* workspace, size_t xh_bytes, int up, const PreOp* prep, const float* addvec, const void* residual,
                               hipStream_t s) {
    // a handful of output channels: one pass over x on the vector ALU instead of a re-layout and a padded MFMA tile
    if (fewk_conv_ok(x, N, C, H, W, K, R, st, dt, nhwc, up, prep && prep->stats, addvec || residual))
        return launch_fewk_conv3x3(x, Wr, bias, y, N, C, H, W, K, nhwc, s);
    IgemmPost post; post.addvec = addvec; post.residual = residual;
    const PreOp pre = prep ? *prep : PreOp();
    ConvGeom g;
    g.up = up; g.Hs = H >> up; g.Ws = W >> up;
    g.N = N; g.C = C; g.Cp = (C + 7) / 8 * 8; g.H = H; g.W = W; g.K = K; g.R = R; g.st = st; g.pad = (R - 1) / 2;
    g.Ho = (H + 2 * g.pad - R) / st + 1; g.Wo = (W + 2 * g.pad - R) / st + 1;
    g.T = N * g.Ho * g.Wo;
    return with_dtype(dt, [&](auto* tag) {
        using E = std::remove_pointer_t<decltype(tag)>;
        return igemm_conv_t<E>(x, Wr, bias, y, g, post, pre, nhwc, workspace, xh_bytes, s);
    });
}

// ---- quantised operands (E4M3, one power-of-two scale per tensor) ---------------------------------------------
// w[K][C][R][R] -> e4m3(w * sw) as Wq[R*R][K][Cq] (Cq = C rounded up to 16), followed by a row of Cq zeros.
template <typename E>
__global__ void __launch_bounds__(256)
igemm_filter_quant_kernel(const E* __restrict__ w, uint8_t* __restrict__ Wq, int K, int C, int Cq, int taps, float sw) {
    const size_t total = (size_t)taps * K * Cq + Cq;
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    uint32_t v = 0;
    if (e < (size_t)taps * K * Cq) {
        const int c = (int)(e % Cq);
        const size_t q = e / Cq;
        const int k = (int)(q % K), tap = (int)(q / K);
        if (c < C) v = quant_e4m3(to_f32<E>(w[((size_t)k * C + c) * taps + tap]) * sw);
    }
    Wq[e] = (uint8_t)v;
}

// x -> e4m3(x' * sx) as xq[N][H][W][Cq], x' = x or SiLU(GroupNorm(x)); four channels (one 32-bit store) per lane.
template <typename E>
__global__ void __launch_bounds__(256)
igemm_quant_nhwc_kernel(const E* __restrict__ x, uint32_t* __restrict__ xq, size_t pixels, size_t pixels_per_image, int C, int Cq,
                        float sx, PreOp pre) {
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    const int quads = Cq / 4;
    if (e >= pixels * quads) return;
    const int c0 = (int)(e % quads) * 4;
    const size_t p = e / quads;
    uint32_t out = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = c0 + i;
        if (c < C) {
            float v = to_f32<E>(x[p * C + c]);
            if (pre.stats) v = pre_apply(v, pre_lane(pre, (int)(p / pixels_per_image), c, C), true);
            out |= quant_e4m3(v * sx) << (8 * i);
        }
    }
    xq[e] = out;
}

// Channel-last source with C a multiple of 8 and 16-byte alignment: one 16-byte load (8 or 2x4 channels) and one
// 8-byte store per lane.
template <typename E>
__global__ void __launch_bounds__(256)
igemm_quant_nhwc_vec_kernel(const E* __restrict__ x, uint2* __restrict__ xq, size_t pixels, size_t pixels_per_image, int C, int Cq,
                            float sx, PreOp pre) {
    constexpr int EPC = 16 / (int)sizeof(E);               // elements per 16-byte load
    constexpr int LOADS = 8 / EPC;                         // loads per 8 output channels
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    const int octs = Cq / 8;
    if (e >= pixels * octs) return;
    const int c0 = (int)(e % octs) * 8;
    const size_t p = e / octs;
    uint32_t out[2] = {0u, 0u};
    if (c0 < C) {                                          // C is a multiple of 8: the whole octet is inside
        const int n = (int)(p / pixels_per_image);
#pragma unroll
        for (int l = 0; l < LOADS; ++l) {
            union { uint4 q; E e[EPC]; } v;
            v.q = *reinterpret_cast<const uint4*>(x + p * C + c0 + l * EPC);
#pragma unroll
            for (int i = 0; i < EPC; ++i) {
                const int j = l * EPC + i;
                float f = to_f32<E>(v.e[i]);
                if (pre.stats) f = pre_apply(f, pre_lane(pre, n, c0 + j, C), true);
                out[j >> 2] |= quant_e4m3(f * sx) << (8 * (j & 3));
            }
        }
    }
    xq[e] = make_uint2(out[0], out[1]);
}

// NCHW source: a 32 (w) x 64 (c) tile of quantised bytes goes through LDS; reads run along w, 32-bit stores along c.
template <typename E>
__global__ void __launch_bounds__(256)
igemm_quant_nchw_kernel(const E* __restrict__ x, uint32_t* __restrict__ xq, int N, int C, int Cq, int H, int W, int wtiles,
                        float sx, PreOp pre) {
    __shared__ uint8_t tile[64][36];
    int b = blockIdx.x;
    const int wt = b % wtiles; b /= wtiles;
    const int h = b % H; const int n = b / H;
    const int c0 = blockIdx.y * 64, w0 = wt * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;     // 32 x 8
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const int c = c0 + ty + 8 * k, wq = w0 + tx;
        uint32_t q = 0;
        if (c < C && wq < W) {
            float v = to_f32<E>(x[(((size_t)n * C + c) * H + h) * W + wq]);
            if (pre.stats) v = pre_apply(v, pre_lane(pre, n, c, C), true);
            q = quant_e4m3(v * sx);
        }
        tile[ty + 8 * k][tx] = (uint8_t)q;
    }
    __syncthreads();
    // 32 pixels x 16 channel quads
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int item = threadIdx.x + 256 * k;
        const int cq = item & 15, wl = item >> 4;
        const int wq = w0 + wl, c = c0 + cq * 4;
        if (wq < W && c < Cq) {
            const uint32_t v = (uint32_t)tile[cq * 4][wl] | ((uint32_t)tile[cq * 4 + 1][wl] << 8) |
                               ((uint32_t)tile[cq * 4 + 2][wl] << 16) | ((uint32_t)tile[cq * 4 + 3][wl] << 24);
            xq[((((size_t)n * H + h) * W + wq) * Cq + c) / 4] = v;
        }
    }
}

// The same with 16-byte accesses on both sides, for rows of whole 16-byte chunks: a tile of 64 channels x TW pixels;
// a lane quantises one chunk along w into LDS bytes and later writes 16 adjacent channels of one pixel.
template <typename E>
__global__ void __launch_bounds__(256)
igemm_quant_nchw_vec_kernel(const E* __restrict__ x, uint4* __restrict__ xq, int N, int C, int Cq, int H, int W, int wtiles,
                            float sx, PreOp pre) {
    constexpr int EPC = 16 / (int)sizeof(E);
    constexpr int TW = 8 * EPC;                            // pixels per tile
    constexpr int PITCH = TW + 4;                          // bytes per channel row (a multiple of 4, an odd number of words)
    __shared__ __attribute__((aligned(16))) uint8_t tile[64 * PITCH];
    int b = blockIdx.x;
    const int wt = b % wtiles; b /= wtiles;
    const int h = b % H; const int n = b / H;
    const int c0 = blockIdx.y * 64, w0 = wt * TW;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int item = threadIdx.x + 256 * k;            // 64 channels x 8 chunks
        const int cl = item >> 3, ch = item & 7;
        const int c = c0 + cl, wq = w0 + ch * EPC;
        uint32_t out[EPC / 4];
#pragma unroll
        for (int i = 0; i < EPC / 4; ++i) out[i] = 0u;
        if (c < C && wq < W) {
            union { uint4 q; E e[EPC]; } v;
            v.q = *reinterpret_cast<const uint4*>(x + (((size_t)n * C + c) * H + h) * W + wq);
            PreLane pl = {0.f, 0.f, false};
            if (pre.stats) pl = pre_lane(pre, n, c, C);
#pragma unroll
            for (int i = 0; i < EPC; ++i) {
                float f = to_f32<E>(v.e[i]);
                if (pre.stats) f = pre_apply(f, pl, true);
                out[i >> 2] |= quant_e4m3(f * sx) << (8 * (i & 3));
            }
        }
        uint32_t* d = reinterpret_cast<uint32_t*>(tile + cl * PITCH + ch * EPC);
#pragma unroll
        for (int i = 0; i < EPC / 4; ++i) d[i] = out[i];
    }
    __syncthreads();
    // out: TW pixels x 4 groups of 16 channels
    for (int item = threadIdx.x; item < TW * 4; item += 256) {
        const int wl = item % TW, cg = item / TW;
        const int wq = w0 + wl, c = c0 + cg * 16;
        if (wq >= W || c >= Cq) continue;
        uint32_t o[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < 16; ++i) o[i >> 2] |= (uint32_t)tile[(cg * 16 + i) * PITCH + wl] << (8 * (i & 3));
        xq[((((size_t)n * H + h) * W + wq) * Cq + c) / 16] = make_uint4(o[0], o[1], o[2], o[3]);
    }
}

hipError_t launch_igemm_fp8_filter_quant(const void* w, void* Wq, int K, int C, int R, int dt, float sw, hipStream_t s) {
    const int Cq = (C + 15) / 16 * 16, taps = R * R;
    const size_t total = (size_t)taps * K * Cq + Cq;
    const size_t blocks = (total + 255) / 256;
    if (blocks > 0x7fffffffULL) return hipErrorInvalidValue;
    return with_dtype(dt, [&](auto* tag) {
        using E = std::remove_pointer_t<decltype(tag)>;
        hipLaunchKernelGGL(igemm_filter_quant_kernel<E>, dim3((unsigned)blocks), dim3(256), 0, s, (const E*)w, (uint8_t*)Wq, K, C, Cq, taps, sw);
        return hipGetLastError();
    });
}

// x and y in `dt`; the workspace holds xq (xq_bytes) and then any partial sums.
hipError_t launch_igemm_fp8_conv2d(const void* x, const void* Wq, const float* bias, void* y,
                                   int N, int C, int H, int W, int K, int R, int st, int dt, bool nhwc,
                                   void* workspace, size_t xq_bytes, int up, const PreOp* prep, const float* addvec,
                                   const void* residual, float sx, float sw, hipStream_t s) {
    IgemmPost post; post.addvec = addvec; post.residual = residual; post.scale = 1.f / (sx * sw);
    const PreOp pre = prep ? *prep : PreOp();
    ConvGeom g;
    g.up = up; g.Hs = H >> up; g.Ws = W >> up;
    g.N = N; g.C = C; g.Cp = (C + 15) / 16 * 16; g.H = H; g.W = W; g.K = K; g.R = R; g.st = st; g.pad = (R - 1) / 2;
    g.Ho = (H + 2 * g.pad - R) / st + 1; g.Wo = (W + 2 * g.pad - R) / st + 1;
    g.T = N * g.Ho * g.Wo;
    return with_dtype(dt, [&](auto* tag) {
        using EO = std::remove_pointer_t<decltype(tag)>;
        const size_t pixels = (size_t)g.N * g.Hs * g.Ws;
        if (nhwc && g.C % 8 == 0) {
            const size_t blocks = (pixels * (g.Cp / 8) + 255) / 256;
            if (blocks > 0x7fffffffULL) return hipErrorInvalidValue;
            hipLaunchKernelGGL(igemm_quant_nhwc_vec_kernel<EO>, dim3((unsigned)blocks), dim3(256), 0, s, (const EO*)x, (uint2*)workspace,
                               pixels, (size_t)g.Hs * g.Ws, g.C, g.Cp, sx, pre);
        } else if (nhwc) {
            const size_t blocks = (pixels * (g.Cp / 4) + 255) / 256;
            if (blocks > 0x7fffffffULL) return hipErrorInvalidValue;
            hipLaunchKernelGGL(igemm_quant_nhwc_kernel<EO>, dim3((unsigned)blocks), dim3(256), 0, s, (const EO*)x, (uint32_t*)workspace,
                               pixels, (size_t)g.Hs * g.Ws, g.C, g.Cp, sx, pre);
        } else {
            constexpr int EPC = 16 / (int)sizeof(EO);
            const bool chunks = g.Ws % EPC == 0;            // x is 16-byte aligned, so every row then is
            const int tw = chunks ? 8 * EPC : 32;
            const int wtiles = (g.Ws + tw - 1) / tw;
            const long long bx = (long long)g.N * g.Hs * wtiles;
            if (bx > 0x7fffffffLL || (g.Cp + 63) / 64 > 65535) return hipErrorInvalidValue;
            if (chunks)
                hipLaunchKernelGGL(igemm_quant_nchw_vec_kernel<EO>, dim3((unsigned)bx, (unsigned)((g.Cp + 63) / 64)), dim3(256), 0, s,
                                   (const EO*)x, (uint4*)workspace, g.N, g.C, g.Cp, g.Hs, g.Ws, wtiles, sx, pre);
            else
                hipLaunchKernelGGL(igemm_quant_nchw_kernel<EO>, dim3((unsigned)bx, (unsigned)((g.Cp + 63) / 64)), dim3(256), 0, s,
                                   (const EO*)x, (uint32_t*)workspace, g.N, g.C, g.Cp, g.Hs, g.Ws, wtiles, sx, pre);
        }
        if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
        const int nsplit = igemm_split(g.T, g.K, g.Cp, g.R, -1);
        float* part = reinterpret_cast<float*>(static_cast<unsigned char*>(workspace) + xq_bytes);
        const fp8_t* xq = static_cast<const fp8_t*>(workspace);
        return nhwc ? launch_igemm_t<fp8_t, EO, true>(xq, (const fp8_t*)Wq, bias, (EO*)y, part, nsplit, g, post, s)
                    : launch_igemm_t<fp8_t, EO, false>(xq, (const fp8_t*)Wq, bias, (EO*)y, part, nsplit, g, post, s);
    });
}

}  // namespace wino
