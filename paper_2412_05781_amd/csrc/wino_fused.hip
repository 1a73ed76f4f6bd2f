// Steps (ii) and (iii) in one kernel (Section "Techniques"; its second paragraph argues for keeping
// dependent steps local): the alpha^2 matrix products and the output transform, for F(2x2,3x3).
//
// Step (iii) is linear in the product M, so the alpha^2 products of one block of (output channels x
// tiles) need not exist together.  A workgroup owns such a block for ALL positions (xi,nu) and walks
// them one after another: the reduction over c for one position leaves M[xi,nu] of the block in the
// MFMA accumulators, which is at once scattered into the m^2 = 4 output accumulators
//     Y[a][b] += A^T[a][xi] * A^T[b][nu] * M[xi,nu]            (coefficients 0, +1, -1)
// and overwritten by the next position.  Cost: five accumulator sets instead of one; gain: M (the
// largest tensor of the unfused path) is never written or read, the output transform launch is gone,
// and a workgroup streams alpha^2 * Cp/64 stages back to back instead of Cp/64, so start-up and drain are
// paid once per 16 products.  The epilogue adds bias (+ the optional vector and residual), crops to the
// image and rounds once to the storage type.
//
// Operand staging is that of the batched GEMM kernel: 128-byte stages per row, global -> LDS directly
// into a ring, XOR-swizzled 16-byte chunks, one barrier per stage, explicit vmcnt waits.
// ROWS_K = true : rows of the block are output channels (U), columns are tiles (V); y is NCHW.
// ROWS_K = false: operands swapped, rows are tiles, columns output channels; y is channel-last.
#include "wino_internal.h"
#include "wino_mma.h"

namespace wino {

namespace {

// A^T of F(2x2,3x3): rows (1 1 1 0) and (0 1 -1 -1); xi is wave-uniform
__device__ __forceinline__ float at2(int a, int xi) {
    return a == 0 ? (xi < 3 ? 1.f : 0.f) : (xi == 0 ? 0.f : (xi == 1 ? 1.f : -1.f));
}

template <typename E> __device__ __forceinline__ uint32_t pack_pair(float a, float b) {
    const E ea = from_f32<E>(a), eb = from_f32<E>(b);
    return (uint32_t)*reinterpret_cast<const uint16_t*>(&ea) | ((uint32_t)*reinterpret_cast<const uint16_t*>(&eb) << 16);
}
template <typename E> __device__ __forceinline__ float half_lo(uint32_t w) { const uint16_t h = (uint16_t)(w & 0xffffu); return to_f32<E>(*reinterpret_cast<const E*>(&h)); }
template <typename E> __device__ __forceinline__ float half_hi(uint32_t w) { const uint16_t h = (uint16_t)(w >> 16); return to_f32<E>(*reinterpret_cast<const E*>(&h)); }

struct FusedGeom { int N, K, H, W, th, tw, T; };

}  // namespace

template <typename E, int BM, int BN, int NST, int WGM, int WGN, bool ROWS_K>
__global__ void __launch_bounds__(WGM * WGN * 64)
wino_fused_f2_kernel(const E* __restrict__ Aop, const E* __restrict__ Bop, const float* __restrict__ bias, E* __restrict__ y,
                     int rowsA, int rowsB, int Cp, FusedGeom g, int tiles_m, int tiles_n, int total_blocks, int blocks_per_xcd,
                     int vec_ok, PostOp post) {
    constexpr int A2 = 16;                                // positions of F(2x2,3x3)
    constexpr int RB = 128;                               // stage bytes per row
    constexpr int CPR = RB / 16;                          // 16-byte chunks per row per stage
    constexpr int BKE = RB / (int)sizeof(E);              // reduction elements per stage
    constexpr int EPC = 16 / (int)sizeof(E);              // elements per chunk
    constexpr int ROWS = BM + BN;
    constexpr int RPL = 1024 / RB;                        // rows covered by one wave-wide load
    constexpr int NW = WGM * WGN;
    constexpr int LPW = ROWS / RPL / NW;                  // wave-wide loads per wave per stage
    constexpr int WTM = BM / WGM, WTN = BN / WGN;
    constexpr int FM = WTM / 32, FN = WTN / 32;
    constexpr int STAGE_BYTES = ROWS * RB;
    static_assert(WTM % 32 == 0 && WTN % 32 == 0 && ROWS % (RPL * NW) == 0, "tile shape");
    static_assert(BM % RPL == 0, "a wave-wide load lies wholly in one operand");
    static_assert(NST >= 2 && NST <= 5 && LPW * (NST - 1) < 64, "ring depth / vmcnt range");

    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];

    // one contiguous range of logical blocks per XCD; the shorter tile dimension runs fastest
    const int bid = blockIdx.x;
    const int logical = (bid % 8) * blocks_per_xcd + bid / 8;
    if (logical >= total_blocks) return;                  // uniform per workgroup, before any barrier
    int tm, tn;
    if (tiles_m <= tiles_n) { tm = logical % tiles_m; tn = logical / tiles_m; }
    else { tn = logical % tiles_n; tm = logical / tiles_n; }

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int row0 = tm * BM, col0 = tn * BN;

    // per-lane source rows of this lane's LPW loads; `cur` walks stage by stage through all positions
    const int lrow = lane / CPR, lchunk = lane % CPR;
    const E* cur[LPW];
    int src_chunk[LPW];
    const size_t planeA = (size_t)rowsA * Cp, planeB = (size_t)rowsB * Cp;
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
        const int row = (wave + NW * i) * RPL + lrow;       // row inside the stage, A rows first
        const int chunk = lchunk ^ ((row >> 1) & (CPR - 1));
        src_chunk[i] = chunk;
        if (row < BM) {
            int r = row0 + row; r = r < rowsA ? r : rowsA - 1;
            cur[i] = Aop + (size_t)r * Cp + chunk * EPC;
        } else {
            int r = col0 + (row - BM); r = r < rowsB ? r : rowsB - 1;
            cur[i] = Bop + (size_t)r * Cp + chunk * EPC;
        }
    }

    const int nk = (Cp + BKE - 1) / BKE;
    const bool ragged = (Cp % BKE) != 0;
    const int total = A2 * nk;

    // issues stage number `s` (position s / nk, reduction stage s % nk); called with s ascending
    int issue_kt = 0;
    auto issue_stage = [&](int s) {
        unsigned char* slot = lds + (s % NST) * STAGE_BYTES;
        if (ragged && issue_kt == nk - 1) {
            // last, partial stage of a position: through registers, chunks beyond Cp become zeros
#pragma unroll
            for (int i = 0; i < LPW; ++i) {
                const int gk = issue_kt * BKE + src_chunk[i] * EPC;
                uint4 v = make_uint4(0, 0, 0, 0);
                if (gk < Cp) v = *reinterpret_cast<const uint4*>(cur[i]);
                *reinterpret_cast<uint4*>(slot + (wave + NW * i) * 1024 + lane * 16) = v;
            }
        } else {
#pragma unroll
            for (int i = 0; i < LPW; ++i) dma_load_1k(cur[i], slot + (wave + NW * i) * 1024);
        }
        if (++issue_kt == nk) {
            issue_kt = 0;
#pragma unroll
            for (int i = 0; i < LPW; ++i) {
                const bool isA = ((wave + NW * i) * RPL) < BM;         // wave-uniform
                cur[i] += (isA ? planeA : planeB) - (size_t)(nk - 1) * BKE;
            }
        } else {
#pragma unroll
            for (int i = 0; i < LPW; ++i) cur[i] += BKE;
        }
    };

    float16_t accM[FM][FN], accY[4][FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) {
#pragma unroll
            for (int r = 0; r < 16; ++r) accM[i][j][r] = 0.f;
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int r = 0; r < 16; ++r) accY[q][i][j][r] = 0.f;
        }

#pragma unroll
    for (int s = 0; s < NST - 1; ++s)
        if (s < total) issue_stage(s);

    const int frag_row = lane & 31, frag_half = lane >> 5;
    int s = 0;
    for (int pos = 0; pos < A2; ++pos) {
        for (int kt = 0; kt < nk; ++kt, ++s) {
            // Stage s must have landed.  Transfers complete in issue order, so it is enough to allow as many
            // outstanding as were issued after it: NST-2 stages in steady state, and once the ring stops
            // refilling simply everything.
            if (s + NST - 1 >= total) wait_vmcnt<0>();
            else wait_vmcnt<(NST - 2) * LPW>();
            __syncthreads();            // stage s visible to all waves; everyone is done with stage s-1
            if (s + NST - 1 < total) issue_stage(s + NST - 1);   // refills the slot stage s-1 used

            const unsigned char* slot = lds + (s % NST) * STAGE_BYTES;
            uint4 fa[CPR / 2][FM], fb[CPR / 2][FN];
#pragma unroll
            for (int ks = 0; ks < CPR / 2; ++ks) {
#pragma unroll
                for (int i = 0; i < FM; ++i) {
                    const int row = wm * WTM + i * 32 + frag_row;
                    const int chunk = (2 * ks + frag_half) ^ ((row >> 1) & (CPR - 1));
                    fa[ks][i] = *reinterpret_cast<const uint4*>(slot + row * RB + chunk * 16);
                }
#pragma unroll
                for (int j = 0; j < FN; ++j) {
                    const int row = BM + wn * WTN + j * 32 + frag_row;
                    const int chunk = (2 * ks + frag_half) ^ ((row >> 1) & (CPR - 1));
                    fb[ks][j] = *reinterpret_cast<const uint4*>(slot + row * RB + chunk * 16);
                }
            }
#pragma unroll
            for (int ks = 0; ks < CPR / 2; ++ks)
#pragma unroll
                for (int i = 0; i < FM; ++i)
#pragma unroll
                    for (int j = 0; j < FN; ++j) Mma<E>::run(fa[ks][i], fb[ks][j], accM[i][j]);
        }
        // step (iii), folded in: scatter this position's product into the four output accumulators
        const int xi = pos >> 2, nu = pos & 3;
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                const float c = at2(a, xi) * at2(b, nu);          // wave-uniform: 0, +1 or -1
                if (c != 0.f) {
#pragma unroll
                    for (int i = 0; i < FM; ++i)
#pragma unroll
                        for (int j = 0; j < FN; ++j)
#pragma unroll
                            for (int r = 0; r < 16; ++r) accY[a * 2 + b][i][j][r] = fmaf(c, accM[i][j][r], accY[a * 2 + b][i][j][r]);
                }
            }
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) accM[i][j][r] = 0.f;
    }

    // ---- epilogue: bias (+ vector, + residual), crop, round once, store ---------------------------------------
    // 32x32 accumulator layout: register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32
    const int H = g.H, W = g.W, K = g.K;
    const E* res = static_cast<const E*>(post.residual);
    if constexpr (ROWS_K) {
        // columns are tiles: a lane owns one tile, its registers run over output channels; the two pixels of an output
        // row of the tile are stored together, and neighbouring lanes hold neighbouring tiles of a tile row
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            int t = col0 + wn * WTN + j * 32 + frag_row;
            const bool t_ok = t < g.T;
            t = t_ok ? t : g.T - 1;
            const int tj = t % g.tw; const int q = t / g.tw;
            const int ti = q % g.th, n = q / g.th;
            const int i0 = 2 * ti, j0 = 2 * tj;
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int k = row0 + wm * WTM + i * 32 + 8 * (r / 4) + 4 * frag_half + (r % 4);
                    if (k < K && t_ok) {
                        const float bb = (bias ? bias[k] : 0.f) + (post.addvec ? post.addvec[(size_t)n * K + k] : 0.f);
                        const size_t off = (((size_t)n * K + k) * H + i0) * W + j0;
#pragma unroll
                        for (int a = 0; a < 2; ++a) {
                            if (i0 + a >= H) continue;
                            float v0 = accY[a * 2 + 0][i][j][r] + bb, v1 = accY[a * 2 + 1][i][j][r] + bb;
                            const size_t o = off + (size_t)a * W;
                            if (vec_ok) {
                                if constexpr (sizeof(E) == 4) {
                                    if (res) { const float2 rr = *reinterpret_cast<const float2*>(res + o); v0 += rr.x; v1 += rr.y; }
                                    *reinterpret_cast<float2*>(y + o) = make_float2(v0, v1);
                                } else {
                                    if (res) { const uint32_t rr = *reinterpret_cast<const uint32_t*>(res + o); v0 += half_lo<E>(rr); v1 += half_hi<E>(rr); }
                                    *reinterpret_cast<uint32_t*>(y + o) = pack_pair<E>(v0, v1);
                                }
                            } else {
                                y[o] = from_f32<E>(v0 + (res ? to_f32<E>(res[o]) : 0.f));
                                if (j0 + 1 < W) y[o + 1] = from_f32<E>(v1 + (res ? to_f32<E>(res[o + 1]) : 0.f));
                            }
                        }
                    }
                }
        }
    } else {
        // columns are output channels: lanes run along k, which is contiguous in a channel-last y
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            const int k = col0 + wn * WTN + j * 32 + frag_row;
            const bool k_ok = k < K;
            const float bk = (bias && k_ok) ? bias[k] : 0.f;
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int t = row0 + wm * WTM + i * 32 + 8 * (r / 4) + 4 * frag_half + (r % 4);
                    if (t < g.T && k_ok) {
                        const int tj = t % g.tw; const int q = t / g.tw;
                        const int ti = q % g.th, n = q / g.th;
                        const float bb = bk + (post.addvec ? post.addvec[(size_t)n * K + k] : 0.f);
#pragma unroll
                        for (int a = 0; a < 2; ++a)
#pragma unroll
                            for (int b = 0; b < 2; ++b) {
                                const int ii = 2 * ti + a, jj = 2 * tj + b;
                                if (ii < H && jj < W) {
                                    const size_t o = (((size_t)n * H + ii) * W + jj) * K + k;
                                    y[o] = from_f32<E>(accY[a * 2 + b][i][j][r] + bb + (res ? to_f32<E>(res[o]) : 0.f));
                                }
                            }
                    }
                }
        }
    }
}

template <typename E, int BM, int BN, int NST, int WGM, int WGN, bool ROWS_K>
static hipError_t launch_fused_cfg(const void* Aop, const void* Bop, int rowsA, int rowsB, const float* bias, void* y,
                                   const Geom& g, const PostOp& post, hipStream_t s) {
    const int tiles_m = (rowsA + BM - 1) / BM, tiles_n = (rowsB + BN - 1) / BN;
    const long long total = (long long)tiles_m * tiles_n;
    if (total > 0x3fffffffLL) return hipErrorInvalidValue;
    const int per_xcd = (int)((total + 7) / 8);
    constexpr int lds_bytes = (BM + BN) * 128 * NST;
    static_assert(lds_bytes <= 160 * 1024, "LDS budget");
    auto kern = wino_fused_f2_kernel<E, BM, BN, NST, WGM, WGN, ROWS_K>;
    // once per instantiation; a function-local static is initialised under the language's own lock
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (attr != hipSuccess) return attr;
    FusedGeom fg{g.N, g.K, g.H, g.W, g.th, g.tw, g.T};
    // paired stores of a tile's output row need even W (the pair then never straddles the row end) and 4-byte alignment
    const int vec_ok = (g.W % 2 == 0) && ((reinterpret_cast<uintptr_t>(y) & 7u) == 0) && ((reinterpret_cast<uintptr_t>(post.residual) & 7u) == 0);
    hipLaunchKernelGGL(kern, dim3((unsigned)(per_xcd * 8)), dim3(WGM * WGN * 64), lds_bytes, s,
                       (const E*)Aop, (const E*)Bop, bias, (E*)y, rowsA, rowsB, g.Cp, fg, tiles_m, tiles_n, (int)total, per_xcd, vec_ok, post);
    return hipGetLastError();
}

// Block shapes on offer (rows x columns of the block, waves): 0 = 64x64 (2x2 waves), 1 = 64x128, 2 = 128x64,
// 3 = 128x128 (each wave 64x64: 320 accumulator registers, one workgroup per compute unit).
int fused_pick_shape(int rows, int cols) {
    auto blocks = [&](int bm, int bn) { return (long long)((rows + bm - 1) / bm) * ((cols + bn - 1) / bn); };
    // the largest block that still leaves at least one workgroup per compute unit
    if (blocks(128, 128) >= 256) return 3;
    if (rows >= cols ? blocks(128, 64) >= 256 : blocks(64, 128) >= 256) return rows >= cols ? 2 : 1;
    if (rows >= cols ? blocks(64, 128) >= 256 : blocks(128, 64) >= 256) return rows >= cols ? 1 : 2;
    return 0;
}

template <typename E, bool ROWS_K>
static hipError_t launch_fused_t(const void* Aop, const void* Bop, int rowsA, int rowsB, const float* bias, void* y,
                                 const Geom& g, const PostOp& post, int shape, hipStream_t s) {
    switch (shape) {
        case 1: return launch_fused_cfg<E, 64, 128, 4, 2, 2, ROWS_K>(Aop, Bop, rowsA, rowsB, bias, y, g, post, s);
        case 2: return launch_fused_cfg<E, 128, 64, 4, 2, 2, ROWS_K>(Aop, Bop, rowsA, rowsB, bias, y, g, post, s);
        case 3: return launch_fused_cfg<E, 128, 128, 4, 2, 2, ROWS_K>(Aop, Bop, rowsA, rowsB, bias, y, g, post, s);
        default: return launch_fused_cfg<E, 64, 64, 4, 2, 2, ROWS_K>(Aop, Bop, rowsA, rowsB, bias, y, g, post, s);
    }
}

hipError_t launch_fused_gemm_output(const void* U, const void* V, const float* bias, void* y, const Geom& g, int dt, bool nhwc,
                                    const PostOp* postp, int shape, hipStream_t s) {
    if (g.m != 2) return hipErrorInvalidValue;
    if (shape < -1 || shape > 3) return hipErrorInvalidValue;
    const PostOp post = postp ? *postp : PostOp();
    return with_dtype(dt, [&](auto* tag) {
        using E = std::remove_pointer_t<decltype(tag)>;
        if (nhwc) return launch_fused_t<E, false>(V, U, g.T, g.K, bias, y, g, post, shape < 0 ? fused_pick_shape(g.T, g.K) : shape, s);
        return launch_fused_t<E, true>(U, V, g.K, g.T, bias, y, g, post, shape < 0 ? fused_pick_shape(g.K, g.T) : shape, s);
    });
}

}  // namespace wino
