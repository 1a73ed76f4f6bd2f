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

// RAGGED = true: Cp is not a multiple of the stage (64 fp16 / 32 fp32 elements); the last stage of every position
// then goes through registers with zero fill.  The common case (RAGGED = false) has no such code in its loop.
template <typename E, int BM, int BN, int NST, int WGM, int WGN, bool ROWS_K, bool RAGGED>
__global__ void __launch_bounds__(WGM * WGN * 64)
wino_fused_f2_kernel(const E* __restrict__ Aop, const E* __restrict__ Bop, const float* __restrict__ bias, E* __restrict__ y,
                     int rowsA, int rowsB, int Cp, FusedGeom g, int tiles_m, int tiles_n, int total_blocks, int blocks_per_xcd,
                     int vec_ok, PostOp post) {
    constexpr int A2 = 16;                                // positions of F(2x2,3x3)
    constexpr int RB = 128;                               // stage bytes per row
    constexpr int CPR = RB / 16;                          // 16-byte chunks per row per stage
    constexpr int BKE = RB / (int)sizeof(E);              // reduction elements per stage
    constexpr int ROWS = BM + BN;
    constexpr int RPL = 1024 / RB;                        // rows covered by one wave-wide load
    constexpr int NW = WGM * WGN;
    constexpr int LPW = ROWS / RPL / NW;                  // wave-wide loads per wave per stage
    constexpr int LA = BM / (RPL * NW);                   // ... of which from the row operand
    constexpr int WTM = BM / WGM, WTN = BN / WGN;
    constexpr int FM = WTM / 32, FN = WTN / 32;
    constexpr int STAGE_BYTES = ROWS * RB;
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "tile shape");
    static_assert(BM % (RPL * NW) == 0 && BN % (RPL * NW) == 0, "load i of every wave lies in the same operand");
    static_assert(NST >= 2 && (NST & (NST - 1)) == 0 && LPW * (NST - 1) < 64, "ring depth: a power of two, within the vmcnt range");

    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];

    // one contiguous range of logical blocks per XCD; the shorter tile dimension runs fastest
    const int bid = blockIdx.x;
    const int logical = (bid % 8) * blocks_per_xcd + bid / 8;
    if (logical >= total_blocks) return;                  // uniform per workgroup, before any barrier
    int tm, tn;
    if (tiles_m <= tiles_n) { tm = logical % tiles_m; tn = logical / tiles_m; }
    else { tn = logical % tiles_n; tm = logical / tiles_n; }

    // Everything that does not depend on the lane is kept in scalar registers (the wave index through readfirstlane),
    // so that the per-stage bookkeeping - LDS destinations, stage bases, slot offsets - runs on the scalar unit: with one
    // or two waves per SIMD every vector instruction spent on addresses is time the MFMA pipe sits idle.
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;
    const int row0 = tm * BM, col0 = tn * BN;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_byte_t*)lds;          // LDS byte address of the ring

    // Global side: one scalar base per operand that walks stage by stage through all positions, plus a fixed 32-bit byte
    // offset per lane and load (row inside the block, clamped to the last valid row, and the swizzled chunk).
    const size_t row_bytes = (size_t)Cp * sizeof(E);
    const int lrow = lane / CPR, lchunk = lane % CPR;
    uint32_t goff[LPW];
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
        const int row = (wave + NW * i) * RPL + lrow;       // row inside the stage, row-operand rows first
        const int chunk = lchunk ^ ((row >> 1) & (CPR - 1));
        int r;
        if (i < LA) { r = row0 + row; r = (r < rowsA ? r : rowsA - 1) - row0; }
        else { r = col0 + (row - BM); r = (r < rowsB ? r : rowsB - 1) - col0; }
        goff[i] = (uint32_t)r * (uint32_t)row_bytes + (uint32_t)chunk * 16u;
    }
    const unsigned char* sA = reinterpret_cast<const unsigned char*>(Aop) + (size_t)row0 * row_bytes;
    const unsigned char* sB = reinterpret_cast<const unsigned char*>(Bop) + (size_t)col0 * row_bytes;
    const size_t planeA = (size_t)rowsA * row_bytes, planeB = (size_t)rowsB * row_bytes;

    const int nk = (Cp + BKE - 1) / BKE;
    const int total = A2 * nk;
    const uint32_t wave_dst = lds0 + (uint32_t)wave * 1024u;

    // issues the next stage in order into ring slot `slot`
    int issue_kt = 0;
    auto issue_stage = [&](int slot) {
        const uint32_t dst = wave_dst + (uint32_t)slot * STAGE_BYTES;
        if (RAGGED && issue_kt == nk - 1) {
            // last, partial stage of a position: through registers, chunks beyond Cp become zeros
#pragma unroll
            for (int i = 0; i < LPW; ++i) {
                const int row = (wave + NW * i) * RPL + lrow;
                const int chunk = lchunk ^ ((row >> 1) & (CPR - 1));
                uint4 v = make_uint4(0, 0, 0, 0);
                if ((size_t)issue_kt * RB + (size_t)chunk * 16 < row_bytes) v = *reinterpret_cast<const uint4*>((i < LA ? sA : sB) + goff[i]);
                *reinterpret_cast<uint4*>(lds + (size_t)slot * STAGE_BYTES + (size_t)(wave + NW * i) * 1024 + lane * 16) = v;
            }
        } else {
#pragma unroll
            for (int i = 0; i < LPW; ++i) dma_load_1k_s(i < LA ? sA : sB, goff[i], dst + (uint32_t)(NW * i) * 1024u);
        }
        if (++issue_kt == nk) {
            issue_kt = 0;
            sA += planeA - (size_t)(nk - 1) * RB;
            sB += planeB - (size_t)(nk - 1) * RB;
        } else {
            sA += RB;
            sB += RB;
        }
    };

    // One product accumulator per 32x32 sub-tile; a wave with a single sub-tile keeps two and alternates between them,
    // so that consecutive MFMAs do not wait for each other.
    constexpr int NACC = (FM * FN == 1) ? 2 : 1;
    float16_t accM[NACC][FM][FN], accY[4][FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) {
#pragma unroll
            for (int q = 0; q < NACC; ++q)
#pragma unroll
                for (int r = 0; r < 16; ++r) accM[q][i][j][r] = 0.f;
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int r = 0; r < 16; ++r) accY[q][i][j][r] = 0.f;
        }

    // The reduction steps of a stage are taken in two halves, and the fragments of the next half are read from LDS while
    // the MFMAs of the current one run (the second half of a stage overlaps with the first reads of the next stage, after
    // the barrier that makes it visible).  Written out explicitly, with scheduling barriers between the phases: left
    // to itself the compiler puts every fragment read directly in front of the MFMA that uses it and waits for it there.
    // Fragment addresses: the swizzled chunk of step ks is chunk(0) ^ 2ks, i.e. the byte address of step 0 with bits 5-6
    // flipped, and sub-tile i lies 32 rows further on; so two per-lane addresses (one per operand) serve a whole stage.
    constexpr int KS = CPR / 2;                           // MFMA steps per stage (one 16-byte chunk pair each)
    constexpr int KH = KS / 2;                            // per half
    static_assert(KS % 2 == 0, "two halves per stage");
    static_assert((FM - 1) * 32 * RB < 65536 && (FN - 1) * 32 * RB < 65536, "sub-tile offsets fit the ds_read offset field");
    u32x4_t fa[2][KH][FM], fb[2][KH][FN];
    const int frag_row = lane & 31, frag_half = lane >> 5;
    const int rowA = wm * WTM + frag_row, rowB = BM + wn * WTN + frag_row;
    const uint32_t fbaseA = lds0 + (uint32_t)rowA * RB + (uint32_t)((frag_half ^ ((rowA >> 1) & (CPR - 1))) << 4);
    const uint32_t fbaseB = lds0 + (uint32_t)rowB * RB + (uint32_t)((frag_half ^ ((rowB >> 1) & (CPR - 1))) << 4);
    constexpr int NREAD = KH * (FM + FN);                 // fragment reads per half
    auto read_half = [&](int slot, auto hc, auto bufc) {
        constexpr int h = decltype(hc)::value, buf = decltype(bufc)::value;
        const uint32_t a0 = fbaseA + (uint32_t)slot * STAGE_BYTES, b0 = fbaseB + (uint32_t)slot * STAGE_BYTES;
        static_for<KH>([&](auto kc) {
            constexpr int kk = decltype(kc)::value;
            const uint32_t flip = (uint32_t)((h * KH + kk) << 5);
            static_for<FM>([&](auto ic) { constexpr int i = decltype(ic)::value; lds_read16_async<i * 32 * RB>(fa[buf][kk][i], a0 ^ flip); });
            static_for<FN>([&](auto jc) { constexpr int j = decltype(jc)::value; lds_read16_async<j * 32 * RB>(fb[buf][kk][j], b0 ^ flip); });
        });
    };
    // everything but the `newer` most recent reads has arrived; ties buffer `buf` to that point
    auto await_half = [&](auto bufc, auto newerc) {
        constexpr int buf = decltype(bufc)::value;
        lds_wait<decltype(newerc)::value>();
#pragma unroll
        for (int kk = 0; kk < KH; ++kk) {
#pragma unroll
            for (int i = 0; i < FM; ++i) pin(fa[buf][kk][i]);
#pragma unroll
            for (int j = 0; j < FN; ++j) pin(fb[buf][kk][j]);
        }
    };
    auto mma_half = [&](auto bufc) {
        constexpr int buf = decltype(bufc)::value;
#pragma unroll
        for (int kk = 0; kk < KH; ++kk)
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j) Mma<E>::run(fa[buf][kk][i], fb[buf][kk][j], accM[kk % NACC][i][j]);
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;

    // prologue: fill the ring, wait for stage 0, read its first half
#pragma unroll
    for (int s = 0; s < NST; ++s)
        if (s < total) issue_stage(s);
    if (NST - 1 >= total) wait_vmcnt<0>();
    else wait_vmcnt<(NST - 1) * LPW>();
    __syncthreads();
    read_half(0, I0(), I0());

    int kt = 0, pos = 0;
    // after the last MFMA of a stage: at the end of a position, step (iii) folded in - the position's product is scattered
    // into the four output accumulators and cleared
    auto end_of_stage = [&]() {
        if (++kt < nk) return;
        kt = 0;
        const int xi = pos >> 2, nu = pos & 3;
        ++pos;
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
                            for (int r = 0; r < 16; ++r) {
                                float m = accM[0][i][j][r];
                                if constexpr (NACC == 2) m += accM[1][i][j][r];
                                accY[a * 2 + b][i][j][r] = fmaf(c, m, accY[a * 2 + b][i][j][r]);
                            }
                }
            }
#pragma unroll
        for (int q = 0; q < NACC; ++q)
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) accM[q][i][j][r] = 0.f;
    };
    // All stages but the last (which is peeled, so that the loop body has no conditional LDS traffic: with one, the
    // compiler's wait insertion falls back to waiting for the newest reads before the second half's MFMAs).
    using NR = std::integral_constant<int, NREAD>;
    for (int s = 0; s < total - 1; ++s) {
        const int slot = s & (NST - 1), next_slot = (s + 1) & (NST - 1);
        // first half: its fragments (buffer 0) were requested one half earlier; request the second half, then multiply
        read_half(slot, I1(), I1());
        await_half(I0(), NR());
        __builtin_amdgcn_sched_barrier(0);
        mma_half(I0());
        __builtin_amdgcn_sched_barrier(0);
        // second half: meanwhile make stage s+1 visible, refill the slot of stage s, and request the first half of stage
        // s+1.  Transfers complete in issue order, so stage s+1 has landed once no more are outstanding than were issued
        // after it (NST-2 stages in steady state; near the end simply everything).
        if (s + NST >= total) wait_vmcnt<0>();
        else wait_vmcnt<(NST - 2) * LPW>();
        await_half(I1(), I0());         // this wave has read all of stage s
        __syncthreads();                // stage s+1 visible to all waves; every wave has read all of stage s
        if (s + NST < total) issue_stage(slot);                  // stage s+NST, into the slot stage s used
        read_half(next_slot, I0(), I0());
        __builtin_amdgcn_sched_barrier(0);
        mma_half(I1());
        __builtin_amdgcn_sched_barrier(0);
        end_of_stage();
    }
    read_half((total - 1) & (NST - 1), I1(), I1());
    await_half(I0(), NR());
    mma_half(I0());
    await_half(I1(), I0());
    mma_half(I1());
    end_of_stage();

    // ---- epilogue: bias (+ vector, + residual), crop, round once, store ---------------------------------------
    // 32x32 accumulator layout: register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32
    const int H = g.H, W = g.W, K = g.K;
    const E* res = static_cast<const E*>(post.residual);
    if constexpr (ROWS_K) {
        // columns are tiles: a lane owns one tile, its registers run over output channels; the two pixels of an output
        // row of the tile are stored together, and neighbouring lanes hold neighbouring tiles of a tile row
        // bias (and the per-image vector) of this lane's 16 x FM output channels: loaded up front from clamped indices, all
        // loads in flight together (inside the guarded store loop each would be waited for on its own)
        float bk[FM][16];
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int k = row0 + wm * WTM + i * 32 + 8 * (r / 4) + 4 * frag_half + (r % 4);
                bk[i][r] = bias ? bias[k < K ? k : K - 1] : 0.f;
            }
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            int t = col0 + wn * WTN + j * 32 + frag_row;
            const bool t_ok = t < g.T;
            t = t_ok ? t : g.T - 1;
            const int tj = t % g.tw; const int q = t / g.tw;
            const int ti = q % g.th, n = q / g.th;
            const int i0 = 2 * ti, j0 = 2 * tj;
            float av[FM][16];
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int k = row0 + wm * WTM + i * 32 + 8 * (r / 4) + 4 * frag_half + (r % 4);
                    av[i][r] = post.addvec ? post.addvec[(size_t)n * K + (k < K ? k : K - 1)] : 0.f;
                }
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int k = row0 + wm * WTM + i * 32 + 8 * (r / 4) + 4 * frag_half + (r % 4);
                    if (k < K && t_ok) {
                        const float bb = bk[i][r] + av[i][r];
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

template <typename E, int BM, int BN, int NST, int WGM, int WGN, bool ROWS_K, bool RAGGED = false>
static hipError_t launch_fused_cfg(const void* Aop, const void* Bop, int rowsA, int rowsB, const float* bias, void* y,
                                   const Geom& g, const PostOp& post, hipStream_t s) {
    const int tiles_m = (rowsA + BM - 1) / BM, tiles_n = (rowsB + BN - 1) / BN;
    const long long total = (long long)tiles_m * tiles_n;
    if (total > 0x3fffffffLL) return hipErrorInvalidValue;
    const int per_xcd = (int)((total + 7) / 8);
    constexpr int lds_bytes = (BM + BN) * 128 * NST;
    static_assert(lds_bytes <= 160 * 1024, "LDS budget");
    // lane offsets are 32-bit: a block's rows must span less than 2 GB
    if ((size_t)g.Cp * sizeof(E) * (size_t)(BM > BN ? BM : BN) >= ((size_t)1 << 31)) return hipErrorInvalidValue;
    auto kern = wino_fused_f2_kernel<E, BM, BN, NST, WGM, WGN, ROWS_K, RAGGED>;
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

// Block shapes on offer (rows x columns of the block): 0 = 64x64, 1 = 64x128, 2 = 128x64, 3 = 128x128 (four waves, 2x2),
// 4 = 128x128, 5 = 128x64, 6 = 64x128 (eight waves: two per SIMD, each with half the accumulators).
// Measured on the SD-shaped layers: the larger blocks pay only while they still fill the chip.
int fused_pick_shape(int rows, int cols) {
    auto blocks = [&](int bm, int bn) { return (long long)((rows + bm - 1) / bm) * ((cols + bn - 1) / bn); };
    if (blocks(128, 128) >= 160) return 4;
    if (rows >= cols ? blocks(64, 128) >= 200 : blocks(128, 64) >= 200) return rows >= cols ? 6 : 5;
    return 0;
}

template <typename E, bool ROWS_K>
static hipError_t launch_fused_t(const void* Aop, const void* Bop, int rowsA, int rowsB, const float* bias, void* y,
                                 const Geom& g, const PostOp& post, int shape, hipStream_t s) {
    // a reduction length that is not a whole number of stages: one block shape with the zero-filling last stage
    if (g.Cp % (128 / (int)sizeof(E)) != 0)
        return launch_fused_cfg<E, 64, 64, 4, 2, 2, ROWS_K, true>(Aop, Bop, rowsA, rowsB, bias, y, g, post, s);
    switch (shape) {
        case 0: return launch_fused_cfg<E, 64, 64, 4, 2, 2, ROWS_K>(Aop, Bop, rowsA, rowsB, bias, y, g, post, s);
        case 1: return launch_fused_cfg<E, 64, 128, 4, 2, 2, ROWS_K>(Aop, Bop, rowsA, rowsB, bias, y, g, post, s);
        case 2: return launch_fused_cfg<E, 128, 64, 4, 2, 2, ROWS_K>(Aop, Bop, rowsA, rowsB, bias, y, g, post, s);
        case 3: return launch_fused_cfg<E, 128, 128, 4, 2, 2, ROWS_K>(Aop, Bop, rowsA, rowsB, bias, y, g, post, s);
        case 4: return launch_fused_cfg<E, 128, 128, 4, 4, 2, ROWS_K>(Aop, Bop, rowsA, rowsB, bias, y, g, post, s);
        case 5: return launch_fused_cfg<E, 128, 64, 4, 4, 2, ROWS_K>(Aop, Bop, rowsA, rowsB, bias, y, g, post, s);
        case 6: return launch_fused_cfg<E, 64, 128, 4, 2, 4, ROWS_K>(Aop, Bop, rowsA, rowsB, bias, y, g, post, s);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_fused_gemm_output(const void* U, const void* V, const float* bias, void* y, const Geom& g, int dt, bool nhwc,
                                    const PostOp* postp, int shape, hipStream_t s) {
    if (g.m != 2) return hipErrorInvalidValue;
    if (shape < -1 || shape > 6) return hipErrorInvalidValue;
    const PostOp post = postp ? *postp : PostOp();
    return with_dtype(dt, [&](auto* tag) {
        using E = std::remove_pointer_t<decltype(tag)>;
        if (nhwc) return launch_fused_t<E, false>(V, U, g.T, g.K, bias, y, g, post, shape < 0 ? fused_pick_shape(g.T, g.K) : shape, s);
        return launch_fused_t<E, true>(U, V, g.K, g.T, bias, y, g, post, shape < 0 ? fused_pick_shape(g.K, g.T) : shape, s);
    });
}

}  // namespace wino
