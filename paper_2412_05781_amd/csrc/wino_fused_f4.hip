// Steps (ii) and (iii) in one kernel for F(4x4,3x3) (Section "Techniques"; its second paragraph argues for keeping
// dependent steps local).  As in the F(2x2) kernel of wino_fused.hip, a workgroup owns a block of (output channels x
// tiles) for ALL 36 positions and walks them one after another, so the product M is never stored.  What differs is the
// bookkeeping of step (iii): an output tile has 16 values per (channel, tile), and with the product and the running sums
// a 32x32 MFMA sub-tile per wave would need more vector registers than exist.  So
//   - a wave owns a 16 x 32 piece (two 16x16 MFMA tiles, v_mfma_f32_16x16x32: four accumulator registers per tile), and
//   - step (iii) is taken one dimension at a time.  Positions run xi-major; while nu runs over a row of the
//     transformed tile the product is folded into four row sums  Z[b] += A^T[b][nu] * M[xi,nu]; at the end of the row
//     Y[a][b] += A^T[a][xi] * Z[b].  That is 22 accumulator sets of 8 registers (16 outputs, 4 row sums, and the product twice:
//     the two MFMA steps of a stage alternate between two accumulators), all in vector registers, and 180 multiply-adds per
//     accumulator register instead of 324.
// The price of the small wave tile is traffic: 3 KB of LDS fragments per 32 reduction elements and wave, and a block of
// at most 64 x 64 per compute unit (the register file holds no more accumulators of this kind), so every byte of U and V is
// fetched into LDS by T/64 and K/64 workgroups.  That fill traffic bounds the kernel; it pays on large images with at
// most 256 channels, where the unfused path is bound by writing and re-reading M.  Two-byte storage types only.
//
// Operand staging is that of the batched GEMM kernel: 128-byte stages per row, global -> LDS directly into a ring,
// XOR-swizzled 16-byte chunks, one barrier per stage, explicit vmcnt waits.
// ROWS_K = true : rows of the block are output channels (U), columns are tiles (V); y is NCHW.
// ROWS_K = false: operands swapped, rows are tiles, columns output channels; y is channel-last.
#include "wino_internal.h"
#include "wino_mma.h"

namespace wino {

namespace {

template <typename E> struct Mma16;
template <> struct Mma16<__half> {
    static __device__ __forceinline__ void run(const u32x4_t& a, const u32x4_t& b, f32x4_t& c) {
        c = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, a), __builtin_bit_cast(half8_t, b), c, 0, 0, 0);
    }
};
template <> struct Mma16<bf16_t> {
    static __device__ __forceinline__ void run(const u32x4_t& a, const u32x4_t& b, f32x4_t& c) {
        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    }
};

// A^T of F(4x4,3x3): rows (1 1 1 1 1 0), (0 1 -1 2 -2 0), (0 1 1 4 4 0), (0 1 -1 8 -8 1); both arguments wave-uniform
__device__ __forceinline__ float at4(int a, int x) {
    if (x == 0) return a == 0 ? 1.f : 0.f;
    if (x == 5) return a == 3 ? 1.f : 0.f;
    const float sign = (x & 1) ? 1.f : -1.f, mag = x <= 2 ? 1.f : 2.f;
    return a == 0 ? 1.f : (a == 1 ? sign * mag : (a == 2 ? mag * mag : sign * mag * mag * mag));
}

template <typename E> __device__ __forceinline__ uint32_t pack2(float a, float b) {
    const E ea = from_f32<E>(a), eb = from_f32<E>(b);
    return (uint32_t)*reinterpret_cast<const uint16_t*>(&ea) | ((uint32_t)*reinterpret_cast<const uint16_t*>(&eb) << 16);
}
template <typename E> __device__ __forceinline__ float lo16(uint32_t w) { const uint16_t h = (uint16_t)(w & 0xffffu); return to_f32<E>(*reinterpret_cast<const E*>(&h)); }
template <typename E> __device__ __forceinline__ float hi16(uint32_t w) { const uint16_t h = (uint16_t)(w >> 16); return to_f32<E>(*reinterpret_cast<const E*>(&h)); }

struct Fused4Geom { int N, K, H, W, th, tw, T; };

}  // namespace

// Block = (WGM * 16) rows x (WGN * 32) columns, one 16 x 32 piece per wave.
// RAGGED = true: Cp is not a multiple of the stage (64 elements); the last stage of every position then goes through
// registers with zero fill.
template <typename E, int NST, int WGM, int WGN, bool ROWS_K, bool RAGGED>
__global__ void __launch_bounds__(WGM * WGN * 64)
wino_fused_f4_kernel(const E* __restrict__ Aop, const E* __restrict__ Bop, const float* __restrict__ bias, E* __restrict__ y,
                     int rowsA, int rowsB, int Cp, Fused4Geom g, int tiles_m, int tiles_n, int total_blocks, int blocks_per_xcd,
                     int vec_ok, PostOp post) {
    static_assert(sizeof(E) == 2, "two-byte storage types");
    constexpr int A2 = 36;                                // positions of F(4x4,3x3)
    constexpr int RB = 128;                               // stage bytes per row
    constexpr int CPR = RB / 16;                          // 16-byte chunks per row per stage
    constexpr int BKE = RB / 2;                           // reduction elements per stage
    constexpr int BM = WGM * 16, BN = WGN * 32;
    constexpr int ROWS = BM + BN;
    constexpr int RPL = 1024 / RB;                        // rows covered by one wave-wide load
    constexpr int NW = WGM * WGN;
    constexpr int LPW = ROWS / RPL / NW;                  // wave-wide loads per wave per stage
    constexpr int LA = BM / (RPL * NW);                   // ... of which from the row operand
    constexpr int STAGE_BYTES = ROWS * RB;
    static_assert(ROWS % (RPL * NW) == 0 && BM % (RPL * NW) == 0, "load i of every wave lies in the same operand");
    static_assert(NST >= 2 && (NST & (NST - 1)) == 0 && LPW * (NST - 1) < 64, "ring depth: a power of two, within the vmcnt range");

    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];

    // one contiguous range of logical blocks per XCD; the shorter tile dimension runs fastest
    const int bid = blockIdx.x;
    const int logical = (bid % 8) * blocks_per_xcd + bid / 8;
    if (logical >= total_blocks) return;                  // uniform per workgroup, before any barrier
    int tm, tn;
    if (tiles_m <= tiles_n) { tm = logical % tiles_m; tn = logical / tiles_m; }
    else { tn = logical % tiles_n; tm = logical / tiles_n; }

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

    int issue_kt = 0;
    auto issue_stage = [&](int slot) __attribute__((always_inline)) {                    // the next stage in order, into ring slot `slot`
        const uint32_t dst = wave_dst + (uint32_t)slot * STAGE_BYTES;
        if (RAGGED && issue_kt == nk - 1) {
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

    // accumulators of the wave's two 16x16 tiles: the product of the current position, the four row sums, the 16 outputs
    f32x4_t accM[2][2], accZ[4][2], accY[4][4][2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        accM[0][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        accM[1][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            accZ[b][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int a = 0; a < 4; ++a) accY[a][b][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        }
    }

    // A stage holds two MFMA steps of 32 reduction elements (four 16-byte chunks each; lanes 16q..16q+15 hold chunk q of the
    // step).  All six fragments of a stage (one row tile and two column tiles per step) are requested as soon as the stage is
    // visible and used one stage later, so that a whole stage of MFMAs and the next barrier lie between request and use; two
    // fragment sets alternate.  The swizzled chunk of step h is chunk(0) ^ 4h, i.e. the byte address of step 0 with bit 6
    // flipped; the second column tile lies 16 rows further on (same swizzle).
    u32x4_t fa[2][2], fb[2][2][2];                        // [set][step], [set][step][column tile]
    const int frag_row = lane & 15, frag_q = lane >> 4;
    const int rowA = wm * 16 + frag_row, rowB = BM + wn * 32 + frag_row;
    const uint32_t fbaseA = lds0 + (uint32_t)rowA * RB + (uint32_t)((frag_q ^ ((rowA >> 1) & (CPR - 1))) << 4);
    const uint32_t fbaseB = lds0 + (uint32_t)rowB * RB + (uint32_t)((frag_q ^ ((rowB >> 1) & (CPR - 1))) << 4);
    auto read_stage = [&](int slot, auto setc) __attribute__((always_inline)) {
        constexpr int set = decltype(setc)::value;
        const uint32_t a0 = fbaseA + (uint32_t)slot * STAGE_BYTES, b0 = fbaseB + (uint32_t)slot * STAGE_BYTES;
        lds_read16_async<0>(fa[set][0], a0);
        lds_read16_async<0>(fb[set][0][0], b0);
        lds_read16_async<16 * RB>(fb[set][0][1], b0);
        lds_read16_async<0>(fa[set][1], a0 ^ 64u);
        lds_read16_async<0>(fb[set][1][0], b0 ^ 64u);
        lds_read16_async<16 * RB>(fb[set][1][1], b0 ^ 64u);
    };
    auto await_stage = [&](auto setc) __attribute__((always_inline)) {                   // every fragment read issued so far has arrived
        constexpr int set = decltype(setc)::value;
        lds_wait<0>();
#pragma unroll
        for (int h = 0; h < 2; ++h) { pin(fa[set][h]); pin(fb[set][h][0]); pin(fb[set][h][1]); }
    };
    auto mma_stage = [&](auto setc) __attribute__((always_inline)) {
        constexpr int set = decltype(setc)::value;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            Mma16<E>::run(fa[set][h], fb[set][h][0], accM[h][0]);
            Mma16<E>::run(fa[set][h], fb[set][h][1], accM[h][1]);
        }
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;

#pragma unroll
    for (int s = 0; s < NST; ++s)
        if (s < total) issue_stage(s);
    if (NST - 1 >= total) wait_vmcnt<0>();
    else wait_vmcnt<(NST - 1) * LPW>();
    __syncthreads();
    read_stage(0, I0());

    int kt = 0, xi = 0, nu = 0;
    // after the last MFMA of a stage: at the end of a position the product is folded into the row sums and cleared; at the
    // end of a row of the transformed tile the row sums are folded into the outputs and cleared
    auto end_of_stage = [&]() __attribute__((always_inline)) {
        if (++kt < nk) return;
        kt = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const float c = at4(b, nu);                   // wave-uniform
            if (c != 0.f) {
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int r = 0; r < 4; ++r) accZ[b][j][r] = fmaf(c, accM[0][j][r] + accM[1][j][r], accZ[b][j][r]);
            }
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) { accM[0][j] = f32x4_t{0.f, 0.f, 0.f, 0.f}; accM[1][j] = f32x4_t{0.f, 0.f, 0.f, 0.f}; }
        if (++nu < 6) return;
        nu = 0;
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const float c = at4(a, xi);
            if (c != 0.f) {
#pragma unroll
                for (int b = 0; b < 4; ++b)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
#pragma unroll
                        for (int r = 0; r < 4; ++r) accY[a][b][j][r] = fmaf(c, accZ[b][j][r], accY[a][b][j][r]);
            }
        }
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int j = 0; j < 2; ++j) accZ[b][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        ++xi;
    };

    // stage s (fragment set s % 2, requested one stage earlier): make stage s+1 visible, refill the slot of stage s, request
    // the fragments of stage s+1, multiply stage s
    auto stage = [&](int s, auto setc, auto nextc) __attribute__((always_inline)) {
        const int slot = s & (NST - 1), next_slot = (s + 1) & (NST - 1);
        // stage s+1 has landed once no more transfers are outstanding than were issued after it
        if (s + NST >= total) wait_vmcnt<0>();
        else wait_vmcnt<(NST - 2) * LPW>();
        await_stage(setc);              // this wave has read all of stage s
        __syncthreads();                // stage s+1 visible to all waves; every wave has read all of stage s
        if (s + NST < total) issue_stage(slot);                  // stage s+NST, into the slot stage s used
        read_stage(next_slot, nextc);
        __builtin_amdgcn_sched_barrier(0);
        mma_stage(setc);
        __builtin_amdgcn_sched_barrier(0);
        end_of_stage();
    };
    // total = 36 * nk is even: stages are taken in pairs so that the fragment sets are compile-time; the last stage is peeled
    for (int s = 0; s < total - 2; s += 2) {
        stage(s, I0(), I1());
        stage(s + 1, I1(), I0());
    }
    stage(total - 2, I0(), I1());
    await_stage(I1());
    mma_stage(I1());
    end_of_stage();

    // ---- epilogue: bias (+ vector, + residual), crop, round once, store ---------------------------------------
    // 16x16 accumulator layout: register r of lane l holds row 4*(l/16) + r, column l%16 of the tile
    const int H = g.H, W = g.W, K = g.K;
    const E* res = static_cast<const E*>(post.residual);
    if constexpr (ROWS_K) {
        // columns are tiles: a lane owns one tile per column tile, its four registers run over output channels; the four
        // pixels of an output row of the tile are stored together, neighbouring lanes hold neighbouring tiles of a tile row
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            int t = col0 + wn * 32 + j * 16 + frag_row;
            const bool t_ok = t < g.T;
            t = t_ok ? t : g.T - 1;
            const int tj = t % g.tw; const int q = t / g.tw;
            const int ti = q % g.th, n = q / g.th;
            const int i0 = 4 * ti, j0 = 4 * tj;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int k = row0 + wm * 16 + 4 * frag_q + r;
                if (!(k < K && t_ok)) continue;
                const float bb = (bias ? bias[k] : 0.f) + (post.addvec ? post.addvec[(size_t)n * K + k] : 0.f);
                const size_t off = (((size_t)n * K + k) * H + i0) * W + j0;
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    if (i0 + a >= H) continue;
                    const size_t o = off + (size_t)a * W;
                    float v[4];
#pragma unroll
                    for (int b = 0; b < 4; ++b) v[b] = accY[a][b][j][r] + bb;
                    if (vec_ok) {
                        if (res) {
                            const uint2 rr = *reinterpret_cast<const uint2*>(res + o);
                            v[0] += lo16<E>(rr.x); v[1] += hi16<E>(rr.x); v[2] += lo16<E>(rr.y); v[3] += hi16<E>(rr.y);
                        }
                        *reinterpret_cast<uint2*>(y + o) = make_uint2(pack2<E>(v[0], v[1]), pack2<E>(v[2], v[3]));
                    } else {
#pragma unroll
                        for (int b = 0; b < 4; ++b)
                            if (j0 + b < W) y[o + b] = from_f32<E>(v[b] + (res ? to_f32<E>(res[o + b]) : 0.f));
                    }
                }
            }
        }
    } else {
        // Columns are output channels, which are contiguous in a channel-last y - but a lane holds one channel and a 16x16
        // tile only 16 of them, so stores straight from the accumulators would be 32-byte pieces.  The block goes through LDS
        // instead (the ring is free by now): for each output row a of the tile, every wave parks its values for the four
        // pixels (a, b) as storage-type elements at [b][tile][channel], and the workgroup then writes them out as 16-byte
        // pieces, eight lanes to a 128-byte line.  Bias, vector and residual are added before the one rounding, as everywhere.
        constexpr int PSTRIDE = BN * 2 + 16;              // bytes per (pixel, tile) row in LDS; the pad spreads the rows over the banks
        constexpr int PIECES = BN / 8;                    // 16-byte pieces per row
        static_assert(4 * BM * PSTRIDE <= NST * STAGE_BYTES, "the parked rows fit the ring's LDS");
        const bool rows16 = (K % 8 == 0);                 // a pixel's channel vector starts on a 16-byte boundary
#pragma unroll
        for (int a = 0; a < 4; ++a) {                     // unrolled: the accumulators are registers, a must be a constant
            __syncthreads();                              // nobody reads the ring (or the previous rows) any more
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int kl = wn * 32 + j * 16 + frag_row, k = col0 + kl;
                const bool k_ok = k < K;
                const float bk = (bias && k_ok) ? bias[k] : 0.f;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int tl = wm * 16 + 4 * frag_q + r, t = row0 + tl;
                    const bool ok = t < g.T && k_ok;
                    const int tc = t < g.T ? t : g.T - 1;
                    const int tj = tc % g.tw; const int q = tc / g.tw;
                    const int ti = q % g.th, n = q / g.th;
                    const float bb = bk + ((post.addvec && ok) ? post.addvec[(size_t)n * K + k] : 0.f);
                    const int ii = 4 * ti + a;
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        const int jj = 4 * tj + b;
                        float v = accY[a][b][j][r] + bb;
                        if (res && ok && ii < H && jj < W) v += to_f32<E>(res[(((size_t)n * H + ii) * W + jj) * K + k]);
                        *reinterpret_cast<E*>(lds + (size_t)(b * BM + tl) * PSTRIDE + (size_t)kl * 2) = from_f32<E>(v);
                    }
                }
            }
            __syncthreads();
            for (int idx = tid; idx < 4 * BM * PIECES; idx += NW * 64) {
                const int piece = idx % PIECES, tl = (idx / PIECES) % BM, b = idx / (PIECES * BM);
                const int t = row0 + tl, k0 = col0 + piece * 8;
                if (t >= g.T || k0 >= K) continue;
                const int tj = t % g.tw; const int q = t / g.tw;
                const int ti = q % g.th, n = q / g.th;
                const int ii = 4 * ti + a, jj = 4 * tj + b;
                if (ii >= H || jj >= W) continue;
                const unsigned char* src = lds + (size_t)(b * BM + tl) * PSTRIDE + (size_t)piece * 16;
                E* dst = y + (((size_t)n * H + ii) * W + jj) * K + k0;
                if (rows16 && k0 + 8 <= K) {
                    *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(src);
                } else {
                    for (int e = 0; e < 8 && k0 + e < K; ++e) dst[e] = reinterpret_cast<const E*>(src)[e];
                }
            }
        }
    }
}

template <typename E, int NST, int WGM, int WGN, bool ROWS_K, bool RAGGED = false>
static hipError_t launch_fused4_cfg(const void* Aop, const void* Bop, int rowsA, int rowsB, const float* bias, void* y,
                                    const Geom& g, const PostOp& post, hipStream_t s) {
    constexpr int BM = WGM * 16, BN = WGN * 32;
    const int tiles_m = (rowsA + BM - 1) / BM, tiles_n = (rowsB + BN - 1) / BN;
    const long long total = (long long)tiles_m * tiles_n;
    if (total > 0x3fffffffLL) return hipErrorInvalidValue;
    const int per_xcd = (int)((total + 7) / 8);
    constexpr int lds_bytes = (BM + BN) * 128 * NST;
    static_assert(lds_bytes <= 160 * 1024, "LDS budget");
    // lane offsets are 32-bit: a block's rows must span less than 2 GB
    if ((size_t)g.Cp * sizeof(E) * (size_t)(BM > BN ? BM : BN) >= ((size_t)1 << 31)) return hipErrorInvalidValue;
    auto kern = wino_fused_f4_kernel<E, NST, WGM, WGN, ROWS_K, RAGGED>;
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (attr != hipSuccess) return attr;
    Fused4Geom fg{g.N, g.K, g.H, g.W, g.th, g.tw, g.T};
    // four-pixel stores of a tile's output row need W % 4 == 0 (the group then never straddles the row end) and 8-byte alignment
    const int vec_ok = (g.W % 4 == 0) && ((reinterpret_cast<uintptr_t>(y) & 7u) == 0) && ((reinterpret_cast<uintptr_t>(post.residual) & 7u) == 0);
    hipLaunchKernelGGL(kern, dim3((unsigned)(per_xcd * 8)), dim3(WGM * WGN * 64), lds_bytes, s,
                       (const E*)Aop, (const E*)Bop, bias, (E*)y, rowsA, rowsB, g.Cp, fg, tiles_m, tiles_n, (int)total, per_xcd, vec_ok, post);
    return hipGetLastError();
}

// Block shapes on offer (rows x columns of the block): 0 = 64x64 with eight waves (4 x 2), 1 = 32x64 with four waves (2 x 2).
int fused4_pick_shape(int rows, int cols) {
    const long long big = (long long)((rows + 63) / 64) * ((cols + 63) / 64);
    return big >= 200 ? 0 : 1;
}

template <typename E, bool ROWS_K>
static hipError_t launch_fused4_t(const void* Aop, const void* Bop, int rowsA, int rowsB, const float* bias, void* y,
                                  const Geom& g, const PostOp& post, int shape, hipStream_t s) {
    if (g.Cp % 64 != 0)       // a reduction length that is not a whole number of stages: the zero-filling last stage
        return launch_fused4_cfg<E, 4, 2, 2, ROWS_K, true>(Aop, Bop, rowsA, rowsB, bias, y, g, post, s);
    switch (shape) {
        case 0: return launch_fused4_cfg<E, 4, 4, 2, ROWS_K>(Aop, Bop, rowsA, rowsB, bias, y, g, post, s);
        case 1: return launch_fused4_cfg<E, 4, 2, 2, ROWS_K>(Aop, Bop, rowsA, rowsB, bias, y, g, post, s);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_fused4_gemm_output(const void* U, const void* V, const float* bias, void* y, const Geom& g, int dt, bool nhwc,
                                     const PostOp* postp, int shape, hipStream_t s) {
    if (g.m != 4 || !two_byte(dt) || dt == DT_I8) return hipErrorInvalidValue;
    if (shape < -1 || shape > 1) return hipErrorInvalidValue;
    const PostOp post = postp ? *postp : PostOp();
    auto run = [&](auto* tag) {
        using E = std::remove_pointer_t<decltype(tag)>;
        if (nhwc) return launch_fused4_t<E, false>(V, U, g.T, g.K, bias, y, g, post, shape < 0 ? fused4_pick_shape(g.T, g.K) : shape, s);
        return launch_fused4_t<E, true>(U, V, g.K, g.T, bias, y, g, post, shape < 0 ? fused4_pick_shape(g.K, g.T) : shape, s);
    };
    return dt == DT_F16 ? run(static_cast<__half*>(nullptr)) : run(static_cast<bf16_t*>(nullptr));
}

}  // namespace wino
