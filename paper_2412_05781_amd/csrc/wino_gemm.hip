// Step (ii) (Section "Techniques"): the "element-wise multiplication" of the
// transformed filter and activation, summed over input channels — i.e. alpha^2
// independent matrix products  M_b[k][t] = sum_c U_b[k][c] * V_b[t][c],
// b = xi*alpha+nu.  This is the one dense contraction of the path and runs on
// the MFMA units with fp32 accumulation.
//
// Both operands are row-major with the reduction index contiguous, so a lane's
// MFMA fragment is one 16-byte LDS read.  A workgroup (WGM x WGN waves) owns a
// BM x BN block of one batch; each wave (BM/WGM)x(BN/WGN) as 32x32 MFMA tiles.
// The reduction is cut into stages of RB bytes per row.  Stages travel
// global -> LDS directly (global_load_lds, 16 bytes per lane, no staging
// registers) through a ring of NST slots; one barrier per stage.  LDS rows are
// unpadded (the transfer writes lanes linearly); bank conflicts are avoided by
// an XOR swizzle of the 16-byte chunk index, applied on the global-address side
// when loading and on the LDS-address side when reading fragments.
// Rows beyond K / T are clamped to the last valid row (their products are never
// stored); a ragged last reduction stage (Cp not a multiple of the stage) goes
// through registers with zero fill instead.
#include "wino_internal.h"
#include "wino_mma.h"
#include <type_traits>

namespace wino {

// 8-bit integer operands carry one quantisation step per row of each operand (rs[nbatch][K] for the first, cs[nbatch][T]
// for the second); the integer sum becomes the product by  float(sum) * rs[batch][k] * cs[batch][t].  For the floating-point
// storage types the accumulator is the product and both pointers are unused.
template <typename E> __device__ __forceinline__ float column_step(const float* cs, int batch, int T, int t) {
    if constexpr (std::is_same_v<E, i8_t>) return t < T ? cs[(size_t)batch * T + t] : 0.f;
    else return 1.f;
}
template <typename E, typename A> __device__ __forceinline__ float product_value(A a, const float* rs, int batch, int K, int k, float cstep) {
    if constexpr (std::is_same_v<E, i8_t>) return (float)a * rs[(size_t)batch * K + k] * cstep;
    else return a;
}

// MT = type the product is stored in: float, or __half for the opt-in half-product mode.
template <typename E, typename MT, int BM, int BN, int RB, int NST, int WGM, int WGN>
__global__ void __launch_bounds__(WGM * WGN * 64)
wino_gemm_kernel(const E* __restrict__ U, const E* __restrict__ V, MT* __restrict__ Mo,
                 int K, int Cp, int T, int tiles_m, int tiles_n, int total_blocks, int blocks_per_xcd,
                 int nbatch, int nsplit, const float* __restrict__ rs, const float* __restrict__ cs) {
    constexpr int CPR = RB / 16;                          // 16-byte chunks per row per stage
    constexpr int BKE = RB / (int)sizeof(E);              // reduction elements per stage
    constexpr int EPC = 16 / (int)sizeof(E);              // elements per chunk
    constexpr int ROWS = BM + BN;
    constexpr int RPL = 1024 / RB;                        // rows covered by one wave-wide load
    constexpr int NW = WGM * WGN;                         // waves per workgroup
    constexpr int LPW = ROWS / RPL / NW;                  // wave-wide loads per wave per stage
    constexpr int SWZ_SHIFT = (RB == 128) ? 1 : 2;        // rows per 256-byte bank wrap = 256/RB
    constexpr int WTM = BM / WGM, WTN = BN / WGN;
    constexpr int FM = WTM / 32, FN = WTN / 32;
    constexpr int STAGE_BYTES = ROWS * RB;
    static_assert(RB == 128 || RB == 64, "stage row bytes");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0 && ROWS % (RPL * NW) == 0, "tile shape");
    static_assert(NST >= 2 && NST <= 4, "ring depth");
    static_assert(LPW * (NST - 1) < 64, "vmcnt range");

    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];

    // XCD-aware mapping: hardware deals workgroups round-robin to the 8 XCDs, so give
    // each XCD a contiguous range of logical blocks (same batch -> same L2).
    const int bid = blockIdx.x;
    const int logical = (bid % 8) * blocks_per_xcd + bid / 8;
    if (logical >= total_blocks) return;                  // uniform per workgroup, before any barrier
    // Inside a batch the shorter tile dimension runs fastest: the workgroups resident together
    // then sweep ALL blocks of the smaller operand (which stays in L2) against a few blocks of
    // the larger one, which is streamed from memory once.
    // With nsplit > 1 the reduction over c is cut into nsplit ranges of whole stages, one workgroup
    // each, and split i writes its partial product to the i-th copy of M (summed by the reader).
    const int bs = logical / (tiles_n * tiles_m);
    const int in_batch = logical - bs * (tiles_n * tiles_m);
    const int batch = bs / nsplit, split = bs - batch * nsplit;
    int tm, tn;
    if (tiles_m <= tiles_n) { tm = in_batch % tiles_m; tn = in_batch / tiles_m; }
    else { tn = in_batch % tiles_n; tm = in_batch / tiles_n; }

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int row_k0 = tm * BM, row_t0 = tn * BN;

    const E* Ub = U + (size_t)batch * K * Cp;
    const E* Vb = V + (size_t)batch * T * Cp;

    // per-lane source rows of this lane's LPW loads (fixed over the reduction loop)
    const int lrow = lane / CPR, lchunk = lane % CPR;
    const E* src[LPW];
    int src_chunk[LPW];
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
        const int row = (wave + NW * i) * RPL + lrow;       // row inside the stage, A rows first
        const int chunk = lchunk ^ ((row >> SWZ_SHIFT) & (CPR - 1));
        src_chunk[i] = chunk;
        if (row < BM) {
            int g = row_k0 + row; g = g < K ? g : K - 1;
            src[i] = Ub + (size_t)g * Cp + chunk * EPC;
        } else {
            int g = row_t0 + (row - BM); g = g < T ? g : T - 1;
            src[i] = Vb + (size_t)g * Cp + chunk * EPC;
        }
    }

    const int nk_all = (Cp + BKE - 1) / BKE;
    const bool ragged = (Cp % BKE) != 0;
    const int kt0 = (int)((long long)split * nk_all / nsplit), nk = (int)((long long)(split + 1) * nk_all / nsplit);

    auto issue_stage = [&](int kt) {
        unsigned char* slot = lds + ((kt - kt0) % NST) * STAGE_BYTES;
        if (ragged && kt == nk_all - 1) {
            // last, partial stage: through registers, chunks beyond Cp become zeros
#pragma unroll
            for (int i = 0; i < LPW; ++i) {
                const int gk = kt * BKE + src_chunk[i] * EPC;
                uint4 v = make_uint4(0, 0, 0, 0);
                if (gk < Cp) v = *reinterpret_cast<const uint4*>(src[i] + kt * BKE);
                *reinterpret_cast<uint4*>(slot + (wave + NW * i) * 1024 + lane * 16) = v;
            }
        } else {
#pragma unroll
            for (int i = 0; i < LPW; ++i) dma_load_1k(src[i] + kt * BKE, slot + (wave + NW * i) * 1024);
        }
    };

    typename Mma<E>::acc_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

#pragma unroll
    for (int s = 0; s < NST - 1; ++s)
        if (kt0 + s < nk) issue_stage(kt0 + s);

    const int frag_row = lane & 31, frag_half = lane >> 5;
    for (int kt = kt0; kt < nk; ++kt) {
        // Stage kt must have landed.  Transfers complete in issue order, so it is enough to allow
        // as many outstanding as were issued after it: NST-2 stages in steady state, and once the
        // ring stops refilling simply everything.
        if (kt + NST - 1 >= nk) wait_vmcnt<0>();
        else wait_vmcnt<(NST - 2) * LPW>();
        __syncthreads();            // stage kt visible to all waves; everyone is done with stage kt-1
        if (kt + NST - 1 < nk) issue_stage(kt + NST - 1);   // refills the slot stage kt-1 used

        // all fragment reads of the stage first, then the MFMAs, so LDS latency is paid once
        const unsigned char* slot = lds + ((kt - kt0) % NST) * STAGE_BYTES;
        uint4 fa[CPR / 2][FM], fb[CPR / 2][FN];
#pragma unroll
        for (int ks = 0; ks < CPR / 2; ++ks) {
#pragma unroll
            for (int i = 0; i < FM; ++i) {
                const int row = wm * WTM + i * 32 + frag_row;
                const int chunk = (2 * ks + frag_half) ^ ((row >> SWZ_SHIFT) & (CPR - 1));
                fa[ks][i] = *reinterpret_cast<const uint4*>(slot + row * RB + chunk * 16);
            }
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                const int row = BM + wn * WTN + j * 32 + frag_row;
                const int chunk = (2 * ks + frag_half) ^ ((row >> SWZ_SHIFT) & (CPR - 1));
                fb[ks][j] = *reinterpret_cast<const uint4*>(slot + row * RB + chunk * 16);
            }
        }
#pragma unroll
        for (int ks = 0; ks < CPR / 2; ++ks)
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j) Mma<E>::run(fa[ks][i], fb[ks][j], acc[i][j]);
    }

    // 32x32 accumulator layout: register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32
    MT* Mb = Mo + ((size_t)split * nbatch + batch) * K * T;
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            const int t = row_t0 + wn * WTN + j * 32 + frag_row;
            const float cstep = column_step<E>(cs, batch, T, t);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int k = row_k0 + wm * WTM + i * 32 + 8 * (r / 4) + 4 * frag_half + (r % 4);
                if (k < K && t < T) Mb[(size_t)k * T + t] = from_f32<MT>(product_value<E>(acc[i][j][r], rs, batch, K, k, cstep));
            }
        }
}

// The same product for reduction lengths that are a whole number of stages (every Stable-Diffusion layer), written for
// the way this chip behaves with one to four waves per SIMD: every instruction a wave spends on addresses, and every
// wait placed by the compiler in front of an MFMA, is time the MFMA pipe idles.  So
//  - everything that does not depend on the lane lives in scalar registers (the wave index through readfirstlane):
//    LDS destinations, stage bases and slot offsets cost scalar instructions only; a transfer is one scalar base plus a
//    fixed 32-bit offset per lane;
//  - a stage's reduction steps are taken in two halves and the fragments of the next half (of the next stage, after the
//    barrier) are requested while the MFMAs of the current half run; the reads are issued from inline assembly and waited
//    for explicitly, because the compiler otherwise waits for the newest read in front of every MFMA;
//  - a wave with a single 32x32 sub-tile alternates between two accumulators.
// Block order, ring, swizzle and the meaning of every argument are those of wino_gemm_kernel.
template <typename E, typename MT, int BM, int BN, int NST, int WGM, int WGN>
__global__ void __launch_bounds__(WGM * WGN * 64)
wino_gemm_lean_kernel(const E* __restrict__ U, const E* __restrict__ V, MT* __restrict__ Mo,
                      int K, int Cp, int T, int tiles_m, int tiles_n, int total_blocks, int blocks_per_xcd,
                      int nbatch, int nsplit, const float* __restrict__ rs, const float* __restrict__ cs) {
    constexpr int RB = 128;
    constexpr int CPR = RB / 16;
    constexpr int BKE = RB / (int)sizeof(E);
    constexpr int ROWS = BM + BN;
    constexpr int RPL = 1024 / RB;
    constexpr int NW = WGM * WGN;
    constexpr int LPW = ROWS / RPL / NW;
    constexpr int LA = BM / (RPL * NW);
    constexpr int WTM = BM / WGM, WTN = BN / WGN;
    constexpr int FM = WTM / 32, FN = WTN / 32;
    constexpr int STAGE_BYTES = ROWS * RB;
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "tile shape");
    static_assert(BM % (RPL * NW) == 0 && BN % (RPL * NW) == 0, "load i of every wave lies in the same operand");
    static_assert(NST >= 2 && NST <= 4 && LPW * (NST - 1) < 64, "ring depth");
    static_assert((FM - 1) * 32 * RB < 65536 && (FN - 1) * 32 * RB < 65536, "sub-tile offsets fit the ds_read offset field");

    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];

    const int bid = blockIdx.x;
    const int logical = (bid % 8) * blocks_per_xcd + bid / 8;
    if (logical >= total_blocks) return;                  // uniform per workgroup, before any barrier
    const int bs = logical / (tiles_n * tiles_m);
    const int in_batch = logical - bs * (tiles_n * tiles_m);
    const int batch = bs / nsplit, split = bs - batch * nsplit;
    int tm, tn;
    if (tiles_m <= tiles_n) { tm = in_batch % tiles_m; tn = in_batch / tiles_m; }
    else { tn = in_batch % tiles_n; tm = in_batch / tiles_n; }

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;
    const int row0 = tm * BM, col0 = tn * BN;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_byte_t*)lds;

    const size_t row_bytes = (size_t)Cp * sizeof(E);
    const int nk_all = Cp / BKE;                          // Cp is a whole number of stages here
    const int kt0 = (int)((long long)split * nk_all / nsplit), kt1 = (int)((long long)(split + 1) * nk_all / nsplit);
    const int total = kt1 - kt0;                          // stages of this workgroup (>= 1: nsplit <= nk_all)

    const int lrow = lane / CPR, lchunk = lane % CPR;
    uint32_t goff[LPW];
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
        const int row = (wave + NW * i) * RPL + lrow;
        const int chunk = lchunk ^ ((row >> 1) & (CPR - 1));
        int r;
        if (i < LA) { r = row0 + row; r = (r < K ? r : K - 1) - row0; }
        else { r = col0 + (row - BM); r = (r < T ? r : T - 1) - col0; }
        goff[i] = (uint32_t)r * (uint32_t)row_bytes + (uint32_t)chunk * 16u;
    }
    const unsigned char* sA = reinterpret_cast<const unsigned char*>(U) + ((size_t)batch * K + row0) * row_bytes + (size_t)kt0 * RB;
    const unsigned char* sB = reinterpret_cast<const unsigned char*>(V) + ((size_t)batch * T + col0) * row_bytes + (size_t)kt0 * RB;
    const uint32_t wave_dst = lds0 + (uint32_t)wave * 1024u;
    auto issue_stage = [&](int slot) {                    // the next stage in order
        const uint32_t dst = wave_dst + (uint32_t)slot * STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < LPW; ++i) dma_load_1k_s(i < LA ? sA : sB, goff[i], dst + (uint32_t)(NW * i) * 1024u);
        sA += RB;
        sB += RB;
    };

    constexpr int NACC = (FM * FN == 1) ? 2 : 1;
    typename Mma<E>::acc_t acc[NACC][FM][FN];
#pragma unroll
    for (int q = 0; q < NACC; ++q)
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[q][i][j][r] = 0;

    constexpr int KS = CPR / 2, KH = KS / 2;
    constexpr int NREAD = KH * (FM + FN);
    u32x4_t fa[2][KH][FM], fb[2][KH][FN];
    const int frag_row = lane & 31, frag_half = lane >> 5;
    const int rowA = wm * WTM + frag_row, rowB = BM + wn * WTN + frag_row;
    const uint32_t fbaseA = lds0 + (uint32_t)rowA * RB + (uint32_t)((frag_half ^ ((rowA >> 1) & (CPR - 1))) << 4);
    const uint32_t fbaseB = lds0 + (uint32_t)rowB * RB + (uint32_t)((frag_half ^ ((rowB >> 1) & (CPR - 1))) << 4);
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
                for (int j = 0; j < FN; ++j) Mma<E>::run(fa[buf][kk][i], fb[buf][kk][j], acc[kk % NACC][i][j]);
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using NR = std::integral_constant<int, NREAD>;

    // prologue: fill the ring, wait for the first stage, request its first half
#pragma unroll
    for (int s = 0; s < NST; ++s)
        if (s < total) issue_stage(s);
    if (NST - 1 >= total) wait_vmcnt<0>();
    else wait_vmcnt<(NST - 1) * LPW>();
    __syncthreads();
    read_half(0, I0(), I0());

    int slot = 0;
    for (int s = 0; s < total - 1; ++s) {
        const int next_slot = slot + 1 == NST ? 0 : slot + 1;
        read_half(slot, I1(), I1());
        await_half(I0(), NR());
        __builtin_amdgcn_sched_barrier(0);
        mma_half(I0());
        __builtin_amdgcn_sched_barrier(0);
        // stage s+1 has landed once no more transfers are outstanding than were issued after it
        if (s + NST >= total) wait_vmcnt<0>();
        else wait_vmcnt<(NST - 2) * LPW>();
        await_half(I1(), I0());         // this wave has read all of stage s
        __syncthreads();                // stage s+1 visible to all waves; every wave has read all of stage s
        if (s + NST < total) issue_stage(slot);                  // stage s+NST, into the slot stage s used
        read_half(next_slot, I0(), I0());
        __builtin_amdgcn_sched_barrier(0);
        mma_half(I1());
        __builtin_amdgcn_sched_barrier(0);
        slot = next_slot;
    }
    read_half(slot, I1(), I1());
    await_half(I0(), NR());
    mma_half(I0());
    await_half(I1(), I0());
    mma_half(I1());

    // 32x32 accumulator layout: register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32.
    // The row part that depends on r is wave-uniform, so each store is a uniform row pointer plus one per-lane offset.
    MT* Mb = Mo + ((size_t)split * nbatch + batch) * K * T;
    if constexpr (NACC == 2) {
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[0][0][0][r] += acc[1][0][0][r];
    }
    const bool full = row0 + BM <= K && col0 + BN <= T && (size_t)K * T * sizeof(MT) < ((size_t)1 << 31);
    if (full) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                const int kb = row0 + wm * WTM + i * 32;                     // uniform
                const uint32_t loff = (uint32_t)(4 * frag_half) * (uint32_t)T + (uint32_t)(col0 + wn * WTN + j * 32 + frag_row);
                const float cstep = column_step<E>(cs, batch, T, col0 + wn * WTN + j * 32 + frag_row);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    MT* rowp = Mb + (size_t)(kb + 8 * (r / 4) + (r % 4)) * T;     // uniform
                    rowp[loff] = from_f32<MT>(product_value<E>(acc[0][i][j][r], rs, batch, K, kb + 8 * (r / 4) + 4 * frag_half + (r % 4), cstep));
                }
            }
    } else {
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j) {
                const int t = col0 + wn * WTN + j * 32 + frag_row;
                const float cstep = column_step<E>(cs, batch, T, t);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int k = row0 + wm * WTM + i * 32 + 8 * (r / 4) + 4 * frag_half + (r % 4);
                    if (k < K && t < T) Mb[(size_t)k * T + t] = from_f32<MT>(product_value<E>(acc[0][i][j][r], rs, batch, K, k, cstep));
                }
            }
    }
}

template <typename E, typename MT, int BM, int BN, int NST, int WGM, int WGN>
static hipError_t launch_gemm_lean(const void* U, const void* V, void* M, int K, int Cp, int T, int nbatch, int nsplit, hipStream_t s,
                                   const float* rs, const float* cs) {
    const int tiles_m = (K + BM - 1) / BM, tiles_n = (T + BN - 1) / BN;
    const long long total = (long long)tiles_m * tiles_n * nbatch * nsplit;
    if (total > 0x3fffffffLL) return hipErrorInvalidValue;
    // lane offsets are 32-bit: a block's rows must span less than 2 GB
    if ((size_t)Cp * sizeof(E) * (size_t)(BM > BN ? BM : BN) >= ((size_t)1 << 31)) return hipErrorInvalidValue;
    const int per_xcd = (int)((total + 7) / 8);
    constexpr int lds_bytes = (BM + BN) * 128 * NST;
    static_assert(lds_bytes <= 160 * 1024, "LDS budget");
    auto kern = wino_gemm_lean_kernel<E, MT, BM, BN, NST, WGM, WGN>;
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL(kern, dim3((unsigned)(per_xcd * 8)), dim3(WGM * WGN * 64), lds_bytes, s, (const E*)U, (const E*)V, (MT*)M,
                       K, Cp, T, tiles_m, tiles_n, (int)total, per_xcd, nbatch, nsplit, rs, cs);
    return hipGetLastError();
}

template <typename E, typename MT, int BM, int BN, int RB, int NST, int WGM = 2, int WGN = 2>
static hipError_t launch_gemm_cfg(const void* U, const void* V, void* M, int K, int Cp, int T, int nbatch, int nsplit, hipStream_t s,
                                  const float* rs, const float* cs) {
    const int tiles_m = (K + BM - 1) / BM, tiles_n = (T + BN - 1) / BN;
    const long long total = (long long)tiles_m * tiles_n * nbatch * nsplit;
    if (total > 0x3fffffffLL) return hipErrorInvalidValue;
    const int per_xcd = (int)((total + 7) / 8);
    constexpr int lds_bytes = (BM + BN) * RB * NST;
    static_assert(lds_bytes <= 160 * 1024, "LDS budget");
    auto kern = wino_gemm_kernel<E, MT, BM, BN, RB, NST, WGM, WGN>;
    // once per instantiation; a function-local static is initialised under the language's own lock
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (attr != hipSuccess) return attr;
    dim3 block(WGM * WGN * 64), grid((unsigned)(per_xcd * 8));
    hipLaunchKernelGGL(kern, grid, block, lds_bytes, s, (const E*)U, (const E*)V, (MT*)M,
                       K, Cp, T, tiles_m, tiles_n, (int)total, per_xcd, nbatch, nsplit, rs, cs);
    return hipGetLastError();
}

// Block shapes on offer (rows of U x rows of V per workgroup).  Rings are two stages of 128 bytes
// per row; measured on the SD-shaped layers, occupancy buys more than ring depth.  The 256x256
// block runs 16 waves (4x4) and halves the L2 traffic per flop; it pays only for very long T.
struct BlockShape { int bm, bn; double eff; };
static const BlockShape kMenu[4] = {{128, 128, 1.00}, {128, 64, 0.85}, {64, 128, 0.90}, {64, 64, 0.70}};

// Pick the shape with the least padded MFMA work per unit of (operand reuse x machine fill).
// Images of 8x8 and 16x16 give T <= 32 columns: the stage is then a pure stream of U, which a
// 128x32 block with four waves stacked along K and a three-slot ring serves best.  Both rules
// have a mirror image for the call with the operands swapped (rows of V x rows of U, which
// leaves the product transposed for channel-last outputs).
static int pick_shape(int K, int T, int nbatch, bool f16) {
    if ((K % 256 == 0 && T >= 4096) || (T % 256 == 0 && K >= 4096)) return 4;
    {   // one 256x256 workgroup (16 waves) per compute unit, nearly all units busy, little padding: measured
        // 18 % faster than any smaller block on 640 x 512 x 640 (SDXL's 64x64 layers)
        const long long tm = (K + 255) / 256, tn = (T + 255) / 256, blocks = tm * tn * nbatch;
        if (f16 && blocks >= 160 && blocks <= 256 && tm * tn * 256 * 256 * 4 <= (long long)K * T * 5) return 4;
    }
    if (T <= 32) return 5;
    if (K <= 32) return 6;
    {   // 128x128 blocks would need a second, mostly empty round (257-384 of them) while 256x128 blocks fit in one:
        // SDXL's 1280-channel 32x32 layers, 360 -> 180 workgroups of 8 waves with three slots, measured 13 % faster
        const long long b128 = (long long)((K + 127) / 128) * ((T + 127) / 128) * nbatch;
        if (f16 && K % 256 == 0 && T % 128 == 0 && b128 > 256 && b128 <= 384) return 8;
    }
    // fp16, at most one 128x128 workgroup per compute unit and next to no padding: nothing else
    // hides a workgroup's load latency, so it gets a third ring slot (measured 10-15 % over the
    // two-slot 128x128 and 64x64; the MFMA-bound fp32 path loses from the lower occupancy)
    if (f16) {
        const long long tm = (K + 127) / 128, tn = (T + 127) / 128;
        if (tm * tn * nbatch <= 256 && tm * tn * 128 * 128 * 20 <= (long long)K * T * 21) return 7;
    }
    int best = 0; double best_score = 1e300;
    for (int i = 0; i < 4; ++i) {
        const double tm = (K + kMenu[i].bm - 1) / kMenu[i].bm, tn = (T + kMenu[i].bn - 1) / kMenu[i].bn;
        const double blocks = tm * tn * nbatch;
        const double padded = tm * kMenu[i].bm * tn * kMenu[i].bn;
        const double fill = blocks >= 512.0 ? 1.0 : blocks / 512.0;     // two resident workgroups per CU
        const double score = padded / (kMenu[i].eff * fill);
        if (score < best_score) { best_score = score; best = i; }
    }
    return best;
}

template <typename E, typename MT>
static hipError_t launch_gemm_t(const void* U, const void* V, void* M, int K, int Cp, int T, int nbatch, int nsplit, int shape, hipStream_t s,
                                const float* rs = nullptr, const float* cs = nullptr) {
    const int sh = shape < 0 ? pick_shape(K, T, nbatch, sizeof(E) == 2) : shape;
    if (Cp % (128 / (int)sizeof(E)) == 0) {               // whole stages: the lean kernel, same block shapes
        switch (sh) {
            case 0: return launch_gemm_lean<E, MT, 128, 128, 2, 2, 2>(U, V, M, K, Cp, T, nbatch, nsplit, s, rs, cs);
            case 1: return launch_gemm_lean<E, MT, 128, 64, 2, 2, 2>(U, V, M, K, Cp, T, nbatch, nsplit, s, rs, cs);
            case 2: return launch_gemm_lean<E, MT, 64, 128, 2, 2, 2>(U, V, M, K, Cp, T, nbatch, nsplit, s, rs, cs);
            case 3: return launch_gemm_lean<E, MT, 64, 64, 2, 2, 2>(U, V, M, K, Cp, T, nbatch, nsplit, s, rs, cs);
            case 5: return launch_gemm_lean<E, MT, 128, 32, 3, 4, 1>(U, V, M, K, Cp, T, nbatch, nsplit, s, rs, cs);
            case 6: return launch_gemm_lean<E, MT, 32, 128, 3, 1, 4>(U, V, M, K, Cp, T, nbatch, nsplit, s, rs, cs);
            case 7: return launch_gemm_lean<E, MT, 128, 128, 3, 2, 2>(U, V, M, K, Cp, T, nbatch, nsplit, s, rs, cs);
            case 8: return launch_gemm_lean<E, MT, 256, 128, 3, 4, 2>(U, V, M, K, Cp, T, nbatch, nsplit, s, rs, cs);
            default: break;                                // 256x256 with 16 waves has no registers for two fragment sets
        }
    }
    switch (sh) {
        case 0: return launch_gemm_cfg<E, MT, 128, 128, 128, 2>(U, V, M, K, Cp, T, nbatch, nsplit, s, rs, cs);
        case 1: return launch_gemm_cfg<E, MT, 128, 64, 128, 2>(U, V, M, K, Cp, T, nbatch, nsplit, s, rs, cs);
        case 2: return launch_gemm_cfg<E, MT, 64, 128, 128, 2>(U, V, M, K, Cp, T, nbatch, nsplit, s, rs, cs);
        case 3: return launch_gemm_cfg<E, MT, 64, 64, 128, 2>(U, V, M, K, Cp, T, nbatch, nsplit, s, rs, cs);
        case 5: return launch_gemm_cfg<E, MT, 128, 32, 128, 3, 4, 1>(U, V, M, K, Cp, T, nbatch, nsplit, s, rs, cs);
        case 6: return launch_gemm_cfg<E, MT, 32, 128, 128, 3, 1, 4>(U, V, M, K, Cp, T, nbatch, nsplit, s, rs, cs);
        case 7: return launch_gemm_cfg<E, MT, 128, 128, 128, 3>(U, V, M, K, Cp, T, nbatch, nsplit, s, rs, cs);
        case 8: return launch_gemm_cfg<E, MT, 256, 128, 128, 3, 4, 2>(U, V, M, K, Cp, T, nbatch, nsplit, s, rs, cs);
        default: return launch_gemm_cfg<E, MT, 256, 256, 128, 2, 4, 4>(U, V, M, K, Cp, T, nbatch, nsplit, s, rs, cs);
    }
}

// Stages are 128 bytes of reduction per row in every block shape.
int gemm_max_split(int Cp, int dt) {
    const int bke = dt == DT_I8 ? 128 : (two_byte(dt) ? 64 : 32);
    const int stages = (Cp + bke - 1) / bke;
    return stages < 1 ? 1 : stages;
}

// Few workgroups and a long reduction (deep UNet layers: 8x8 and 16x16 images, 1280+ channels): the
// stage is a stream of U that one workgroup per compute unit, each waiting on its own loads, cannot
// keep busy.  Cutting the reduction multiplies the workgroups in flight; the price is nsplit
// copies of the (small) product.
int gemm_split(int rows, int cols, int Cp, int nbatch, int dt) {
    const bool f16 = two_byte(dt);
    const int shape = pick_shape(rows, cols, nbatch, f16);
    const int bm = (shape == 4 || shape == 8) ? 256 : (shape == 6 ? 32 : ((shape == 2 || shape == 3) ? 64 : 128));
    const int bn = shape == 4 ? 256 : (shape == 5 ? 32 : ((shape == 1 || shape == 3) ? 64 : 128));
    const long long blocks = (long long)((rows + bm - 1) / bm) * ((cols + bn - 1) / bn) * nbatch;
    const int max_split = gemm_max_split(Cp, dt);
    int sp = 1;
    if (nbatch <= 16 && (bm < 128 || bn < 128) && blocks <= 320 && rows >= cols) {
        // measured: pays 6-10 % for F(2x2) with narrow blocks (images of 8x8, and 16x16 at batch 1)
        // while there are about as many workgroups as compute units; with the 36 batches of
        // F(4x4) the extra copies of the product cost more than the GEMM stage gains, and so they do with the
        // operands swapped (channel-last: few rows, many columns)
        sp = (int)(640 / blocks);
        if (sp > 3) sp = 3;
        if (sp > max_split / 4) sp = max_split / 4;               // at least four stages per workgroup
    }
    if (sp > max_split) sp = max_split;
    return sp < 1 ? 1 : sp;
}

hipError_t launch_batched_gemm(const void* U, const void* V, void* M, int K, int Cp, int T, int nbatch, int nsplit, int dt, bool half_product,
                               hipStream_t s, int shape) {
    if (nsplit < 1 || nsplit > gemm_max_split(Cp, dt)) return hipErrorInvalidValue;
    if (shape < -1 || shape > 8) return hipErrorInvalidValue;
    if (half_product && (dt != DT_F16 || nsplit != 1)) return hipErrorInvalidValue;      // fp16 storage, unsplit reduction only
    if (half_product) return launch_gemm_t<__half, __half>(U, V, M, K, Cp, T, nbatch, nsplit, shape, s);
    return with_dtype(dt, [&](auto* tag) {
        using E = std::remove_pointer_t<decltype(tag)>;
        return launch_gemm_t<E, float>(U, V, M, K, Cp, T, nbatch, nsplit, shape, s);
    });
}

hipError_t launch_batched_gemm_i8(const void* Uq, const float* dU, const void* Vq, const float* dV, float* M, int K, int Cq, int T,
                                  int nbatch, int nsplit, hipStream_t s, int shape) {
    if (nsplit < 1 || nsplit > gemm_max_split(Cq, DT_I8)) return hipErrorInvalidValue;
    if (shape < -1 || shape > 8 || !dU || !dV || Cq % 16 != 0) return hipErrorInvalidValue;
    return launch_gemm_t<i8_t, float>(Uq, Vq, M, K, Cq, T, nbatch, nsplit, shape, s, dU, dV);
}

}  // namespace wino
