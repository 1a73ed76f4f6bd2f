// Step (ii) (Section "Techniques"): the "element-wise multiplication" of the
// transformed filter and activation, summed over input channels — i.e. alpha^2
// independent matrix products  M_b[k][t] = sum_c U_b[k][c] * V_b[t][c],
// b = xi*alpha+nu.  This is the one dense contraction of the path and runs on
// the MFMA units with fp32 accumulation.
//
// Both operands are row-major with the reduction index contiguous, so a lane's
// MFMA fragment is one 16-byte load.  A workgroup owns a BM x BN block of one
// batch; 4 waves in a 2x2 grid, each wave (BM/2)x(BN/2) as 32x32 MFMA tiles.
// Stages of 128 bytes per row (64 fp16 / 32 fp32 reduction elements) go global
// -> registers -> LDS (rows padded by 16 bytes: conflict-free 128-bit reads),
// double-buffered so the next stage's global loads fly during the MFMAs.
// Rows beyond K / T and reduction chunks beyond Cp are staged as zeros.
#include "wino_internal.h"

namespace wino {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef float float16_t __attribute__((ext_vector_type(16)));

constexpr int kRowBytes = 128;                 // reduction bytes per row per stage
constexpr int kPitch = kRowBytes + 16;         // LDS row pitch
constexpr int kChunksPerRow = kRowBytes / 16;  // 8

template <typename E> struct Mma;
template <> struct Mma<__half> {
    // one 16-byte chunk = 8 reduction elements; lanes 0-31 and 32-63 hold different chunks
    static __device__ __forceinline__ void run(const uint4& a, const uint4& b, float16_t& c) {
        c = __builtin_amdgcn_mfma_f32_32x32x16_f16(*reinterpret_cast<const half8_t*>(&a),
                                                    *reinterpret_cast<const half8_t*>(&b), c, 0, 0, 0);
    }
};
template <> struct Mma<float> {
    static __device__ __forceinline__ void run(const uint4& a, const uint4& b, float16_t& c) {
        const float* fa = reinterpret_cast<const float*>(&a);
        const float* fb = reinterpret_cast<const float*>(&b);
#pragma unroll
        for (int j = 0; j < 4; ++j) c = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[j], fb[j], c, 0, 0, 0);
    }
};

template <typename E, int BM, int BN>
__global__ void __launch_bounds__(256)
wino_gemm_kernel(const E* __restrict__ U, const E* __restrict__ V, float* __restrict__ Mo,
                 int K, int Cp, int T, int tiles_m, int tiles_n, int total_blocks, int blocks_per_xcd) {
    constexpr int BKE = kRowBytes / (int)sizeof(E);       // reduction elements per stage
    constexpr int EPC = 16 / (int)sizeof(E);              // elements per 16-byte chunk
    constexpr int WTM = BM / 2, WTN = BN / 2;             // wave tile
    constexpr int FM = WTM / 32, FN = WTN / 32;           // 32x32 MFMA tiles per wave
    constexpr int A_CHUNKS = BM * kChunksPerRow / 256;    // 16-byte chunks per thread per stage
    constexpr int B_CHUNKS = BN * kChunksPerRow / 256;
    static_assert(BM % 64 == 0 && BN % 64 == 0, "wave tile must be a multiple of 32");

    __shared__ __attribute__((aligned(16))) unsigned char lds[2][(BM + BN) * kPitch];

    // XCD-aware mapping: hardware deals workgroups round-robin to the 8 XCDs, so give
    // each XCD a contiguous range of logical blocks (same batch -> same L2).
    const int bid = blockIdx.x;
    const int logical = (bid % 8) * blocks_per_xcd + bid / 8;
    if (logical >= total_blocks) return;                  // uniform per workgroup, before any barrier
    const int tn = logical % tiles_n;
    const int tm = (logical / tiles_n) % tiles_m;
    const int batch = logical / (tiles_n * tiles_m);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int row_k0 = tm * BM, row_t0 = tn * BN;

    const E* Ub = U + (size_t)batch * K * Cp;
    const E* Vb = V + (size_t)batch * T * Cp;

    uint4 ra[A_CHUNKS], rb[B_CHUNKS];
    auto load_stage = [&](int kt) {
        const int kbase = kt * BKE;
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i) {
            const int q = tid + i * 256;
            const int r = q / kChunksPerRow, ch = q % kChunksPerRow;
            const int gr = row_k0 + r, gk = kbase + ch * EPC;
            ra[i] = (gr < K && gk < Cp) ? *reinterpret_cast<const uint4*>(Ub + (size_t)gr * Cp + gk)
                                        : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < B_CHUNKS; ++i) {
            const int q = tid + i * 256;
            const int r = q / kChunksPerRow, ch = q % kChunksPerRow;
            const int gr = row_t0 + r, gk = kbase + ch * EPC;
            rb[i] = (gr < T && gk < Cp) ? *reinterpret_cast<const uint4*>(Vb + (size_t)gr * Cp + gk)
                                        : make_uint4(0, 0, 0, 0);
        }
    };
    auto store_stage = [&](int buf) {
        unsigned char* la = lds[buf];
        unsigned char* lb = lds[buf] + BM * kPitch;
#pragma unroll
        for (int i = 0; i < A_CHUNKS; ++i) {
            const int q = tid + i * 256;
            *reinterpret_cast<uint4*>(la + (q / kChunksPerRow) * kPitch + (q % kChunksPerRow) * 16) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < B_CHUNKS; ++i) {
            const int q = tid + i * 256;
            *reinterpret_cast<uint4*>(lb + (q / kChunksPerRow) * kPitch + (q % kChunksPerRow) * 16) = rb[i];
        }
    };

    float16_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int nk = (Cp + BKE - 1) / BKE;
    load_stage(0);
    store_stage(0);
    __syncthreads();

    const int frag_row = lane & 31, frag_half = lane >> 5;
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) load_stage(kt + 1);
        const unsigned char* la = lds[buf] + (wm * WTM + frag_row) * kPitch + frag_half * 16;
        const unsigned char* lb = lds[buf] + BM * kPitch + (wn * WTN + frag_row) * kPitch + frag_half * 16;
#pragma unroll
        for (int ks = 0; ks < kChunksPerRow / 2; ++ks) {
            uint4 fa[FM], fb[FN];
#pragma unroll
            for (int i = 0; i < FM; ++i) fa[i] = *reinterpret_cast<const uint4*>(la + i * 32 * kPitch + ks * 32);
#pragma unroll
            for (int j = 0; j < FN; ++j) fb[j] = *reinterpret_cast<const uint4*>(lb + j * 32 * kPitch + ks * 32);
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j) Mma<E>::run(fa[i], fb[j], acc[i][j]);
        }
        if (kt + 1 < nk) store_stage(buf ^ 1);
        __syncthreads();
    }

    // 32x32 accumulator layout: register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32
    float* Mb = Mo + (size_t)batch * K * T;
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            const int t = row_t0 + wn * WTN + j * 32 + frag_row;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int k = row_k0 + wm * WTM + i * 32 + 8 * (r / 4) + 4 * frag_half + (r % 4);
                if (k < K && t < T) Mb[(size_t)k * T + t] = acc[i][j][r];
            }
        }
}

template <typename E, int BM, int BN>
static hipError_t launch_gemm_cfg(const void* U, const void* V, float* M, int K, int Cp, int T, int nbatch, hipStream_t s) {
    const int tiles_m = (K + BM - 1) / BM, tiles_n = (T + BN - 1) / BN;
    const long long total = (long long)tiles_m * tiles_n * nbatch;
    if (total > 0x3fffffffLL) return hipErrorInvalidValue;
    const int per_xcd = (int)((total + 7) / 8);
    dim3 block(256), grid((unsigned)(per_xcd * 8));
    hipLaunchKernelGGL((wino_gemm_kernel<E, BM, BN>), grid, block, 0, s, (const E*)U, (const E*)V, M,
                       K, Cp, T, tiles_m, tiles_n, (int)total, per_xcd);
    return hipGetLastError();
}

hipError_t launch_batched_gemm(const void* U, const void* V, float* M, int K, int Cp, int T, int nbatch, bool f16, hipStream_t s) {
    // narrow T (small images): 64-wide column blocks waste fewer MFMA columns
    if (f16) {
        if (T <= 64) return launch_gemm_cfg<__half, 128, 64>(U, V, M, K, Cp, T, nbatch, s);
        return launch_gemm_cfg<__half, 128, 128>(U, V, M, K, Cp, T, nbatch, s);
    }
    if (T <= 64) return launch_gemm_cfg<float, 128, 64>(U, V, M, K, Cp, T, nbatch, s);
    return launch_gemm_cfg<float, 128, 128>(U, V, M, K, Cp, T, nbatch, s);
}

}  // namespace wino
