// Step (i), activation side (Section "Techniques"): V = B^T d B for every
// overlapping alpha x alpha window d of the zero-padded image, per channel.
//
// x is NCHW (W contiguous) but the GEMM stage wants the reduction index c
// contiguous, V[alpha^2][T][Cp].  A workgroup therefore stages a patch of
// CB channels x alpha rows x (m*TJ+2) columns in LDS with loads that run along
// W, then each lane takes one channel of one tile, transforms it in fp32 and
// stores with lanes running along c.  Out-of-image taps and channels >= C are
// staged as zeros, so V's padded reduction columns are exact zeros.
// Four kernels: a scalar one for any row length, the chunked strip kernel, the
// sliding-window kernel for long rows, and the channel-last kernel, which needs no
// transposition.  All of them can apply SiLU(GroupNorm(.)) to what they load and
// read x through a 2x nearest-neighbour upsampling.
// Bound by HBM/L2 traffic: reads x once (plus the 2-row/2-column halo), writes V.
#include "wino_internal.h"
#include "wino_transforms.h"

namespace wino {

template <int M, typename E, int CB, int TJ, bool PRE>
__global__ void __launch_bounds__(256)
input_transform_nchw_kernel(const E* __restrict__ x, E* __restrict__ V,
                            int N, int C, int H, int W, int th, int tw, int T, int Cp, int strips_per_row, PreOp pre) {
    constexpr int A = M + 2;
    constexpr int PW = M * TJ + 2;                       // patch width (elements)
    // channel stride: odd number of 32-bit words so lanes (= channels) hit distinct banks
    constexpr int RAW = A * PW;
    constexpr int EPW = 4 / (int)sizeof(E);              // elements per 32-bit word
    constexpr int WORDS = (RAW + EPW - 1) / EPW;
    constexpr int CS = ((WORDS % 2 == 0) ? WORDS + 1 : WORDS) * EPW;
    __shared__ E patch[CB * CS];

    const int tid = threadIdx.x;
    int sidx = blockIdx.x;
    const int js = sidx % strips_per_row; sidx /= strips_per_row;
    const int ti = sidx % th;
    const int n = sidx / th;
    const int tj0 = js * TJ;
    const int c0 = blockIdx.y * CB;
    const int row0 = M * ti - 1;
    const int col0 = M * tj0 - 1;

    // ---- stage the patch: consecutive lanes walk along W -------------------------------
    for (int e = tid; e < CB * RAW; e += 256) {
        const int cc = e / RAW;
        const int rem = e - cc * RAW;
        const int a = rem / PW;
        const int b = rem - a * PW;
        const int r = row0 + a, q = col0 + b, c = c0 + cc;
        E v = from_f32<E>(0.f);
        if (c < C && r >= 0 && r < H && q >= 0 && q < W)
            v = x[(((size_t)n * C + c) * (H >> pre.up) + (r >> pre.up)) * (W >> pre.up) + (q >> pre.up)];
        patch[cc * CS + rem] = v;
    }
    __syncthreads();

    // ---- transform: lane = channel, one tile per wave per iteration ----------------------
    const int cc = tid % CB;
    const int c = c0 + cc;
    constexpr int TILES_PER_ITER = 256 / CB;
    const size_t plane = (size_t)T * Cp;
    for (int tl = tid / CB; tl < TJ; tl += TILES_PER_ITER) {
        const int tj = tj0 + tl;
        if (tj >= tw || c >= Cp) continue;
        const E* p = patch + cc * CS + M * tl;
        float d[A][A];
        PreLane pl = {0.f, 0.f, false};
        if (PRE) pl = pre_lane(pre, n, c, C);
#pragma unroll
        for (int a = 0; a < A; ++a)
#pragma unroll
            for (int b = 0; b < A; ++b) {
                d[a][b] = to_f32<E>(p[a * PW + b]);
                if (PRE) {
                    const int r = M * ti - 1 + a, q = M * tj - 1 + b;
                    d[a][b] = pre_apply(d[a][b], pl, r >= 0 && r < H && q >= 0 && q < W);
                }
            }
        // columns: tmp[:, b] = B^T d[:, b]
        float tmp[A][A];
#pragma unroll
        for (int b = 0; b < A; ++b) {
            float in[A], out[A];
#pragma unroll
            for (int a = 0; a < A; ++a) in[a] = d[a][b];
            bt_1d<M>(in, out);
#pragma unroll
            for (int a = 0; a < A; ++a) tmp[a][b] = out[a];
        }
        const size_t t = ((size_t)n * th + ti) * tw + tj;
        E* dst = V + t * Cp + c;
#pragma unroll
        for (int xi = 0; xi < A; ++xi) {
            float out[A];
            bt_1d<M>(tmp[xi], out);                      // rows: (B^T d) B = (B^T (B^T d)^T)^T
#pragma unroll
            for (int nu = 0; nu < A; ++nu) dst[(size_t)(xi * A + nu) * plane] = from_f32<E>(out[nu]);
        }
    }
}

// Fast path for rows that are whole 16-byte chunks (W*sizeof(E) a multiple of 16): the patch is
// fetched as 16-byte chunks, all loads of a lane issued before the first LDS write, so one global
// round trip covers the whole patch.  Patch columns run from m*tj0 - EPC to m*(tj0+TJ) + EPC
// (EPC = elements per chunk); a chunk is either wholly inside the image or wholly outside (zero).
template <int M, typename E, int CB, int TJ, bool PRE>
__global__ void __launch_bounds__(256)
input_transform_nchw_vec_kernel(const E* __restrict__ x, E* __restrict__ V,
                                int N, int C, int H, int W, int th, int tw, int T, int Cp, int strips_per_row,
                                int total_blocks, int blocks_per_xcd, PreOp pre) {
    constexpr int A = M + 2;
    constexpr int EPC = 16 / (int)sizeof(E);
    static_assert((M * TJ) % EPC == 0, "strip width must be whole chunks");
    constexpr int NCH = (M * TJ) / EPC + 2;              // chunks per patch row
    constexpr int ROWW = NCH * 4;                        // 32-bit words per patch row
    constexpr int CSW = (A * ROWW) | 1;                  // words per channel, odd: lanes = channels hit distinct banks
    __shared__ uint32_t patch[CB * CSW];

    const int tid = threadIdx.x;
    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of
    // (channel chunk, n, tile row, strip) so neighbours that share halo rows share an L2.
    const int logical = (blockIdx.x % 8) * blocks_per_xcd + blockIdx.x / 8;
    if (logical >= total_blocks) return;                 // uniform, before the barrier
    int sidx = logical;
    const int js = sidx % strips_per_row; sidx /= strips_per_row;
    const int ti = sidx % th; sidx /= th;
    const int n = sidx % N;
    const int c0 = (sidx / N) * CB;
    const int tj0 = js * TJ;
    const int row0 = M * ti - 1;
    const int col0 = M * tj0 - EPC;

    // 32-bit lane offsets against wave-uniform 64-bit bases keep the address arithmetic off the
    // vector ALU (the transform itself is only ~200 operations per tile and channel).
    const int Hs = H >> pre.up, Ws = W >> pre.up;         // the stored image (half size when it is read upsampled)
    const unsigned char* xb = reinterpret_cast<const unsigned char*>(x + ((size_t)n * C + c0) * Hs * Ws);
    // a lane owns one (channel, chunk column) and walks the alpha patch rows: one add per load
    constexpr int ITEMS = CB * NCH;
    constexpr int PASSES = (ITEMS + 255) / 256;
    uint4 reg[PASSES][A];
#pragma unroll
    for (int ps = 0; ps < PASSES; ++ps) {
        const int item = tid + ps * 256;
        const int cc = item / NCH, ch = item - cc * NCH;
        const int col = col0 + ch * EPC;
        const bool ok = item < ITEMS && (c0 + cc) < C && col >= 0 && col + EPC <= W;
        const unsigned off0 = (unsigned)(((cc * H + row0) * W + col) * (int)sizeof(E));   // may wrap for row0 = -1; only used when the row is valid
#pragma unroll
        for (int a = 0; a < A; ++a) {
            const int r = row0 + a;
            reg[ps][a] = make_uint4(0, 0, 0, 0);
            if (ok && r >= 0 && r < H) {
                if (pre.up)   // 8 source bytes under the 16-byte chunk, every element twice
                    reg[ps][a] = dup_elements<E>(*reinterpret_cast<const uint2*>(
                        xb + (unsigned)(((cc * Hs + (r >> 1)) * Ws + (col >> 1)) * (int)sizeof(E))));
                else
                    reg[ps][a] = *reinterpret_cast<const uint4*>(xb + (off0 + (unsigned)(a * W * (int)sizeof(E))));
            }
        }
    }
#pragma unroll
    for (int ps = 0; ps < PASSES; ++ps) {
        const int item = tid + ps * 256;
        if (item < ITEMS) {
            const int cc = item / NCH, ch = item - cc * NCH;
            uint32_t* dst = patch + cc * CSW + ch * 4;
#pragma unroll
            for (int a = 0; a < A; ++a) {
                dst[a * ROWW + 0] = reg[ps][a].x; dst[a * ROWW + 1] = reg[ps][a].y;
                dst[a * ROWW + 2] = reg[ps][a].z; dst[a * ROWW + 3] = reg[ps][a].w;
            }
        }
    }
    __syncthreads();

    // one tile per wave per iteration (lane = channel), so the tile index is wave-uniform
    static_assert(CB == 64, "lane = channel");
    const int cc = tid & 63;
    const int c = c0 + cc;
    const size_t plane = (size_t)T * Cp;
    const E* pch = reinterpret_cast<const E*>(patch + cc * CSW);
    for (int tl = __builtin_amdgcn_readfirstlane(tid >> 6); tl < TJ; tl += 4) {
        const int tj = tj0 + tl;
        if (tj >= tw) break;                              // wave-uniform
        const E* p = pch + (EPC - 1) + M * tl;
        float d[A][A];
        PreLane pl = {0.f, 0.f, false};
        if (PRE) pl = pre_lane(pre, n, c, C);
#pragma unroll
        for (int a = 0; a < A; ++a)
#pragma unroll
            for (int b = 0; b < A; ++b) {
                d[a][b] = to_f32<E>(p[a * (NCH * EPC) + b]);
                if (PRE) {
                    const int r = M * ti - 1 + a, q = M * tj - 1 + b;
                    d[a][b] = pre_apply(d[a][b], pl, r >= 0 && r < H && q >= 0 && q < W);
                }
            }
        float tmp[A][A];
#pragma unroll
        for (int b = 0; b < A; ++b) {
            float in[A], out[A];
#pragma unroll
            for (int a = 0; a < A; ++a) in[a] = d[a][b];
            bt_1d<M>(in, out);
#pragma unroll
            for (int a = 0; a < A; ++a) tmp[a][b] = out[a];
        }
        const size_t t = ((size_t)n * th + ti) * tw + tj;  // wave-uniform
        E* rowp = V + t * Cp;                              // wave-uniform base; lane offset is just c
        const unsigned coff = (unsigned)c * (unsigned)sizeof(E);
        if (c < Cp) {
            unsigned char* pp = reinterpret_cast<unsigned char*>(rowp);     // walks the alpha^2 planes
            const size_t plane_bytes = plane * sizeof(E);
#pragma unroll
            for (int xi = 0; xi < A; ++xi) {
                float out[A];
                bt_1d<M>(tmp[xi], out);
#pragma unroll
                for (int nu = 0; nu < A; ++nu) {
                    *reinterpret_cast<E*>(pp + coff) = from_f32<E>(out[nu]);
                    pp += plane_bytes;
                }
            }
        }
    }
}

// Long rows: a workgroup slides along one tile row.  The row is cut into 64-byte bodies (TJ tiles
// wide); LDS keeps the last two bodies of every (channel, patch row), and step s transforms the
// TJ tiles that straddle the seam between bodies s-1 and s, whose windows lie wholly inside those
// two bodies.  Every body is therefore fetched from memory once per workgroup, as aligned 64-byte
// runs, instead of once per strip plus halo chunks on either side; body s+1 is in flight while
// step s computes and stores.  Tiles outside [0, tw) are replaced by the nearest tile inside, which
// the same step computes anyway: the duplicate writes the same values, and every wave issues the
// same number of stores per step, so the wait for the prefetched body leaves those stores pending.
// Needs Cp % 64 == 0 (no lane is idle) and rows of whole 16-byte chunks.
template <int M, typename E, int TJ, bool PRE>
__global__ void __launch_bounds__(256)
input_transform_nchw_slide_kernel(const E* __restrict__ x, E* __restrict__ V,
                                  int N, int C, int H, int W, int th, int tw, int T, int Cp, int steps_per_row,
                                  int spb, int total_blocks, int blocks_per_xcd, PreOp pre) {
    constexpr int A = M + 2;
    constexpr int EPC = 16 / (int)sizeof(E);             // elements per 16-byte chunk
    constexpr int BODYE = 64 / (int)sizeof(E);           // elements per body
    constexpr int EPW = 4 / (int)sizeof(E);              // elements per 32-bit word
    static_assert(TJ * M == BODYE && TJ % 4 == 0, "a body is TJ tiles wide, TJ/4 tiles per wave");
    constexpr int ROWW = 32;                             // words per patch row: two bodies
    constexpr int CSW = (A * ROWW) | 1;                  // words per channel, odd: lanes = channels hit distinct banks
    __shared__ uint32_t patch[64 * CSW];

    const int tid = threadIdx.x;
    const int logical = (blockIdx.x % 8) * blocks_per_xcd + blockIdx.x / 8;   // one contiguous range per XCD
    if (logical >= total_blocks) return;                 // uniform, before any barrier
    const int groups_per_row = (steps_per_row + spb - 1) / spb;
    int sidx = logical;
    const int jg = sidx % groups_per_row; sidx /= groups_per_row;
    const int ti = sidx % th; sidx /= th;
    const int n = sidx % N;
    const int c0 = (sidx / N) * 64;
    const int s0 = jg * spb;
    const int s1 = min(s0 + spb, steps_per_row);
    const int row0 = M * ti - 1;

    const int Hs = H >> pre.up, Ws = W >> pre.up;         // the stored image (half size when it is read upsampled)
    const unsigned char* xb = reinterpret_cast<const unsigned char*>(x + ((size_t)n * C + c0) * Hs * Ws);
    // loader role: lane = (channel, chunk of the body), walks the alpha patch rows
    const int lc = tid >> 2, lch = tid & 3;
    const bool lc_ok = (c0 + lc) < C;
    uint4 reg[A];
    auto fetch = [&](int body) {
        const int col = body * BODYE + lch * EPC;
        const bool ok = lc_ok && body >= 0 && col < W;   // W is a multiple of EPC: a chunk is inside or outside as a whole
        const unsigned off0 = (unsigned)(((lc * H + row0) * W + col) * (int)sizeof(E));   // only used when row and col are valid
#pragma unroll
        for (int a = 0; a < A; ++a) {
            const int r = row0 + a;
            reg[a] = make_uint4(0, 0, 0, 0);
            if (ok && r >= 0 && r < H) {
                if (pre.up)   // 8 source bytes under the 16-byte chunk, every element twice
                    reg[a] = dup_elements<E>(*reinterpret_cast<const uint2*>(
                        xb + (unsigned)(((lc * Hs + (r >> 1)) * Ws + (col >> 1)) * (int)sizeof(E))));
                else
                    reg[a] = *reinterpret_cast<const uint4*>(xb + (off0 + (unsigned)(a * W * (int)sizeof(E))));
            }
        }
    };
    auto stash = [&](int body) {
        uint32_t* dst = patch + lc * CSW + (body & 1) * 16 + lch * 4;
#pragma unroll
        for (int a = 0; a < A; ++a) {
            dst[a * ROWW + 0] = reg[a].x; dst[a * ROWW + 1] = reg[a].y;
            dst[a * ROWW + 2] = reg[a].z; dst[a * ROWW + 3] = reg[a].w;
        }
    };

    // transform role: lane = channel, TJ/4 tiles per wave and step
    const int cc = tid & 63;
    const int c = c0 + cc;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const size_t plane_bytes = (size_t)T * Cp * sizeof(E);
    const E* pch = reinterpret_cast<const E*>(patch + cc * CSW);
    const unsigned coff = (unsigned)c * (unsigned)sizeof(E);
    PreLane pl = {0.f, 0.f, false};
    if (PRE) pl = pre_lane(pre, n, c, C);

    fetch(s0 - 1);
    stash(s0 - 1);
    fetch(s0);
    stash(s0);
    __syncthreads();
    for (int s = s0; s < s1; ++s) {
        if (s + 1 < s1) fetch(s + 1);                     // in flight while this step is transformed
#pragma unroll
        for (int i = 0; i < TJ / 4; ++i) {
            int tj = TJ * s - TJ / 2 + wave + 4 * i;
            tj = min(max(tj, 0), tw - 1);                 // wave-uniform; duplicates write identical values
            const int g0 = M * tj - 1;                    // first window column (global), -1 for the left border
            int colofs[A];
#pragma unroll
            for (int b = 0; b < A; ++b) colofs[b] = (g0 + b) & (2 * BODYE - 1);
            float d[A][A];
#pragma unroll
            for (int a = 0; a < A; ++a)
#pragma unroll
                for (int b = 0; b < A; ++b) {
                    d[a][b] = to_f32<E>(pch[a * (ROWW * EPW) + colofs[b]]);
                    if (PRE) {
                        const int r = M * ti - 1 + a, q = g0 + b;
                        d[a][b] = pre_apply(d[a][b], pl, r >= 0 && r < H && q >= 0 && q < W);
                    }
                }
            float tmp[A][A];
#pragma unroll
            for (int b = 0; b < A; ++b) {
                float in[A], out[A];
#pragma unroll
                for (int a = 0; a < A; ++a) in[a] = d[a][b];
                bt_1d<M>(in, out);
#pragma unroll
                for (int a = 0; a < A; ++a) tmp[a][b] = out[a];
            }
            const size_t t = ((size_t)n * th + ti) * tw + tj;                  // wave-uniform
            unsigned char* pp = reinterpret_cast<unsigned char*>(V + t * Cp);  // walks the alpha^2 planes
#pragma unroll
            for (int xi = 0; xi < A; ++xi) {
                float out[A];
                bt_1d<M>(tmp[xi], out);
#pragma unroll
                for (int nu = 0; nu < A; ++nu) {
                    *reinterpret_cast<E*>(pp + coff) = from_f32<E>(out[nu]);
                    pp += plane_bytes;
                }
            }
        }
        if (s + 1 < s1) {
            __syncthreads();                              // everyone is done with body s-1
            stash(s + 1);                                 // overwrites it
            __syncthreads();
        }
    }
}

// NHWC activations (channels contiguous): no transposition is needed, V's rows are channel-
// contiguous too.  One lane owns CPT adjacent channels of one tile, reads its alpha x alpha window
// straight from global memory (neighbouring lanes read neighbouring channels, so every load is
// one contiguous run; the 2.25x / 4x window overlap is served by L1/L2) and stores CPT values
// per transformed position.  Channels in [C, Cp) are written as zeros.
template <int M, typename E, int CPT, bool PRE>
__global__ void __launch_bounds__(256)
input_transform_nhwc_kernel(const E* __restrict__ x, E* __restrict__ V,
                            int N, int C, int H, int W, int th, int tw, int T, int Cp, int per_xcd, PreOp pre) {
    constexpr int A = M + 2;
    const int groups = Cp / CPT;                               // Cp is a multiple of 8
    // workgroups go round-robin to the 8 XCDs: give each XCD one contiguous range of tiles, so
    // that the window overlap between neighbouring tiles is served by that XCD's own L2
    const size_t logical = (size_t)(blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    const size_t item = logical * 256 + threadIdx.x;
    if (item >= (size_t)T * groups) return;
    const int gidx = (int)(item % groups);
    int t = (int)(item / groups);
    const int c = gidx * CPT;
    const int tj = t % tw; int q = t / tw;
    const int ti = q % th;
    const int n = q / th;
    const bool live = c < C;                                   // CPT divides C on this path
    PreLane pl[CPT];
#pragma unroll
    for (int u = 0; u < CPT; ++u) { pl[u].sc = 0.f; pl[u].sh = 0.f; pl[u].on = false; if (PRE) pl[u] = pre_lane(pre, n, c + u, C); }
    // Every load is issued unconditionally from a clamped (always valid) address and the loaded
    // bits are ANDed with an all-ones / all-zeros mask, so that the alpha^2 loads of a lane are all
    // in flight together.  The masks pass through an empty asm statement: seen as a select on the
    // bounds test, the compiler moves each load into a branch of its own and waits for it there.
    const int us = pre.up;                                      // 1: x is stored at half size and read upsampled
    const E* xb = x + (size_t)n * (H >> us) * (W >> us) * C + (live ? c : 0);
    uint32_t rmask[A], cmask[A];
#pragma unroll
    for (int a = 0; a < A; ++a) {
        const int r = M * ti - 1 + a, col = M * tj - 1 + a;
        rmask[a] = (live && r >= 0 && r < H) ? 0xffffffffu : 0u;
        cmask[a] = (col >= 0 && col < W) ? 0xffffffffu : 0u;
        asm("" : "+v"(rmask[a]));
        asm("" : "+v"(cmask[a]));
    }
    float d[CPT][A][A];
#pragma unroll
    for (int a = 0; a < A; ++a) {
        const int r = M * ti - 1 + a;
        const E* xr = xb + (size_t)(min(max(r, 0), H - 1) >> us) * (W >> us) * C;
#pragma unroll
        for (int b = 0; b < A; ++b) {
            const int col = M * tj - 1 + b;
            const E* p = xr + (size_t)(min(max(col, 0), W - 1) >> us) * C;
            const uint32_t msk = rmask[a] & cmask[b];
            union { uint32_t w; E e[4 / sizeof(E)]; } v;
            if constexpr (CPT == 2) v.w = *reinterpret_cast<const uint32_t*>(p);
            else if constexpr (sizeof(E) == 4) v.w = *reinterpret_cast<const uint32_t*>(p);
            else v.w = *reinterpret_cast<const uint16_t*>(p);
            v.w &= msk;
#pragma unroll
            for (int u = 0; u < CPT; ++u) {
                d[u][a][b] = to_f32<E>(v.e[u]);
                if (PRE) d[u][a][b] = pre_apply(d[u][a][b], pl[u], msk != 0u);
            }
        }
    }
    float o[CPT][A][A];
#pragma unroll
    for (int u = 0; u < CPT; ++u) {
        float tmp[A][A];
#pragma unroll
        for (int b = 0; b < A; ++b) {
            float in[A], out[A];
#pragma unroll
            for (int a = 0; a < A; ++a) in[a] = d[u][a][b];
            bt_1d<M>(in, out);
#pragma unroll
            for (int a = 0; a < A; ++a) tmp[a][b] = out[a];
        }
#pragma unroll
        for (int xi = 0; xi < A; ++xi) bt_1d<M>(tmp[xi], o[u][xi]);
    }
    const size_t plane = (size_t)T * Cp;
    E* dst = V + (size_t)t * Cp + c;
#pragma unroll
    for (int xi = 0; xi < A; ++xi)
#pragma unroll
        for (int nu = 0; nu < A; ++nu) {
            E v[CPT];
#pragma unroll
            for (int u = 0; u < CPT; ++u) v[u] = from_f32<E>(o[u][xi][nu]);
            E* p = dst + (size_t)(xi * A + nu) * plane;
            if constexpr (CPT == 2) { *reinterpret_cast<uint32_t*>(p) = *reinterpret_cast<const uint32_t*>(v); }
            else { p[0] = v[0]; }
        }
}

template <int M, typename E>
static hipError_t launch_it_nhwc(const void* x, void* V, const Geom& g, const PreOp* pre, hipStream_t s) {
    const PreOp po = pre ? *pre : PreOp();
    const bool gn = po.stats != nullptr;
    // two fp16 channels per lane (4-byte accesses) when channel pairs never straddle C
    const bool pair = sizeof(E) == 2 && g.C % 2 == 0 && (reinterpret_cast<uintptr_t>(x) & 3u) == 0;
    const int cpt = pair ? 2 : 1;
    const size_t items = (size_t)g.T * (g.Cp / cpt);
    const size_t blocks = (items + 255) / 256;
    if (blocks > 0x3fffffffULL) return hipErrorInvalidValue;
    const int per_xcd = (int)((blocks + 7) / 8);
    dim3 block(256), grid((unsigned)per_xcd * 8);
    if (pair) {
        if constexpr (sizeof(E) == 2) {
            if (gn) hipLaunchKernelGGL((input_transform_nhwc_kernel<M, E, 2, true>), grid, block, 0, s, (const E*)x, (E*)V, g.N, g.C, g.H, g.W, g.th, g.tw, g.T, g.Cp, per_xcd, po);
            else     hipLaunchKernelGGL((input_transform_nhwc_kernel<M, E, 2, false>), grid, block, 0, s, (const E*)x, (E*)V, g.N, g.C, g.H, g.W, g.th, g.tw, g.T, g.Cp, per_xcd, po);
        }
    } else {
        if (gn) hipLaunchKernelGGL((input_transform_nhwc_kernel<M, E, 1, true>), grid, block, 0, s, (const E*)x, (E*)V, g.N, g.C, g.H, g.W, g.th, g.tw, g.T, g.Cp, per_xcd, po);
        else     hipLaunchKernelGGL((input_transform_nhwc_kernel<M, E, 1, false>), grid, block, 0, s, (const E*)x, (E*)V, g.N, g.C, g.H, g.W, g.th, g.tw, g.T, g.Cp, per_xcd, po);
    }
    return hipGetLastError();
}

template <int M, typename E, int CB, int TJ>
static hipError_t launch_it_cfg(const void* x, void* V, const Geom& g, const PreOp* pre, hipStream_t s) {
    const PreOp po = pre ? *pre : PreOp();
    const bool gn = po.stats != nullptr;
    const int strips = (g.tw + TJ - 1) / TJ;
    dim3 block(256), grid((unsigned)(g.N * g.th * strips), (unsigned)((g.Cp + CB - 1) / CB));
    // fast path: rows are whole 16-byte chunks and a 64-channel slab of x spans < 2 GB (32-bit lane offsets)
    const bool rows_are_chunks = ((size_t)g.W * sizeof(E)) % 16 == 0 && (reinterpret_cast<uintptr_t>(x) & 15u) == 0 &&
                                 (size_t)CB * g.H * g.W * sizeof(E) < ((size_t)1 << 31);
    constexpr int STJ = 64 / (int)sizeof(E) / M;          // tiles per 64-byte body
    if (rows_are_chunks && g.Cp % 64 == 0) {
        const int steps = (g.tw + STJ / 2 + STJ - 1) / STJ;
        // Measured over the SD-shaped layers: with fp16 F(2x2) (16 tiles per body) the aligned fetch
        // alone pays from 16 tiles per row on; otherwise the strip kernel wins until a row has
        // eight steps.  Two steps per workgroup keep the grid large and the tail short.
        const bool wide_body = sizeof(E) == 2 && M == 2;
        const bool pays = wide_body ? g.tw >= STJ : steps >= 8;
        const int spb = steps >= 8 ? 2 : 1;
        const long long total = (long long)g.N * g.th * (g.Cp / 64) * ((steps + spb - 1) / spb);
        if (pays && total <= 0x3fffffffLL) {
            const int per_xcd = (int)((total + 7) / 8);
            if (gn) hipLaunchKernelGGL((input_transform_nchw_slide_kernel<M, E, STJ, true>), dim3((unsigned)(per_xcd * 8)), block, 0, s,
                                        (const E*)x, (E*)V, g.N, g.C, g.H, g.W, g.th, g.tw, g.T, g.Cp, steps, spb, (int)total, per_xcd, po);
            else     hipLaunchKernelGGL((input_transform_nchw_slide_kernel<M, E, STJ, false>), dim3((unsigned)(per_xcd * 8)), block, 0, s,
                                        (const E*)x, (E*)V, g.N, g.C, g.H, g.W, g.th, g.tw, g.T, g.Cp, steps, spb, (int)total, per_xcd, po);
            return hipGetLastError();
        }
    }
    if (rows_are_chunks) {
        const long long total = (long long)grid.x * grid.y;
        if (total > 0x3fffffffLL) return hipErrorInvalidValue;
        const int per_xcd = (int)((total + 7) / 8);
        if (gn) hipLaunchKernelGGL((input_transform_nchw_vec_kernel<M, E, CB, TJ, true>), dim3((unsigned)(per_xcd * 8)), block, 0, s,
                                    (const E*)x, (E*)V, g.N, g.C, g.H, g.W, g.th, g.tw, g.T, g.Cp, strips, (int)total, per_xcd, po);
        else     hipLaunchKernelGGL((input_transform_nchw_vec_kernel<M, E, CB, TJ, false>), dim3((unsigned)(per_xcd * 8)), block, 0, s,
                                    (const E*)x, (E*)V, g.N, g.C, g.H, g.W, g.th, g.tw, g.T, g.Cp, strips, (int)total, per_xcd, po);
    } else {
        if (gn) hipLaunchKernelGGL((input_transform_nchw_kernel<M, E, CB, TJ, true>), grid, block, 0, s,
                                    (const E*)x, (E*)V, g.N, g.C, g.H, g.W, g.th, g.tw, g.T, g.Cp, strips, po);
        else     hipLaunchKernelGGL((input_transform_nchw_kernel<M, E, CB, TJ, false>), grid, block, 0, s,
                                    (const E*)x, (E*)V, g.N, g.C, g.H, g.W, g.th, g.tw, g.T, g.Cp, strips, po);
    }
    return hipGetLastError();
}

template <int M, typename E>
static hipError_t launch_it(const void* x, void* V, const Geom& g, const PreOp* pre, hipStream_t s) {
    constexpr int Q = 8 / M;      // TJ multiples that keep strips whole 16-byte chunks for fp16
    return launch_it_cfg<M, E, 64, 2 * Q>(x, V, g, pre, s);      // measured best of 1, 2, 4, 8 x Q tiles per strip
}

hipError_t launch_input_transform(const void* x, void* V, const Geom& g, int dt, bool nhwc, const PreOp* pre, hipStream_t s) {
    return with_dtype(dt, [&](auto* tag) {
        using E = std::remove_pointer_t<decltype(tag)>;
        if (nhwc) return g.m == 2 ? launch_it_nhwc<2, E>(x, V, g, pre, s) : launch_it_nhwc<4, E>(x, V, g, pre, s);
        return g.m == 2 ? launch_it<2, E>(x, V, g, pre, s) : launch_it<4, E>(x, V, g, pre, s);
    });
}

}  // namespace wino
