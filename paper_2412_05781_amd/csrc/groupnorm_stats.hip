// Mean and 1/sqrt(var + eps) per (image, channel group): the statistics that the activation
// transform needs to apply GroupNorm + SiLU while it loads x (the operators next to the 3x3
// convolution inside a residual block; the paper's Section "Techniques" argues for keeping such
// dependent steps local).  Two launches: partial (sum, sum of squares) per slice of a group, fp32
// per lane and fp64 from the block reduction on; then one lane per group merges the slices.
// Deterministic (fixed reduction trees, no atomics).  Bound by reading x once from HBM.
#include "wino_internal.h"

namespace wino {

constexpr int kMaxSplit = 32;

size_t groupnorm_stats_bytes(int N, int groups) {
    const size_t ng = (size_t)N * groups;
    return ((ng * 2 * sizeof(float) + 255) / 256) * 256 + ng * kMaxSplit * 2 * sizeof(double);
}

// block reduction of (s, q): fp32 inside a wave (shuffles), fp64 across the four waves
__device__ __forceinline__ void block_reduce_store(float s, float q, double* dst) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) { s += __shfl_down(s, off, 64); q += __shfl_down(q, off, 64); }
    __shared__ double ws[4], wq[4];
    if ((threadIdx.x & 63) == 0) { ws[threadIdx.x >> 6] = (double)s; wq[threadIdx.x >> 6] = (double)q; }
    __syncthreads();
    if (threadIdx.x == 0) { dst[0] = ws[0] + ws[1] + ws[2] + ws[3]; dst[1] = wq[0] + wq[1] + wq[2] + wq[3]; }
}

// NCHW fast path: a group is one contiguous run of cpg*H*W elements; 16-byte loads.
template <typename E>
__global__ void __launch_bounds__(256)
groupnorm_partial_vec_kernel(const E* __restrict__ x, double* __restrict__ partial, size_t group_elems, int split,
                             size_t per_slice) {
    constexpr int EPC = 16 / (int)sizeof(E);
    const int ng = blockIdx.x, sl = blockIdx.y;
    const E* base = x + (size_t)ng * group_elems;          // groups of all images are laid end to end
    const size_t lo = (size_t)sl * per_slice;
    size_t hi = lo + per_slice; hi = hi < group_elems ? hi : group_elems;
    float s = 0.f, q = 0.f;
    for (size_t e = lo + (size_t)threadIdx.x * EPC; e < hi; e += 256 * EPC) {
        const uint4 raw = *reinterpret_cast<const uint4*>(base + e);
        const E* v = reinterpret_cast<const E*>(&raw);
#pragma unroll
        for (int u = 0; u < EPC; ++u) { const float f = to_f32<E>(v[u]); s += f; q = fmaf(f, f, q); }
    }
    block_reduce_store(s, q, partial + ((size_t)ng * split + sl) * 2);
}

template <typename E, bool NHWC>
__global__ void __launch_bounds__(256)
groupnorm_partial_kernel(const E* __restrict__ x, double* __restrict__ partial, int C, int HW, int groups, int cpg,
                         int split, size_t per_slice) {
    const int ng = blockIdx.x, sl = blockIdx.y;
    const int n = ng / groups, g = ng % groups;
    const size_t elems = (size_t)cpg * HW;
    const size_t lo = (size_t)sl * per_slice;
    size_t hi = lo + per_slice; hi = hi < elems ? hi : elems;
    float s = 0.f, q = 0.f;
    for (size_t e = lo + threadIdx.x; e < hi; e += 256) {
        size_t idx;
        if (NHWC) { const size_t p = e / cpg; const int j = (int)(e - p * cpg); idx = ((size_t)n * HW + p) * C + (size_t)g * cpg + j; }
        else idx = ((size_t)n * C + (size_t)g * cpg) * HW + e;
        const float v = to_f32<E>(x[idx]);
        s += v; q = fmaf(v, v, q);
    }
    block_reduce_store(s, q, partial + ((size_t)ng * split + sl) * 2);
}

__global__ void groupnorm_finalize_kernel(const double* __restrict__ partial, float* __restrict__ stats, int total,
                                          int split, double inv_count, float eps) {
    const int ng = blockIdx.x * blockDim.x + threadIdx.x;
    if (ng >= total) return;
    double s = 0.0, q = 0.0;
    for (int i = 0; i < split; ++i) { s += partial[((size_t)ng * split + i) * 2]; q += partial[((size_t)ng * split + i) * 2 + 1]; }
    const double mean = s * inv_count;
    double var = q * inv_count - mean * mean;
    var = var > 0.0 ? var : 0.0;
    stats[(size_t)ng * 2 + 0] = (float)mean;
    stats[(size_t)ng * 2 + 1] = (float)(1.0 / sqrt(var + (double)eps));
}

hipError_t launch_groupnorm_stats(const void* x, float* stats, int N, int C, int H, int W, int groups, float eps,
                                  int dt, bool nhwc, hipStream_t s) {
    const int cpg = C / groups, HW = H * W, total = N * groups;
    const size_t elems = (size_t)cpg * HW;
    const size_t esz = two_byte(dt) ? 2 : 4, epc = 16 / esz;
    // slices are whole numbers of block-wide 16-byte loads (256 lanes x 16 bytes)
    const size_t quantum = 256 * epc;
    int split = (int)((elems + 2 * quantum - 1) / (2 * quantum));
    split = split < 1 ? 1 : (split > kMaxSplit ? kMaxSplit : split);
    size_t per_slice = (elems + split - 1) / split;
    per_slice = (per_slice + quantum - 1) / quantum * quantum;
    double* partial = reinterpret_cast<double*>(reinterpret_cast<unsigned char*>(stats) +
                                                (((size_t)total * 2 * sizeof(float) + 255) / 256) * 256);
    dim3 grid((unsigned)total, (unsigned)split), block(256);
    const bool vec = !nhwc && (elems * esz) % 16 == 0 && (reinterpret_cast<uintptr_t>(x) & 15u) == 0;
    (void)with_dtype(dt, [&](auto* tag) {
        using E = std::remove_pointer_t<decltype(tag)>;
        if (vec)       hipLaunchKernelGGL((groupnorm_partial_vec_kernel<E>), grid, block, 0, s, (const E*)x, partial, elems, split, per_slice);
        else if (nhwc) hipLaunchKernelGGL((groupnorm_partial_kernel<E, true>), grid, block, 0, s, (const E*)x, partial, C, HW, groups, cpg, split, per_slice);
        else           hipLaunchKernelGGL((groupnorm_partial_kernel<E, false>), grid, block, 0, s, (const E*)x, partial, C, HW, groups, cpg, split, per_slice);
        return hipSuccess;
    });
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(groupnorm_finalize_kernel, dim3((unsigned)((total + 63) / 64)), dim3(64), 0, s,
                       (const double*)partial, stats, total, split, 1.0 / (double)elems, eps);
    return hipGetLastError();
}

}  // namespace wino
