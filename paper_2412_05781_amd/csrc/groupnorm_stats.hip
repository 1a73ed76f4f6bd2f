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
    __shared__ double ss[256], qq[256];
    ss[threadIdx.x] = (double)s; qq[threadIdx.x] = (double)q;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) { ss[threadIdx.x] += ss[threadIdx.x + w]; qq[threadIdx.x] += qq[threadIdx.x + w]; }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        partial[((size_t)ng * split + sl) * 2 + 0] = ss[0];
        partial[((size_t)ng * split + sl) * 2 + 1] = qq[0];
    }
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
                                  bool f16, bool nhwc, hipStream_t s) {
    const int cpg = C / groups, HW = H * W, total = N * groups;
    const size_t elems = (size_t)cpg * HW;
    int split = (int)((elems + 16383) / 16384);
    split = split < 1 ? 1 : (split > kMaxSplit ? kMaxSplit : split);
    const size_t per_slice = (elems + split - 1) / split;
    double* partial = reinterpret_cast<double*>(reinterpret_cast<unsigned char*>(stats) +
                                                (((size_t)total * 2 * sizeof(float) + 255) / 256) * 256);
    dim3 grid((unsigned)total, (unsigned)split), block(256);
    if (f16) {
        if (nhwc) hipLaunchKernelGGL((groupnorm_partial_kernel<__half, true>), grid, block, 0, s, (const __half*)x, partial, C, HW, groups, cpg, split, per_slice);
        else      hipLaunchKernelGGL((groupnorm_partial_kernel<__half, false>), grid, block, 0, s, (const __half*)x, partial, C, HW, groups, cpg, split, per_slice);
    } else {
        if (nhwc) hipLaunchKernelGGL((groupnorm_partial_kernel<float, true>), grid, block, 0, s, (const float*)x, partial, C, HW, groups, cpg, split, per_slice);
        else      hipLaunchKernelGGL((groupnorm_partial_kernel<float, false>), grid, block, 0, s, (const float*)x, partial, C, HW, groups, cpg, split, per_slice);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(groupnorm_finalize_kernel, dim3((unsigned)((total + 63) / 64)), dim3(64), 0, s,
                       (const double*)partial, stats, total, split, 1.0 / (double)elems, eps);
    return hipGetLastError();
}

}  // namespace wino
