// calibration: plain read / write / copy kernels, grid-stride with 16-byte accesses
#include <hip/hip_runtime.h>
#include <cstdio>
#include <vector>
__global__ void k_copy(const uint4* __restrict__ a, uint4* __restrict__ b, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) b[i] = a[i];
}
__global__ void k_read(const uint4* __restrict__ a, uint4* __restrict__ b, size_t n) {
    uint4 acc = make_uint4(0,0,0,0);
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) { uint4 v = a[i]; acc.x ^= v.x; acc.y ^= v.y; acc.z ^= v.z; acc.w ^= v.w; }
    if (acc.x == 0x12345678u && acc.y == 0x9abcdef0u) b[0] = acc;
}
__global__ void k_write(uint4* __restrict__ b, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) b[i] = make_uint4(1,2,3,4);
}
__global__ void k_empty() {}
int main() {
    const size_t MAXB = 512u << 20;
    uint4 *a, *b; hipMalloc(&a, MAXB); hipMalloc(&b, MAXB);
    hipMemset(a, 1, MAXB); hipMemset(b, 0, MAXB);
    hipEvent_t e0, e1; hipEventCreate(&e0); hipEventCreate(&e1);
    size_t sizes[] = {5u<<20, 12u<<20, 24u<<20, 48u<<20, 96u<<20, 384u<<20};
    for (size_t sz : sizes) {
        size_t n = sz / 16;
        int blocks = (int)((n + 255) / 256); if (blocks > 256 * 16) blocks = 256 * 16;
        for (int mode = 0; mode < 3; ++mode) {
            float best = 1e9;
            for (int rep = 0; rep < 6; ++rep) {
                hipEventRecord(e0);
                for (int it = 0; it < 20; ++it) {
                    if (mode == 0) hipLaunchKernelGGL(k_read, dim3(blocks), dim3(256), 0, 0, a, b, n);
                    else if (mode == 1) hipLaunchKernelGGL(k_write, dim3(blocks), dim3(256), 0, 0, b, n);
                    else hipLaunchKernelGGL(k_copy, dim3(blocks), dim3(256), 0, 0, a, b, n);
                }
                hipEventRecord(e1); hipEventSynchronize(e1);
                float ms; hipEventElapsedTime(&ms, e0, e1); if (ms / 20 < best) best = ms / 20;
            }
            const char* nm[] = {"read", "write", "copy"};
            double bytes = (mode == 2 ? 2.0 : 1.0) * sz;
            printf("%5zu MB %-5s %8.2f us  %7.2f TB/s\n", sz >> 20, nm[mode], best * 1e3, bytes / (best * 1e-3) / 1e12);
        }
    }
    float best = 1e9;
    for (int rep = 0; rep < 5; ++rep) { hipEventRecord(e0); for (int it = 0; it < 100; ++it) hipLaunchKernelGGL(k_empty, dim3(256), dim3(256), 0, 0); hipEventRecord(e1); hipEventSynchronize(e1); float ms; hipEventElapsedTime(&ms, e0, e1); if (ms/100 < best) best = ms/100; }
    printf("empty kernel back-to-back: %.2f us\n", best * 1e3);
    return 0;
}
