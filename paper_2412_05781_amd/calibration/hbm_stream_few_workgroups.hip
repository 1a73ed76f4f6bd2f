// Cold HBM streaming through (a) plain global loads into registers, (b) LDS-DMA loads, at a fixed
// number of workgroups, each wave keeping DEPTH 1-KB loads in flight.  Region 1.5 GB (>> 256 MB cache).
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdint>
typedef __attribute__((address_space(3))) unsigned char lds_byte_t;
template <int N> __device__ __forceinline__ void wait_vmcnt() { asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory"); }

template <int MODE, int DEPTH>
__global__ void __launch_bounds__(256) k(const unsigned char* __restrict__ buf, size_t per_wg, uint4* out) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const unsigned char* base = buf + (size_t)blockIdx.x * per_wg + (size_t)wave * 1024 + lane * 16;
    const int steps = (int)(per_wg / 4096);          // each step: 4 waves x 1 KB
    uint4 acc = make_uint4(0, 0, 0, 0);
    if (MODE == 0) {
        uint4 r[DEPTH];
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) if (d < steps) r[d] = *reinterpret_cast<const uint4*>(base + (size_t)d * 4096);
        for (int s = 0; s < steps; s += DEPTH) {
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) {
                const uint4 v = r[d];
                if (s + DEPTH + d < steps) r[d] = *reinterpret_cast<const uint4*>(base + (size_t)(s + DEPTH + d) * 4096);
                acc.x ^= v.x; acc.y ^= v.y; acc.z ^= v.z; acc.w ^= v.w;
            }
        }
    } else {
        unsigned char* slot = lds + wave * (DEPTH * 1024);
        auto dma = [&](int s) {
            const uint32_t m0v = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_byte_t*)(slot + (s % DEPTH) * 1024));
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" :: "s"(m0v), "v"(base + (size_t)s * 4096) : "memory");
        };
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) if (d < steps) dma(d);
        for (int s = 0; s < steps; ++s) {
            if (s + DEPTH <= steps) wait_vmcnt<DEPTH - 1>(); else wait_vmcnt<0>();
            if (s + DEPTH < steps) dma(s + DEPTH);
        }
        acc = *reinterpret_cast<uint4*>(slot + lane * 16);
    }
    if (acc.x == 0x12345678u && acc.y == 77u) out[0] = acc;
}

int main() {
    const size_t SZ = (size_t)3 << 29;   // 1.5 GB
    unsigned char* buf; uint4* out; hipMalloc(&buf, SZ); hipMalloc(&out, 64); hipMemset(buf, 1, SZ);
    hipEvent_t e0, e1; hipEventCreate(&e0); hipEventCreate(&e1);
    for (int wgs : {160, 256, 512, 1024, 2048}) {
        const size_t per_wg = (SZ / wgs) & ~(size_t)4095;
        for (int mode = 0; mode < 2; ++mode) for (int depth : {4, 16}) {
            float best = 1e9;
            for (int rep = 0; rep < 3; ++rep) {
                hipEventRecord(e0);
                if (mode == 0 && depth == 4) hipLaunchKernelGGL((k<0, 4>), dim3(wgs), dim3(256), 0, 0, buf, per_wg, out);
                if (mode == 0 && depth == 16) hipLaunchKernelGGL((k<0, 16>), dim3(wgs), dim3(256), 0, 0, buf, per_wg, out);
                if (mode == 1 && depth == 4) hipLaunchKernelGGL((k<1, 4>), dim3(wgs), dim3(256), 4 * 4 * 1024, 0, buf, per_wg, out);
                if (mode == 1 && depth == 16) hipLaunchKernelGGL((k<1, 16>), dim3(wgs), dim3(256), 4 * 16 * 1024, 0, buf, per_wg, out);
                hipEventRecord(e1); hipEventSynchronize(e1);
                float ms; hipEventElapsedTime(&ms, e0, e1); if (ms < best) best = ms;
            }
            printf("wgs %5d mode %s depth %2d: %8.1f us %6.2f TB/s\n", wgs, mode ? "lds-dma" : "regs   ", depth, best * 1e3, (double)per_wg * wgs / (best * 1e-3) / 1e12);
            fflush(stdout);
        }
    }
    return 0;
}
