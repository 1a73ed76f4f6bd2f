// Streaming a [rows][pitch] matrix from HBM the way the step (ii) kernel reads the transformed filter: a workgroup owns a
// panel of 128 rows and walks along the rows in stages of SW bytes per row (direct-to-LDS transfers, 16 bytes per lane), a ring
// of NST stages, with the kernel's XOR permutation of the 16-byte chunks inside a row or without it.  Compared with the same
// bytes read as one contiguous run per workgroup.  Footprints of 419 MB come from HBM; the 52-210 MB runs fit the 256 MB
// memory-side cache after the first repetition and show its rate instead.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdint>
typedef __attribute__((address_space(3))) unsigned char lds_byte_t;
__device__ __forceinline__ void dma16(const void* src, unsigned char* lds_dst) {
    const uint32_t m0v = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_byte_t*)lds_dst);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" :: "s"(m0v), "v"(src) : "memory", "m0");
}
// SW: bytes per row per stage (128, 256, 512); panel = 128 rows; 4 waves; a stage = 128*SW bytes = SW/8 loads per wave... (128*SW/1024/4)
template <int SW, int NST, bool CONTIG, bool SWZ = false>
__global__ void __launch_bounds__(256) k(const unsigned char* __restrict__ buf, int pitch, int panels_per_wg, uint4* out) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    constexpr int STAGE = 128 * SW;             // bytes per stage
    constexpr int LPW = STAGE / 1024 / 4;       // loads per wave per stage
    constexpr int LPR = SW / 16;                // lanes per row
    constexpr int RPL = 64 / LPR;               // rows per load
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nstage = pitch / SW;
    for (int p = 0; p < panels_per_wg; ++p) {
        const size_t panel = (size_t)blockIdx.x * panels_per_wg + p;
        const unsigned char* base = buf + panel * 128 * (size_t)pitch;
        auto issue = [&](int s) {
#pragma unroll
            for (int i = 0; i < LPW; ++i) {
                const unsigned char* src;
                if (CONTIG) src = base + (size_t)s * STAGE + (size_t)((wave * LPW + i) * 1024 + lane * 16);
                else { const int row = (wave * LPW + i) * RPL + lane / LPR; const int ch = SWZ ? ((lane % LPR) ^ ((row >> 1) & (LPR - 1))) : (lane % LPR); src = base + (size_t)row * pitch + (size_t)s * SW + ch * 16; }
                dma16(src, lds + (s % NST) * STAGE + (wave * LPW + i) * 1024);
            }
        };
        for (int s = 0; s < NST - 1 && s < nstage; ++s) issue(s);
        for (int s = 0; s < nstage; ++s) {
            if (s + NST - 1 < nstage) { issue(s + NST - 1); asm volatile("s_waitcnt vmcnt(%0)" :: "n"(LPW * (NST - 1)) : "memory"); }
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
        }
    }
    uint4 acc = *reinterpret_cast<uint4*>(lds + tid * 16);
    if (acc.x == 0x12345678u && acc.y == 77u) out[0] = acc;
}
template <int SW, int NST, bool CONTIG, bool SWZ = false>
void run(const unsigned char* buf, uint4* out, int blocks, int pitch, int ppw) {
    hipEvent_t e0, e1; hipEventCreate(&e0); hipEventCreate(&e1);
    float best = 1e9;
    const int lds = 128 * SW * NST;
    hipFuncSetAttribute(reinterpret_cast<const void*>(k<SW, NST, CONTIG, SWZ>), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    for (int rep = 0; rep < 4; ++rep) {
        hipEventRecord(e0);
        hipLaunchKernelGGL((k<SW, NST, CONTIG, SWZ>), dim3(blocks), dim3(256), lds, 0, buf, pitch, ppw, out);
        hipEventRecord(e1); hipEventSynchronize(e1);
        float ms; hipEventElapsedTime(&ms, e0, e1); if (ms < best) best = ms;
    }
    const double bytes = (double)blocks * ppw * 128.0 * pitch;
    printf("%s%s stage %3d B/row ring %d blocks %4d pitch %5d panels/wg %d: %7.1f us %6.2f TB/s (%.0f MB)\n", CONTIG ? "contiguous" : "row-walk  ", SWZ ? " swizzled" : "         ", SW, NST, blocks, pitch, ppw,
           best * 1e3, bytes / (best * 1e-3) / 1e12, bytes / 1e6);
    fflush(stdout);
}
// One launch over `bytes` of a 1 GB buffer, the region advancing with every launch so that each launch reads from HBM:
// what a single short kernel (the weight-streaming layers read 52-105 MB per launch) can reach, start-up and drain included.
template <int SW, int NST>
void run_cold(const unsigned char* buf, uint4* out, int blocks, int pitch) {
    hipEvent_t e0, e1; hipEventCreate(&e0); hipEventCreate(&e1);
    const int lds = 128 * SW * NST;
    hipFuncSetAttribute(reinterpret_cast<const void*>(k<SW, NST, false, true>), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    const size_t region = (size_t)blocks * 128 * pitch;
    const int nreg = (int)(((size_t)1 << 30) / region);
    const int launches = 2 * nreg;
    hipLaunchKernelGGL((k<SW, NST, false, true>), dim3(blocks), dim3(256), lds, 0, buf, pitch, 1, out);
    hipDeviceSynchronize();
    hipEventRecord(e0);
    for (int i = 0; i < launches; ++i)
        hipLaunchKernelGGL((k<SW, NST, false, true>), dim3(blocks), dim3(256), lds, 0, buf + (size_t)(i % nreg) * region, pitch, 1, out);
    hipEventRecord(e1); hipEventSynchronize(e1);
    float ms; hipEventElapsedTime(&ms, e0, e1);
    const double us = ms * 1e3 / launches;
    printf("cold single launch, row-walk swizzled stage %3d B/row ring %d blocks %4d pitch %5d: %7.1f us per launch %6.2f TB/s (%.0f MB per launch, %d regions)\n",
           SW, NST, blocks, pitch, us, region / (us * 1e-6) / 1e12, region / 1e6, nreg);
    fflush(stdout);
}
int main() {
    unsigned char* buf; uint4* out; const size_t SZ = (size_t)1 << 30;
    hipMalloc(&buf, SZ); hipMalloc(&out, 64); hipMemset(buf, 1, SZ);
    // footprint 419 MB (> 256 MB memory-side cache): e.g. 640 panels of 128 rows x 5120 B
    for (int pitch : {2560, 5120}) {
        for (int blocks : {160, 320, 640}) {
            const int ppw = (int)((400u << 20) / ((size_t)blocks * 128 * pitch));
            run<128, 3, false>(buf, out, blocks, pitch, ppw);
            run<128, 3, false, true>(buf, out, blocks, pitch, ppw);
            run<128, 3, true>(buf, out, blocks, pitch, ppw);
            if (ppw > 1) { run<128, 3, false>(buf, out, blocks, pitch, 1); run<128, 3, false, true>(buf, out, blocks, pitch, 1); }
        }
    }
    for (int pitch : {2560, 5120})
        for (int blocks : {160, 320, 480}) {
            run_cold<128, 3>(buf, out, blocks, pitch);
            run_cold<256, 3>(buf, out, blocks, pitch);
        }
    return 0;
}
