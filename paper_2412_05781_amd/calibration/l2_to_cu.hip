// microbenchmark: per-CU bandwidth from L2 (hot) with (a) plain 16B loads, (b) LDS-DMA 16B loads
#include <hip/hip_runtime.h>
#include <cstdio>
typedef __attribute__((address_space(3))) unsigned char lds_byte_t;
__device__ __forceinline__ void dma16(const void* src, unsigned char* lds_dst) {
    const uint32_t m0v = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_byte_t*)lds_dst);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" :: "s"(m0v), "v"(src) : "memory");
}
// each WG streams over `span` bytes starting at a WG-dependent offset inside a region of `region` bytes, `iters` times
template <int MODE, int ROWB>
__global__ void __launch_bounds__(256) k(const unsigned char* __restrict__ buf, size_t region, size_t span, int iters, uint4* out) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const size_t base = ((size_t)blockIdx.x * 65536) % region;
    uint4 acc = make_uint4(0, 0, 0, 0);
    // row-structured access like the GEMM: a wave-load covers 1024/ROWB rows of ROWB bytes, rows 640 B... use pitch
    const size_t pitch = 1024;   // bytes between rows
    const int rpl = 1024 / ROWB;
    const int lrow = lane / (ROWB / 16), lch = lane % (ROWB / 16);
    for (int it = 0; it < iters; ++it) {
        for (size_t off = 0; off < span; off += 4 * 8 * rpl * pitch) {
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const size_t row = (size_t)(wave * 8 + u) * rpl + lrow;
                const size_t a = (base + off + row * pitch + lch * 16 + (it & 7) * ROWB) % region;
                if (MODE == 0) { uint4 v = *reinterpret_cast<const uint4*>(buf + a); acc.x ^= v.x; acc.y ^= v.y; acc.z ^= v.z; acc.w ^= v.w; }
                else dma16(buf + a, lds + (wave * 8 + u) * 1024);
            }
        }
    }
    if (MODE == 1) { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); __syncthreads(); acc = *reinterpret_cast<uint4*>(lds + tid * 16); }
    if (acc.x == 0x12345678u && acc.y == 77u) out[0] = acc;
}
template <int MODE, int ROWB>
void run(const char* name, const unsigned char* buf, size_t region, uint4* out, int blocks) {
    const size_t span = 1 << 20; const int iters = 16;
    hipEvent_t e0, e1; hipEventCreate(&e0); hipEventCreate(&e1);
    float best = 1e9;
    for (int rep = 0; rep < 4; ++rep) {
        hipEventRecord(e0);
        hipLaunchKernelGGL((k<MODE, ROWB>), dim3(blocks), dim3(256), 32768, 0, buf, region, span, iters, out);
        hipEventRecord(e1); hipEventSynchronize(e1);
        float ms; hipEventElapsedTime(&ms, e0, e1); if (ms < best) best = ms;
    }
    // bytes actually loaded per WG: per off-step 4 waves * 8 loads * 1KB = 32 KB; steps = span / (32*rpl*pitch)
    const int rpl = 1024 / ROWB;
    const double steps = (double)span / (4.0 * 8 * rpl * 1024);
    const double bytes = (double)blocks * iters * steps * 32768.0;
    printf("%-28s region %4zu MB blocks %5d: %8.1f us  %6.2f TB/s  %5.1f B/clk/CU@2.4GHz\n", name, region >> 20, blocks, best * 1e3,
           bytes / (best * 1e-3) / 1e12, bytes / (best * 1e-3) / 256 / 2.4e9);
}
int main() {
    unsigned char* buf; uint4* out; const size_t SZ = 512u << 20;
    hipMalloc(&buf, SZ); hipMalloc(&out, 64); hipMemset(buf, 1, SZ);
    for (size_t region : {(size_t)2 << 20, (size_t)16 << 20, (size_t)128 << 20}) {
        for (int blocks : {256, 512, 1024, 2048}) {
            run<0, 128>("plain 16B, 128B rows", buf, region, out, blocks);
            run<1, 128>("dma 16B, 128B rows", buf, region, out, blocks);
            run<0, 64>("plain 16B, 64B rows", buf, region, out, blocks);
            run<1, 64>("dma 16B, 64B rows", buf, region, out, blocks);
        }
    }
    return 0;
}
