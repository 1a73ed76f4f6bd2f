// Fill bandwidth of a compute unit from L1, from L2 and from beyond, for the two ways the kernels fetch operands: ordinary
// 16-byte loads into registers and direct-to-LDS transfers (global_load_lds_dwordx4).  No address arithmetic in the loop beyond
// an add and a mask.  Each workgroup walks a window of WIN bytes (a power of two) repeatedly; the windows are private and
// L1-sized, private and L2-sized (all windows of an XCD fit its 4 MB), one window shared by every workgroup, or private and
// far larger than the caches.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdint>
typedef __attribute__((address_space(3))) unsigned char lds_byte_t;
__device__ __forceinline__ void dma16(const void* src, unsigned char* lds_dst) {
    const uint32_t m0v = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_byte_t*)lds_dst);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" :: "s"(m0v), "v"(src) : "memory", "m0");
}
// MODE 0: plain 16B/lane to registers; 1: LDS-DMA 16B/lane; 3: both, alternating (half of the bytes each way)
// PAT 0: wave reads 1 KB contiguous; 1: 8 rows of 128 B at 640 B pitch
template <int MODE, int PAT>
__global__ void __launch_bounds__(256) k(const unsigned char* __restrict__ buf, unsigned win_mask, int iters, size_t wg_stride, uint4* out) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const unsigned char* base = buf + (size_t)blockIdx.x * wg_stride;
    unsigned off;
    if (PAT == 0) off = wave * 1024 + lane * 16;
    else off = wave * 8 * 640 + (lane >> 3) * 640 + (lane & 7) * 16;
    const unsigned step = PAT == 0 ? 4096 : 4 * 8 * 640;
    uint4 acc = make_uint4(0, 0, 0, 0);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const unsigned char* p = base + (off & win_mask);
            if (MODE == 0) { uint4 v = *reinterpret_cast<const uint4*>(p); acc.x ^= v.x; acc.y ^= v.y; acc.z ^= v.z; acc.w ^= v.w; }
            else if (MODE == 3 && (u & 1)) { uint4 v = *reinterpret_cast<const uint4*>(p); acc.x ^= v.x; acc.y ^= v.y; acc.z ^= v.z; acc.w ^= v.w; }
            else dma16(p, lds + (wave * 8 + u) * 1024);
            off += step;
        }
        if (MODE == 1) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        if (MODE == 3) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    }
    if (MODE == 1 || MODE == 3) { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); __syncthreads(); uint4 t = *reinterpret_cast<uint4*>(lds + tid * 16); acc.x ^= t.x; acc.y ^= t.y; }
    if (acc.x == 0x12345678u && acc.y == 77u) out[0] = acc;
}
template <int MODE, int PAT>
void run(const char* name, const unsigned char* buf, uint4* out, int blocks, unsigned win, size_t wg_stride) {
    const int iters = 512;
    hipEvent_t e0, e1; hipEventCreate(&e0); hipEventCreate(&e1);
    float best = 1e9;
    for (int rep = 0; rep < 4; ++rep) {
        hipEventRecord(e0);
        hipLaunchKernelGGL((k<MODE, PAT>), dim3(blocks), dim3(256), 32768, 0, buf, win - 1, iters, wg_stride, out);
        hipEventRecord(e1); hipEventSynchronize(e1);
        float ms; hipEventElapsedTime(&ms, e0, e1); if (ms < best) best = ms;
    }
    const double bytes = (double)blocks * iters * 8 * 4 * 1024.0;
    printf("%-34s blocks %5d window %4u KB stride %5zu KB: %8.1f us  %6.2f TB/s  %5.1f B/clk/CU@2.4GHz\n", name, blocks, win >> 10, wg_stride >> 10,
           best * 1e3, bytes / (best * 1e-3) / 1e12, bytes / (best * 1e-3) / 256 / 2.4e9);
    fflush(stdout);
}
int main() {
    unsigned char* buf; uint4* out; const size_t SZ = (1024u << 20) + (4u << 20);
    hipMalloc(&buf, SZ); hipMalloc(&out, 64); hipMemset(buf, 1, SZ);
    for (int blocks : {256, 512, 1024, 2048}) {
        // L1-resident (16 KB window per workgroup), L2-resident private windows (64 KB each; all windows of an XCD fit its 4 MB),
        // shared window (every workgroup reads the same 1 MB: L2 hits, fetched once), far (private 1 MB windows: MALL / HBM)
        for (int cfg = 0; cfg < 4; ++cfg) {
            const unsigned win = cfg == 0 ? 16u << 10 : (cfg == 1 ? 64u << 10 : 1u << 20);
            const size_t stride = cfg == 0 ? (16u << 10) : (cfg == 1 ? (64u << 10) : (cfg == 2 ? 0 : (size_t)((1u << 20) / (blocks > 1024 ? 2 : 1))));
            const char* tag = cfg == 0 ? "L1 16K" : (cfg == 1 ? "L2 private 64K" : (cfg == 2 ? "L2 shared 1M" : "far private"));
            char nm[96];
            snprintf(nm, sizeof nm, "plain16 contiguous  %s", tag); run<0, 0>(nm, buf, out, blocks, win, stride);
            snprintf(nm, sizeof nm, "dma16   contiguous  %s", tag); run<1, 0>(nm, buf, out, blocks, win, stride);
            snprintf(nm, sizeof nm, "dma16   128B rows   %s", tag); run<1, 1>(nm, buf, out, blocks, win, stride);
            snprintf(nm, sizeof nm, "both    contiguous  %s", tag); run<3, 0>(nm, buf, out, blocks, win, stride);
        }
    }
    return 0;
}
