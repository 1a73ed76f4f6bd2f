// Device helpers shared by the kernels that feed the MFMA units from LDS: the 32x32 MFMA step per
// storage type, the explicit vmcnt wait, and the global -> LDS transfer.
#ifndef WINO_MMA_H
#define WINO_MMA_H
#include "wino_internal.h"

namespace wino {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));      // a 16-byte fragment as a native vector (inline-asm operand)
typedef float f32x4_t __attribute__((ext_vector_type(4)));

typedef int int16v_t __attribute__((ext_vector_type(16)));
typedef int int4v_t __attribute__((ext_vector_type(4)));

// acc_t: the sixteen accumulator registers of one 32x32 tile (fp32; int32 for 8-bit integer operands)
template <typename E> struct Mma;
template <> struct Mma<__half> {
    using acc_t = float16_t;
    // one 16-byte chunk = 8 reduction elements; lanes 0-31 and 32-63 hold different chunks
    static __device__ __forceinline__ void run(const uint4& a, const uint4& b, float16_t& c) {
        c = __builtin_amdgcn_mfma_f32_32x32x16_f16(*reinterpret_cast<const half8_t*>(&a),
                                                    *reinterpret_cast<const half8_t*>(&b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ void run(const u32x4_t& a, const u32x4_t& b, float16_t& c) {
        c = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, a), __builtin_bit_cast(half8_t, b), c, 0, 0, 0);
    }
};
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
template <> struct Mma<bf16_t> {
    using acc_t = float16_t;
    static __device__ __forceinline__ void run(const uint4& a, const uint4& b, float16_t& c) {
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8_t*>(&a),
                                                     *reinterpret_cast<const bf16x8_t*>(&b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ void run(const u32x4_t& a, const u32x4_t& b, float16_t& c) {
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    }
};
template <> struct Mma<float> {
    using acc_t = float16_t;
    static __device__ __forceinline__ void run(const uint4& a, const uint4& b, float16_t& c) {
        const float* fa = reinterpret_cast<const float*>(&a);
        const float* fb = reinterpret_cast<const float*>(&b);
#pragma unroll
        for (int j = 0; j < 4; ++j) c = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[j], fb[j], c, 0, 0, 0);
    }
    static __device__ __forceinline__ void run(const u32x4_t& a, const u32x4_t& b, float16_t& c) {
        const f32x4_t fa = __builtin_bit_cast(f32x4_t, a), fb = __builtin_bit_cast(f32x4_t, b);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(fa.x, fb.x, c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(fa.y, fb.y, c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(fa.z, fb.z, c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(fa.w, fb.w, c, 0, 0, 0);
    }
};

// 8-bit integer operands, exact int32 accumulation: one 16-byte chunk = 16 reduction elements per lane (32 per step)
template <> struct Mma<i8_t> {
    using acc_t = int16v_t;
    static __device__ __forceinline__ void run(const uint4& a, const uint4& b, int16v_t& c) {
        c = __builtin_amdgcn_mfma_i32_32x32x32_i8(*reinterpret_cast<const int4v_t*>(&a), *reinterpret_cast<const int4v_t*>(&b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ void run(const u32x4_t& a, const u32x4_t& b, int16v_t& c) {
        c = __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(int4v_t, a), __builtin_bit_cast(int4v_t, b), c, 0, 0, 0);
    }
};

// 8-bit floating-point operands: one 32x32x64 step takes 32 bytes per lane and operand, i.e. two 16-byte chunks (lanes 0-31
// and 32-63 hold different chunk pairs).  Which byte lands on which k inside the instruction does not matter as
// long as both operands are loaded the same way.  Format selectors 0 = E4M3; scale bytes 0x7f = 2^0.
typedef int int8v_t __attribute__((ext_vector_type(8)));
template <> struct Mma<fp8_t> {
    static __device__ __forceinline__ void run2(const uint4& a0, const uint4& a1, const uint4& b0, const uint4& b1, float16_t& c) {
        int8v_t a, b;
        a[0] = a0.x; a[1] = a0.y; a[2] = a0.z; a[3] = a0.w; a[4] = a1.x; a[5] = a1.y; a[6] = a1.z; a[7] = a1.w;
        b[0] = b0.x; b[1] = b0.y; b[2] = b0.z; b[3] = b0.w; b[4] = b1.x; b[5] = b1.y; b[6] = b1.z; b[7] = b1.w;
        c = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 0, 0, 0x7f7f7f7f, 0, 0x7f7f7f7f);
    }
};
// chunks per lane, operand and MFMA step
template <typename E> struct MmaChunks { static constexpr int value = 1; };
template <> struct MmaChunks<fp8_t> { static constexpr int value = 2; };

template <int N> __device__ __forceinline__ void wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// One wave-wide global -> LDS transfer: lane l's 16 bytes at `src` land at lds_dst + 16*l
// (lds_dst wave-uniform).  Written as inline assembly on purpose: the compiler then does not
// track the transfer and does not drain every outstanding one before each barrier and LDS read;
// the kernel waits with explicit vmcnt values instead (see the reduction loop).
typedef __attribute__((address_space(3))) unsigned char lds_byte_t;
// m0 is set and consumed inside the one asm statement and is named as clobbered, so the compiler
// re-creates any m0 value of its own after it (the clobber reaches the machine code as an implicit
// definition; clang's generic warning about clobbering a reserved register is switched off here).
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void dma_load_1k(const void* src, unsigned char* lds_dst) {
    const uint32_t m0v = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_byte_t*)lds_dst);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :: "s"(m0v), "v"(src) : "memory", "m0");
}
// The same transfer with the global address split into a wave-uniform 64-bit base (scalar registers) and a 32-bit
// byte offset per lane, and the LDS destination given as a wave-uniform LDS byte address: nothing per-lane has to be
// recomputed from stage to stage, the base moves on the scalar unit.
__device__ __forceinline__ void dma_load_1k_s(const void* base, uint32_t lane_off, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_addr), "v"(lane_off), "s"(base) : "memory", "m0");
}
#pragma clang diagnostic pop

// Fragment reads under explicit control.  The read is issued from inline assembly, so the compiler does not track it
// (it would otherwise place its own lgkmcnt waits, and in loops it falls back to waiting for the newest read); the
// kernel waits with lds_wait<N>() and then passes every register the reads wrote through pin(), which ties the
// MFMAs that consume them to a point after the wait.  LDS reads return in order, so lds_wait<N>() guarantees everything
// but the N most recently issued reads.
template <int OFF> __device__ __forceinline__ void lds_read16_async(u32x4_t& dst, uint32_t addr) {
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF));
}
template <int N> __device__ __forceinline__ void lds_wait() {
    asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ void pin(u32x4_t& v) { asm volatile("" : "+v"(v)); }

// compile-time loop: f(std::integral_constant<int, 0>()), ..., f(std::integral_constant<int, N-1>())
template <int N, typename F> __device__ __forceinline__ void static_for(F&& f) {
    if constexpr (N > 0) {
        static_for<N - 1>(f);
        f(std::integral_constant<int, N - 1>());
    }
}

}  // namespace wino
#endif
