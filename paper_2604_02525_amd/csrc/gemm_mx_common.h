// Device helpers shared by the block-scaled FP4 GEMM kernels (gfx950): matrix-core wrappers, the
// global -> LDS copy instruction, and the scheduling pin.
#pragma once
#include "common.h"

namespace adahop {

namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

__device__ __forceinline__ v16f mfma_fp4(uint4 a, uint4 b, v16f c, int sa, int sb)
{
    v8i av = {(int)a.x, (int)a.y, (int)a.z, (int)a.w, 0, 0, 0, 0};
    v8i bv = {(int)b.x, (int)b.y, (int)b.z, (int)b.w, 0, 0, 0, 0};
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av, bv, c, 4, 4, 0, sa, 0, sb);
}

__device__ __forceinline__ v16f mfma_bf16(uint4 a, uint4 b, v16f c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b), c, 0, 0, 0);
}

// Copies from global memory straight into LDS: lane i's 16 bytes, read at base + voff, land at
// lds_addr + 16 i (base and lds_addr wave-uniform, voff a 32-bit per-lane byte offset).  Inline
// assembly on purpose: with the builtin the compiler's wait-count pass makes every later LDS read
// wait for ALL outstanding copies (it cannot tell that they target the other stage), which
// serialises the copies with the matrix-core work.  The kernel waits for the copies itself
// (s_waitcnt vmcnt(0) before the stage barrier).  M0 is written here (and declared clobbered) and used
// by nothing else in these kernels (no dynamic register indexing, no other DMA).
__device__ __forceinline__ const uint8_t *uniform_ptr(const uint8_t *p)
{
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const uint8_t *>(((uint64_t)hi << 32) | lo);
}

__device__ __forceinline__ void dma16(const uint8_t *base, uint32_t voff, uint32_t lds_addr)
{
    // Both are wave-uniform by construction; reading them through the first lane makes sure they sit
    // in scalar registers, which the instruction requires, whatever the register allocator did.
    base = uniform_ptr(base);
    lds_addr = __builtin_amdgcn_readfirstlane(lds_addr);
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(voff), "s"(base), "s"(lds_addr)
                 : "memory", "m0");
}

__device__ __forceinline__ uint32_t lds_address(const void *p)
{
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void *)p;
}

// Keeps the instruction scheduler from moving anything across this point (one wave per SIMD: the
// order written here is what hides the LDS and copy-issue latency behind the matrix cores).
#define ADAHOP_PIN() __builtin_amdgcn_sched_barrier(0)

} // namespace

} // namespace adahop
