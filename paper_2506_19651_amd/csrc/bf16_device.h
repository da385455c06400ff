// Device helpers shared by the bf16 MFMA attention kernels (gfx950).
#pragma once
#include "common.h"

namespace pevlm {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T *)(p))

// 16-byte-per-lane load from global memory straight into LDS (no register staging).  The LDS
// destination of lane i is lds_addr + 16 i; lds_addr must be wavefront-uniform.  Issued through
// inline assembly so that the tile being consumed can be read while the next one is in flight: the
// wait for completion is the explicit vmcnt(0) at the top of the tile loop.
__device__ __forceinline__ void load_lds_16(const void *gptr, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off\n" ::"s"(lds_addr), "v"(gptr) : "memory");
}

__device__ __forceinline__ float max3f(float a, float b, float c)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// Same, with a wavefront-uniform 64-bit base address and a per-lane 32-bit byte offset.
__device__ __forceinline__ void load_lds_16_base(const void *sbase, uint32_t voff, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2\n" ::"s"(lds_addr), "v"(voff), "s"(sbase) : "memory");
}

// Marks a pointer that is the same in every lane as wavefront-uniform (scalar registers).
template <typename T>
__device__ __forceinline__ const T *uniform_ptr(const T *p)
{
    const uint64_t v = (uint64_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (const T *)(((uint64_t)hi << 32) | lo);
}

}  // namespace pevlm
