// Device helpers shared by the bf16 MFMA attention kernels (gfx950 only): vector types, the fence-free barrier, the
// hand-tracked direct-to-LDS tile loads and the cross-half maximum.  Internal: not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dr {
namespace mfma {

typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef __bf16 v4bf __attribute__((ext_vector_type(4)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
typedef short v4s __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));

// log2(e) / sqrt(128): the factor that turns a d = 128 dot product into an exponent of 2.
constexpr float kExpScale = (float)(1.4426950408889634 / 11.313708498984760);
// The fast pass multiplies Q by kExpScale and rounds the product to bf16 again: a logit error that grows with
// |logit| (about |logit| * 2^-9 per channel, random in sign).  Rows whose largest exponent, in units of log2, is
// beyond this limit in magnitude (44 in natural units) are taken again with the scale applied in fp32.
constexpr float kExactLimit = 64.0f;

// The barrier carries no memory fence on purpose: a fence would drain the prefetch of the next
// chunk.  Ordering of the direct-to-LDS loads is enforced by the explicit vmcnt waits.
#define DR_BARRIER() asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory")
#define DR_WAIT_VMCNT0() asm volatile("s_waitcnt vmcnt(0)" ::: "memory")

// 16 bytes per lane from (base + voff) straight into LDS at m0_base + 16 * lane.  Issued through inline
// assembly so that the compiler's wait-count insertion does not see an LDS write it cannot disambiguate
// (it would drain the prefetch before every LDS read); completion is tracked by hand with vmcnt waits.
// m0 is named as clobbered: the compiler must not carry a value of its own in it across a tile load.
__device__ __forceinline__ void dma16(uint32_t voff, uint64_t base, uint32_t m0_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(voff), "s"(base), "s"(m0_base) : "memory", "m0");
}
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}
__device__ __forceinline__ uint64_t uniform64(uint64_t x) {
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)x);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(x >> 32));
    return ((uint64_t)hi << 32) | lo;
}
// max of a value with its copy in the lane 32 away (v_permlane32_swap: no LDS round trip)
__device__ __forceinline__ float max_across_halves(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

}  // namespace mfma
}  // namespace dr
