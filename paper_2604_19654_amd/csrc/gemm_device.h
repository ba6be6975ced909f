// Device-side helpers shared by the grouped GEMM kernels (forward and backward).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "feplb.h"

namespace feplb {
namespace dev {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) const void gptr_t;
typedef __attribute__((address_space(3))) void lptr_t;

constexpr int XCDS = 8;   // workgroups are dealt round-robin to the 8 XCDs, each with its own L2

// 16-byte-per-lane load from global memory straight into LDS (LDS-DMA): lane l's data lands at
// LDS byte address lds_base + 16*l (lds_base is wave-uniform and travels in M0).  Written as
// inline assembly so that the loads' completion is tracked by the explicit s_waitcnt vmcnt(n)
// of the pipeline below: the compiler's own tracking would wait for ALL outstanding loads
// before any LDS read in a loop, i.e. also for the tiles requested for later steps.
// The address is a wave-uniform base (scalar register pair) plus a 32-bit per-lane byte offset.
__device__ __forceinline__ void load_to_lds_16(const char* base, uint32_t lane_off, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(lane_off), "s"(base), "s"(lds_base)
               : "memory", "m0");
}
__device__ __forceinline__ const char* wave_uniform(const void* p) {
  const uint64_t v = (uint64_t)(uintptr_t)p;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return (const char*)(uintptr_t)(((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ uint32_t lds_offset(const void* p) {
  return (uint32_t)(uintptr_t)p;   // low half of a generic LDS address is the LDS byte offset
}

// per-group matrix pointers passed by value as a kernel argument
struct WeightTable {
  const void* w0[FEPLB_MAX_GROUPS];  // gate (gate_up) or the only matrix of the GEMM
  const void* w1[FEPLB_MAX_GROUPS];  // up (gate_up only)
};

// a * sigmoid(a) with the hardware reciprocal (1 ulp): the result is rounded to bf16 anyway
__device__ __forceinline__ float silu(float a) { return a * __builtin_amdgcn_rcpf(1.0f + __expf(-a)); }

// two floats -> two bf16 (round to nearest even) in one 32-bit word, first argument in the low half
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// bf16 (upper half of an fp32) -> float
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xffff0000u); }

}  // namespace dev
}  // namespace feplb
