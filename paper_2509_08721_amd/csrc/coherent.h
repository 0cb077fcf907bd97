// Loads and stores for data that workgroups of ONE launch hand to each other (gfx950).  Workgroups of a launch may run
// on different XCDs whose L2s do not see each other's lines inside a kernel: what another workgroup will read is
// stored write-through (sc0 sc1), what another workgroup wrote is loaded past the L2 (sc0 sc1), and nothing is
// invalidated or written back wholesale (an L2 invalidate costs more than a decode step).  These are buffer
// instructions with the cache-policy operand set (the compiler keeps its usual count of them).  COH = false gives the
// plain access (a kernel boundary makes a producer's stores visible to its consumer).
#pragma once
#include "common.h"

namespace sapo {

typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------------------
// memory access with or without the coherence bits: (buffer base, byte offset below 2 GiB)
// ---------------------------------------------------------------------------------------
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
constexpr int kCohPolicy = 17;   // sc0 | sc1 of a buffer instruction's cache policy operand

__device__ __forceinline__ __amdgpu_buffer_rsrc_t coh_rsrc(const void* base) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, 0x7fffffff, 0x00020000);
}
template <bool COH> __device__ __forceinline__ u32x4 ld_u4(const void* base, size_t off) {
  if (COH) return __builtin_amdgcn_raw_buffer_load_b128(coh_rsrc(base), (int)off, 0, kCohPolicy);
  return *(const u32x4*)((const char*)base + off);
}
template <bool COH> __device__ __forceinline__ float ld_f32(const void* base, size_t off) {
  if (COH) return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(coh_rsrc(base), (int)off, 0, kCohPolicy));
  return *(const float*)((const char*)base + off);
}
template <bool COH> __device__ __forceinline__ void st_u4(void* base, size_t off, u32x4 v) {
  if (COH) __builtin_amdgcn_raw_buffer_store_b128(v, coh_rsrc(base), (int)off, 0, kCohPolicy);
  else *(u32x4*)((char*)base + off) = v;
}
template <bool COH> __device__ __forceinline__ void st_f4(void* base, size_t off, float4 v) {
  const u32x4 u = {__float_as_uint(v.x), __float_as_uint(v.y), __float_as_uint(v.z), __float_as_uint(v.w)};
  st_u4<COH>(base, off, u);
}
template <bool COH> __device__ __forceinline__ void st_h4(void* base, size_t off, f16x4 v) {
  if (COH) {
    union { f16x4 h; u32x2 u; } c;
    c.h = v;
    __builtin_amdgcn_raw_buffer_store_b64(c.u, coh_rsrc(base), (int)off, 0, kCohPolicy);
  } else {
    *(f16x4*)((char*)base + off) = v;
  }
}
template <bool COH> __device__ __forceinline__ void st_f32(void* base, size_t off, float v) {
  if (COH) __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), coh_rsrc(base), (int)off, 0, kCohPolicy);
  else *(float*)((char*)base + off) = v;
}
__device__ __forceinline__ float4 as_f4(const u32x4& u) {
  return make_float4(__uint_as_float(u[0]), __uint_as_float(u[1]), __uint_as_float(u[2]), __uint_as_float(u[3]));
}
// every load and store issued so far has completed (a producer calls this before it reports its output as written)
__device__ __forceinline__ void coh_drain() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

}  // namespace sapo
