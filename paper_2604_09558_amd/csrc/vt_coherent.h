// 16-byte stores and loads that are coherent across the whole device (all compute dies), for
// data that one workgroup hands to another inside a launch.  They carry the same cache
// policy as a device-scope atomic access (written through / read past the per-die caches) but
// move 16 bytes per lane, so a wave transfers whole cache lines instead of 64 separate words.
// The compiler does not see these memory operations: the caller orders them with explicit
// waits (a store is complete after s_waitcnt vmcnt(0); the load helper waits itself).
#pragma once

#include <hip/hip_runtime.h>

namespace vt {

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void store_device_b128(void* p, u32x4_t v) {
  asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(p), "v"(v) : "memory");
}

// Four independent 16-byte loads in flight, then one wait.
__device__ __forceinline__ void load_device_4xb128(const void* p0, const void* p1, const void* p2, const void* p3,
                                                   u32x4_t* v) {
  asm volatile(
      "global_load_dwordx4 %0, %4, off sc1\n\t"
      "global_load_dwordx4 %1, %5, off sc1\n\t"
      "global_load_dwordx4 %2, %6, off sc1\n\t"
      "global_load_dwordx4 %3, %7, off sc1\n\t"
      "s_waitcnt vmcnt(0)"
      : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3])
      : "v"(p0), "v"(p1), "v"(p2), "v"(p3)
      : "memory");
}

// Eight in flight (the split merge of the attention kernel reads eight partial results at once).
__device__ __forceinline__ void load_device_8xb128(const void* const* p, u32x4_t* v) {
  asm volatile(
      "global_load_dwordx4 %0, %8, off sc1\n\t"
      "global_load_dwordx4 %1, %9, off sc1\n\t"
      "global_load_dwordx4 %2, %10, off sc1\n\t"
      "global_load_dwordx4 %3, %11, off sc1\n\t"
      "global_load_dwordx4 %4, %12, off sc1\n\t"
      "global_load_dwordx4 %5, %13, off sc1\n\t"
      "global_load_dwordx4 %6, %14, off sc1\n\t"
      "global_load_dwordx4 %7, %15, off sc1\n\t"
      "s_waitcnt vmcnt(0)"
      : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3]), "=&v"(v[4]), "=&v"(v[5]), "=&v"(v[6]), "=&v"(v[7])
      : "v"(p[0]), "v"(p[1]), "v"(p[2]), "v"(p[3]), "v"(p[4]), "v"(p[5]), "v"(p[6]), "v"(p[7])
      : "memory");
}

}  // namespace vt
