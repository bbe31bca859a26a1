// Kernel arguments reach a wave through the scalar cache, one 64-byte line per miss.  A kernel
// whose prologue walks a large by-value parameter structure (segment tables, axis maps) reads
// those lines in several rounds, each waiting for the one before (data-dependent indices, or
// simply the order in which the values are needed): a chain of cold misses before the first
// useful load can be issued.  The function below asks for one word of each of the first lines of
// the kernel-argument segment at once and waits once, so that the reads that follow hit the scalar
// cache.  Reads only; the values are dropped.  Every word read must lie inside the arguments
// (15 * 64 + 4 <= sizeof(arguments) and also + 68 <= sizeof(arguments)), which the caller asserts.
// All loads and the wait sit in one asm statement: the registers they write are not handed out
// again before the data has arrived.
#pragma once

#include <hip/hip_runtime.h>

namespace vt {

// lines 0..15 (bytes 0..1023) and the two lines from byte `also` (a multiple of 64)
__device__ __forceinline__ void warm_kernarg_16_and_2(uint32_t also) {
  typedef __attribute__((address_space(4))) const char* karg_t;
  const karg_t base = (karg_t)__builtin_amdgcn_kernarg_segment_ptr();
  const uint64_t p = (uint64_t)base, q = (uint64_t)(base + also);
  uint32_t d0, d1, d2, d3, d4, d5, d6, d7, d8, d9, d10, d11, d12, d13, d14, d15, d16, d17;
  asm volatile(
      "s_load_dword %0, %18, 0x0\n\t"
      "s_load_dword %1, %18, 0x40\n\t"
      "s_load_dword %2, %18, 0x80\n\t"
      "s_load_dword %3, %18, 0xc0\n\t"
      "s_load_dword %4, %18, 0x100\n\t"
      "s_load_dword %5, %18, 0x140\n\t"
      "s_load_dword %6, %18, 0x180\n\t"
      "s_load_dword %7, %18, 0x1c0\n\t"
      "s_load_dword %8, %18, 0x200\n\t"
      "s_load_dword %9, %18, 0x240\n\t"
      "s_load_dword %10, %18, 0x280\n\t"
      "s_load_dword %11, %18, 0x2c0\n\t"
      "s_load_dword %12, %18, 0x300\n\t"
      "s_load_dword %13, %18, 0x340\n\t"
      "s_load_dword %14, %18, 0x380\n\t"
      "s_load_dword %15, %18, 0x3c0\n\t"
      "s_load_dword %16, %19, 0x0\n\t"
      "s_load_dword %17, %19, 0x40\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&s"(d0), "=&s"(d1), "=&s"(d2), "=&s"(d3), "=&s"(d4), "=&s"(d5), "=&s"(d6), "=&s"(d7), "=&s"(d8), "=&s"(d9), "=&s"(d10), "=&s"(d11), "=&s"(d12), "=&s"(d13), "=&s"(d14), "=&s"(d15), "=&s"(d16), "=&s"(d17)
      : "s"(p), "s"(q)
      : "memory");
}

// lines 0..7 (bytes 0..511): for kernels whose walked arguments fit there (7 * 64 + 4 <= sizeof(arguments))
__device__ __forceinline__ void warm_kernarg_8() {
  typedef __attribute__((address_space(4))) const char* karg_t;
  const uint64_t p = (uint64_t)(karg_t)__builtin_amdgcn_kernarg_segment_ptr();
  uint32_t d0, d1, d2, d3, d4, d5, d6, d7;
  asm volatile(
      "s_load_dword %0, %8, 0x0\n\t"
      "s_load_dword %1, %8, 0x40\n\t"
      "s_load_dword %2, %8, 0x80\n\t"
      "s_load_dword %3, %8, 0xc0\n\t"
      "s_load_dword %4, %8, 0x100\n\t"
      "s_load_dword %5, %8, 0x140\n\t"
      "s_load_dword %6, %8, 0x180\n\t"
      "s_load_dword %7, %8, 0x1c0\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&s"(d0), "=&s"(d1), "=&s"(d2), "=&s"(d3), "=&s"(d4), "=&s"(d5), "=&s"(d6), "=&s"(d7)
      : "s"(p)
      : "memory");
}

// lines 0..26 (bytes 0..1727): two block walks (26 * 64 + 4 <= sizeof(arguments))
__device__ __forceinline__ void warm_kernarg_27() {
  typedef __attribute__((address_space(4))) const char* karg_t;
  const uint64_t p = (uint64_t)(karg_t)__builtin_amdgcn_kernarg_segment_ptr();
  uint32_t d[27];
  asm volatile(
      "s_load_dword %0, %27, 0x0\n\t"
      "s_load_dword %1, %27, 0x40\n\t"
      "s_load_dword %2, %27, 0x80\n\t"
      "s_load_dword %3, %27, 0xc0\n\t"
      "s_load_dword %4, %27, 0x100\n\t"
      "s_load_dword %5, %27, 0x140\n\t"
      "s_load_dword %6, %27, 0x180\n\t"
      "s_load_dword %7, %27, 0x1c0\n\t"
      "s_load_dword %8, %27, 0x200\n\t"
      "s_load_dword %9, %27, 0x240\n\t"
      "s_load_dword %10, %27, 0x280\n\t"
      "s_load_dword %11, %27, 0x2c0\n\t"
      "s_load_dword %12, %27, 0x300\n\t"
      "s_load_dword %13, %27, 0x340\n\t"
      "s_load_dword %14, %27, 0x380\n\t"
      "s_load_dword %15, %27, 0x3c0\n\t"
      "s_load_dword %16, %27, 0x400\n\t"
      "s_load_dword %17, %27, 0x440\n\t"
      "s_load_dword %18, %27, 0x480\n\t"
      "s_load_dword %19, %27, 0x4c0\n\t"
      "s_load_dword %20, %27, 0x500\n\t"
      "s_load_dword %21, %27, 0x540\n\t"
      "s_load_dword %22, %27, 0x580\n\t"
      "s_load_dword %23, %27, 0x5c0\n\t"
      "s_load_dword %24, %27, 0x600\n\t"
      "s_load_dword %25, %27, 0x640\n\t"
      "s_load_dword %26, %27, 0x680\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&s"(d[0]), "=&s"(d[1]), "=&s"(d[2]), "=&s"(d[3]), "=&s"(d[4]), "=&s"(d[5]), "=&s"(d[6]), "=&s"(d[7]), "=&s"(d[8]), "=&s"(d[9]), "=&s"(d[10]), "=&s"(d[11]), "=&s"(d[12]), "=&s"(d[13]), "=&s"(d[14]), "=&s"(d[15]), "=&s"(d[16]), "=&s"(d[17]), "=&s"(d[18]), "=&s"(d[19]), "=&s"(d[20]), "=&s"(d[21]), "=&s"(d[22]), "=&s"(d[23]), "=&s"(d[24]), "=&s"(d[25]), "=&s"(d[26])
      : "s"(p)
      : "memory");
}

}  // namespace vt
