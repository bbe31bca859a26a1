// Per-workgroup timestamps for the hand-scheduled kernels, compiled in only with -DVT_PROFILE
// (build.py builds that variant as libvt_profile.so next to libvt.so; the ordinary library
// contains none of this).  A kernel marks up to 8 points per workgroup with the 100 MHz
// wall clock; slot 7 is reserved for the compute die (XCC) the workgroup ran on.  The host
// reads and clears the marks of the last launch with vt_profile_read_<kernel>.
#ifndef VT_PROFILE_H_
#define VT_PROFILE_H_

#ifdef VT_PROFILE
#include <hip/hip_runtime.h>

#include <vector>

namespace vt {
constexpr int kProfSlots = 8;
constexpr int kProfMaxWg = 16384;
}  // namespace vt

// hardware register 20 (XCC_ID), bits [3:0]: s_getreg immediate = (size - 1) << 11 | offset << 6 | id
#define VT_PROF_XCC_ID() ((long long)(__builtin_amdgcn_s_getreg((3 << 11) | 20) & 15))

// ticks of the wall clock per microsecond on the current device
static inline double vt_profile_ticks_per_us() {
  int dev = 0, khz = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 100.0;
  if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess || khz <= 0) return 100.0;
  return khz / 1000.0;
}

#define VT_PROF_DECLARE(name)                                                                        \
  extern "C" double vt_profile_ticks_per_us_##name(void) { return vt_profile_ticks_per_us(); }       \
  static __device__ long long g_prof_##name[vt::kProfMaxWg * vt::kProfSlots];                        \
  extern "C" int vt_profile_read_##name(long long* out, int n_wg) {                                  \
    if (!out || n_wg < 1 || n_wg > vt::kProfMaxWg) return 1;                                         \
    const size_t bytes = sizeof(long long) * (size_t)n_wg * vt::kProfSlots;                          \
    if (hipDeviceSynchronize() != hipSuccess) return 6;                                              \
    if (hipMemcpyFromSymbol(out, HIP_SYMBOL(g_prof_##name), bytes) != hipSuccess) return 6;          \
    std::vector<long long> z((size_t)n_wg * vt::kProfSlots, 0);                                      \
    return hipMemcpyToSymbol(HIP_SYMBOL(g_prof_##name), z.data(), bytes) == hipSuccess ? 0 : 6;      \
  }
// Marks are kept in LDS while the kernel runs (an LDS write does not count among the vector
// memory operations whose order the kernels' waits rely on) and written out by VT_PROF_FLUSH at
// every exit of the kernel.  VT_PROF_BEGIN goes to the top of the kernel body.
#define VT_PROF_BEGIN()                                                                              \
  __shared__ long long vt_prof_sh[vt::kProfSlots];                                                   \
  if (threadIdx.x == 0) {                                                                            \
    for (int vt_k = 0; vt_k < vt::kProfSlots - 1; ++vt_k) vt_prof_sh[vt_k] = 0;                      \
    vt_prof_sh[vt::kProfSlots - 1] = VT_PROF_XCC_ID();                                               \
  }
#define VT_PROF(k)                                                                                   \
  do {                                                                                               \
    if (threadIdx.x == 0) vt_prof_sh[(k)] = wall_clock64();                                          \
  } while (0)
// the shader's own cycle counter at a point (against the wall clock it gives the clock the
// compute unit actually ran at)
#define VT_PROF_CYCLES(k)                                                                            \
  do {                                                                                               \
    if (threadIdx.x == 0) vt_prof_sh[(k)] = clock64();                                               \
  } while (0)
// a point inside a hot loop, taken the first time it is reached
#define VT_PROF_ONCE(k)                                                                              \
  do {                                                                                               \
    if (threadIdx.x == 0 && vt_prof_sh[(k)] == 0) vt_prof_sh[(k)] = wall_clock64();                  \
  } while (0)
#define VT_PROF_FLUSH(name, wg)                                                                      \
  do {                                                                                               \
    if (threadIdx.x == 0 && (wg) < vt::kProfMaxWg)                                                   \
      for (int vt_k = 0; vt_k < vt::kProfSlots; ++vt_k) g_prof_##name[(wg) * vt::kProfSlots + vt_k] = vt_prof_sh[vt_k]; \
  } while (0)
#else
#define VT_PROF_DECLARE(name)
#define VT_PROF_BEGIN() do { } while (0)
#define VT_PROF(k) do { } while (0)
#define VT_PROF_ONCE(k) do { } while (0)
#define VT_PROF_CYCLES(k) do { } while (0)
#define VT_PROF_FLUSH(name, wg) do { } while (0)
#endif

#endif  // VT_PROFILE_H_
