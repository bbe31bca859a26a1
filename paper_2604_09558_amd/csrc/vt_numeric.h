// Storage types and conversions used by the kernels (device only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace vt {

struct bf16_t {
  uint16_t bits;
};
typedef _Float16 f16_t;

template <typename T, int N>
struct __attribute__((aligned(sizeof(T) * N))) Vec {
  T v[N];
};

__device__ __forceinline__ float to_float(float x) { return x; }
__device__ __forceinline__ float to_float(f16_t x) { return (float)x; }
__device__ __forceinline__ float to_float(bf16_t x) { return __uint_as_float((uint32_t)x.bits << 16); }

// float -> bf16, round to nearest even (gfx950 converts in hardware: v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  return __builtin_bit_cast(uint16_t, static_cast<__bf16>(f));
}

template <typename T>
__device__ __forceinline__ T from_float(float x);
template <>
__device__ __forceinline__ float from_float<float>(float x) {
  return x;
}
template <>
__device__ __forceinline__ f16_t from_float<f16_t>(float x) {
  return (f16_t)x;
}
template <>
__device__ __forceinline__ bf16_t from_float<bf16_t>(float x) {
  bf16_t r;
  r.bits = f32_to_bf16_bits(x);
  return r;
}


// Sum over the LPR (8 or 16) consecutive lanes that share a row, on the VALU's data-parallel
// primitives (mirror within 16 / 8 lanes, then the two quad permutes): every lane gets the total.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, false));
}
template <int LPR>
__device__ __forceinline__ float group_sum(float v) {
  if (LPR == 16) v += dpp_move<0x140>(v);   // row_mirror: lane i <-> 15 - i
  v += dpp_move<0x141>(v);                  // row_half_mirror: i <-> 7 - i
  v += dpp_move<0xB1>(v);                   // quad_perm [1,0,3,2]
  v += dpp_move<0x4E>(v);                   // quad_perm [2,3,0,1]
  return v;
}

}  // namespace vt
