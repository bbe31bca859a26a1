// Pieces shared by the GEMM consumers: axis maps (the separable form row_offset(m) +
// col_offset(k) of a 2-D operand's index map), their device evaluators, MFMA wrappers.
#pragma once

#include <hip/hip_runtime.h>

#include <cstring>
#include <string>
#include <vector>

#include "vt_device.h"
#include "vt_numeric.h"

namespace vt {
namespace gemm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

template <int ND>
struct AxisMap {
  FastDiv radix[ND];        // outer -> inner
  int64_t stride[ND];       // elements
  const int32_t* table;     // digit `tdig` is looked up in this table first (index_select), or NULL
  int32_t nd, tdig;
};

// Offset contributed by index v along an axis.  Unused digits are padded on the host with
// radix 1 / stride 0 (in the outer slots), so the walk is branch-free.
template <int ND>
__device__ __forceinline__ int64_t axis_off(const AxisMap<ND>& a, uint32_t v) {
  int64_t off = 0;
#pragma unroll
  for (int d = ND - 1; d >= 0; --d) {
    uint32_t r;
    if (d > 0) {
      uint32_t q = fdiv(v, a.radix[d]);
      r = v - q * a.radix[d].d;
      v = q;
    } else {
      r = v;
    }
    off += (int64_t)r * a.stride[d];
  }
  return off;
}

// The same with an index table on digit a.tdig (index_select): only the row axis of A can
// carry one, and it is evaluated once per thread before the K loop.
template <int ND>
__device__ __forceinline__ int64_t axis_off_table(const AxisMap<ND>& a, uint32_t v) {
  int64_t off = 0;
  uint32_t rt = 0;
  int64_t st = 0;
#pragma unroll
  for (int d = ND - 1; d >= 0; --d) {
    uint32_t r;
    if (d > 0) {
      uint32_t q = fdiv(v, a.radix[d]);
      r = v - q * a.radix[d].d;
      v = q;
    } else {
      r = v;
    }
    const bool is_t = d == a.tdig;
    rt = is_t ? r : rt;
    st = is_t ? a.stride[d] : st;
    off += is_t ? 0 : (int64_t)r * a.stride[d];
  }
  return off + (int64_t)a.table[rt] * st;
}

__device__ __forceinline__ uint32_t word(const uint4& v, int i) { return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w; }

template <typename T>
struct Mma;
template <>
struct Mma<bf16_t> {
  typedef bf16x8 vec;
  static __device__ __forceinline__ f32x16 run(vec a, vec b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
  }
};
template <>
struct Mma<f16_t> {
  typedef f16x8 vec;
  static __device__ __forceinline__ f32x16 run(vec a, vec b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
  }
};

// ---------------------------------------------------------------- host: descriptor -> axis maps
// Concatenates the digit groups of dims [d0, d1) of a single-piece, single-stage descriptor.
template <int ND>
int make_axis(const vt_desc& d, const Piece& p, int d0, int d1, AxisMap<ND>* out, const char* what, bool allow_table = false) {
  memset(out, 0, sizeof(*out));
  out->tdig = -1;
  std::vector<Digit> dg;
  for (int i = d0; i < d1; ++i)
    for (const Digit& g : p.v.groups[i]) dg.push_back(g);
  // merge neighbours that form one dense digit
  std::vector<Digit> m;
  for (const Digit& g : dg) {
    if (!m.empty() && m.back().table < 0 && g.table < 0 && m.back().stride == g.stride * g.radix) {
      m.back().radix *= g.radix;
      m.back().stride = g.stride;
    } else {
      m.push_back(g);
    }
  }
  if ((int)m.size() > ND) return fail(VT_ERR_UNSUPPORTED, std::string(what) + ": too many index digits for the GEMM loader");
  out->nd = (int)m.size();
  for (int i = 0; i < ND; ++i) {        // padding: digits that are always 0
    out->radix[i] = make_fastdiv(1);
    out->stride[i] = 0;
  }
  // real digits occupy the innermost slots so that slot 0 (which takes what is left of the
  // index without a division) is either the outermost real digit or padding over a zero
  const int shift = ND - (int)m.size();
  for (size_t i0 = 0; i0 < m.size(); ++i0) {
    const int i = (int)i0 + shift;
    const Digit& mi = m[i0];
    if (mi.radix >= (1ll << 31)) return fail(VT_ERR_UNSUPPORTED, std::string(what) + ": extent too large");
    out->radix[i] = make_fastdiv((uint32_t)mi.radix);
    out->stride[i] = mi.stride;
    if (mi.table >= 0) {
      if (!allow_table) return fail(VT_ERR_UNSUPPORTED, std::string(what) + ": index_select is only supported on the rows of A");
      if (out->table) return fail(VT_ERR_UNSUPPORTED, std::string(what) + ": two index tables on one axis");
      const Table& t = d.tables[mi.table];
      if (!t.dev) return fail(VT_ERR_INVALID_ARG, std::string(what) + ": index table without a device pointer");
      out->table = t.dev + mi.table_off;
      out->tdig = i;
    }
  }
  return VT_OK;
}

template <int ND>
bool strides_multiple_of(const AxisMap<ND>& a, int64_t q, int skip_inner) {
  for (int i = 0; i < ND - skip_inner; ++i)
    if (a.stride[i] % q) return false;
  return true;
}

}  // namespace gemm
}  // namespace vt
