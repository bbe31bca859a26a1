// Host-side representation of a virtual-tensor descriptor (internal to the library).
//
// The mapping function of Eq. 1, f(I) = S.I + b(I), is held per *piece* (the region of the
// virtual index space that one physical source serves; pieces arise from Concat) as a stack
// of mixed-radix strided stages:
//
//   top stage : every virtual dim i owns a group of digits (outer -> inner).  The local
//               coordinate x_i - lo_i is written in the mixed radix of its group and each
//               digit contributes digit * stride (or table[digit] * stride for a digit
//               that carries an index table: the table-driven part of b(I)).
//   lower stages : take the number produced by the stage above as a linear index, write it
//               in their own mixed radix and again sum digit * stride + base.
//
// The last stage yields the element offset into the source.  A reshape that cannot be
// expressed by splitting or merging digits (for instance after a slice that is not aligned
// to the inner dims) pushes a new top stage; everything else edits the top stage in place.
// A stride of zero is a broadcast digit (Expand).
#pragma once

#include <cstdint>
#include <string>
#include <vector>

#include "vt.h"

namespace vt {

constexpr int kMaxStages = 3;     // top + lower
constexpr int kMaxDigits = 12;    // per stage
constexpr int kMaxPieces = 16;

struct Digit {
  int64_t radix = 1;
  int64_t stride = 0;
  int table = -1;          // index into Desc::tables, -1 = plain digit
  int64_t table_off = 0;   // first table entry this digit uses
};

struct Stage {
  std::vector<Digit> digits;   // outer -> inner
  int64_t base = 0;
};

struct View {
  std::vector<int64_t> shape;                 // local extents
  std::vector<std::vector<Digit>> groups;     // top stage, one group per dim
  int64_t base = 0;                           // top stage base
  std::vector<Stage> lower;                   // evaluated in order after the top stage
};

struct Piece {
  int src = 0;
  std::vector<int64_t> lo, hi;   // box in the virtual index space
  View v;                        // maps (x - lo) to an element offset of source `src`
  int64_t run = 1;               // contiguous run in elements (filled by finalize)
  int64_t align = 0;             // gcd of the offsets at which a run can start in the source (0 = only offset 0)
};

struct Table {
  const int32_t* dev = nullptr;
  std::vector<int32_t> host;
};

}  // namespace vt

struct vt_desc {
  int dtype = VT_F32;
  std::vector<int64_t> shape;
  std::vector<vt::Piece> pieces;
  std::vector<vt_source> sources;
  std::vector<vt::Table> tables;
  int64_t run = 1;
};

namespace vt {

void set_error(const std::string& msg);
int fail(int code, const std::string& msg);

// Evaluate one piece's map at a local index (x - lo); tables are read from their host copy.
int64_t eval_view(const vt_desc& d, const View& v, const int64_t* local);
// Index of the piece whose box holds x, or -1.
int find_piece(const vt_desc& d, const int64_t* x);

inline int dtype_size(int dt) { return dt == VT_F32 ? 4 : 2; }

}  // namespace vt
