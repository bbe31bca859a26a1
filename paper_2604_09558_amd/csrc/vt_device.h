// Device-side form of a descriptor (a POD passed to kernels by value) and its evaluator.
//
// The generic evaluator applies the whole map to one index: it is the fallback every
// consumer can use on any descriptor.  The fast paths of the consumers do not call it per
// element: they resolve a tile origin once and walk the tile with a few strides (the
// paper's block-wise virtual tensor I/O, Sec. 4.2).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "vt_desc.h"

namespace vt {

constexpr int kDevPieces = 8;
constexpr int kDevStages = 10;   // pool shared by all pieces
constexpr int kDevDigits = 24;   // pool shared by all stages
constexpr int kDevTables = 4;

// n / d for n < 2^31 as (n * magic) >> (31 + shift), magic = ceil(2^(31+shift) / d),
// shift = ceil(log2 d): exact for every n < 2^31 (Granlund-Montgomery with N = 31).
struct FastDiv {
  uint32_t d, magic, shift;
};

struct DevDigit {
  int64_t stride;
  FastDiv radix;
  uint32_t table_off;
  int32_t table;     // index into DevDesc::tables or -1
};

struct DevStage {
  int64_t base;
  uint8_t first, count;   // digits [first, first+count) of the pool, outer -> inner
};

struct DevPiece {
  const void* ptr;
  int32_t lo[VT_MAX_DIMS], hi[VT_MAX_DIMS];
  uint8_t group_begin[VT_MAX_DIMS + 1];   // top stage: dim i owns digits [gb[i], gb[i+1]) (absolute pool indices)
  uint8_t stage_first, n_stages;          // stage_first = top stage; the lower ones follow it
};

struct DevDesc {
  int32_t ndim, n_pieces, elem_size, outer_dims;   // dims [0,outer_dims) are indexed by the launch's outer index
  FastDiv shape[VT_MAX_DIMS];
  DevPiece pieces[kDevPieces];
  DevStage stages[kDevStages];
  DevDigit digits[kDevDigits];
  const int32_t* tables[kDevTables];
};

FastDiv make_fastdiv(uint32_t d);
// Fills `out` from a host descriptor.  VT_ERR_UNSUPPORTED if it exceeds the device pools or a
// 31-bit index range.  `inner_elems` receives the product of the dims that are addressed by
// the 32-bit inner index (all dims unless the tensor has 2^31 elements or more).
// `host_tables` makes the table pointers name the host copies (for evaluation on the CPU) and
// tolerates sources without device pointers.
int to_device(const vt_desc& d, DevDesc* out, int64_t* outer_count, int64_t* inner_elems, bool host_tables = false);

__host__ __device__ __forceinline__ uint32_t fdiv(uint32_t n, const FastDiv& f) {
  return (uint32_t)(((uint64_t)n * f.magic) >> (31u + f.shift));
}

// Entry i of an index table.  On the device the tables live in device memory: the pointer comes
// out of the descriptor, so the compiler would emit a generic access (one that also checks the
// LDS and scratch apertures); naming the address space makes it a global load.
__host__ __device__ __forceinline__ int32_t table_at(const int32_t* t, uint32_t i) {
#if defined(__HIP_DEVICE_COMPILE__)
  return reinterpret_cast<const __attribute__((address_space(1))) int32_t*>(reinterpret_cast<uintptr_t>(t))[i];
#else
  return t[i];
#endif
}

// Element offset and source pointer of the element at (outer index o, inner linear index L).
// Returns the piece index (always found for a well-formed descriptor).
__host__ __device__ __forceinline__ int vtd_eval(const DevDesc& D, uint32_t o, uint32_t L, int64_t* off_out,
                                                 const void** ptr_out) {
  uint32_t x[VT_MAX_DIMS];
  for (int i = D.ndim - 1; i >= D.outer_dims; --i) {
    uint32_t q = fdiv(L, D.shape[i]);
    x[i] = L - q * D.shape[i].d;
    L = q;
  }
  for (int i = D.outer_dims - 1; i >= 0; --i) {
    uint32_t q = o / D.shape[i].d;
    x[i] = o - q * D.shape[i].d;
    o = q;
  }
  int found = -1;
  int64_t off = 0;
  const void* ptr = nullptr;
  for (int p = 0; p < D.n_pieces; ++p) {
    const DevPiece& pc = D.pieces[p];
    bool in = true;
    for (int i = 0; i < D.ndim; ++i) in = in && (int32_t)x[i] >= pc.lo[i] && (int32_t)x[i] < pc.hi[i];
    if (!in) continue;
    found = p;
    ptr = pc.ptr;
    int64_t acc = D.stages[pc.stage_first].base;
    for (int i = 0; i < D.ndim; ++i) {
      uint32_t v = x[i] - (uint32_t)pc.lo[i];
      for (int k = (int)pc.group_begin[i + 1] - 1; k >= (int)pc.group_begin[i]; --k) {
        const DevDigit& dg = D.digits[k];
        uint32_t q = fdiv(v, dg.radix);
        uint32_t r = v - q * dg.radix.d;
        v = q;
        int64_t val = dg.table >= 0 ? (int64_t)table_at(D.tables[dg.table], dg.table_off + r) : (int64_t)r;
        acc += val * dg.stride;
      }
    }
    for (int s = 1; s < pc.n_stages; ++s) {
      const DevStage& st = D.stages[pc.stage_first + s];
      uint32_t v = (uint32_t)acc;
      acc = st.base;
      for (int k = (int)st.first + st.count - 1; k >= (int)st.first; --k) {
        const DevDigit& dg = D.digits[k];
        uint32_t q = fdiv(v, dg.radix);
        uint32_t r = v - q * dg.radix.d;
        v = q;
        int64_t val = dg.table >= 0 ? (int64_t)table_at(D.tables[dg.table], dg.table_off + r) : (int64_t)r;
        acc += val * dg.stride;
      }
    }
    off = acc;
  }
  *off_out = off;
  *ptr_out = ptr;
  return found;
}

#ifdef __HIPCC__
// Loads and stores of 2, 4, 8 or 16 bytes at an address that a map produced.  Such an address
// names device memory, which the compiler cannot see (it is an integer, or a pointer read out of
// a descriptor): these helpers say so, and the access becomes a global one instead of a generic
// one.  STREAM: the bytes are read once (a streaming load that does not displace other lines).
// Stores stay ordinary: a copy's output is what the next kernel reads, and a streaming store would
// send it past the caches (isolated copies measured 6 % faster with streaming stores, the
// materialized chains of the benchmark up to 15 % slower).
template <int BYTES> struct RawVec;
template <> struct RawVec<2> { typedef uint16_t type; };
template <> struct RawVec<4> { typedef uint32_t type; };
template <> struct RawVec<8> { typedef uint32_t type __attribute__((ext_vector_type(2))); };
template <> struct RawVec<16> { typedef uint32_t type __attribute__((ext_vector_type(4))); };

template <typename V, bool STREAM = false>
__device__ __forceinline__ V ld_global(uint64_t addr) {
  typedef typename RawVec<sizeof(V)>::type R;
  const __attribute__((address_space(1))) R* p = reinterpret_cast<const __attribute__((address_space(1))) R*>(addr);
  const R r = STREAM ? __builtin_nontemporal_load(p) : *p;
  V v;
  __builtin_memcpy(&v, &r, sizeof(V));
  return v;
}
template <typename V, bool STREAM = false>
__device__ __forceinline__ V ld_global(const void* p) { return ld_global<V, STREAM>(reinterpret_cast<uint64_t>(p)); }

template <typename V>
__device__ __forceinline__ void st_global(uint64_t addr, const V& v) {
  typedef typename RawVec<sizeof(V)>::type R;
  R r;
  __builtin_memcpy(&r, &v, sizeof(V));
  *reinterpret_cast<__attribute__((address_space(1))) R*>(addr) = r;
}
template <typename V>
__device__ __forceinline__ void st_global(void* p, const V& v) { st_global<V>(reinterpret_cast<uint64_t>(p), v); }

// The evaluator walks a map with per-lane indices (which piece, which digits): read from the
// kernel arguments every step of that walk is a dependent read of memory.  The kernels that
// evaluate per lane copy their maps to LDS first, with one coalesced read.
template <int N>
__device__ __forceinline__ void stage_maps(DevDesc* dst, const DevDesc* const (&src)[N]) {
#pragma unroll
  for (int k = 0; k < N; ++k) {
    const uint32_t* s = reinterpret_cast<const uint32_t*>(src[k]);
    uint32_t* d = reinterpret_cast<uint32_t*>(&dst[k]);
    for (uint32_t i = threadIdx.x; i < sizeof(DevDesc) / 4; i += blockDim.x) d[i] = s[i];
  }
  __syncthreads();
}
#endif

// Largest vector width (elements, a power of two, at most 16 bytes) with which aligned groups
// of consecutive virtual elements can be moved as one access: it divides every piece's run,
// every piece boundary and every offset at which a run can start, and the source pointers are
// 16-byte aligned.  Always >= 1.
int vector_width(const vt_desc& d);
// Largest power of two c <= cap such that aligned groups of c consecutive virtual elements are
// one contiguous range of one source each (the block form of vector_width; no alignment claim).
int64_t block_elems(const vt_desc& d, int64_t cap);

// Where the host can resolve an operand's map into a few segments in which the block address is
// affine in the row and in at most two levels of the block index, the kernel needs no evaluator:
// a segment covers the blocks [blk_lo, blk_hi) of the rows [row_lo, row_hi), its first block
// starts at `base`, one row further the address moves by row_stride bytes, and block blk_lo + j
// lies (j % blk_group) * blk_stride + (j / blk_group) * group_stride bytes from the first
// (blk_group = 0: one level, j * blk_stride).  n = 0: not resolved.
constexpr int kRowSegs = 4;
struct RowSeg {
  uint64_t base;
  int64_t row_stride;
  uint32_t blk_stride, group_stride;   // a segment's blocks of one row span less than 4 GiB
  uint32_t row_lo, row_hi, blk_lo, blk_hi;
  FastDiv blk_group;                   // d = 0: one level
  uint32_t pad;
};
struct RowWalk {
  RowSeg seg[kRowSegs];
  int32_t n;
  int32_t two_level;                   // some segment has a blk_group
};
// Resolves the [R, C] operand d, read in aligned blocks of `be` columns, into such segments.
// Every piece must be a single stage without tables whose row digits collapse to one stride and
// whose column digits above the block collapse to one or two; the result is checked against the
// evaluator at the corners and the centre of every segment.  False (w->n = 0) for any other map.
bool resolve_row_walk(const vt_desc& d, int64_t be, RowWalk* w);

// The general form of the same idea, for any index space cut into equal units (blocks of a copy,
// rows of a row-wise consumer): unit u of the virtual tensor, in row-major order, starts at
//   base + sum over terms of ((u / div) % mod) * coef        bytes,
// in the piece that holds it.  Every single-stage map without tables has this form: each digit of
// each dim is one term, digits whose strides nest collapse into one, digits below the unit vanish.
// A piece that does not span a dim completely (Concat) is recognised by a test on that dim's
// coordinate, lo <= x < hi with x = (u / t_div) % t_mod (one such dim per piece), and the digits
// of that dim are terms in x - lo instead of u (a piece that is a range of the outermost dim is a
// range of the units, and all its digits are terms in the unit's index within that range).  A dozen instructions per term, against several
// hundred for the evaluator's walk over the map.
constexpr int kWalkPieces = 4;
constexpr int kWalkTerms = 5;
struct WalkTerm {
  FastDiv div, mod;        // mod.d == 0: no modulo (the outermost term)
  uint32_t coef;           // bytes; a piece's units span less than 4 GiB
  uint32_t on_coord;       // the term is a function of x - lo (the tested dim's local coordinate), not of u
};
struct WalkPiece {
  uint64_t base;
  WalkTerm term[kWalkTerms];   // unused ones: div 1, no modulo, coefficient 0
  int32_t n_terms;
  int32_t has_test;            // 0: t_div 1, no modulo, [t_lo, t_hi) = [0, 2^32 - 1): always true
  FastDiv t_div, t_mod;
  uint32_t t_lo, t_hi;
};
struct BlockWalk {
  WalkPiece piece[kWalkPieces];
  int32_t n;               // 0: not resolved
  int32_t pad;
};
// Resolves d, cut into units of `unit` elements (unit divides the element count; the caller
// guarantees that a unit is one contiguous range of a source if it relies on that), into this
// form; the result is checked against the evaluator on a sample of units.  False (w->n = 0) for
// maps with tables, several stages, more pieces or terms than the form holds, 2^31 elements or more.
bool resolve_block_walk(const vt_desc& d, int64_t unit, BlockWalk* w);

// Address of unit u.  W: a pointer to the walk (generic, or into the kernel-argument segment).
// A piece is copied as a whole (a few wide reads) and evaluated without branches: the host fills
// unused terms with coefficient 0 and a piece without a test with one that always holds.
template <typename WalkPtr>
__host__ __device__ __forceinline__ uint64_t walk_address(WalkPtr W, uint32_t u) {
  uint64_t addr = 0;
  const int n = W->n;
#pragma unroll
  for (int p = 0; p < kWalkPieces; ++p) {
    if (p < n) {
      WalkPiece pc;
      __builtin_memcpy(&pc, &W->piece[p], sizeof(WalkPiece));
      const uint32_t xq = fdiv(u, pc.t_div), x = xq - fdiv(xq, pc.t_mod) * pc.t_mod.d;
      const bool in = x >= pc.t_lo && x < pc.t_hi;
      const uint32_t v = x - pc.t_lo;                   // local coordinate of the tested dim
      uint32_t off = 0;
#pragma unroll
      for (int t = 0; t < kWalkTerms; ++t) {
        uint32_t q = fdiv(pc.term[t].on_coord ? v : u, pc.term[t].div);
        q -= fdiv(q, pc.term[t].mod) * pc.term[t].mod.d;   // mod.d == 0 (no modulo): magic 0 gives 0
        off += q * pc.term[t].coef;
      }
      addr = in ? pc.base + off : addr;
    }
  }
  return addr;
}

// launch bookkeeping shared by the kernels' host wrappers
int check_launch(const char* what);
// VT_OK if the descriptor can be the target of a store: no two virtual elements share a physical one.
int check_store_map(const vt_desc& d, const char* who);

}  // namespace vt
