// Host helpers: conversion of a descriptor to its device form, vector-width analysis.
#include <algorithm>
#include <cstring>
#include <vector>

#include "vt_device.h"

namespace vt {

FastDiv make_fastdiv(uint32_t d) {
  FastDiv f;
  f.d = d;
  uint32_t l = 0;
  while ((1ull << l) < d) ++l;
  f.shift = l;
  unsigned __int128 num = (unsigned __int128)1 << (31 + l);
  f.magic = (uint32_t)((num + d - 1) / d);
  return f;
}

static bool fits31(int64_t v) { return v >= 0 && v < (1ll << 31); }

int to_device(const vt_desc& d, DevDesc* out, int64_t* outer_count, int64_t* inner_elems, bool host_tables) {
  memset(out, 0, sizeof(*out));
  int n = (int)d.shape.size();
  out->ndim = n;
  out->elem_size = dtype_size(d.dtype);
  if ((int)d.pieces.size() > kDevPieces) return fail(VT_ERR_UNSUPPORTED, "descriptor has more pieces than the generic kernels take (8)");
  if ((int)d.tables.size() > kDevTables) return fail(VT_ERR_UNSUPPORTED, "descriptor has more index tables than the generic kernels take (4)");
  out->n_pieces = (int)d.pieces.size();
  int64_t inner = 1;
  int k = n;
  while (k > 0 && inner * d.shape[k - 1] < (1ll << 31)) inner *= d.shape[--k];
  int64_t outer = 1;
  for (int i = 0; i < k; ++i) outer *= d.shape[i];
  if (!fits31(outer)) return fail(VT_ERR_UNSUPPORTED, "tensor too large for the generic kernels");
  out->outer_dims = k;
  if (outer_count) *outer_count = outer;
  if (inner_elems) *inner_elems = inner;
  for (int i = 0; i < n; ++i) {
    if (!fits31(d.shape[i])) return fail(VT_ERR_UNSUPPORTED, "extent >= 2^31");
    out->shape[i] = make_fastdiv((uint32_t)d.shape[i]);
  }
  for (size_t t = 0; t < d.tables.size(); ++t) {
    if (host_tables) {
      out->tables[t] = d.tables[t].host.data();
      continue;
    }
    if (!d.tables[t].dev) return fail(VT_ERR_INVALID_ARG, "descriptor was built without the device pointer of an index table");
    out->tables[t] = d.tables[t].dev;
  }
  int ns = 0, nd = 0;
  auto put_digit = [&](const Digit& g) -> bool {
    if (nd >= kDevDigits || !fits31(g.radix)) return false;
    DevDigit& o = out->digits[nd++];
    o.stride = g.stride;
    o.radix = make_fastdiv((uint32_t)g.radix);
    o.table = g.table;
    o.table_off = (uint32_t)g.table_off;
    return true;
  };
  for (size_t p = 0; p < d.pieces.size(); ++p) {
    const Piece& pc = d.pieces[p];
    DevPiece& o = out->pieces[p];
    o.ptr = d.sources[pc.src].ptr;
    if (!o.ptr && !host_tables) return fail(VT_ERR_INVALID_ARG, "descriptor was built from a source without a device pointer");
    for (int i = 0; i < n; ++i) {
      o.lo[i] = (int32_t)pc.lo[i];
      o.hi[i] = (int32_t)pc.hi[i];
    }
    if (ns + 1 + (int)pc.v.lower.size() > kDevStages) return fail(VT_ERR_UNSUPPORTED, "descriptor has more stages than the generic kernels take");
    o.stage_first = (uint8_t)ns;
    o.n_stages = (uint8_t)(1 + pc.v.lower.size());
    DevStage& top = out->stages[ns++];
    top.base = pc.v.base;
    top.first = (uint8_t)nd;
    for (int i = 0; i < n; ++i) {
      o.group_begin[i] = (uint8_t)nd;
      for (const Digit& g : pc.v.groups[i])
        if (!put_digit(g)) return fail(VT_ERR_UNSUPPORTED, "descriptor has more digits than the generic kernels take");
    }
    o.group_begin[n] = (uint8_t)nd;
    top.count = (uint8_t)(nd - top.first);
    for (const Stage& s : pc.v.lower) {
      DevStage& st = out->stages[ns++];
      st.base = s.base;
      st.first = (uint8_t)nd;
      int64_t span = 1;
      for (const Digit& g : s.digits) {
        span *= g.radix;
        if (!fits31(span)) return fail(VT_ERR_UNSUPPORTED, "stacked stage spans 2^31 elements or more");
        if (!put_digit(g)) return fail(VT_ERR_UNSUPPORTED, "descriptor has more digits than the generic kernels take");
      }
      st.count = (uint8_t)(nd - st.first);
    }
  }
  return VT_OK;
}

int vector_width(const vt_desc& d) {
  int n = (int)d.shape.size();
  int esz = dtype_size(d.dtype);
  int vec = 16 / esz;
  auto ok = [&](int v) {
    if (d.shape[n - 1] % v) return false;
    for (const Piece& p : d.pieces) {
      if (p.run % v) return false;
      if (p.align % v) return false;
      if (p.lo[n - 1] % v || p.hi[n - 1] % v) return false;
      if ((uintptr_t)d.sources[p.src].ptr % 16) return false;
    }
    return true;
  };
  while (vec > 1 && !ok(vec)) vec >>= 1;
  return vec;
}

// The block form of vector_width (block-wise virtual tensor I/O, Sec. 4.2): the largest power of
// two c <= cap such that every aligned group of c consecutive elements of the virtual tensor (in
// row-major order) lies in one piece and is one contiguous range of its source.  Conditions, per
// piece: c divides the piece's run; where the piece is narrower than the tensor along a dim, c
// divides the row-major positions at which the piece starts, ends and repeats along that dim.
// c = 1 always holds.
int64_t block_elems(const vt_desc& d, int64_t cap) {
  const int n = (int)d.shape.size();
  std::vector<int64_t> suffix(n + 1, 1);
  for (int i = n - 1; i >= 0; --i) suffix[i] = suffix[i + 1] * d.shape[i];
  auto ok = [&](int64_t c) {
    if (suffix[0] % c) return false;
    for (const Piece& p : d.pieces) {
      if (p.run % c) return false;
      for (int i = 0; i < n; ++i) {
        if (p.lo[i] == 0 && p.hi[i] == d.shape[i]) continue;
        if ((p.lo[i] * suffix[i + 1]) % c || (p.hi[i] * suffix[i + 1]) % c || suffix[i] % c) return false;
      }
    }
    return true;
  };
  int64_t c = 1;
  while (c * 2 <= cap && ok(c * 2)) c *= 2;
  return c;
}

// A physical tensor may be written through a map only if no two virtual elements share a
// physical one.  Sufficient conditions checked here: no broadcast digit, no index table, no
// stacked stage; inside a piece the digits, ordered by stride, nest (each stride at least the
// span of the smaller ones); pieces of one source cover disjoint offset ranges.
int check_store_map(const vt_desc& d, const char* who) {
  const std::string w(who);
  struct Range {
    int src;
    int64_t lo, hi;
  };
  std::vector<Range> ranges;
  for (const Piece& p : d.pieces) {
    if (!p.v.lower.empty()) return fail(VT_ERR_UNSUPPORTED, w + ": output with stacked index stages");
    std::vector<std::pair<int64_t, int64_t>> dg;    // (|stride|, radix)
    int64_t lo = p.v.base, hi = p.v.base;
    for (const auto& grp : p.v.groups)
      for (const Digit& g : grp) {
        if (g.radix <= 1) continue;
        if (g.table >= 0) return fail(VT_ERR_UNSUPPORTED, w + ": output through an index table");
        if (g.stride == 0) return fail(VT_ERR_NOT_ONE_TO_ONE, w + ": the output map sends several elements to one place (broadcast)");
        dg.push_back({g.stride < 0 ? -g.stride : g.stride, g.radix});
        (g.stride < 0 ? lo : hi) += (g.radix - 1) * g.stride;
      }
    std::sort(dg.begin(), dg.end());
    int64_t span = 1;
    for (const auto& sr : dg) {
      if (sr.first < span) return fail(VT_ERR_NOT_ONE_TO_ONE, w + ": the output map is not one to one (overlapping strides)");
      span = sr.first * (sr.second - 1) + span;
    }
    for (const Range& r : ranges)
      if (r.src == p.src && !(hi < r.lo || r.hi < lo))
        return fail(VT_ERR_NOT_ONE_TO_ONE, w + ": two pieces of the output may overlap in one tensor");
    ranges.push_back({p.src, lo, hi});
  }
  return VT_OK;
}


}  // namespace vt

// The kernels' own evaluator, run on the CPU over the device form of the descriptor: lets the
// host tests check the structure the kernels will walk before anything is launched.
extern "C" int vt_eval_device_form(const vt_desc* d, const int64_t* vindex, int* piece, int64_t* elem_offset) {
  using namespace vt;
  if (!d || !vindex) return fail(VT_ERR_INVALID_ARG, "vt_eval_device_form: NULL argument");
  DevDesc D;
  int64_t outer, inner;
  int rc = to_device(*d, &D, &outer, &inner, true);
  if (rc != VT_OK) return rc;
  int n = (int)d->shape.size();
  uint64_t o = 0, L = 0;
  for (int i = 0; i < D.outer_dims; ++i) o = o * d->shape[i] + vindex[i];
  for (int i = D.outer_dims; i < n; ++i) L = L * d->shape[i] + vindex[i];
  int64_t off;
  const void* ptr;
  int p = vtd_eval(D, (uint32_t)o, (uint32_t)L, &off, &ptr);
  if (p < 0) return fail(VT_ERR_RANGE, "vt_eval_device_form: no piece holds the index");
  if (piece) *piece = p;
  if (elem_offset) *elem_offset = off;
  return VT_OK;
}

extern "C" int vt_desc_block(const vt_desc* d, int64_t cap_elems, int64_t* block_elems_out) {
  if (!d || !block_elems_out || cap_elems < 1) return vt::fail(VT_ERR_INVALID_ARG, "vt_desc_block: NULL argument or cap < 1");
  *block_elems_out = vt::block_elems(*d, cap_elems);
  return VT_OK;
}

extern "C" int vt_desc_row_walk(const vt_desc* d, int64_t block_elems_in, int* n_segments, int64_t* segments) {
  if (!d || !n_segments || !segments || block_elems_in < 1) return vt::fail(VT_ERR_INVALID_ARG, "vt_desc_row_walk: NULL argument or block < 1");
  if (d->shape.size() != 2) return vt::fail(VT_ERR_SHAPE, "vt_desc_row_walk: the tensor must be [R, C]");
  vt::RowWalk w;
  vt::resolve_row_walk(*d, block_elems_in, &w);
  *n_segments = w.n;
  for (int k = 0; k < w.n; ++k) {
    const vt::RowSeg& sg = w.seg[k];
    int64_t* o = segments + 9 * k;
    o[0] = sg.row_lo, o[1] = sg.row_hi, o[2] = sg.blk_lo, o[3] = sg.blk_hi;
    o[4] = (int64_t)sg.base, o[5] = sg.row_stride, o[6] = sg.blk_stride, o[7] = sg.blk_group.d, o[8] = sg.group_stride;
  }
  return VT_OK;
}

extern "C" int vt_desc_walk_addresses(const vt_desc* d, int64_t unit_elems, int64_t first, int64_t count, int* resolved,
                                      uint64_t* addresses) {
  if (!d || !resolved || unit_elems < 1 || first < 0 || count < 0 || (count > 0 && !addresses))
    return vt::fail(VT_ERR_INVALID_ARG, "vt_desc_walk_addresses: NULL argument or negative range");
  vt::BlockWalk w;
  *resolved = vt::resolve_block_walk(*d, unit_elems, &w) ? 1 : 0;
  if (!*resolved) return VT_OK;
  int64_t numel = 1;
  for (int64_t e : d->shape) numel *= e;
  if (first + count > numel / unit_elems) return vt::fail(VT_ERR_RANGE, "vt_desc_walk_addresses: units past the end of the tensor");
  for (int64_t k = 0; k < count; ++k) addresses[k] = vt::walk_address(static_cast<const vt::BlockWalk*>(&w), (uint32_t)(first + k));
  return VT_OK;
}

namespace vt {

// Terms of a digit group as a function of u, where the local coordinate is v = u * unit: every
// digit becomes coef * ((u / div) % mod).  False if a digit cuts through `unit` unevenly or reads a table.
struct AffTerm {
  int64_t div, mod, coef;
};
static bool group_terms(const std::vector<Digit>& g, int64_t unit, std::vector<AffTerm>* terms) {
  int64_t below = 1;                                  // product of the radices inner to the digit
  for (int k = (int)g.size() - 1; k >= 0; --k) {
    const Digit& dg = g[k];
    if (dg.table >= 0) return false;
    if (below % unit == 0) terms->push_back({below / unit, dg.radix, dg.stride});
    else if (unit % below == 0) {
      const int64_t m = unit / below;                 // the digit's value is (u * m) % radix
      if (dg.radix % m == 0) terms->push_back({1, dg.radix / m, dg.stride * m});
      else if (m % dg.radix != 0) return false;       // else: always zero
    } else return false;
    below *= dg.radix;
  }
  return true;
}
// Is the sum of the terms, on [0, extent), of the form (u % group) * s0 + (u / group) * s1?
// One level (affine in u) gives group = 0.
static bool terms_two_level(const std::vector<AffTerm>& terms, int64_t extent, int64_t* s0, int64_t* group, int64_t* s1) {
  *s0 = *s1 = *group = 0;
  bool have = false;
  for (const AffTerm& t : terms) {
    if (t.div >= extent || t.mod == 1) continue;      // never leaves zero
    if (!have) {
      if (t.div != 1) return false;                   // the values below this digit would be dropped
      *s0 = t.coef;
      have = true;
    } else if (*group == 0) {
      if (t.coef == *s0 * t.div) continue;
      *group = t.div;                                 // the second level starts at this digit
      *s1 = t.coef;
    } else if (t.coef != *s1 * (t.div / *group) || t.div % *group) return false;
  }
  return true;
}

bool resolve_row_walk(const vt_desc& d, int64_t be, RowWalk* w) {
  memset(w, 0, sizeof(*w));
  if (d.shape.size() != 2 || d.pieces.size() > (size_t)kRowSegs || be < 1) return false;
  if (block_elems(d, be) != be || d.shape[1] % be) return false;   // the blocks themselves must be contiguous ranges
  const int esz = dtype_size(d.dtype);
  int n = 0;
  for (const Piece& p : d.pieces) {
    if (!p.v.lower.empty() || p.v.groups.size() != 2) return false;
    if (p.lo[1] % be || p.hi[1] % be) return false;
    const int64_t rows = p.hi[0] - p.lo[0], blks = (p.hi[1] - p.lo[1]) / be;
    if (rows < 1 || blks < 1) continue;
    std::vector<AffTerm> tr, tb;
    int64_t rs, r_group, r1, bs, b_group, b1;
    if (!group_terms(p.v.groups[0], 1, &tr) || !terms_two_level(tr, rows, &rs, &r_group, &r1) || r_group != 0) return false;
    if (!group_terms(p.v.groups[1], be, &tb) || !terms_two_level(tb, blks, &bs, &b_group, &b1)) return false;
    const char* src = static_cast<const char*>(d.sources[p.src].ptr);
    if (!src) return false;
    // the kernel adds the block's distance from the row's first block as an unsigned 32-bit number
    if (bs < 0 || b1 < 0) return false;
    const int64_t span = b_group ? (b_group - 1) * bs + ((blks - 1) / b_group) * b1 : (blks - 1) * bs;
    if (span * esz >= (1ll << 32) || blks >= (1ll << 31)) return false;
    RowSeg& sg = w->seg[n++];
    const int64_t zero[2] = {0, 0};
    sg.base = reinterpret_cast<uint64_t>(src) + (uint64_t)(eval_view(d, p.v, zero) * esz);
    sg.row_stride = rs * esz;
    sg.blk_stride = (uint32_t)(bs * esz);
    sg.group_stride = (uint32_t)(b1 * esz);
    if (b_group) {
      sg.blk_group = make_fastdiv((uint32_t)b_group);
      w->two_level = 1;
    }
    sg.row_lo = (uint32_t)p.lo[0];
    sg.row_hi = (uint32_t)p.hi[0];
    sg.blk_lo = (uint32_t)(p.lo[1] / be);
    sg.blk_hi = (uint32_t)(p.hi[1] / be);
    // the evaluator has the last word: corners and centre of the segment, and the blocks around a group boundary
    const int64_t rr[3] = {0, rows / 2, rows - 1};
    const int64_t bb[5] = {0, blks / 2, blks - 1, std::min<int64_t>(blks - 1, b_group), std::min<int64_t>(blks - 1, std::max<int64_t>(0, b_group - 1))};
    for (int64_t r : rr)
      for (int64_t b : bb) {
        const int64_t local[2] = {r, b * be};
        const uint64_t want = reinterpret_cast<uint64_t>(src) + (uint64_t)(eval_view(d, p.v, local) * esz);
        const int64_t hi = b_group ? b / b_group : 0, lo = b - hi * b_group;
        if (want != sg.base + (uint64_t)(r * sg.row_stride) + (uint64_t)((uint32_t)lo * sg.blk_stride + (uint32_t)hi * sg.group_stride)) return false;
      }
  }
  w->n = n;
  return n > 0;
}

// ---- resolve_block_walk
namespace {
struct RawTerm {
  int64_t div, mod, coef;   // ((L / div) % mod) * coef, L and coef in elements; mod = 0: no modulo
  bool on_coord = false;    // a function of the tested dim's local coordinate instead of L
};
// The same term as a function of u = L / unit (L a multiple of unit).  0: vanishes, 1: converted, -1: neither.
int term_in_units(const RawTerm& t, int64_t unit, RawTerm* out) {
  if (t.div % unit == 0) {
    *out = {t.div / unit, t.mod, t.coef, t.on_coord};
    return 1;
  }
  if (unit % t.div) return -1;
  const int64_t m = unit / t.div;                      // the digit's value at L = u * unit is (u * m) % mod
  if (t.mod == 0) {                                    // no modulo: u * m
    *out = {1, 0, t.coef * m, t.on_coord};
    return 1;
  }
  if (m % t.mod == 0) return 0;
  if (t.mod % m) return -1;
  *out = {1, t.mod / m, t.coef * m, t.on_coord};
  return 1;
}
}  // namespace

bool resolve_block_walk(const vt_desc& d, int64_t unit, BlockWalk* w) {
  memset(w, 0, sizeof(*w));
  const int n = (int)d.shape.size();
  if (n < 1 || d.pieces.empty() || d.pieces.size() > (size_t)kWalkPieces || unit < 1) return false;
  int64_t numel = 1;
  for (int64_t e : d.shape) numel *= e;
  if (numel < 1 || numel >= (1ll << 31) || numel % unit) return false;
  const int64_t units = numel / unit;
  const int esz = dtype_size(d.dtype);
  std::vector<int64_t> Q(n, 1);                        // elements per step of dim i
  for (int i = n - 2; i >= 0; --i) Q[i] = Q[i + 1] * d.shape[i + 1];
  int np = 0;
  for (const Piece& p : d.pieces) {
    if (!p.v.lower.empty() || (int)p.v.groups.size() != n) return false;
    const char* src = static_cast<const char*>(d.sources[p.src].ptr);
    if (!src) return false;
    bool empty = false;
    for (int i = 0; i < n; ++i) empty = empty || p.hi[i] <= p.lo[i];
    if (empty) continue;
    std::vector<RawTerm> raw;                           // terms of L (or of the index within the piece's range), in elements
    std::vector<RawTerm> ut;                            // terms in units
    int restricted = -1;
    bool starts_no_unit = false;
    int64_t extent_v = 0;                               // extent of the tested dim's local coordinate, in its units
    WalkPiece& wp = w->piece[np];
    memset(&wp, 0, sizeof(wp));
    // what the branch-free evaluation needs of unused fields: terms that add nothing, a test that holds
    for (WalkTerm& t : wp.term) t.div = make_fastdiv(1);
    wp.t_div = make_fastdiv(1);
    wp.t_hi = 0xffffffffu;
    // A piece that is a range of the OUTERMOST dim only (Concat along dim 0) is a tensor of its
    // own: a range [lo, hi) of the units, and every digit a function of the unit's index in it.
    bool own_range = p.lo[0] != 0 || p.hi[0] != d.shape[0];
    for (int i = 1; i < n; ++i) own_range = own_range && p.lo[i] == 0 && p.hi[i] == d.shape[i];
    if ((p.lo[0] * Q[0]) % unit || (p.hi[0] * Q[0]) % unit) own_range = false;   // a unit across the range's end: the general form
    if (own_range) {
      wp.has_test = 1;                                  // t_div 1, no modulo: the coordinate is u itself
      wp.t_lo = (uint32_t)(p.lo[0] * Q[0] / unit);
      wp.t_hi = (uint32_t)(p.hi[0] * Q[0] / unit);
      extent_v = (p.hi[0] - p.lo[0]) * Q[0] / unit;
      restricted = 0;
    }
    for (int i = 0; i < n && !starts_no_unit; ++i) {
      const std::vector<Digit>& g = p.v.groups[i];
      const int64_t S = d.shape[i];
      for (const Digit& dg : g)
        if (dg.table >= 0) return false;
      if (own_range && i == 0) {
        int64_t below = 1;
        for (int k = (int)g.size() - 1; k >= 0; --k) {   // digits of the index within the range, divided by Q[0]
          raw.push_back({Q[0] * below, k == 0 ? 0 : g[k].radix, g[k].stride, true});
          below *= g[k].radix;
        }
      } else if (own_range || (p.lo[i] == 0 && p.hi[i] == S)) {
        int64_t below = 1;
        for (int k = (int)g.size() - 1; k >= 0; --k) {
          if (S % below || (k > 0 && S % (below * g[k].radix))) return false;
          const int64_t mod = k == 0 ? S / below : g[k].radix;     // the outermost digit takes what is left
          raw.push_back({Q[i] * below, mod, g[k].stride, own_range});
          below *= g[k].radix;
        }
      } else {
        if (restricted >= 0) return false;
        restricted = i;
        RawTerm c;
        const int r = term_in_units({Q[i], S, 1, false}, unit, &c);   // the coordinate: ((u / c.div) % c.mod) * c.coef
        if (r < 0) return false;
        if (r == 0) {                                   // 0 at every unit start: local coordinate 0, or not this piece
          starts_no_unit = p.lo[i] != 0;
          continue;
        }
        const int64_t m = c.coef;
        if (p.lo[i] % m || p.hi[i] % m) return false;
        wp.has_test = 1;
        wp.t_div = make_fastdiv((uint32_t)c.div);
        wp.t_mod = make_fastdiv((uint32_t)c.mod);
        wp.t_lo = (uint32_t)(p.lo[i] / m);
        wp.t_hi = (uint32_t)(p.hi[i] / m);
        extent_v = (p.hi[i] - p.lo[i]) / m;
        int64_t below = 1;
        for (int k = (int)g.size() - 1; k >= 0; --k) {   // digits of the local coordinate v = (x - lo) * m
          RawTerm o;
          const int rr = term_in_units({below, k == 0 ? 0 : g[k].radix, g[k].stride, true}, m, &o);
          if (rr < 0) return false;
          if (rr > 0) ut.push_back(o);
          below *= g[k].radix;
        }
      }
    }
    if (starts_no_unit) continue;
    {
      // digits whose strides nest are one digit: merged in elements first, so that a unit may cut
      // through them (rows of 40 elements in units of 64, when the rows follow each other in the source)
      std::sort(raw.begin(), raw.end(), [](const RawTerm& a, const RawTerm& b) { return a.div < b.div; });
      std::vector<RawTerm> nested;
      for (const RawTerm& t : raw) {
        if (t.coef == 0 || t.mod == 1) continue;
        if (!nested.empty()) {
          RawTerm& m = nested.back();
          if (m.mod > 0 && t.div == m.div * m.mod && t.coef == m.coef * m.mod) {
            m.mod = t.mod == 0 ? 0 : m.mod * t.mod;
            continue;
          }
        }
        nested.push_back(t);
      }
      for (const RawTerm& t : nested) {
        RawTerm o;
        const int r = term_in_units(t, unit, &o);
        if (r < 0) return false;
        if (r > 0) ut.push_back(o);
      }
    }
    // drop what never leaves zero, sort, merge digits whose strides nest
    std::vector<RawTerm> kept;
    for (RawTerm t : ut) {
      const int64_t range = t.on_coord ? extent_v : units;
      if (t.coef == 0 || t.mod == 1 || t.div >= range) continue;
      if (t.mod == 0 || t.div * t.mod >= range) t.mod = 0;             // never wraps: no modulo needed
      kept.push_back(t);
    }
    std::sort(kept.begin(), kept.end(), [](const RawTerm& a, const RawTerm& b) { return a.on_coord != b.on_coord ? a.on_coord < b.on_coord : a.div < b.div; });
    std::vector<RawTerm> merged;
    for (const RawTerm& t : kept) {
      if (!merged.empty()) {
        RawTerm& m = merged.back();
        if (m.on_coord == t.on_coord && m.mod > 0 && t.div == m.div * m.mod && t.coef == m.coef * m.mod) {
          m.mod = t.mod == 0 ? 0 : m.mod * t.mod;
          continue;
        }
      }
      merged.push_back(t);
    }
    if ((int)merged.size() > kWalkTerms) return false;
    int64_t span = 0;
    for (const RawTerm& t : merged) {
      if (t.coef < 0 || t.coef * esz >= (1ll << 32)) return false;
      const int64_t range = t.on_coord ? extent_v : units;
      span += (t.mod ? t.mod - 1 : (range - 1) / t.div) * t.coef;
    }
    if (span * esz >= (1ll << 32)) return false;
    wp.base = reinterpret_cast<uint64_t>(src) + (uint64_t)(p.v.base * esz);
    wp.n_terms = (int)merged.size();
    for (size_t k = 0; k < merged.size(); ++k) {
      wp.term[k].div = make_fastdiv((uint32_t)merged[k].div);
      if (merged[k].mod) wp.term[k].mod = make_fastdiv((uint32_t)merged[k].mod);
      wp.term[k].coef = (uint32_t)(merged[k].coef * esz);
      wp.term[k].on_coord = merged[k].on_coord ? 1u : 0u;
    }
    ++np;
  }
  if (np == 0) return false;
  w->n = np;
  // the evaluator has the last word, on the first and last units and a spread of others
  const int64_t samples = std::min<int64_t>(units, 29);    // this runs at every launch: a few microseconds
  std::vector<int64_t> x(n), local(n);
  for (int64_t k = 0; k < samples + 2; ++k) {
    const int64_t u = k == samples ? units - 1 : k == samples + 1 ? units / 2 : (k * 2654435761ll) % units;
    int64_t L = u * unit;
    for (int i = n - 1; i >= 0; --i) {
      x[i] = L % d.shape[i];
      L /= d.shape[i];
    }
    const int pi = find_piece(d, x.data());
    if (pi < 0) {
      w->n = 0;
      return false;
    }
    const Piece& p = d.pieces[pi];
    for (int i = 0; i < n; ++i) local[i] = x[i] - p.lo[i];
    const uint64_t want = reinterpret_cast<uint64_t>(d.sources[p.src].ptr) + (uint64_t)(eval_view(d, p.v, local.data()) * esz);
    if (walk_address(static_cast<const BlockWalk*>(w), (uint32_t)u) != want) {
      w->n = 0;
      return false;
    }
  }
  return true;
}

int check_launch(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(VT_ERR_DEVICE, std::string(what) + ": " + hipGetErrorString(e));
  return VT_OK;
}

}  // namespace vt
