// Descriptor builder: composes a chain of data-movement operators into one index map
// (Sec. 4.1 "mapping function composition"; Eq. 1 form; Def. 4/5 contiguity).  Host only.
#include <algorithm>
#include <cstdio>
#include <cstring>
#include <numeric>
#include <sstream>

#include "vt_desc.h"

namespace vt {

static thread_local std::string g_err;
void set_error(const std::string& msg) { g_err = msg; }
int fail(int code, const std::string& msg) {
  g_err = msg;
  return code;
}
const char* last_error() { return g_err.c_str(); }

struct Err {
  int code;
  std::string msg;
};
[[noreturn]] static void raise(int code, const std::string& msg) { throw Err{code, msg}; }

static int64_t prod(const std::vector<int64_t>& v) {
  int64_t p = 1;
  for (int64_t x : v) p *= x;
  return p;
}

// ---------------------------------------------------------------- digit-group helpers
static bool mergeable(const Digit& outer, const Digit& inner) {
  return outer.table < 0 && inner.table < 0 && outer.stride == inner.stride * inner.radix;
}

static void normalize(std::vector<Digit>& g) {
  std::vector<Digit> out;
  for (const Digit& d : g) {
    if (d.radix == 1) {
      // a digit that is always 0 contributes table[off]*stride or nothing
      continue;
    }
    if (!out.empty() && mergeable(out.back(), d)) {
      out.back().radix *= d.radix;
      out.back().stride = d.stride;
    } else {
      out.push_back(d);
    }
  }
  g.swap(out);
}

static int stage_count(const View& v) { return 1 + (int)v.lower.size(); }

// A radix-1 digit with a table is not droppable in general (table[off] may be non-zero);
// fold it into the base instead.  Called before normalize on groups that may hold tables.
static void fold_unit_table_digits(const vt_desc& d, View& v) {
  for (auto& g : v.groups)
    for (Digit& dg : g)
      if (dg.radix == 1 && dg.table >= 0) {
        v.base += (int64_t)d.tables[dg.table].host[dg.table_off] * dg.stride;
        dg.table = -1;
        dg.stride = 0;
      }
}

static std::vector<Digit> flatten(const View& v) {
  std::vector<Digit> all;
  for (const auto& g : v.groups)
    for (const Digit& d : g) all.push_back(d);
  return all;
}

// Move the current top stage below a fresh identity top stage over v.shape.
static void push_stage(View& v) {
  if (stage_count(v) + 1 > kMaxStages)
    raise(VT_ERR_UNSUPPORTED, "chain needs more than 3 stacked index stages");
  Stage s;
  s.digits = flatten(v);
  // keep radix-1 plain digits out; the linear index is unaffected by them
  s.digits.erase(std::remove_if(s.digits.begin(), s.digits.end(),
                                [](const Digit& d) { return d.radix == 1 && d.table < 0; }),
                 s.digits.end());
  s.base = v.base;
  v.lower.insert(v.lower.begin(), s);
  v.base = 0;
  int n = (int)v.shape.size();
  v.groups.assign(n, {});
  int64_t st = 1;
  for (int i = n - 1; i >= 0; --i) {
    if (v.shape[i] > 1) v.groups[i].push_back(Digit{v.shape[i], st, -1, 0});
    st *= v.shape[i];
  }
}

// ---------------------------------------------------------------- single-view operators
static void view_permute(View& v, const std::vector<int>& perm) {
  View o = v;
  for (size_t i = 0; i < perm.size(); ++i) {
    o.shape[i] = v.shape[perm[i]];
    o.groups[i] = v.groups[perm[i]];
  }
  v = o;
}

static void view_slice(const vt_desc& d, View& v, int dim, int64_t start, int64_t n, int64_t step) {
  if (start == 0 && n == v.shape[dim] && step == 1) return;
  fold_unit_table_digits(d, v);
  normalize(v.groups[dim]);
  auto& g = v.groups[dim];
  if (g.empty()) return;  // size-1 dim: only the full slice is possible (checked by caller)
  if (g.size() == 1) {
    Digit& dg = g[0];
    if (dg.table < 0) {
      v.base += start * dg.stride;
      dg.radix = n;
      dg.stride *= step;
      v.shape[dim] = n;
      return;
    }
    if (step == 1) {
      dg.table_off += start;
      dg.radix = n;
      v.shape[dim] = n;
      return;
    }
  } else {
    int64_t inner = 1;
    for (size_t i = 1; i < g.size(); ++i) inner *= g[i].radix;
    if (step == 1 && g[0].table < 0 && start % inner == 0 && n % inner == 0) {
      v.base += (start / inner) * g[0].stride;
      g[0].radix = n / inner;
      v.shape[dim] = n;
      return;
    }
  }
  push_stage(v);
  Digit& dg = v.groups[dim][0];
  v.base += start * dg.stride;
  dg.radix = n;
  dg.stride *= step;
  v.shape[dim] = n;
}

static void view_unsqueeze(View& v, int dim) {
  v.shape.insert(v.shape.begin() + dim, 1);
  v.groups.insert(v.groups.begin() + dim, std::vector<Digit>{});
}

static void view_expand(const vt_desc& d, View& v, int dim, int64_t n) {
  fold_unit_table_digits(d, v);
  v.groups[dim].clear();
  v.groups[dim].push_back(Digit{n, 0, -1, 0});
  v.shape[dim] = n;
}

static void view_reshape(const vt_desc& d, View& v, const std::vector<int64_t>& ns) {
  fold_unit_table_digits(d, v);
  std::vector<Digit> dg = flatten(v);
  normalize(dg);
  const int64_t total = prod(ns);
  bool ok = true;
  // every suffix product of the new shape must be a digit boundary (split digits if needed)
  int64_t P = 1;
  for (int j = (int)ns.size() - 1; j >= 1 && ok; --j) {
    P *= ns[j];
    if (P == 1 || P == total) continue;
    int64_t lo = 1;
    for (int i = (int)dg.size() - 1; i >= 0; --i) {
      int64_t hi = lo * dg[i].radix;
      if (P == lo || P == hi) break;
      if (P > lo && P < hi) {
        int64_t q = P / lo;
        if (P % lo != 0 || dg[i].radix % q != 0 || dg[i].table >= 0) {
          ok = false;
          break;
        }
        Digit outer = dg[i], inner = dg[i];
        outer.radix = dg[i].radix / q;
        outer.stride = dg[i].stride * q;
        inner.radix = q;
        dg[i] = outer;
        dg.insert(dg.begin() + i + 1, inner);
        break;
      }
      lo = hi;
    }
  }
  if (!ok) {
    push_stage(v);  // top becomes the identity over the OLD shape ...
    // ... whose digits are one dense row-major number, so any new shape regroups it
    v.shape = ns;
    v.groups.assign(ns.size(), {});
    int64_t st = 1;
    for (int i = (int)ns.size() - 1; i >= 0; --i) {
      if (ns[i] > 1) v.groups[i].push_back(Digit{ns[i], st, -1, 0});
      st *= ns[i];
    }
    return;
  }
  std::vector<std::vector<Digit>> groups(ns.size());
  size_t k = 0;
  for (size_t j = 0; j < ns.size(); ++j) {
    int64_t need = ns[j];
    while (need > 1) {
      if (k >= dg.size() || need % dg[k].radix != 0)
        raise(VT_ERR_UNSUPPORTED, "internal: reshape regrouping failed");
      need /= dg[k].radix;
      groups[j].push_back(dg[k++]);
    }
  }
  v.shape = ns;
  v.groups = groups;
  for (auto& g : v.groups) normalize(g);
}

static void view_index_select(vt_desc& d, View& v, int dim, int table, int64_t n) {
  fold_unit_table_digits(d, v);
  normalize(v.groups[dim]);
  auto& g = v.groups[dim];
  if (g.empty()) {  // size-1 dim: every index is 0 (validated by the caller)
    if (n > 1) g.push_back(Digit{n, 0, -1, 0});
    v.shape[dim] = n;
    return;
  }
  if (!(g.size() == 1 && g[0].table < 0)) push_stage(v);
  Digit& dg = v.groups[dim][0];
  dg.table = table;
  dg.table_off = 0;
  dg.radix = n;
  v.shape[dim] = n;
}

// ---------------------------------------------------------------- multi-piece values
struct Value {
  std::vector<int64_t> shape;
  std::vector<Piece> pieces;
};

static Value from_source(const vt_source& s, int id) {
  Value v;
  int n = s.ndim;
  v.shape.assign(s.shape, s.shape + n);
  bool dense = true;
  for (int i = 0; i < n; ++i) dense = dense && s.stride[i] == 0;
  Piece p;
  p.src = id;
  p.lo.assign(n, 0);
  p.hi = v.shape;
  p.v.shape = v.shape;
  p.v.groups.assign(n, {});
  int64_t st = 1;
  for (int i = n - 1; i >= 0; --i) {
    int64_t stride = dense ? st : s.stride[i];
    if (s.shape[i] > 1) p.v.groups[i].push_back(Digit{s.shape[i], stride, -1, 0});
    st *= s.shape[i];
  }
  v.pieces.push_back(p);
  return v;
}

static void check_dim(int64_t dim, size_t nd, const char* what) {
  if (dim < 0 || dim >= (int64_t)nd) raise(VT_ERR_RANGE, std::string(what) + ": dim out of range");
}

static Value op_permute(const Value& in, const vt_op& op) {
  size_t n = in.shape.size();
  if ((size_t)op.ndim != n) raise(VT_ERR_SHAPE, "permute: perm length differs from rank");
  std::vector<int> perm(n);
  std::vector<bool> seen(n, false);
  for (size_t i = 0; i < n; ++i) {
    if (op.a[i] < 0 || op.a[i] >= (int64_t)n || seen[op.a[i]])
      raise(VT_ERR_INVALID_ARG, "permute: not a permutation");
    seen[op.a[i]] = true;
    perm[i] = (int)op.a[i];
  }
  Value out = in;
  for (size_t i = 0; i < n; ++i) out.shape[i] = in.shape[perm[i]];
  for (Piece& p : out.pieces) {
    std::vector<int64_t> lo = p.lo, hi = p.hi;
    for (size_t i = 0; i < n; ++i) {
      p.lo[i] = lo[perm[i]];
      p.hi[i] = hi[perm[i]];
    }
    view_permute(p.v, perm);
  }
  return out;
}

static Value op_slice(const vt_desc& d, const Value& in, int dim, int64_t start, int64_t stop, int64_t step) {
  check_dim(dim, in.shape.size(), "slice");
  if (step < 1) raise(VT_ERR_RANGE, "slice: step must be >= 1");
  if (start < 0 || stop > in.shape[dim] || start >= stop) raise(VT_ERR_RANGE, "slice: range outside the dim or empty");
  Value out;
  out.shape = in.shape;
  out.shape[dim] = (stop - start + step - 1) / step;
  for (const Piece& p0 : in.pieces) {
    // new coordinate x' <-> old x = start + step*x'; keep those with lo <= x < hi
    int64_t lo = p0.lo[dim], hi = std::min(p0.hi[dim], stop);
    int64_t xlo = lo <= start ? 0 : (lo - start + step - 1) / step;
    int64_t xhi = hi <= start ? 0 : (hi - start + step - 1) / step;
    if (xhi <= xlo) continue;
    Piece p = p0;
    int64_t first_local = start + step * xlo - lo;
    view_slice(d, p.v, dim, first_local, xhi - xlo, step);
    p.lo[dim] = xlo;
    p.hi[dim] = xhi;
    out.pieces.push_back(p);
  }
  return out;
}

static Value op_concat(const std::vector<const Value*>& ins, int dim) {
  const Value& f = *ins[0];
  check_dim(dim, f.shape.size(), "concat");
  Value out;
  out.shape = f.shape;
  out.shape[dim] = 0;
  for (const Value* v : ins) {
    if (v->shape.size() != f.shape.size()) raise(VT_ERR_SHAPE, "concat: ranks differ");
    for (size_t i = 0; i < f.shape.size(); ++i)
      if ((int)i != dim && v->shape[i] != f.shape[i]) raise(VT_ERR_SHAPE, "concat: shapes differ off the concat dim");
    for (Piece p : v->pieces) {
      p.lo[dim] += out.shape[dim];
      p.hi[dim] += out.shape[dim];
      out.pieces.push_back(p);
    }
    out.shape[dim] += v->shape[dim];
  }
  if ((int)out.pieces.size() > kMaxPieces) raise(VT_ERR_UNSUPPORTED, "more than 16 pieces");
  return out;
}

static Value op_unsqueeze(const Value& in, int dim) {
  if (dim < 0 || dim > (int)in.shape.size()) raise(VT_ERR_RANGE, "unsqueeze: dim out of range");
  if (in.shape.size() + 1 > VT_MAX_DIMS) raise(VT_ERR_UNSUPPORTED, "more than 8 dims");
  Value out = in;
  out.shape.insert(out.shape.begin() + dim, 1);
  for (Piece& p : out.pieces) {
    p.lo.insert(p.lo.begin() + dim, 0);
    p.hi.insert(p.hi.begin() + dim, 1);
    view_unsqueeze(p.v, dim);
  }
  return out;
}

static Value op_expand(const vt_desc& d, const Value& in, const vt_op& op) {
  size_t n = in.shape.size();
  if ((size_t)op.ndim != n) raise(VT_ERR_SHAPE, "expand: rank must be kept (unsqueeze first)");
  Value out = in;
  for (size_t i = 0; i < n; ++i) {
    if (op.a[i] == in.shape[i]) continue;
    if (in.shape[i] != 1 || op.a[i] < 1) raise(VT_ERR_SHAPE, "expand: only size-1 dims broadcast");
    out.shape[i] = op.a[i];
    for (Piece& p : out.pieces) {
      p.hi[i] = op.a[i];
      view_expand(d, p.v, (int)i, op.a[i]);
    }
  }
  return out;
}

static Value op_index_select(vt_desc& d, const Value& in, int dim, int table) {
  check_dim(dim, in.shape.size(), "index_select");
  const std::vector<int32_t>& t = d.tables[table].host;
  for (int32_t x : t)
    if (x < 0 || x >= in.shape[dim]) raise(VT_ERR_RANGE, "index_select: index outside the dim");
  const int64_t n = (int64_t)t.size();
  Value out = in;
  out.shape[dim] = n;
  bool cut = false;
  for (const Piece& p : in.pieces) cut = cut || p.lo[dim] != 0 || p.hi[dim] != in.shape[dim];
  if (!cut) {
    for (Piece& p : out.pieces) {
      view_index_select(d, p.v, dim, table, n);
      p.hi[dim] = n;
    }
    return out;
  }
  // The dim is cut into pieces (a Concat below): a table entry decides which piece an output
  // index reads.  The pieces are boxes, so between two neighbouring cut points every piece spans
  // the whole slab; consecutive output indices whose entries fall into one slab form a run, and
  // each run becomes its own set of pieces [j0, j1) that read entries j0.. of the same table.  The
  // entries stay global: entry * stride - lo * stride, the second term goes into the base.
  std::vector<int64_t> cuts;
  for (const Piece& p : in.pieces) {
    cuts.push_back(p.lo[dim]);
    cuts.push_back(p.hi[dim]);
  }
  std::sort(cuts.begin(), cuts.end());
  cuts.erase(std::unique(cuts.begin(), cuts.end()), cuts.end());
  auto slab_of = [&](int64_t x) { return (int)(std::upper_bound(cuts.begin(), cuts.end(), x) - cuts.begin()) - 1; };
  out.pieces.clear();
  for (int64_t j0 = 0; j0 < n;) {
    const int slab = slab_of(t[j0]);
    int64_t j1 = j0 + 1;
    while (j1 < n && slab_of(t[j1]) == slab) ++j1;
    for (const Piece& p0 : in.pieces) {
      if (!(p0.lo[dim] <= cuts[slab] && cuts[slab + 1] <= p0.hi[dim])) continue;
      Piece p = p0;
      view_index_select(d, p.v, dim, table, j1 - j0);
      auto& g = p.v.groups[dim];
      if (!g.empty() && g[0].table >= 0) {
        g[0].table_off = j0;
        p.v.base -= p0.lo[dim] * g[0].stride;
      }
      p.lo[dim] = j0;
      p.hi[dim] = j1;
      out.pieces.push_back(p);
      if ((int)out.pieces.size() > kMaxPieces) raise(VT_ERR_UNSUPPORTED, "index_select over a concatenated dim needs more than 16 pieces");
    }
    j0 = j1;
  }
  return out;
}

static Value op_reshape(const vt_desc& d, const Value& in, const vt_op& op) {
  std::vector<int64_t> ns(op.a, op.a + op.ndim);
  for (int64_t x : ns)
    if (x < 1) raise(VT_ERR_SHAPE, "reshape: extents must be >= 1");
  if (prod(ns) != prod(in.shape)) raise(VT_ERR_SHAPE, "reshape: element counts differ");
  Value out;
  out.shape = ns;
  // match minimal chunks of equal product between old and new dims (size-1 dims set aside)
  std::vector<int> od, nd;
  for (size_t i = 0; i < in.shape.size(); ++i)
    if (in.shape[i] > 1) od.push_back((int)i);
  for (size_t j = 0; j < ns.size(); ++j)
    if (ns[j] > 1) nd.push_back((int)j);
  struct Chunk {
    std::vector<int> o, n;
  };
  std::vector<Chunk> chunks;
  size_t i = 0, j = 0;
  while (i < od.size() || j < nd.size()) {
    Chunk c;
    int64_t po = 1, pn = 1;
    do {
      if (po <= pn && i < od.size()) {
        po *= in.shape[od[i]];
        c.o.push_back(od[i++]);
      } else if (j < nd.size()) {
        pn *= ns[nd[j]];
        c.n.push_back(nd[j++]);
      } else {
        raise(VT_ERR_SHAPE, "reshape: internal chunking error");
      }
    } while (po != pn);
    chunks.push_back(c);
  }
  // A piece that a Concat made narrower than the tensor inside a chunk is, in the chunk's linear
  // index, a set of intervals: one per choice of the indices of the old dims outside the innermost
  // narrowed one.  Over the new dims an interval is a few boxes (the rest of a row, whole rows, the
  // start of a row, recursively per new dim).  Each box becomes a piece of the result whose view
  // is the old piece's view, cut down to the interval (slices of the old dims, then of the
  // chunk's dims merged into one) and regrouped.
  struct Part {
    std::vector<int64_t> lo, hi;                       // over c.n
    std::vector<std::pair<int, int64_t>> fix;          // old dims held at one local index
    int64_t merged_len = 1, start = 0, len = -1;       // slice of the merged dim (len < 0: none)
  };
  for (const Piece& p0 : in.pieces) {
    std::vector<std::vector<Part>> options;      // per chunk
    for (const Chunk& c : chunks) {
      std::vector<Part> parts;
      const size_t ko = c.o.size(), m = c.n.size();
      int q = -1;                                      // innermost narrowed old dim of the chunk
      for (size_t k = 0; k < ko; ++k)
        if (p0.lo[c.o[k]] != 0 || p0.hi[c.o[k]] != in.shape[c.o[k]]) q = (int)k;
      if (q < 0) {
        Part pt;
        for (int n : c.n) {
          pt.lo.push_back(0);
          pt.hi.push_back(ns[n]);
          pt.merged_len *= ns[n];
        }
        parts.push_back(pt);
        options.push_back(parts);
        continue;
      }
      std::vector<int64_t> so(ko + 1, 1), inner(m + 1, 1);      // suffix products: old dims, new dims
      for (size_t k = ko; k-- > 0;) so[k] = so[k + 1] * in.shape[c.o[k]];
      for (size_t k = m; k-- > 0;) inner[k] = inner[k + 1] * ns[c.n[k]];
      std::vector<int64_t> x(q, 0);
      for (int k = 0; k < q; ++k) x[k] = p0.lo[c.o[k]];
      while (true) {
        int64_t a = p0.lo[c.o[q]] * so[q + 1];
        for (int k = 0; k < q; ++k) a += x[k] * so[k + 1];
        const int64_t b = a + (p0.hi[c.o[q]] - p0.lo[c.o[q]]) * so[q + 1];
        struct Job {
          int64_t u, v;      // interval of the chunk's linear index
          size_t level;      // new dims before `level` are fixed by u
        };
        std::vector<Job> todo{{a, b, 0}};
        while (!todo.empty()) {
          const Job jb = todo.back();
          todo.pop_back();
          if (jb.u >= jb.v) continue;
          const int64_t in1 = inner[jb.level + 1];     // elements per index of new dim `level`
          const int64_t base = jb.u / inner[jb.level] * inner[jb.level];
          const int64_t u = jb.u - base, v = jb.v - base;
          if (jb.level + 1 == m || (u % in1 == 0 && v % in1 == 0)) {
            Part pt;
            int64_t rem = base;
            for (size_t k = 0; k < m; ++k) {
              if (k < jb.level) {
                const int64_t xi = rem / inner[k + 1];
                rem -= xi * inner[k + 1];
                pt.lo.push_back(xi);
                pt.hi.push_back(xi + 1);
              } else if (k == jb.level) {
                pt.lo.push_back(u / in1);
                pt.hi.push_back(v / in1);
              } else {
                pt.lo.push_back(0);
                pt.hi.push_back(ns[c.n[k]]);
              }
            }
            for (int k = 0; k < q; ++k) pt.fix.push_back({c.o[k], x[k] - p0.lo[c.o[k]]});
            pt.merged_len = b - a;
            pt.start = jb.u - a;
            pt.len = jb.v - jb.u;
            parts.push_back(pt);
            if (parts.size() > (size_t)kMaxPieces) raise(VT_ERR_UNSUPPORTED, "reshape across a concat cut needs more than 16 pieces");
            continue;
          }
          const int64_t first = u / in1, last = (v - 1) / in1;
          if (first == last) {
            todo.push_back({jb.u, jb.v, jb.level + 1});
            continue;
          }
          const int64_t head_end = u % in1 ? (first + 1) * in1 : u, tail_begin = v % in1 ? last * in1 : v;
          if (u < head_end) todo.push_back({base + u, base + head_end, jb.level + 1});
          if (head_end < tail_begin) todo.push_back({base + head_end, base + tail_begin, jb.level});
          if (tail_begin < v) todo.push_back({base + tail_begin, base + v, jb.level + 1});
        }
        int k = q - 1;
        while (k >= 0 && ++x[k] == p0.hi[c.o[k]]) {
          x[k] = p0.lo[c.o[k]];
          --k;
        }
        if (k < 0) break;
      }
      options.push_back(parts);
    }
    // every combination of one part per chunk is a piece of the result
    std::vector<size_t> pick(chunks.size(), 0);
    while (true) {
      Piece p = p0;
      std::vector<int64_t> lo(ns.size(), 0), hi(ns.size(), 1), local(ns.size(), 1), merged;
      bool cut = false;
      for (size_t ci = 0; ci < chunks.size(); ++ci) {
        const Chunk& c = chunks[ci];
        const Part& pt = options[ci][pick[ci]];
        for (size_t k = 0; k < c.n.size(); ++k) {
          lo[c.n[k]] = pt.lo[k];
          hi[c.n[k]] = pt.hi[k];
          local[c.n[k]] = pt.hi[k] - pt.lo[k];
        }
        for (const auto& f : pt.fix) view_slice(d, p.v, f.first, f.second, 1, 1);
        merged.push_back(pt.merged_len);
        cut = cut || (pt.len >= 0 && pt.len != pt.merged_len);
      }
      if (cut) {
        if (merged.empty()) merged.push_back(1);
        view_reshape(d, p.v, merged);
        for (size_t ci = 0; ci < chunks.size(); ++ci) {
          const Part& pt = options[ci][pick[ci]];
          if (pt.len >= 0 && pt.len != pt.merged_len) view_slice(d, p.v, (int)ci, pt.start, pt.len, 1);
        }
      }
      view_reshape(d, p.v, local);
      p.lo = lo;
      p.hi = hi;
      out.pieces.push_back(p);
      if ((int)out.pieces.size() > kMaxPieces) raise(VT_ERR_UNSUPPORTED, "reshape across a concat cut needs more than 16 pieces");
      size_t ci = 0;
      while (ci < chunks.size() && ++pick[ci] == options[ci].size()) pick[ci++] = 0;
      if (ci == chunks.size()) break;
    }
  }
  return out;
}

// ---------------------------------------------------------------- contiguity (Def. 4/5)
static int64_t gcd64(int64_t a, int64_t b) {
  a = a < 0 ? -a : a;
  b = b < 0 ? -b : b;
  while (b) {
    int64_t t = a % b;
    a = b;
    b = t;
  }
  return a;
}

static void finalize_piece(const vt_desc& d, Piece& p) {
  fold_unit_table_digits(d, p.v);
  for (auto& g : p.v.groups) normalize(g);
  for (Stage& s : p.v.lower) {
    for (Digit& dg : s.digits)
      if (dg.radix == 1 && dg.table >= 0) {
        s.base += (int64_t)d.tables[dg.table].host[dg.table_off] * dg.stride;
        dg.table = -1;
        dg.stride = 0;
      }
    normalize(s.digits);
  }
  // top stage: walk digits from the innermost dim while they form a dense suffix
  int n = (int)p.v.shape.size();
  int64_t run = 1, expect = 1;
  int64_t g = 0;  // gcd of everything that positions a run in the next stage's index space
  bool open = true;
  for (int i = n - 1; i >= 0; --i) {
    const auto& grp = p.v.groups[i];
    for (int k = (int)grp.size() - 1; k >= 0; --k) {
      const Digit& dg = grp[k];
      if (open && dg.table < 0 && dg.stride == expect) {
        run *= dg.radix;
        expect *= dg.radix;
      } else {
        open = false;
        g = gcd64(g, dg.stride);
      }
    }
    if (p.hi[i] - p.lo[i] != d.shape[i]) open = false;  // the piece is narrower than the tensor here
  }
  g = gcd64(g, p.v.base);
  // A piece that is one run as a whole sits at cur .. cur + run - 1 of the next stage's index space;
  // while that range stays inside one dense run of the stage below, it remains one range (its
  // extent decides, not the alignment of its start).
  int64_t piece_size = 1;
  for (int i = 0; i < n; ++i) piece_size *= p.hi[i] - p.lo[i];
  bool whole = run == piece_size && p.v.base >= 0;
  int64_t cur = p.v.base;
  for (const Stage& s : p.v.lower) {
    int64_t r2 = 1, e2 = 1, g2 = 0;
    bool op2 = true;
    for (int k = (int)s.digits.size() - 1; k >= 0; --k) {
      const Digit& dg = s.digits[k];
      if (op2 && dg.table < 0 && dg.stride == e2) {
        r2 *= dg.radix;
        e2 *= dg.radix;
      } else {
        op2 = false;
        g2 = gcd64(g2, dg.stride);
      }
    }
    if (whole && cur % r2 + run <= r2) {
      int64_t x = cur;
      cur = s.base;
      for (int k = (int)s.digits.size() - 1; k >= 0; --k) {
        int64_t dig = x % s.digits[k].radix;
        x /= s.digits[k].radix;
        if (s.digits[k].table >= 0) dig = d.tables[s.digits[k].table].host[s.digits[k].table_off + dig];
        cur += dig * s.digits[k].stride;
      }
      g = cur;                     // the one offset at which the range starts below
      whole = cur >= 0;
      continue;
    }
    whole = false;
    // blocks of c consecutive indices are contiguous below iff c | run, c | r2 and c divides
    // every offset at which a run of the stage above can start
    int64_t c = gcd64(run, r2);
    if (g != 0) c = gcd64(c, g);
    run = c;
    g = gcd64(g2, s.base);
  }
  p.run = run;
  p.align = g;
}

}  // namespace vt

using namespace vt;

// ---------------------------------------------------------------- evaluation on the host
int64_t vt::eval_view(const vt_desc& d, const View& v, const int64_t* local) {
  int64_t off = v.base;
  for (size_t i = 0; i < v.groups.size(); ++i) {
    int64_t x = local[i];
    const auto& g = v.groups[i];
    for (int k = (int)g.size() - 1; k >= 0; --k) {
      int64_t dig = x % g[k].radix;
      x /= g[k].radix;
      if (g[k].table >= 0) dig = d.tables[g[k].table].host[g[k].table_off + dig];
      off += dig * g[k].stride;
    }
  }
  for (const Stage& s : v.lower) {
    int64_t x = off;
    off = s.base;
    for (int k = (int)s.digits.size() - 1; k >= 0; --k) {
      int64_t dig = x % s.digits[k].radix;
      x /= s.digits[k].radix;
      if (s.digits[k].table >= 0) dig = d.tables[s.digits[k].table].host[s.digits[k].table_off + dig];
      off += dig * s.digits[k].stride;
    }
  }
  return off;
}

int vt::find_piece(const vt_desc& d, const int64_t* x) {
  for (size_t p = 0; p < d.pieces.size(); ++p) {
    bool in = true;
    for (size_t i = 0; i < d.shape.size() && in; ++i) in = x[i] >= d.pieces[p].lo[i] && x[i] < d.pieces[p].hi[i];
    if (in) return (int)p;
  }
  return -1;
}

// ---------------------------------------------------------------- C ABI
extern "C" {

const char* vt_last_error(void) { return vt::last_error(); }
const char* vt_version(void) { return "vt 0.1 (gfx950)"; }

int vt_build(const vt_source* src, int n_src, const vt_op* ops, int n_ops, int result_value, vt_desc** out) {
  if (!out) return fail(VT_ERR_INVALID_ARG, "vt_build: out is NULL");
  *out = nullptr;
  if (!src || n_src < 1 || n_ops < 0 || (n_ops > 0 && !ops)) return fail(VT_ERR_INVALID_ARG, "vt_build: bad arguments");
  if (result_value >= n_ops || result_value < -n_src) return fail(VT_ERR_INVALID_ARG, "vt_build: result_value names nothing");
  vt_desc* d = new vt_desc();
  try {
    d->dtype = src[0].dtype;
    for (int i = 0; i < n_src; ++i) {
      const vt_source& s = src[i];
      if (s.dtype != d->dtype) raise(VT_ERR_INVALID_ARG, "sources of one virtual tensor must share a dtype");
      if (s.dtype < VT_F32 || s.dtype > VT_BF16) raise(VT_ERR_INVALID_ARG, "bad dtype");
      if (s.ndim < 1 || s.ndim > VT_MAX_DIMS) raise(VT_ERR_INVALID_ARG, "source rank must be 1..8");
      for (int k = 0; k < s.ndim; ++k)
        if (s.shape[k] < 1 || s.stride[k] < 0) raise(VT_ERR_SHAPE, "source extents must be >= 1 and strides >= 0");
      d->sources.push_back(s);
    }
    std::vector<Value> vals(n_ops);
    std::vector<Value> srcv;
    for (int i = 0; i < n_src; ++i) srcv.push_back(from_source(src[i], i));
    auto get = [&](int id, int at) -> const Value& {
      if (id < 0) {
        if (-1 - id >= n_src) raise(VT_ERR_INVALID_ARG, "statement names a source that does not exist");
        return srcv[-1 - id];
      }
      if (id >= at) raise(VT_ERR_INVALID_ARG, "statement names a later statement");
      return vals[id];
    };
    for (int k = 0; k < n_ops; ++k) {
      const vt_op& op = ops[k];
      if (op.n_in < 1 || op.n_in > VT_MAX_OP_INPUTS) raise(VT_ERR_INVALID_ARG, "bad number of inputs");
      if (op.kind != VT_OP_CONCAT && op.n_in != 1) raise(VT_ERR_INVALID_ARG, "only concat takes several inputs");
      if (op.ndim < 0 || op.ndim > VT_MAX_DIMS) raise(VT_ERR_INVALID_ARG, "bad ndim in statement");
      const Value& in0 = get(op.in[0], k);
      switch (op.kind) {
        case VT_OP_RESHAPE:
          if (op.ndim < 1) raise(VT_ERR_SHAPE, "reshape: empty shape");
          vals[k] = op_reshape(*d, in0, op);
          break;
        case VT_OP_PERMUTE:
          vals[k] = op_permute(in0, op);
          break;
        case VT_OP_SLICE:
          vals[k] = op_slice(*d, in0, (int)op.a[0], op.a[1], op.a[2], op.a[3] == 0 ? 1 : op.a[3]);
          break;
        case VT_OP_SPLIT: {
          int dim = (int)op.a[0];
          check_dim(dim, in0.shape.size(), "split");
          if (op.ndim < 1 || op.out_index < 0 || op.out_index >= op.ndim) raise(VT_ERR_RANGE, "split: out_index outside the outputs");
          int64_t sum = 0, off = 0;
          for (int t = 0; t < op.ndim; ++t) {
            if (op.b[t] < 1) raise(VT_ERR_RANGE, "split: sizes must be >= 1");
            if (t < op.out_index) off += op.b[t];
            sum += op.b[t];
          }
          if (sum != in0.shape[dim]) raise(VT_ERR_RANGE, "split: sizes do not add up to the dim");
          vals[k] = op_slice(*d, in0, dim, off, off + op.b[op.out_index], 1);
          break;
        }
        case VT_OP_CONCAT: {
          std::vector<const Value*> ins;
          for (int t = 0; t < op.n_in; ++t) ins.push_back(&get(op.in[t], k));
          vals[k] = op_concat(ins, (int)op.a[0]);
          break;
        }
        case VT_OP_EXPAND:
          vals[k] = op_expand(*d, in0, op);
          break;
        case VT_OP_UNSQUEEZE:
          vals[k] = op_unsqueeze(in0, (int)op.a[0]);
          break;
        case VT_OP_INDEX_SELECT: {
          if (!op.index_host || op.n_index < 1) raise(VT_ERR_INVALID_ARG, "index_select: host copy of the table is required");
          Table t;
          t.dev = op.index;
          t.host.assign(op.index_host, op.index_host + op.n_index);
          d->tables.push_back(t);
          vals[k] = op_index_select(*d, in0, (int)op.a[0], (int)d->tables.size() - 1);
          break;
        }
        default:
          raise(VT_ERR_INVALID_ARG, "unknown operator kind");
      }
      for (const Piece& p : vals[k].pieces) {
        if (stage_count(p.v) > kMaxStages) raise(VT_ERR_UNSUPPORTED, "too many stages");
      }
    }
    const Value& r = get(result_value, n_ops);
    d->shape = r.shape;
    d->pieces = r.pieces;
    if (d->shape.size() > VT_MAX_DIMS) raise(VT_ERR_UNSUPPORTED, "more than 8 dims");
    d->run = INT64_MAX;
    for (Piece& p : d->pieces) {
      finalize_piece(*d, p);
      size_t nd = 0;
      for (const auto& g : p.v.groups) nd += g.size();
      if (nd > (size_t)kMaxDigits) raise(VT_ERR_UNSUPPORTED, "more than 12 digits in one stage");
      for (const Stage& s : p.v.lower)
        if (s.digits.size() > (size_t)kMaxDigits) raise(VT_ERR_UNSUPPORTED, "more than 12 digits in one stage");
      d->run = std::min(d->run, p.run);
    }
  } catch (const Err& e) {
    delete d;
    return fail(e.code, e.msg);
  } catch (const std::exception& e) {
    delete d;
    return fail(VT_ERR_INVALID_ARG, std::string("vt_build: ") + e.what());
  }
  *out = d;
  return VT_OK;
}

int vt_free(vt_desc* d) {
  delete d;
  return VT_OK;
}

int vt_desc_info(const vt_desc* d, int* ndim, int64_t* shape, int* dtype, int64_t* contiguous_run, int* n_pieces) {
  if (!d) return fail(VT_ERR_INVALID_ARG, "vt_desc_info: NULL descriptor");
  if (ndim) *ndim = (int)d->shape.size();
  if (shape)
    for (size_t i = 0; i < d->shape.size(); ++i) shape[i] = d->shape[i];
  if (dtype) *dtype = d->dtype;
  if (contiguous_run) *contiguous_run = d->run;
  if (n_pieces) *n_pieces = (int)d->pieces.size();
  return VT_OK;
}

int vt_desc_as_strided(const vt_desc* d, int* is_strided, int64_t* stride, int64_t* offset) {
  if (!d || !is_strided) return fail(VT_ERR_INVALID_ARG, "vt_desc_as_strided: NULL argument");
  *is_strided = 0;
  if (d->pieces.size() != 1 || !d->pieces[0].v.lower.empty()) return VT_OK;
  const Piece& p = d->pieces[0];
  for (size_t i = 0; i < d->shape.size(); ++i) {
    const auto& g = p.v.groups[i];
    if (g.size() > 1 || (g.size() == 1 && g[0].table >= 0)) return VT_OK;
    if (stride) stride[i] = g.empty() ? 0 : g[0].stride;
  }
  if (offset) *offset = p.v.base;
  *is_strided = 1;
  return VT_OK;
}

int vt_classify(const vt_desc* d, int64_t unit_bytes, int* access_class, int64_t* min_run_bytes) {
  if (!d || !access_class) return fail(VT_ERR_INVALID_ARG, "vt_classify: NULL argument");
  if (unit_bytes < 0) return fail(VT_ERR_INVALID_ARG, "vt_classify: negative unit");
  if (unit_bytes == 0) unit_bytes = 128;
  const int64_t esz = d->dtype == VT_F32 ? 4 : 2;
  int64_t numel = 1;
  for (int64_t e : d->shape) numel *= e;
  const int64_t run_bytes = d->run * esz;
  if (min_run_bytes) *min_run_bytes = run_bytes;
  // one piece whose run spans the whole tensor: minimal contiguous dimension 1 (Def. 5)
  if (d->pieces.size() == 1 && d->run >= numel) *access_class = VT_ACCESS_FULL;
  else if (run_bytes >= unit_bytes) *access_class = VT_ACCESS_PARTIAL;
  else *access_class = VT_ACCESS_SCATTERED;
  return VT_OK;
}

int vt_desc_piece(const vt_desc* d, int p, int64_t* lo, int64_t* hi, int* src_id, int64_t* run) {
  if (!d || p < 0 || p >= (int)d->pieces.size()) return fail(VT_ERR_INVALID_ARG, "vt_desc_piece: no such piece");
  const Piece& pc = d->pieces[p];
  for (size_t i = 0; i < d->shape.size(); ++i) {
    if (lo) lo[i] = pc.lo[i];
    if (hi) hi[i] = pc.hi[i];
  }
  if (src_id) *src_id = pc.src;
  if (run) *run = pc.run;
  return VT_OK;
}

int vt_eval_host(const vt_desc* d, const int64_t* vindex, int* src_id, int64_t* elem_offset) {
  if (!d || !vindex) return fail(VT_ERR_INVALID_ARG, "vt_eval_host: NULL argument");
  for (size_t i = 0; i < d->shape.size(); ++i)
    if (vindex[i] < 0 || vindex[i] >= d->shape[i]) return fail(VT_ERR_RANGE, "vt_eval_host: index outside the tensor");
  int p = find_piece(*d, vindex);
  if (p < 0) return fail(VT_ERR_RANGE, "vt_eval_host: index not covered by any piece");
  int64_t local[VT_MAX_DIMS];
  for (size_t i = 0; i < d->shape.size(); ++i) local[i] = vindex[i] - d->pieces[p].lo[i];
  if (src_id) *src_id = d->pieces[p].src;
  if (elem_offset) *elem_offset = eval_view(*d, d->pieces[p].v, local);
  return VT_OK;
}

int vt_desc_dump(const vt_desc* d, char* buf, size_t cap) {
  if (!d || !buf || cap == 0) return fail(VT_ERR_INVALID_ARG, "vt_desc_dump: NULL argument");
  std::ostringstream os;
  os << "shape[";
  for (size_t i = 0; i < d->shape.size(); ++i) os << (i ? "," : "") << d->shape[i];
  os << "] dtype=" << d->dtype << " run=" << d->run << " pieces=" << d->pieces.size() << "\n";
  auto dig = [&](const Digit& g) {
    os << "(" << g.radix << "," << g.stride;
    if (g.table >= 0) os << ",T" << g.table << "+" << g.table_off;
    os << ")";
  };
  for (const Piece& p : d->pieces) {
    os << " piece src=" << p.src << " box";
    for (size_t i = 0; i < d->shape.size(); ++i) os << "[" << p.lo[i] << "," << p.hi[i] << ")";
    os << " run=" << p.run << " base=" << p.v.base << " top:";
    for (const auto& g : p.v.groups) {
      os << " {";
      for (const Digit& x : g) dig(x);
      os << "}";
    }
    for (const Stage& s : p.v.lower) {
      os << " | base=" << s.base << " ";
      for (const Digit& x : s.digits) dig(x);
    }
    os << "\n";
  }
  std::string s = os.str();
  size_t n = std::min(cap - 1, s.size());
  memcpy(buf, s.data(), n);
  buf[n] = 0;
  return VT_OK;
}

}  // extern "C"
