// Split-K flash-decoding attention for grouped queries that reads Q, K and V through
// virtual-tensor descriptors (Sec. 3.1: the attention kernel reads the un-expanded cache and
// the freshly projected K/V rows where the producer left them).  gfx950, wave64, MFMA.
//
// Work split: one workgroup per (batch b, kv head g, context split s); WAVES waves share the
// split's rows in tiles of 32.  All G query heads of the group are served from one read of
// K and V (the broadcast digit of the descriptor, i.e. the Expand that is never executed).
// The context is cut into segments at the piece boundaries of the two descriptors (the
// Concat that is never executed).  Inside a segment a row address is one wave-uniform base
// plus a per-lane constant; a tile in which a segment ends continues in the next one with
// per-lane row addresses (so the fresh K/V row behind the cached ones costs no tile of its own).
//
// Per tile of 32 context rows and per wave:
//   S^T = K . Q^T   on v_mfma_f32_16x16x32 (rows = context, cols = the group's heads, padded
//                   to 16).  K rows are fetched with fully coalesced 16-byte loads (16 lanes
//                   per 256-byte row), staged through an XOR-swizzled LDS tile and read back in
//                   the matrix-core operand layout without bank conflicts.
//   softmax         in the accumulator layout (lane = head, 4 rows per 16-row block) against a
//                   reference maximum that is only moved (and the accumulators rescaled) when
//                   a score exceeds it by more than a threshold: the common tile costs one
//                   fma and one exp2 per score and no cross-lane traffic.
//   O^T += V^T . P^T on the same instruction.  V never touches LDS: each lane loads 8 rows of
//                   its own 8-column chunk (again whole rows per 16 lanes), transposes the 8x8
//                   block inside its registers (v_perm_b32) and feeds it as the A operand;
//                   the contraction index is permuted identically for P, which the softmax
//                   already holds in exactly that layout.
// The workgroup that finishes last for a (b, g) merges the splits' partial results (a ticket
// counter per (b, g) in the workspace; no second launch, no spinning).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstddef>
#include <cstring>
#include <mutex>
#include <numeric>
#include <string>

#include "vt_coherent.h"
#include "vt_kernarg.h"
#include "vt_device.h"
#include "vt_numeric.h"
#include "vt_profile.h"

using namespace vt;

// profile marks: 0 start, 1 first K tile staged, 2 tile loop done (all waves), 3 partial results
// stored, 4 ticket taken, 5 merge written, 6 merge loads landed, 7 compute die
VT_PROF_DECLARE(attn)
#define ATTN_WG (blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z))

namespace {

constexpr int kD = 128;          // head dim
constexpr int kTile = 32;        // context rows per wave step
constexpr int kMaxAttnPieces = 4;
constexpr int kMaxSegs = 8;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// A stretch of the context [t_lo, t_hi) in which K rows come from one source region and V
// rows from one source region (the union of the piece boundaries of the two descriptors).
// An operand whose rows sit in pages picked through an index table (paged KV cache: the map has
// table digit, Sec. 4.1 / the table-driven part of b(I) in Eq. 1).  With (batch b, stored head
// h, page pg, row-in-page o):
//   L = L0 + b Lb + h Lh + pg Lp + o Lo          (what the table digit and its stage see)
//   X = X0 + b Xb + h Xh + o Xo                  (strided terms outside the table's stage)
//   element offset = tab[L / W] * ps + L % W + X
// Two-stage form (the table dim was reshaped: the top stage builds a linear index that the second
// stage cuts into table entry and remainder): X terms are 0 except X0 = the second stage's base.
// One-stage form (the table digit sits in the context group itself): L = pg, W = 1.
struct PagedOperand {
  const int32_t* tab;    // NULL: the operand is not paged in this segment
  int64_t L0, Lb, Lh, Lp, Lo;
  int64_t X0, Xb, Xh, Xo;
  int64_t ps;
  FastDiv W, page;       // elements per table entry; rows per page (a multiple of 32, or the whole segment)
};

// (what every tile walk reads comes first, in 72 bytes: two lines of the kernel arguments at most)
struct AttnSeg {
  int32_t t_lo, t_hi;
  int32_t paged;         // bit 0: K is paged in this segment, bit 1: V is
  int32_t k_hdiv, v_hdiv;           // head group g reads stored head g / hdiv (1 unless this operand is
                                    // broadcast over more heads than the group size G both operands share)
  uint32_t k_st, v_st;              // bytes per context row
  int32_t pad;
  const char* k;         // K element (b=0, g=0, t=t_lo, d=0); for a paged operand: element 0 of its source
  const char* v;
  int64_t k_sb, k_sh, v_sb, v_sh;   // bytes per batch / per stored head
  PagedOperand kp, vp;
};
struct AttnParams {
  AttnSeg seg[kMaxSegs];
  int32_t n_seg;
  const char* q_ptr;
  int64_t q_sb, q_sh;    // bytes
  int32_t B, Hkv, G, S, n_splits, rows_per_split;
  float scale_log2;      // softmax scale * log2(e)
  uint32_t* tickets;     // [B, Hkv], zero between launches
  float* ws_ml;          // [B, Hkv, n_splits, G, 2]
  float* ws_o;           // [B, Hkv, n_splits, G, D]
  void* out;             // [B, Hq, D]
  float* lse;            // [B, Hq] or NULL
};

template <typename T>
struct Mfma;
template <>
struct Mfma<bf16_t> {
  typedef bf16x8 vec;
  static constexpr float kThreshold = 16.0f;   // p <= 2^16: far inside the bf16 exponent range
  static __device__ __forceinline__ f32x4 run(vec a, vec b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
  }
};
template <>
struct Mfma<f16_t> {
  typedef f16x8 vec;
  static constexpr float kThreshold = 0.0f;    // keep p <= 1 (f16 tops out at 65504)
  static __device__ __forceinline__ f32x4 run(vec a, vec b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
  }
};

struct Regs16 {
  uint32_t w[4];
};

// K and V rows are read exactly once per launch: streaming (nontemporal) loads keep them from
// displacing each other in the caches (measured: 29.6 -> 26.9 us on the benchmark's decode step).
__device__ __forceinline__ Regs16 load16(const char* base, uint32_t off) {
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + off));
  Regs16 r;
  r.w[0] = t[0]; r.w[1] = t[1]; r.w[2] = t[2]; r.w[3] = t[3];
  return r;
}

// The 32-row tiles of a split [t_begin, t_end) are taken one after the other.  A tile lies in one
// segment, or - where a segment ends inside it - continues into the next one (rows >= cut come
// from there): the fresh K/V row appended behind 4095 cached rows then costs no extra tile.
// Tiles do not continue across a boundary with a paged operand (a tile has one page).  All
// values are wave-uniform.
struct TileWalk {
  const char* k;         // K row t_lo of this (b, g) in the tile's (first) segment
  const char* v;
  uint32_t k_st, v_st;   // bytes per context row
  int t_lo;              // first row of that segment
  int r0, end;           // the tile: rows [r0, end), at most 32
  int seg_end;           // end of the tile's (first) segment, clipped to the split
  int seg;               // its (first) segment, P.n_seg when the walk is over
  int paged;             // that segment's paged bits
  int cut, seg2;         // rows >= cut belong to segment seg2 (cut = INT_MAX, seg2 = -1: one segment only)
  const char* k2;        // K row `cut` of this (b, g) in segment seg2
  const char* v2;
  uint32_t k2_st, v2_st;
};

// One table entry, read on the scalar unit (the table is read-only for the kernel; a vector
// load would queue behind the K/V rows already in flight).
__device__ __forceinline__ int32_t table_entry(const int32_t* tab, uint32_t idx) {
  // table and index are wave-uniform by construction; readfirstlane states it, so that the scalar
  // operands below do not depend on what the compiler's uniformity analysis can prove
  const uint64_t t = reinterpret_cast<uint64_t>(tab);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)t), hi = __builtin_amdgcn_readfirstlane((uint32_t)(t >> 32));
  const int32_t* utab = reinterpret_cast<const int32_t*>(((uint64_t)hi << 32) | lo);
  const uint32_t off = __builtin_amdgcn_readfirstlane(idx * 4u);
  int32_t v;
  asm volatile("s_load_dword %0, %1, %2\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(utab), "s"(off) : "memory");
  return v;
}

// Pointer p such that p + (r0 - t_lo) * st is row r0 of this (b, g): the form the loads use.
__device__ __forceinline__ const char* paged_base(const PagedOperand& o, const char* src, uint32_t st, int b, int h, int rel) {
  const uint32_t pg = fdiv((uint32_t)rel, o.page);
  const int64_t row = rel - (int)(pg * o.page.d);
  const int64_t L = o.L0 + b * o.Lb + h * o.Lh + (int64_t)pg * o.Lp + row * o.Lo;
  const int64_t X = o.X0 + b * o.Xb + h * o.Xh + row * o.Xo;
  const uint32_t j = fdiv((uint32_t)L, o.W);
  const int64_t off = (int64_t)table_entry(o.tab, j) * o.ps + (L - (int64_t)j * o.W.d) + X;
  return src + off * 2 - (int64_t)rel * st;
}

// the tile at w.r0 moved: paged operands look their page up again
__device__ __forceinline__ void walk_locate(const AttnParams& P, TileWalk& w, int b, int g) {
  const AttnSeg& sg = P.seg[w.seg];
  if (w.paged & 1) w.k = paged_base(sg.kp, sg.k, sg.k_st, b, g / sg.k_hdiv, w.r0 - sg.t_lo);
  if (w.paged & 2) w.v = paged_base(sg.vp, sg.v, sg.v_st, b, g / sg.v_hdiv, w.r0 - sg.t_lo);
}

// The tile that starts at row r0 of segment seg (r0 inside the segment and the split).
__device__ __forceinline__ void walk_place(const AttnParams& P, TileWalk& w, int seg, int r0, int t_end) {
  w.seg = seg;
  w.r0 = r0;
  w.cut = 0x7fffffff;
  w.seg2 = -1;
  const int seg_end = min(P.seg[seg].t_hi, t_end);
  w.paged = P.seg[seg].paged;
  w.seg_end = seg_end;
  w.end = min(r0 + kTile, seg_end);
  if (w.end < r0 + kTile && seg_end < t_end && seg + 1 < P.n_seg) {
    const AttnSeg& B = P.seg[seg + 1];
    if ((w.paged | B.paged) == 0) {
      w.cut = seg_end;
      w.seg2 = seg + 1;
      w.end = min(r0 + kTile, min(B.t_hi, t_end));
    }
  }
}

// The tile after the current one; w.seg = P.n_seg when there is none.
__device__ __forceinline__ void walk_next(const AttnParams& P, TileWalk& w, int t_end) {
  const int r0 = w.end;
  int seg = w.seg2 >= 0 ? w.seg2 : w.seg;
  while (seg < P.n_seg && r0 >= min(P.seg[seg].t_hi, t_end)) ++seg;
  if (seg >= P.n_seg || r0 >= t_end) {
    w.seg = P.n_seg;
    return;
  }
  walk_place(P, w, seg, r0, t_end);
}

// Row pointers and pitches of the tile that walk_place / walk_next chose.
__device__ __forceinline__ void walk_fetch(const AttnParams& P, TileWalk& w, int b, int g) {
  const AttnSeg& sg = P.seg[w.seg];
  w.k = sg.k + b * sg.k_sb + (g / sg.k_hdiv) * sg.k_sh;
  w.v = sg.v + b * sg.v_sb + (g / sg.v_hdiv) * sg.v_sh;
  w.k_st = sg.k_st;
  w.v_st = sg.v_st;
  w.t_lo = sg.t_lo;
  if (w.paged) walk_locate(P, w, b, g);
  if (w.seg2 >= 0) {
    const AttnSeg& s2 = P.seg[w.seg2];
    w.k2 = s2.k + b * s2.k_sb + (g / s2.k_hdiv) * s2.k_sh + (int64_t)(w.cut - s2.t_lo) * s2.k_st;
    w.v2 = s2.v + b * s2.v_sb + (g / s2.v_hdiv) * s2.v_sh + (int64_t)(w.cut - s2.t_lo) * s2.v_st;
    w.k2_st = s2.k_st;
    w.v2_st = s2.v_st;
  }
}

// n tiles forward (n >= 0), then the pointers of the tile reached
__device__ __forceinline__ void walk_advance(const AttnParams& P, TileWalk& w, int n, int b, int g, int t_end) {
  if (w.seg >= P.n_seg) return;
  const bool fetched = n > 0 && w.k != nullptr;
  if (w.seg2 < 0 && w.r0 + kTile * (n + 1) <= w.seg_end) {
    // the usual case: n full tiles further inside the same segment
    w.r0 += kTile * n;
    w.end = w.r0 + kTile;
    if (fetched) {                       // same segment: only a paged operand has to look its page up again
      if (w.paged) walk_locate(P, w, b, g);
      return;
    }
  } else {
    for (int i = 0; i < n && w.seg < P.n_seg; ++i) walk_next(P, w, t_end);
  }
  if (w.seg < P.n_seg) walk_fetch(P, w, b, g);
}

template <typename T, int WAVES, int OCC>
__global__ void __launch_bounds__(WAVES * 64) __attribute__((amdgpu_waves_per_eu(OCC, OCC)))
k_decode_attn(const AttnParams P) {
  typedef Mfma<T> M;
  typedef typename M::vec opvec;
  __shared__ uint4 lds[WAVES][kTile * 16];   // per wave: 32 rows x 16 chunks of 16 bytes, swizzled
  __shared__ float red_ml[WAVES * 16 * 2];   // [WAVES][16][2]
  __shared__ uint32_t ticket_sh;

  // the tile walk below reads the segment table with data-dependent indices: have its first lines
  // (three segments) and the scalars behind the table in the scalar cache before the chain of
  // dependent reads starts
  static_assert(offsetof(AttnParams, n_seg) >= 1024 && offsetof(AttnParams, n_seg) / 64 * 64 + 68 <= sizeof(AttnParams),
                "the warmed lines lie inside the arguments");
  warm_kernarg_16_and_2(offsetof(AttnParams, n_seg) / 64 * 64);
  VT_PROF_BEGIN();
  VT_PROF(0);
  const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int l16 = lane & 15, lg = lane >> 4;
  const int t_begin = split * P.rows_per_split;
  const int t_end = min(P.S, t_begin + P.rows_per_split);
  const float c = P.scale_log2;

  // Q^T operand: lane (head l16, k-group lg) holds 8 consecutive d for each of the 4 k-steps
  opvec qreg[4];
  {
    const char* qp = P.q_ptr + b * P.q_sb + (int64_t)(g * P.G + l16) * P.q_sh;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      uint4 raw = make_uint4(0, 0, 0, 0);
      if (l16 < P.G) raw = *reinterpret_cast<const uint4*>(qp + (kk * 32 + lg * 8) * 2);
      qreg[kk] = __builtin_bit_cast(opvec, raw);
    }
  }

  float m_ref = -1.0e30f;   // reference maximum (log2 domain) of head l16, identical in the 4 lane groups
  float l_run = 0.0f;       // this lane's share of the denominator, relative to m_ref
  f32x4 acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = f32x4{0.f, 0.f, 0.f, 0.f};

  // Loads of one tile.  K: instruction j covers rows 4j..4j+3 (16 lanes per 256-byte row);
  // V: instruction j is contraction slot j of the lane group, row (j>>2)*16 + lg*4 + (j&3).
  // In a full tile the address is a wave-uniform base per instruction plus ONE per-lane
  // offset; a partial tile (last of a segment) clamps its rows onto the last valid one.
  Regs16 kst[8], vst[8];
  auto issue_k = [&](const TileWalk& tp) {
    const uint32_t st = tp.k_st;
    const char* kb = tp.k + (int64_t)(tp.r0 - tp.t_lo) * st;
    if (tp.r0 + kTile <= tp.end && tp.seg2 < 0) {
      const uint32_t off = lg * st + l16 * 16;
#pragma unroll
      for (int j = 0; j < 8; ++j) kst[j] = load16(kb + (size_t)(4 * j) * st, off);
    } else {
      // a short tile (rows past its end repeat the last valid one) or one that continues in the
      // next segment: per-lane row addresses
      const int span = tp.end - 1 - tp.r0, ncut = tp.cut - tp.r0;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int rr = min(4 * j + lg, span);
        const bool in2 = rr >= ncut;
        kst[j] = load16(in2 ? tp.k2 : kb, (in2 ? (uint32_t)(rr - ncut) * tp.k2_st : (uint32_t)rr * st) + l16 * 16);
      }
    }
  };
  auto issue_v = [&](const TileWalk& tp) {
    const uint32_t st = tp.v_st;
    const char* vb = tp.v + (int64_t)(tp.r0 - tp.t_lo) * st;
    if (tp.r0 + kTile <= tp.end && tp.seg2 < 0) {
      const uint32_t off = lg * 4 * st + l16 * 16;
#pragma unroll
      for (int j = 0; j < 8; ++j) vst[j] = load16(vb + (size_t)((j >> 2) * 16 + (j & 3)) * st, off);
    } else {
      const int span = tp.end - 1 - tp.r0, ncut = tp.cut - tp.r0;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int rr = min((j >> 2) * 16 + lg * 4 + (j & 3), span);
        const bool in2 = rr >= ncut;
        vst[j] = load16(in2 ? tp.v2 : vb, (in2 ? (uint32_t)(rr - ncut) * tp.v2_st : (uint32_t)rr * st) + l16 * 16);
      }
    }
  };

  uint4* my_lds = lds[wave];
  // this wave's tiles: wave, wave + WAVES, ... of the split
  TileWalk cur;
  {
    int seg0 = 0;
    while (seg0 < P.n_seg && t_begin >= min(P.seg[seg0].t_hi, t_end)) ++seg0;
    cur.seg = P.n_seg;
    cur.k = nullptr;                     // pointers not fetched yet
    if (seg0 < P.n_seg && t_begin < t_end) walk_place(P, cur, seg0, t_begin, t_end);
  }
  walk_advance(P, cur, wave, b, g, t_end);
  if (cur.seg < P.n_seg) {
    issue_k(cur);
    issue_v(cur);
  }
  while (cur.seg < P.n_seg) {
    const int r0 = cur.r0, r_end = cur.end;
    const bool partial = r0 + kTile > r_end;
    walk_advance(P, cur, WAVES, b, g, t_end);              // cur is now the next tile of this wave
    const bool more = cur.seg < P.n_seg;
    // ---- stage K through LDS (swizzle: chunk c of row r sits at unit c ^ (r & 15))
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      int r = 4 * j + lg;
      my_lds[r * 16 + (l16 ^ (r & 15))] = make_uint4(kst[j].w[0], kst[j].w[1], kst[j].w[2], kst[j].w[3]);
    }
    VT_PROF_ONCE(1);
    if (more) issue_k(cur);              // next tile's K is in flight during this tile's math

    // ---- S^T = K . Q^T : two 16-row blocks, 4 k-steps each
    f32x4 s[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      s[u] = f32x4{0.f, 0.f, 0.f, 0.f};
      int r = u * 16 + l16;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        uint4 raw = my_lds[r * 16 + ((kk * 4 + lg) ^ l16)];
        s[u] = M::run(__builtin_bit_cast(opvec, raw), qreg[kk], s[u]);
      }
    }
    // ---- softmax; lane holds head l16 and rows r0 + (j>>2)*16 + lg*4 + (j&3), j = 0..7
    float sv[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) sv[j] = s[j >> 2][j & 3];
    if (partial) {
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (r0 + (j >> 2) * 16 + lg * 4 + (j & 3) >= r_end) sv[j] = -3.0e38f;
    }
    float tmax = fmaxf(fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])), fmaxf(fmaxf(sv[4], sv[5]), fmaxf(sv[6], sv[7])));
    tmax = fmaxf(tmax * c, -1.0e30f);
    if (__builtin_amdgcn_ballot_w64(tmax > m_ref + M::kThreshold) != 0) {
      // move the reference maximum of every head to its new maximum and rescale what was
      // accumulated against the old one (rare after the first tiles)
      float mn = fmaxf(m_ref, tmax);
      mn = fmaxf(mn, __shfl_xor(mn, 16, 64));
      mn = fmaxf(mn, __shfl_xor(mn, 32, 64));
      const float alpha = __builtin_amdgcn_exp2f(m_ref - mn);
      m_ref = mn;
      l_run *= alpha;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        acc[e][0] *= alpha; acc[e][1] *= alpha; acc[e][2] *= alpha; acc[e][3] *= alpha;
      }
    }
    float pv[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) pv[j] = __builtin_amdgcn_exp2f(fmaf(sv[j], c, -m_ref));   // masked rows: exp2(-huge) = 0
    l_run += ((pv[0] + pv[1]) + (pv[2] + pv[3])) + ((pv[4] + pv[5]) + (pv[6] + pv[7]));
    uint4 praw = make_uint4(M::pack2(pv[0], pv[1]), M::pack2(pv[2], pv[3]), M::pack2(pv[4], pv[5]),
                            M::pack2(pv[6], pv[7]));
    const opvec pop = __builtin_bit_cast(opvec, praw);
    // ---- O^T += V^T . P^T : transpose the lane's 8x8 block, one MFMA per column e
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
      uint32_t w[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) w[u] = __builtin_amdgcn_perm(vst[2 * u + 1].w[e >> 1], vst[2 * u].w[e >> 1], sel);
      uint4 traw = make_uint4(w[0], w[1], w[2], w[3]);
      acc[e] = M::run(__builtin_bit_cast(opvec, traw), pop, acc[e]);
    }
    if (more) issue_v(cur);              // next tile's V: lands while the next K tile is being scored
  }

  // Everything the rest of the kernel needs from the arguments is fetched here, in one batch, and
  // pinned in registers (the empty statement makes the values opaque, so they cannot be fetched
  // again later): the steps below are a chain of round trips to memory, and a reload of a pointer
  // from the argument segment in front of each of them would lengthen every link.
  uint32_t* a_tickets = P.tickets;
  float* a_ws_ml = P.ws_ml;
  float* a_ws_o = P.ws_o;
  T* a_out = static_cast<T*>(P.out);
  float* a_lse = P.lse;
  int a_G = P.G, a_ns = P.n_splits, a_Hkv = P.Hkv;
  asm volatile("" : "+s"(a_tickets), "+s"(a_ws_ml), "+s"(a_ws_o), "+s"(a_out), "+s"(a_lse), "+s"(a_G), "+s"(a_ns), "+s"(a_Hkv));

  // ---- merge the waves of the workgroup through LDS, then write the split's partial result
  l_run += __shfl_xor(l_run, 16, 64);
  l_run += __shfl_xor(l_run, 32, 64);
  __syncthreads();                       // every wave is done with its K tile
  VT_PROF(2);
  float* red_o = reinterpret_cast<float*>(&lds[0][0]);    // [WAVES][G][D] floats: at most the K tiles' 32 KB
  const int G = a_G;
  if (l16 < G) {
#pragma unroll
    for (int e = 0; e < 8; ++e)
#pragma unroll
      for (int i = 0; i < 4; ++i) red_o[(wave * G + l16) * kD + (lg * 4 + i) * 8 + e] = acc[e][i];
    if (lg == 0) {
      red_ml[(wave * 16 + l16) * 2 + 0] = m_ref;
      red_ml[(wave * 16 + l16) * 2 + 1] = l_run;
    }
  }
  __syncthreads();
  const int bg = b * a_Hkv + g;
  const size_t unit = (size_t)bg * a_ns + split;
  // four consecutive d per thread; partial results go out as 16-byte device-coherent stores
  // (written through to where every compute die sees them), whole cache lines per wave
  for (int idx = threadIdx.x * 4; idx < G * kD; idx += WAVES * 64 * 4) {
    const int h = idx / kD;
    float mx = -1.0e30f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) mx = fmaxf(mx, red_ml[(w * 16 + h) * 2]);
    float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
    float l = 0.f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
      const float sc = __builtin_amdgcn_exp2f(red_ml[(w * 16 + h) * 2] - mx);
      const float4 r = *reinterpret_cast<const float4*>(&red_o[(w * G + h) * kD + (idx - h * kD)]);
      o.x += r.x * sc; o.y += r.y * sc; o.z += r.z * sc; o.w += r.w * sc;
      l += red_ml[(w * 16 + h) * 2 + 1] * sc;
    }
    store_device_b128(&a_ws_o[unit * G * kD + idx], __builtin_bit_cast(u32x4_t, o));
    if (idx == h * kD) {
      __hip_atomic_store(&a_ws_ml[(unit * G + h) * 2 + 0], mx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(&a_ws_ml[(unit * G + h) * 2 + 1], l, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }

  // ---- the last workgroup of this (b, g) to arrive merges the splits.  The barrier waits for
  // every wave's stores to complete before one thread takes the ticket (a device-scope atomic);
  // the merging workgroup reads the partial results with device-scope atomic loads, which do
  // not hit stale cache lines.  atomicInc wraps to 0 at n_splits - 1, which leaves the counter
  // ready for the next launch.  No wave ever waits for another workgroup.
  __builtin_amdgcn_s_waitcnt(0);         // this wave's stores have completed (vmcnt = 0)
  __syncthreads();
  VT_PROF(3);
  if (threadIdx.x == 0) ticket_sh = atomicInc(&a_tickets[bg], (uint32_t)(a_ns - 1));
  __syncthreads();
  VT_PROF(4);
  if (ticket_sh != (uint32_t)(a_ns - 1)) {
    VT_PROF_FLUSH(attn, ATTN_WG);
    return;
  }
  const size_t u0 = (size_t)bg * a_ns;
  const int ns = a_ns;
  T* out = a_out;
  auto ld = [](const float* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); };
  // (m, l) of every split and head go to LDS (ns * G * 2 contiguous floats; the K tiles' LDS is
  // free now).  Each thread merges four consecutive d of one head; the first eight splits'
  // partial outputs are requested in the same breath as (m, l), with 16-byte device-coherent
  // loads, so that the merge costs one memory round trip, not two.
  float* ml_sh = reinterpret_cast<float*>(&lds[0][0]);
  const int idx0 = threadIdx.x * 4;                   // G * kD / 4 >= 32 threads are busy; the rest idle through
  const int h0 = min(idx0 / kD, G - 1), d0 = idx0 % kD;
  const int i_ml = threadIdx.x;                       // ns * G * 2 <= 256 * 32 ... a thread may own several
  float ml_first = 0.f;
  if (i_ml < ns * G * 2) ml_first = ld(&a_ws_ml[u0 * G * 2 + i_ml]);
  u32x4_t v0[8];
  {
    const void* q[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) q[u] = &a_ws_o[((u0 + min(u, ns - 1)) * G + h0) * kD + d0];
    load_device_8xb128(q, v0);
  }
  VT_PROF(6);
  if (i_ml < ns * G * 2) ml_sh[i_ml] = ml_first;
  for (int i = i_ml + WAVES * 64; i < ns * G * 2; i += WAVES * 64) ml_sh[i] = ld(&a_ws_ml[u0 * G * 2 + i]);
  __syncthreads();
  for (int idx = idx0; idx < G * kD; idx += WAVES * 64 * 4) {
    const int h = idx / kD, d = idx - h * kD;
    float mx = -1.0e30f;
    for (int sp = 0; sp < ns; ++sp) mx = fmaxf(mx, ml_sh[(sp * G + h) * 2]);
    float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
    float l = 0.f;
    for (int sp0 = 0; sp0 < ns; sp0 += 8) {
      u32x4_t v[8];
      if (idx == idx0 && sp0 == 0) {
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = v0[u];
      } else {
        const void* q[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) q[u] = &a_ws_o[((u0 + min(sp0 + u, ns - 1)) * G + h) * kD + d];
        load_device_8xb128(q, v);
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (sp0 + u < ns) {
          const float sc = __builtin_amdgcn_exp2f(ml_sh[((sp0 + u) * G + h) * 2] - mx);
          const float4 r = __builtin_bit_cast(float4, v[u]);
          o.x += r.x * sc; o.y += r.y * sc; o.z += r.z * sc; o.w += r.w * sc;
          l += ml_sh[((sp0 + u) * G + h) * 2 + 1] * sc;
        }
      }
    }
    const size_t hq = (size_t)bg * G + h;      // = b * Hq + g * G + h
    Vec<T, 4> r;
    r.v[0] = from_float<T>(o.x / l); r.v[1] = from_float<T>(o.y / l);
    r.v[2] = from_float<T>(o.z / l); r.v[3] = from_float<T>(o.w / l);
    *reinterpret_cast<Vec<T, 4>*>(&out[hq * kD + d]) = r;
    if (a_lse && d == 0) a_lse[hq] = (mx + log2f(l)) * 0.6931471805599453f;
  }
#ifdef VT_PROFILE
  __builtin_amdgcn_s_waitcnt(0);
  VT_PROF(5);
  VT_PROF_FLUSH(attn, ATTN_WG);
#endif
}

// ------------------------------------------------------------------------------------------
// The same attention for ANY maps the descriptors can hold and any head dim (tables anywhere,
// stacked index stages, pieces along any dim, rows that are not contiguous): every element of Q,
// K and V is found through the generic evaluator.  One workgroup per (batch, query head) walks the
// context in chunks of 256 keys with a running maximum and sum (fp32); thread t scores key t of
// the chunk, then thread d accumulates output column d.  Correct for every representable chain,
// and slow: the kernel above takes over whenever the maps have the form it plans for.
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) k_decode_attn_generic(const DevDesc Q_, const DevDesc K_, const DevDesc V_, T* __restrict__ out,
                                                             float* __restrict__ lse, int Hq, int S, int D, float scale) {
  __shared__ float p_sh[256];
  __shared__ float red[256];
  __shared__ DevDesc maps[3];                        // the evaluator reads the maps from LDS
  {
    const DevDesc* const from[3] = {&Q_, &K_, &V_};
    stage_maps(maps, from);
  }
  const DevDesc& Q = maps[0];
  const DevDesc& K = maps[1];
  const DevDesc& V = maps[2];
  const int h = blockIdx.x, b = blockIdx.y, t = threadIdx.x;
  const uint32_t q_lin = (uint32_t)(b * Hq + h) * (uint32_t)D;              // [B,Hq,1,D]
  const uint32_t kv_lin = (uint32_t)(b * Hq + h) * (uint32_t)S * (uint32_t)D;   // [B,Hq,S,D]
  auto at = [](const DevDesc& X, uint32_t lin) {
    int64_t off;
    const void* ptr;
    vtd_eval(X, 0, lin, &off, &ptr);
    return to_float(static_cast<const T*>(ptr)[off]);
  };
  float m_run = -3.0e38f, l_run = 0.f;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};             // output columns t, t + 256, ... (D <= 1024)
  for (int t0 = 0; t0 < S; t0 += 256) {
    const int key = t0 + t;
    float sc = -3.0e38f;
    if (key < S) {
      sc = 0.f;
      for (int d = 0; d < D; ++d) sc += at(Q, q_lin + d) * at(K, kv_lin + (uint32_t)key * D + d);
      sc *= scale;
    }
    red[t] = sc;
    __syncthreads();
    for (int w = 128; w >= 1; w >>= 1) {
      if (t < w) red[t] = fmaxf(red[t], red[t + w]);
      __syncthreads();
    }
    const float m_new = fmaxf(m_run, red[0]);
    __syncthreads();
    const float alpha = __expf(m_run - m_new), pv = key < S ? __expf(sc - m_new) : 0.f;
    p_sh[t] = pv;
    red[t] = pv;
    __syncthreads();
    for (int w = 128; w >= 1; w >>= 1) {
      if (t < w) red[t] += red[t + w];
      __syncthreads();
    }
    l_run = l_run * alpha + red[0];
    m_run = m_new;
    const int n_keys = min(256, S - t0);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int d = t + 256 * c;
      if (d < D) {
        float a = acc[c] * alpha;
        for (int j = 0; j < n_keys; ++j) a += p_sh[j] * at(V, kv_lin + (uint32_t)(t0 + j) * D + d);
        acc[c] = a;
      }
    }
    __syncthreads();
  }
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const int d = t + 256 * c;
    if (d < D) out[(size_t)(b * Hq + h) * D + d] = from_float<T>(acc[c] / l_run);
  }
  if (lse && t == 0) lse[b * Hq + h] = m_run + __logf(l_run);
}

__global__ void k_zero_words(uint32_t* p, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
}

// ---------------------------------------------------------------- host: descriptor -> plan
struct HeadMap {
  int64_t stride;   // elements per kv head
  int64_t G;        // query heads per kv head (trailing broadcast digits)
};

// A digit group that acts as ONE strided digit: a single plain digit, or several that nest
// densely (each stride = the next stride x the next radix, as a reshape of a dense buffer
// leaves them).
bool single_plain(const std::vector<Digit>& g, int64_t* stride) {
  if (g.empty()) {
    *stride = 0;
    return true;
  }
  for (size_t i = 0; i < g.size(); ++i) {
    if (g[i].table >= 0) return false;
    if (i + 1 < g.size() && g[i].stride != g[i + 1].stride * g[i + 1].radix) return false;
  }
  *stride = g.back().stride;
  return true;
}

// Trailing zero-stride digits of the head group = heads that share rows.
int64_t broadcast_factor(const std::vector<Digit>& g) {
  int64_t f = 1;
  for (int k = (int)g.size() - 1; k >= 0 && g[k].stride == 0 && g[k].table < 0; --k) f *= g[k].radix;
  return f;
}

struct PlanPiece {
  const char* ptr;
  int64_t sb, sh;
  int32_t hdiv;
  uint32_t st;
  int32_t t_lo, t_hi;
  PagedOperand pg;       // pg.tab != NULL: rows through a page table (ptr is then element 0 of the source)
  int64_t page_rows;
};
struct AttnOperand {
  PlanPiece pc[kMaxAttnPieces];
  int n;
};

int plan_operand(const vt_desc& d, const char* name, int64_t G, AttnOperand* out) {
  const int esz = 2;
  if (d.pieces.size() > (size_t)kMaxAttnPieces) return fail(VT_ERR_UNSUPPORTED, std::string(name) + ": more than 4 pieces along the context");
  std::vector<const Piece*> ps;
  for (const Piece& p : d.pieces) ps.push_back(&p);
  std::sort(ps.begin(), ps.end(), [](const Piece* a, const Piece* b) { return a->lo[2] < b->lo[2]; });
  int64_t expect = 0;
  out->n = (int)ps.size();
  for (size_t i = 0; i < ps.size(); ++i) {
    const Piece& p = *ps[i];
    for (int dim : {0, 1, 3})
      if (p.lo[dim] != 0 || p.hi[dim] != d.shape[dim]) return fail(VT_ERR_UNSUPPORTED, std::string(name) + ": pieces must split the context dim only");
    if (p.lo[2] != expect) return fail(VT_ERR_UNSUPPORTED, std::string(name) + ": pieces do not tile the context");
    expect = p.hi[2];
    if (p.v.lower.size() > 1) return fail(VT_ERR_UNSUPPORTED, std::string(name) + ": more than two index stages");
    const bool two_stage = p.v.lower.size() == 1;
    bool paged = two_stage;
    const Digit* ctx_table = nullptr;      // one-stage paged form: the table digit in the context group
    int64_t sb, st, sd, lp = 0, page_rows = p.hi[2] - p.lo[2];
    if (!single_plain(p.v.groups[0], &sb) || !single_plain(p.v.groups[3], &sd))
      return fail(VT_ERR_UNSUPPORTED, std::string(name) + ": batch and feature dims must each be one strided digit");
    if (!single_plain(p.v.groups[2], &st)) {
      // a paged context: [pages] x [rows of a page (stride st)]
      const std::vector<Digit>& cg = p.v.groups[2];
      if (cg.size() != 2 || cg[1].table >= 0 || (cg[0].table >= 0) == two_stage)
        return fail(VT_ERR_UNSUPPORTED, std::string(name) + ": the context dim must be one strided digit (or pages x rows under a page table)");
      if (cg[0].table >= 0) ctx_table = &cg[0];
      paged = true;
      lp = cg[0].stride;
      page_rows = cg[1].radix;
      st = cg[1].stride;
    }
    if (sd != 1) return fail(VT_ERR_UNSUPPORTED, std::string(name) + ": rows must be contiguous along the head dim");
    // head group: [kv heads (stride sh)] x [G broadcast]
    std::vector<Digit> hg = p.v.groups[1];
    int32_t a_hdiv = 1;
    int64_t left = G;
    while (left > 1) {
      if (hg.empty() || hg.back().stride != 0 || hg.back().table >= 0 || (left % hg.back().radix != 0 && hg.back().radix % left != 0))
        return fail(VT_ERR_UNSUPPORTED, std::string(name) + ": head broadcast structure not recognised");
      if (hg.back().radix <= left) {
        left /= hg.back().radix;
        hg.pop_back();
      } else {
        hg.back().radix /= left;
        left = 1;
      }
    }
    // heads this operand still shares beyond G (the other operand is broadcast less, or not at
    // all: the group size is the factor common to both): consecutive groups read one stored head
    int64_t hdiv = 1;
    while (!hg.empty() && hg.back().stride == 0 && hg.back().table < 0) {
      hdiv *= hg.back().radix;
      hg.pop_back();
    }
    if (hdiv >= (1ll << 31)) return fail(VT_ERR_UNSUPPORTED, std::string(name) + ": head broadcast too wide");
    a_hdiv = (int32_t)hdiv;
    int64_t sh;
    if (!single_plain(hg, &sh)) return fail(VT_ERR_UNSUPPORTED, std::string(name) + ": kv-head dim must be one strided digit");
    const vt_source& src = d.sources[p.src];
    if (!src.ptr) return fail(VT_ERR_INVALID_ARG, std::string(name) + ": source without a device pointer");
    PlanPiece& a = out->pc[i];
    memset(&a.pg, 0, sizeof(a.pg));
    a.page_rows = page_rows;
    a.hdiv = a_hdiv;
    a.ptr = static_cast<const char*>(src.ptr) + p.v.base * esz;
    a.sb = sb * esz;
    a.sh = sh * esz;
    if (paged) {
      const int64_t rows = p.hi[2] - p.lo[2];
      const Digit* T = ctx_table;
      int64_t W = 1;
      if (two_stage) {
        // second stage: one table digit, then digits that together are the identity on [0, W)
        const Stage& lo = p.v.lower[0];
        if (lo.digits.empty() || lo.digits[0].table < 0) return fail(VT_ERR_UNSUPPORTED, std::string(name) + ": second index stage without a leading table digit");
        for (size_t k = lo.digits.size(); k-- > 1;) {
          if (lo.digits[k].table >= 0 || lo.digits[k].stride != W) return fail(VT_ERR_UNSUPPORTED, std::string(name) + ": second index stage must be a page table over dense pages");
          W *= lo.digits[k].radix;
        }
        T = &lo.digits[0];
        // a context dim that is ONE digit of the top stage (one kv head per page: page stride =
        // rows x row stride) still walks through the table: W / st rows per entry
        if (lp == 0 && st > 0 && W % st == 0 && W / st < rows) {
          page_rows = W / st;
          lp = W;
        }
        // No carries: the table entry must depend only on digits whose stride is a multiple of W,
        // and everything else must add up to less than W - then the rows of a page are equally
        // spaced in the source, which is what a tile relies on.
        int64_t sub = p.v.base % W + (page_rows - 1) * st + d.shape[3];
        if (sb % W) sub += (d.shape[0] - 1) * sb;
        if (sh % W) sub += (d.shape[1] / (G * a_hdiv) - 1) * sh;
        if (lp % W || sub > W) return fail(VT_ERR_UNSUPPORTED, std::string(name) + ": paged map: rows of a page are not equally spaced in the source");
        int64_t span = p.v.base;     // largest value of the top stage: must stay a 31-bit index
        for (const auto& grp : p.v.groups)
          for (const Digit& g : grp) span += (g.radix - 1) * (g.stride > 0 ? g.stride : 0);
        if (span >= (1ll << 31) || W >= (1ll << 31)) return fail(VT_ERR_UNSUPPORTED, std::string(name) + ": paged index space too large");
        if (p.v.base % 8 || lp % 8 || W % 8 || lo.base % 8) return fail(VT_ERR_UNSUPPORTED, std::string(name) + ": paged rows are not 16-byte aligned");
        a.pg.L0 = p.v.base; a.pg.Lb = sb; a.pg.Lh = sh; a.pg.Lp = lp; a.pg.Lo = st;
        a.pg.X0 = lo.base;
      } else {
        if (p.v.base % 8) return fail(VT_ERR_UNSUPPORTED, std::string(name) + ": paged rows are not 16-byte aligned");
        a.pg.Lp = 1;                 // L = page number within the piece
        a.pg.X0 = p.v.base; a.pg.Xb = sb; a.pg.Xh = sh; a.pg.Xo = st;
      }
      if (!(page_rows % kTile == 0 || page_rows >= rows)) return fail(VT_ERR_UNSUPPORTED, std::string(name) + ": pages must hold a multiple of 32 rows");
      const Table& tb = d.tables[T->table];
      if (!tb.dev) return fail(VT_ERR_INVALID_ARG, std::string(name) + ": page table without a device pointer");
      if (sb % 8 || sh % 8 || T->stride % 8) return fail(VT_ERR_UNSUPPORTED, std::string(name) + ": paged rows are not 16-byte aligned");
      a.ptr = static_cast<const char*>(src.ptr);
      a.pg.tab = tb.dev + T->table_off;
      a.pg.ps = T->stride;
      a.pg.W = make_fastdiv((uint32_t)W);
      a.pg.page = make_fastdiv((uint32_t)page_rows);
      // the closed form above against the descriptor's own evaluator, on sampled rows
      if (!tb.host.empty()) {
        const int64_t Hq = d.shape[1];
        uint64_t rng = 0x9E3779B97F4A7C15ull;
        for (int smp = 0; smp < 48; ++smp) {
          rng = rng * 6364136223846793005ull + 1442695040888963407ull;
          const int64_t bb = (int64_t)((rng >> 33) % (uint64_t)d.shape[0]);
          const int64_t hh = (int64_t)((rng >> 13) % (uint64_t)Hq);
          const int64_t rr = smp == 0 ? rows - 1 : (int64_t)((rng >> 23) % (uint64_t)rows);
          const int64_t local[4] = {bb, hh, rr, 0};
          const int64_t want = eval_view(d, p.v, local);
          const int64_t hs = hh / (G * a_hdiv), pgi = rr / page_rows, row = rr - pgi * page_rows;
          const int64_t L = a.pg.L0 + bb * a.pg.Lb + hs * a.pg.Lh + pgi * a.pg.Lp + row * a.pg.Lo;
          const int64_t X = a.pg.X0 + bb * a.pg.Xb + hs * a.pg.Xh + row * a.pg.Xo;
          const int64_t got = (int64_t)tb.host[T->table_off + L / W] * T->stride + L % W + X;
          if (got != want) return fail(VT_ERR_UNSUPPORTED, std::string(name) + ": paged map does not have the page-table form");
        }
      }
    }
    a.page_rows = page_rows;
    if (st * esz >= (1ll << 32) || st < 0) return fail(VT_ERR_UNSUPPORTED, std::string(name) + ": context stride too large");
    a.st = (uint32_t)(st * esz);
    a.t_lo = (int32_t)p.lo[2];
    a.t_hi = (int32_t)p.hi[2];
    if ((uintptr_t)a.ptr % 16 || a.sb % 16 || a.sh % 16 || a.st % 16)
      return fail(VT_ERR_UNSUPPORTED, std::string(name) + ": rows are not 16-byte aligned");
  }
  if (expect != d.shape[2]) return fail(VT_ERR_UNSUPPORTED, std::string(name) + ": pieces do not cover the context");
  return VT_OK;
}

// About two workgroups per compute unit, and at least one 32-row tile per wave.
int choose_splits(int units, int S, int n_splits) {
  if (n_splits > 0) return n_splits;
  int max_splits = std::max(1, (S + 127) / 128);
  int want = std::max(1, (512 + units - 1) / units);
  return std::min(want, max_splits);
}

constexpr int kWaves = 4;

}  // namespace

static size_t ticket_bytes(int64_t B, int64_t Hq) { return (size_t)((B * Hq * 4 + 255) / 256 * 256); }

// Workspace of vt_decode_attn_static: a fixed array in the code object's own device memory, so
// that the call needs no allocation.  Every GPU the library runs on holds its own copy at its
// own address; the name below is only a host-side handle, the address is asked from the runtime
// once per device and kept.
constexpr size_t kScratchBytes = 4u << 20;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
static void* g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mutex;

static int scratch_address(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
    return fail(VT_ERR_DEVICE, "vt_decode_attn_static: no current device (or device number above 63)");
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p)
      return fail(VT_ERR_DEVICE, std::string("vt_decode_attn_static: hipGetSymbolAddress failed: ") + hipGetErrorString(e));
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return VT_OK;
}

extern "C" {

size_t vt_decode_attn_workspace(int B, int Hq, int D, int S, int n_splits) {
  if (B < 1 || Hq < 1 || D < 1 || S < 1 || n_splits < 0) return 0;
  // an upper bound that does not need the grouping: the fewest kv heads (16 query heads each)
  // give the most splits
  int ns = choose_splits(B * std::max(1, Hq / 16), S, n_splits);
  return ticket_bytes(B, Hq) + (size_t)B * Hq * ns * ((size_t)D + 2) * sizeof(float);
}

int vt_decode_attn_workspace_init(void* workspace, size_t workspace_bytes, void* stream) {
  if (!workspace || (uintptr_t)workspace % 16) return fail(VT_ERR_INVALID_ARG, "vt_decode_attn_workspace_init: NULL or misaligned workspace");
  size_t words = workspace_bytes / 4;
  if (words == 0) return VT_OK;
  hipLaunchKernelGGL(k_zero_words, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, (hipStream_t)stream, (uint32_t*)workspace, words);
  return check_launch("vt_decode_attn_workspace_init");
}

// Everything vt_decode_attn decides on the host: group size, segments, paged operands, splits.
// Fills P except for the workspace, output and scale fields.
static int plan_attention(const vt_desc* Q, const vt_desc* K, const vt_desc* V, int n_splits, AttnParams& P) {
  if (!Q || !K || !V) return fail(VT_ERR_INVALID_ARG, "vt_decode_attn: NULL argument");
  if (Q->dtype == VT_F32 || K->dtype != Q->dtype || V->dtype != Q->dtype)
    return fail(VT_ERR_INVALID_ARG, "vt_decode_attn: Q, K, V must share a 16-bit dtype");
  if (Q->shape.size() != 4 || K->shape.size() != 4 || V->shape != K->shape)
    return fail(VT_ERR_SHAPE, "vt_decode_attn: Q must be [B,Hq,1,D], K and V [B,Hq,S,D]");
  const int64_t B = K->shape[0], Hq = K->shape[1], S = K->shape[2], D = K->shape[3];
  if (Q->shape[0] != B || Q->shape[1] != Hq || Q->shape[2] != 1 || Q->shape[3] != D)
    return fail(VT_ERR_SHAPE, "vt_decode_attn: Q does not match K");
  if (D != kD) return fail(VT_ERR_UNSUPPORTED, "vt_decode_attn: head dim must be 128");
  if (B > 65535 || Hq > 65535 || S >= (1ll << 31)) return fail(VT_ERR_UNSUPPORTED, "vt_decode_attn: extents too large");
  if (n_splits < 0) return fail(VT_ERR_INVALID_ARG, "vt_decode_attn: n_splits < 0");

  // query heads that share K/V rows: common broadcast factor over all pieces of K and V
  int64_t G = 0;
  for (const vt_desc* X : {K, V})
    for (const Piece& p : X->pieces) {
      int64_t f = broadcast_factor(p.v.groups[1]);
      G = G == 0 ? f : std::gcd(G, f);
    }
  if (G < 1) G = 1;
  {
    // the matrix-core tile holds at most 16 heads: the largest group size that divides the
    // broadcast factor every piece shares (so that a group never straddles two stored heads)
    int64_t g = std::min<int64_t>(G, 16);
    while (G % g || Hq % g) --g;
    G = g;
  }
  memset(&P, 0, sizeof(P));
  AttnOperand ko, vo;
  int rc = plan_operand(*K, "K", G, &ko);
  if (rc != VT_OK) return rc;
  rc = plan_operand(*V, "V", G, &vo);
  if (rc != VT_OK) return rc;
  {  // segments = union of the piece boundaries of K and V
    int ik = 0, iv = 0, t = 0, n = 0;
    while (t < S) {
      while (ko.pc[ik].t_hi <= t) ++ik;
      while (vo.pc[iv].t_hi <= t) ++iv;
      int e = std::min(ko.pc[ik].t_hi, vo.pc[iv].t_hi);
      if (n >= kMaxSegs) return fail(VT_ERR_UNSUPPORTED, "vt_decode_attn: more than 8 context segments");
      AttnSeg& sg = P.seg[n++];
      sg.k = ko.pc[ik].ptr + (int64_t)(t - ko.pc[ik].t_lo) * ko.pc[ik].st;
      sg.v = vo.pc[iv].ptr + (int64_t)(t - vo.pc[iv].t_lo) * vo.pc[iv].st;
      sg.k_sb = ko.pc[ik].sb; sg.k_sh = ko.pc[ik].sh; sg.k_st = ko.pc[ik].st; sg.k_hdiv = ko.pc[ik].hdiv;
      sg.v_sb = vo.pc[iv].sb; sg.v_sh = vo.pc[iv].sh; sg.v_st = vo.pc[iv].st; sg.v_hdiv = vo.pc[iv].hdiv;
      sg.t_lo = t;
      sg.t_hi = e;
      // paged operands: the segment must start on a page boundary and on the 32-row tile grid,
      // so that no tile straddles two pages
      for (int which = 0; which < 2; ++which) {
        const PlanPiece& pc = which == 0 ? ko.pc[ik] : vo.pc[iv];
        PagedOperand& dst = which == 0 ? sg.kp : sg.vp;
        dst = pc.pg;
        if (!pc.pg.tab) continue;
        sg.paged |= 1 << which;
        const int64_t rel = t - pc.t_lo;
        if (rel % pc.page_rows || t % kTile) return fail(VT_ERR_UNSUPPORTED, "vt_decode_attn: a paged operand's segment does not start on a page boundary");
        dst.L0 += rel / pc.page_rows * pc.pg.Lp;
        (which == 0 ? sg.k : sg.v) = pc.ptr;
      }
      t = e;
    }
    P.n_seg = n;
  }
  // Q: one piece, one stage, contiguous rows
  if (Q->pieces.size() != 1 || !Q->pieces[0].v.lower.empty()) return fail(VT_ERR_UNSUPPORTED, "Q: must be a single strided piece");
  {
    const Piece& p = Q->pieces[0];
    int64_t sb, sh, sd;
    if (!single_plain(p.v.groups[0], &sb) || !single_plain(p.v.groups[1], &sh) || !single_plain(p.v.groups[3], &sd) || sd != 1)
      return fail(VT_ERR_UNSUPPORTED, "Q: batch and head dims must each be one strided digit, rows contiguous");
    const vt_source& src = Q->sources[p.src];
    if (!src.ptr) return fail(VT_ERR_INVALID_ARG, "Q: source without a device pointer");
    P.q_ptr = static_cast<const char*>(src.ptr) + p.v.base * 2;
    P.q_sb = sb * 2;
    P.q_sh = sh * 2;
    if ((uintptr_t)P.q_ptr % 16 || P.q_sb % 16 || P.q_sh % 16) return fail(VT_ERR_UNSUPPORTED, "Q: rows are not 16-byte aligned");
  }
  const int Hkv = (int)(Hq / G);
  const int ns = choose_splits((int)B * Hkv, (int)S, n_splits);
  int rows = (int)((S + ns - 1) / ns);
  rows = (rows + kTile - 1) / kTile * kTile;
  const int ns_eff = (int)((S + rows - 1) / rows);
  if ((int64_t)ns_eff * G * 2 > kWaves * kTile * 64) return fail(VT_ERR_UNSUPPORTED, "vt_decode_attn: too many splits");
  P.B = (int)B;
  P.Hkv = Hkv;
  P.G = (int)G;
  P.S = (int)S;
  P.n_splits = ns_eff;
  P.rows_per_split = rows;
  return VT_OK;
}

int vt_decode_attn_plan(const vt_desc* Q, const vt_desc* K, const vt_desc* V, int n_splits, int* group_size,
                        int* n_segments, int* splits, int* paged_segments) {
  AttnParams P;
  int rc = plan_attention(Q, K, V, n_splits, P);
  if (rc != VT_OK) return rc;
  if (group_size) *group_size = P.G;
  if (n_segments) *n_segments = P.n_seg;
  if (splits) *splits = P.n_splits;
  if (paged_segments) {
    *paged_segments = 0;
    for (int i = 0; i < P.n_seg; ++i) *paged_segments += P.seg[i].paged ? 1 : 0;
  }
  return VT_OK;
}

// Everything after the plan: workspace carving, launch.  `clear_tickets` queues a small fill
// kernel over the arrival counters first (for a workspace whose previous contents are not known
// to be zero).
static int launch_attention(const vt_desc* Q, const vt_desc* K, const vt_desc* V, float scale, void* out, float* lse,
                            void* workspace, size_t workspace_bytes, int n_splits, bool clear_tickets,
                            const char* who, void* stream) {
  if (!out || !workspace) return fail(VT_ERR_INVALID_ARG, std::string(who) + ": NULL argument");
  AttnParams P;
  int rc = plan_attention(Q, K, V, n_splits, P);
  if (rc == VT_ERR_UNSUPPORTED) {
    // maps or a head dim the planned kernel does not take: the generic kernel, if the shapes allow
    const std::string why = vt_last_error();
    const int64_t B = K->shape[0], Hq = K->shape[1], S = K->shape[2], D = K->shape[3];
    DevDesc DQ, DK, DV;
    int64_t o1, i1, o2, i2, o3, i3;
    if (D > 1024 || B > 65535 || to_device(*Q, &DQ, &o1, &i1) != VT_OK || to_device(*K, &DK, &o2, &i2) != VT_OK ||
        to_device(*V, &DV, &o3, &i3) != VT_OK || o1 != 1 || o2 != 1 || o3 != 1)
      return fail(VT_ERR_UNSUPPORTED, why);
    hipStream_t gs = (hipStream_t)stream;
    dim3 grid((unsigned)Hq, (unsigned)B);
    if (Q->dtype == VT_BF16) hipLaunchKernelGGL((k_decode_attn_generic<bf16_t>), grid, dim3(256), 0, gs, DQ, DK, DV, (bf16_t*)out, lse, (int)Hq, (int)S, (int)D, scale);
    else hipLaunchKernelGGL((k_decode_attn_generic<f16_t>), grid, dim3(256), 0, gs, DQ, DK, DV, (f16_t*)out, lse, (int)Hq, (int)S, (int)D, scale);
    return check_launch(who);
  }
  if (rc != VT_OK) return rc;
  const int64_t B = P.B, Hq = (int64_t)P.Hkv * P.G;
  const int ns_eff = P.n_splits, Hkv = P.Hkv;
  const size_t need = ticket_bytes(B, Hq) + (size_t)B * Hq * ns_eff * ((size_t)kD + 2) * sizeof(float);
  if (workspace_bytes < need)
    return fail(VT_ERR_INVALID_ARG, std::string(who) + ": workspace too small (" + std::to_string(need) + " bytes needed, " +
                                        std::to_string(workspace_bytes) + " available)");
  if ((uintptr_t)workspace % 16 || (uintptr_t)out % 8) return fail(VT_ERR_INVALID_ARG, std::string(who) + ": misaligned workspace or out (16 and 8 bytes)");
  P.scale_log2 = scale * 1.4426950408889634f;
  P.tickets = static_cast<uint32_t*>(workspace);
  P.ws_ml = reinterpret_cast<float*>(static_cast<char*>(workspace) + ticket_bytes(B, Hq));
  P.ws_o = P.ws_ml + (size_t)B * Hq * ns_eff * 2;
  P.out = out;
  P.lse = lse;
  hipStream_t st = (hipStream_t)stream;
  if (clear_tickets) {
    const size_t words = ticket_bytes(B, Hq) / 4;
    hipLaunchKernelGGL(k_zero_words, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, st, P.tickets, words);
    rc = check_launch(who);
    if (rc != VT_OK) return rc;
  }
  dim3 grid(ns_eff, Hkv, (unsigned)B);
  // compiled for three waves per SIMD (two workgroups of four waves per compute unit and room for
  // a third); the build for two measures the same on the benchmark's shape
  if (Q->dtype == VT_BF16) hipLaunchKernelGGL((k_decode_attn<bf16_t, kWaves, 3>), grid, dim3(kWaves * 64), 0, st, P);
  else hipLaunchKernelGGL((k_decode_attn<f16_t, kWaves, 3>), grid, dim3(kWaves * 64), 0, st, P);
  return check_launch(who);
}

int vt_decode_attn(const vt_desc* Q, const vt_desc* K, const vt_desc* V, float scale, void* out, float* lse,
                   void* workspace, size_t workspace_bytes, int n_splits, void* stream) {
  return launch_attention(Q, K, V, scale, out, lse, workspace, workspace_bytes, n_splits, false, "vt_decode_attn", stream);
}

size_t vt_decode_attn_static_capacity(void) { return kScratchBytes; }

int vt_decode_attn_static(const vt_desc* Q, const vt_desc* K, const vt_desc* V, float scale, void* out, float* lse,
                          int n_splits, void* stream) {
  void* ws = nullptr;
  int rc = scratch_address(&ws);
  if (rc != VT_OK) return rc;
  return launch_attention(Q, K, V, scale, out, lse, ws, kScratchBytes, n_splits, true, "vt_decode_attn_static", stream);
}

}  // extern "C"
